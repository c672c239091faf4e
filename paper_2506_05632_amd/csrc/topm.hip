// Algorithm 1 on candidate lists (paper Section 4.4: with top-K sampling only M << N tokens
// per distribution survive).  A row is a few hundred (token id, value) pairs, so there is
// nothing to prune: one workgroup per row evaluates every key exactly in fp64 -- the random
// word of (row, k, token id) from its two Philox blocks, ln S - x/T + ln sum exp(x/T) for
// logits and log-weights, S/p for probabilities -- and reduces with the usual tie rule
// (smaller key, then smaller token id, then smaller k).
#include "scan.hpp"

namespace llc {
namespace {

constexpr int kTopmMaxK = 1024;

struct Best {
  double key;
  int id, k;
  double sec;  // the smallest key seen at another id (the runner-up that a near-tie is judged by)
};

// a beats b: smaller key; equal keys: smaller id, then smaller k.  id < 0 = nothing yet.
__device__ __forceinline__ bool better(const Best &a, const Best &b) {
  if (a.id < 0) return false;
  if (b.id < 0) return true;
  if (a.key != b.key) return a.key < b.key;
  if (a.id != b.id) return a.id < b.id;
  return a.k < b.k;
}

// Fold one more state into a running one.  The loser's winner is a runner-up candidate unless it
// sits at the winner's id; the loser's own runner-up is then the candidate (it excludes that id).
__device__ __forceinline__ void fold(Best &v, const Best &o) {
  if (o.id < 0) return;
  if (better(o, v)) {
    double sec = o.sec;
    if (v.id >= 0) sec = fmin(sec, v.id != o.id ? v.key : v.sec);
    v = o;
    v.sec = sec;
  } else {
    v.sec = fmin(v.sec, o.id != v.id ? o.key : o.sec);
  }
}

__device__ __forceinline__ Best wave_best(Best v) {
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) {
    Best o;
    o.key = __shfl_xor(v.key, d);
    o.id = __shfl_xor(v.id, d);
    o.k = __shfl_xor(v.k, d);
    o.sec = __shfl_xor(v.sec, d);
    fold(v, o);
  }
  return v;
}

// Relative distance (in S/p) between the winner and the runner-up below 1e-6 (log-domain keys differ
// by the log of the ratio).
__device__ __forceinline__ bool near_tie(const Best &v, bool probs) {
  if (v.id < 0 || !(v.sec < __builtin_huge_val())) return false;
  if (!probs) return expm1(v.sec - v.key) < 1e-6;
  return v.key > 0.0 ? (v.sec - v.key) / v.key < 1e-6 : !(v.sec > 0.0);
}

__device__ __forceinline__ float widen_at(const void *base, int dtype, long long off) {
  if (dtype == LLC_F32) return reinterpret_cast<const float *>(base)[off];
  return __uint_as_float((uint32_t) reinterpret_cast<const uint16_t *>(base)[off] << 16);
}

// does the entry carry mass?  (empty slot, NaN, +inf, and for probabilities <= 0: no)
__device__ __forceinline__ bool has_mass(int id, float v, bool probs) {
  if (id < 0) return false;
  if (probs) return v > 0.0f && v < __builtin_huge_valf();
  return v < __builtin_huge_valf() && v > -__builtin_huge_valf();
}

__device__ __forceinline__ uint32_t word_of(uint32_t id, uint32_t k, uint32_t row_lo, uint32_t row_hi,
                                            uint32_t k0, uint32_t k1) {
  uint32_t up[4], lo[4];
  philox_block(row_lo, id >> 2, row_hi, k >> 1, k0, k1, up);
  philox_block(row_lo, id >> 2, row_hi, (k >> 1) | kLowBlock, k0, k1, lo);
  const int j = (int)(id & 3u);
  const uint32_t uw = j == 0 ? up[0] : j == 1 ? up[1] : j == 2 ? up[2] : up[3];
  const uint32_t lw = j == 0 ? lo[0] : j == 1 ? lo[1] : j == 2 ? lo[2] : lo[3];
  return element_word(uw, lw, (int)(k & 1u));
}

__global__ void __launch_bounds__(256) topm_kernel(const TopmParams p) {
  __shared__ double s_lse[kTopmMaxK + 1];  // ln sum exp(x/T) of draft list k, of the target list at [K]
  __shared__ int s_x[kTopmMaxK];
  __shared__ Best s_pool[4];
  __shared__ int s_match, s_y;
  __shared__ unsigned long long s_evals;
  __shared__ unsigned s_degenerate, s_near;

  const long long b = blockIdx.x;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int K = p.K;
  const bool probs = p.kind == LLC_PROBS;
  const bool logits = p.kind == LLC_LOGITS;
  const unsigned long long row = p.row_offset + (unsigned long long)b;
  const uint32_t row_lo = (uint32_t)row, row_hi = (uint32_t)(row >> 32);
  const int32_t *t_ids = p.target_ids + b * p.target_stride_b;
  const long long t_off = b * p.target_stride_b;
  const float inf = __builtin_huge_valf();

  if (tid == 0) { s_match = 0x7FFFFFFF; s_evals = 0; s_degenerate = 0; s_near = 0; }

  // ---- normalisers: list l < K is draft l, list K the target; one wavefront per list
  if (!probs) {
    const bool one_list = p.draft_stride_k == 0 && p.temp_draft == nullptr;
    for (int l = wave; l <= K; l += 4) {
      if (l < K && one_list && l > 0) continue;  // filled from list 0 below
      const bool target = l == K;
      const int M = target ? p.Mt : p.Md;
      const long long off = target ? t_off : b * p.draft_stride_b + (long long)l * p.draft_stride_k;
      const int32_t *ids = target ? t_ids : p.draft_ids + off;
      const void *val = target ? p.target_val : p.draft_val;
      float T = 1.0f;
      if (logits) T = target ? p.temp_target : (p.temp_draft != nullptr ? p.temp_draft[l] : p.temp_draft_all);
      float m = -inf;
      for (int e = lane; e < M; e += 64) {
        const float v = widen_at(val, p.dtype, off + e);
        if (has_mass(ids[e], v, false)) m = fmaxf(m, v);
      }
#pragma unroll
      for (int d = 32; d >= 1; d >>= 1) m = fmaxf(m, __shfl_xor(m, d));
      double sum = 0.0;
      if (m > -inf) {
        for (int e = lane; e < M; e += 64) {
          const float v = widen_at(val, p.dtype, off + e);
          if (has_mass(ids[e], v, false)) sum += exp(((double)v - (double)m) / (double)T);
        }
      }
#pragma unroll
      for (int d = 32; d >= 1; d >>= 1) sum += __shfl_xor(sum, d);
      if (lane == 0) {
        const bool ok = m > -inf && T > 0.0f && T < inf;
        s_lse[l] = ok ? (double)m / (double)T + log(sum) : -__builtin_huge_val();
      }
    }
    __syncthreads();
    if (one_list)
      for (int k = 1 + tid; k < K; k += 256) s_lse[k] = s_lse[0];
  }
  __syncthreads();

  unsigned long long evals = 0;
  // ---- draft side: one wavefront per list, lanes over its entries
  for (int k = wave; k < K; k += 4) {
    const long long off = b * p.draft_stride_b + (long long)k * p.draft_stride_k;
    const int32_t *ids = p.draft_ids + off;
    float T = 1.0f;
    if (logits) T = p.temp_draft != nullptr ? p.temp_draft[k] : p.temp_draft_all;
    const bool t_ok = T > 0.0f && T < inf;
    const double lse = probs ? 0.0 : s_lse[k];
    Best best = {__builtin_huge_val(), -1, k, __builtin_huge_val()};
    for (int e = lane; e < p.Md; e += 64) {
      const int id = ids[e];
      const float v = widen_at(p.draft_val, p.dtype, off + e);
      if (!t_ok || !has_mass(id, v, probs)) continue;
      const double S = exact_race_time(word_of((uint32_t)id, (uint32_t)k, row_lo, row_hi, p.seed_lo, p.seed_hi));
      Best c = {probs ? S / (double)v : log(S) - (double)v / (double)T + lse, id, k, __builtin_huge_val()};
      ++evals;
      fold(best, c);
    }
    best = wave_best(best);
    if (lane == 0) {
      if (near_tie(best, probs)) atomicAdd(&s_near, 1u);
      s_x[k] = best.id;
      p.X[b * K + k] = best.id;
      if (p.keyX != nullptr)
        p.keyX[b * K + k] = best.id >= 0 ? (float)(probs ? best.key : exp(best.key)) : inf;
      if (best.id < 0) atomicAdd(&s_degenerate, 1u);
    }
  }

  // ---- pool: all (k, target entry) pairs over the workgroup
  {
    const double lse = probs ? 0.0 : s_lse[K];
    const float T = logits ? p.temp_target : 1.0f;
    Best best = {__builtin_huge_val(), -1, 0, __builtin_huge_val()};
    const long long items = (long long)K * p.Mt;
    for (long long it = tid; it < items; it += 256) {
      const int k = (int)(it / p.Mt), e = (int)(it % p.Mt);
      const int id = t_ids[e];
      const float v = widen_at(p.target_val, p.dtype, t_off + e);
      if (!has_mass(id, v, probs)) continue;
      const double S = exact_race_time(word_of((uint32_t)id, (uint32_t)k, row_lo, row_hi, p.seed_lo, p.seed_hi));
      Best c = {probs ? S / (double)v : log(S) - (double)v / (double)T + lse, id, k, __builtin_huge_val()};
      ++evals;
      fold(best, c);
    }
    best = wave_best(best);
    if (lane == 0) s_pool[wave] = best;
  }
  __syncthreads();
  if (tid == 0) {
    Best best = s_pool[0];
    for (int w = 1; w < 4; ++w) fold(best, s_pool[w]);
    if (near_tie(best, probs)) atomicAdd(&s_near, 1u);
    s_y = best.id;
    p.Y[b] = best.id;
    if (p.keyY != nullptr) p.keyY[b] = best.id >= 0 ? (float)(probs ? best.key : exp(best.key)) : inf;
    if (best.id < 0) atomicAdd(&s_degenerate, 1u);
  }
  __syncthreads();
  const int y = s_y;
  if (y >= 0)
    for (int k = tid; k < K; k += 256)
      if (s_x[k] == y) atomicMin(&s_match, k);
  if (p.stats != nullptr && evals) atomicAdd(&s_evals, evals);
  __syncthreads();
  if (tid == 0) {
    const bool hit = s_match != 0x7FFFFFFF;
    p.accept[b] = hit ? 1 : 0;
    if (p.match_k != nullptr) p.match_k[b] = hit ? s_match : -1;
    if (p.stats != nullptr) {
      if (s_evals) atomicAdd(&p.stats->exact_evals, s_evals);
      if (s_degenerate) atomicAdd(&p.stats->degenerate, (unsigned long long)s_degenerate);
      if (s_near) atomicAdd(&p.stats->near_ties, (unsigned long long)s_near);
    }
  }
}

}  // namespace

hipError_t launch_topm(hipStream_t s, const TopmParams &p) {
  if (p.B == 0) return hipSuccess;
  hipLaunchKernelGGL(topm_kernel, dim3((unsigned)p.B), dim3(256), 0, s, p);
  return hipGetLastError();
}

}  // namespace llc
