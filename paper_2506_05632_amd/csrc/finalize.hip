// Finalize: merge the per-chunk partial argmins of a row and take Algorithm 1's
// last step, accept = [Y in {X^(1..K)}] (paper Section 3).  Also the row
// normalisers ln sum exp(x/T) that turn log-domain keys into S/p with p
// normalised (Section 3 defines p and q as distributions; Appendix C normalises
// the importance weights the same way).
#include "finalize_row.hpp"

namespace llc {

namespace {

__global__ void __launch_bounds__(64) finalize_kernel(const FinalizeParams p) {
  __shared__ FinalizeShared sh;
  finalize_row<64>(p, (long long)blockIdx.x, (int)threadIdx.x, sh);
}

// ln sum_i exp(x_i / T) of one input row, in one pass over the row: every thread keeps a
// running maximum and the sum of exp relative to it (fp32 terms, four at a time, into an fp64
// running sum that is rescaled when the maximum moves).  NaN and +inf entries carry no mass.
template <typename E>
__device__ __forceinline__ void load_group(const E *row, int i0, int V, bool vec, float (&v)[4]);
template <>
__device__ __forceinline__ void load_group<float>(const float *row, int i0, int V, bool vec, float (&v)[4]) {
  if (vec && i0 + 3 < V) {
    const float4 t = *reinterpret_cast<const float4 *>(row + i0);
    v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w;
  } else {
#pragma unroll
    for (int j = 0; j < 4; ++j) v[j] = (i0 + j < V) ? row[i0 + j] : -__builtin_huge_valf();
  }
}
template <>
__device__ __forceinline__ void load_group<uint16_t>(const uint16_t *row, int i0, int V, bool vec, float (&v)[4]) {
  if (vec && i0 + 3 < V) {
    const uint2 t = *reinterpret_cast<const uint2 *>(row + i0);
    v[0] = __uint_as_float(t.x << 16);
    v[1] = __uint_as_float(t.x & 0xFFFF0000u);
    v[2] = __uint_as_float(t.y << 16);
    v[3] = __uint_as_float(t.y & 0xFFFF0000u);
  } else {
#pragma unroll
    for (int j = 0; j < 4; ++j)
      v[j] = (i0 + j < V) ? __uint_as_float((uint32_t)row[i0 + j] << 16) : -__builtin_huge_valf();
  }
}

template <typename E>
__global__ void __launch_bounds__(256) lse_kernel(const LseParams p) {
  __shared__ float s_max[4];
  __shared__ double s_sum[4];
  const int kd = p.per_k ? p.K : 1;  // distinct draft rows
  const int nd = p.with_drafts ? kd : 0;
  const int per_b = nd + (p.with_target ? 1 : 0);
  const long long b = blockIdx.x / (unsigned)per_b;
  int which = (int)(blockIdx.x % (unsigned)per_b);
  if (which == nd) which = kd;  // kd = the target row
  const int tid = threadIdx.x;
  const E *row;
  float T;
  long long extra = 0;
  if (p.draft_row_off != nullptr) {
    extra = p.draft_row_off[b];
    if (extra < 0) return;  // the row is not wanted
  }
  if (which == kd) {
    row = reinterpret_cast<const E *>(p.target) + p.map.target_off(b);
    T = p.temp_target;
  } else {
    row = reinterpret_cast<const E *>(p.draft) + p.map.draft_off(b) + extra + (long long)which * p.draft_stride_k;
    T = p.temp_draft != nullptr ? p.temp_draft[which] : p.temp_draft_all;
  }
  if (!p.is_logits) T = 1.0f;
  const float inf = __builtin_huge_valf();
  const bool vec = p.vector_loads != 0;
  // log2(e)/T as a two-float sum, so that the exponent carries no systematic rounding of 1/T
  const double c64 = 1.4426950408889634 / (double)T;
  const float c_hi = (float)c64;
  const float c_lo = (float)(c64 - (double)c_hi);

  float m = -inf;     // running maximum of the entries that carry mass
  double sum = 0.0;   // sum of exp((x - m)/T) over the entries seen
  const int G = (p.V + 3) >> 2;
  // binned candidates: a draft row only lives on the announced bin (the target row is not masked)
  const bool binned = p.bins != nullptr && which != kd;
  const uint8_t *brow = binned ? p.bins + b * p.bins_stride_b : nullptr;
  int announced = -1;
  if (binned) {
    const int y = p.bin_of[b];
    if (y >= 0 && y < p.V) announced = (int)brow[y];
  }
  for (int g = tid; g < G; g += 256) {
    float v[4];
    load_group<E>(row, g * 4, p.V, vec, v);
    if (binned) {
#pragma unroll
      for (int j = 0; j < 4; ++j)
        if (g * 4 + j < p.V && (int)brow[g * 4 + j] != announced) v[j] = -inf;
    }
    float gm = -inf;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      if (!(v[j] < inf)) v[j] = -inf;  // NaN, +inf: no mass
      gm = fmaxf(gm, v[j]);
    }
    if (gm > m) {
      if (m > -inf) {
        const float d = m - gm;
        sum *= (double)__builtin_amdgcn_exp2f(fmaf(d, c_hi, d * c_lo));
      }
      m = gm;
    }
    if (m > -inf) {
      float part = 0.0f;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        // <= 0; entries without mass are clamped to a finite distance whose term is exactly 0
        // (an infinite one would meet c_lo's sign in the two-float product)
        const float d = fmaxf(v[j] - m, -65536.0f);
        part += __builtin_amdgcn_exp2f(fmaf(d, c_hi, d * c_lo));
      }
      sum += (double)part;
    }
  }
  float bm = m;
  for (int d = 32; d >= 1; d >>= 1) bm = fmaxf(bm, __shfl_xor(bm, d));
  if ((tid & 63) == 0) s_max[tid >> 6] = bm;
  __syncthreads();
  bm = fmaxf(fmaxf(s_max[0], s_max[1]), fmaxf(s_max[2], s_max[3]));
  if (m > -inf && m < bm) sum *= exp2(((double)m - (double)bm) * c64);
  if (!(m > -inf)) sum = 0.0;
  for (int d = 32; d >= 1; d >>= 1) sum += __shfl_xor(sum, d);
  if ((tid & 63) == 0) s_sum[tid >> 6] = sum;
  __syncthreads();
  if (tid == 0) {
    sum = (s_sum[0] + s_sum[1]) + (s_sum[2] + s_sum[3]);
    const bool ok = (bm > -inf) && (T > 0.0f) && (T < inf);
    const double lse = ok ? (double)bm / (double)T + log(sum) : -__builtin_huge_val();
    double *out = p.lse + b * (p.K + 1);
    if (which == kd) {
      out[p.K] = lse;
    } else if (kd == 1) {
      for (int k = 0; k < p.K; ++k) out[k] = lse;
    } else {
      out[which] = lse;
    }
  }
}

// Algorithm 2, the loop over positions (Section 4.2): Y_j is the candidate of the viable draft
// with the smallest key (ties: smaller index, then smaller k); drafts whose token differs from
// Y_j stop being viable; the loop ends when none is left or after the bonus position.
// One wavefront per sequence, lane k holds draft k (K <= 64); positions are fetched eight at a
// time so that the loop itself only waits for memory once per eight positions.
__global__ void __launch_bounds__(64) verify_kernel(const VerifyParams p) {
  const long long s = blockIdx.x;
  const int lane = threadIdx.x;
  const int L = p.L, K = p.K;
  const int32_t *cand = p.cand + s * (L + 1) * K;
  const double *ckey = p.cand_key + s * (L + 1) * K;
  const double *csec = p.cand_sec + s * (L + 1) * K;
  int32_t *Y = p.Y + s * (L + 1);
  float *keyY = p.keyY != nullptr ? p.keyY + s * (L + 1) : nullptr;
  bool viable = lane < K;
  bool done = false;
  int n = 0;
  unsigned long long near = 0;
  for (int j0 = 0; j0 <= L && !done; j0 += 8) {
    double key[8], sec[8];
    int idx[8], tok[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int j = j0 + u;
      key[u] = sec[u] = __builtin_huge_val(); idx[u] = -1; tok[u] = -2;
      if (j <= L && lane < K) {
        key[u] = ckey[(long long)j * K + lane];
        sec[u] = csec[(long long)j * K + lane];
        idx[u] = cand[(long long)j * K + lane];
        if (j < L) tok[u] = p.tokens[s * p.tok_stride_s + (long long)j * p.tok_stride_j + lane];
      }
    }
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int j = j0 + u;
      if (j > L || done) break;  // uniform
      double bkey = (viable && idx[u] >= 0) ? key[u] : __builtin_huge_val();
      int bidx = (viable && idx[u] >= 0) ? idx[u] : -1;
      int bk = lane;
#pragma unroll
      for (int d = 32; d >= 1; d >>= 1) {
        const double okey = __shfl_xor(bkey, d);
        const int oidx = __shfl_xor(bidx, d);
        const int ok = __shfl_xor(bk, d);
        if (beats(okey, oidx, ok, bkey, bidx, bk)) { bkey = okey; bidx = oidx; bk = ok; }
      }
      if (lane == 0) {
        Y[j] = bidx;
        if (keyY != nullptr) keyY[j] = bidx >= 0 ? (float)exp(bkey) : __builtin_huge_valf();
      }
      if (p.stats != nullptr && bidx >= 0) {
        // the pool's runner-up at another index: a viable draft whose own winner sits at the
        // pool's index offers its own runner-up, the others their winner
        double r = __builtin_huge_val();
        if (viable && idx[u] >= 0) r = idx[u] != bidx ? key[u] : sec[u];
#pragma unroll
        for (int d = 32; d >= 1; d >>= 1) r = fmin(r, __shfl_xor(r, d));
        if (near_tie(bkey, r, 1)) ++near;
      }
      n = j + 1;
      if (j == L) { done = true; break; }
      viable = viable && tok[u] == bidx;
      if (__ballot(viable) == 0ull) done = true;
    }
  }
  if (lane == 0 && near) atomicAdd(&p.stats->near_ties, near);
  for (int j = n + lane; j <= L; j += 64) {
    Y[j] = -1;
    if (keyY != nullptr) keyY[j] = __builtin_huge_valf();
  }
  if (lane == 0) p.n_out[s] = n;
  if (p.active != nullptr && lane < K) p.active[s * K + lane] = viable ? 1 : 0;
}

// One position of the loop in its strong form (Appendix B).  One wavefront per sequence, lane k
// holds draft k.  At j == 0 the state is set up (every draft viable).
__global__ void __launch_bounds__(64) strong_step_kernel(const StrongStepParams p) {
  const long long s = blockIdx.x;
  const int lane = threadIdx.x;
  const int L = p.L, K = p.K, j = p.j;
  int32_t *Y = p.Y + s * (L + 1);
  float *keyY = p.keyY != nullptr ? p.keyY + s * (L + 1) : nullptr;
  bool viable = lane < K;
  bool running = true;
  if (j == 0 && p.tau_all != nullptr) {
    // the scans of the later positions find their rows' running bests reset
    for (int t = lane; t < L * (K + 1); t += 64)
      p.tau_all[((long long)(t / (K + 1)) * p.S + s) * (K + 1) + t % (K + 1)] = 0x7F800000;
  }
  if (j > 0) {
    viable = lane < K && p.viable[s * K + lane] != 0;
    running = p.running[s] != 0;
  }
  if (!running) {  // uniform: the loop ended at an earlier position
    if (lane == 0) {
      Y[j] = -1;
      if (keyY != nullptr) keyY[j] = __builtin_huge_valf();
      p.next_off[s] = -1;
    }
    return;
  }
  double key = __builtin_huge_val(), sec = __builtin_huge_val();
  int idx = -1;
  if (lane < K) {
    if (viable) {
      key = p.cand_key[(s * (L + 1) + j) * K + lane];
      sec = p.cand_sec[(s * (L + 1) + j) * K + lane];
      idx = p.cand[(s * (L + 1) + j) * K + lane];
    } else {
      // merge the chunks of this draft's scan (as the finalize kernel does) and normalise
      const long long o = (s * K + lane) * p.n_chunks;
      for (int c = 0; c < p.n_chunks; ++c) {
        const double ckey = p.part_key[o + c];
        const int cidx = p.part_idx[o + c];
        if (beats(ckey, cidx, 0, key, idx, 0)) {
          if (idx >= 0) sec = fmin(sec, key);
          key = ckey; idx = cidx;
        } else if (cidx >= 0) {
          sec = fmin(sec, ckey);
        }
        sec = fmin(sec, p.part_sec[o + c]);
      }
      const double norm = p.lse_sel[s * (K + 1) + lane];
      sec = (idx >= 0 && sec < __builtin_huge_val()) ? sec + norm : __builtin_huge_val();
      key = idx >= 0 ? key + norm : __builtin_huge_val();
    }
  }
  double bkey = idx >= 0 ? key : __builtin_huge_val();
  int bidx = idx, bk = lane;
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) {
    const double okey = __shfl_xor(bkey, d);
    const int oidx = __shfl_xor(bidx, d);
    const int ok = __shfl_xor(bk, d);
    if (beats(okey, oidx, ok, bkey, bidx, bk)) { bkey = okey; bidx = oidx; bk = ok; }
  }
  if (lane == 0) {
    Y[j] = bidx;
    if (keyY != nullptr) keyY[j] = bidx >= 0 ? (float)exp(bkey) : __builtin_huge_valf();
  }
  if (p.stats != nullptr && bidx >= 0) {
    // the runner-up at another index, over all K drafts' race times
    double r = __builtin_huge_val();
    if (lane < K && idx >= 0) r = idx != bidx ? key : sec;
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) r = fmin(r, __shfl_xor(r, d));
    if (lane == 0 && near_tie(bkey, r, 1)) atomicAdd(&p.stats->near_ties, 1ull);
  }
  bool more = j < L;
  if (more) {
    const int tok = lane < K ? p.tokens[s * p.tok_stride_s + (long long)j * p.tok_stride_j + lane] : -2;
    viable = viable && tok == bidx;
    more = __ballot(viable) != 0ull;
  }
  const unsigned long long mask = __ballot(viable);
  if (lane < K) p.viable[s * K + lane] = viable ? 1 : 0;
  if (lane == 0) {
    p.running[s] = more ? 1 : 0;
    if (!more) p.n_out[s] = j + 1;
    // the next position prices the dropped drafts with the first viable draft's row, if there are any
    const bool some_dropped = __popcll(mask) < K;
    p.next_off[s] = (more && some_dropped) ? (long long)(__ffsll((long long)mask) - 1) * p.stride_k : -1;
  }
  if (more && lane < K) {
    const int kref = __ffsll((long long)mask) - 1;
    p.lse_sel[s * (K + 1) + lane] = p.lse[(s * (L + 1) + j + 1) * (K + 1) + kref];
  }
  if (!more && p.active != nullptr && lane < K) p.active[s * K + lane] = viable ? 1 : 0;
}

__global__ void __launch_bounds__(256) fill_kernel(int32_t *dst, long long n, int32_t value) {
  const long long i = (long long)blockIdx.x * 256 + threadIdx.x;
  if (i < n) dst[i] = value;
}

}  // namespace

hipError_t launch_fill(hipStream_t s, int32_t *dst, long long n, int32_t value) {
  if (n == 0) return hipSuccess;
  hipLaunchKernelGGL(fill_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, dst, n, value);
  return hipGetLastError();
}

hipError_t launch_verify(hipStream_t s, const VerifyParams &p) {
  if (p.S == 0) return hipSuccess;
  hipLaunchKernelGGL(verify_kernel, dim3((unsigned)p.S), dim3(64), 0, s, p);
  return hipGetLastError();
}

hipError_t launch_strong_step(hipStream_t s, const StrongStepParams &p) {
  if (p.S == 0) return hipSuccess;
  hipLaunchKernelGGL(strong_step_kernel, dim3((unsigned)p.S), dim3(64), 0, s, p);
  return hipGetLastError();
}

hipError_t launch_finalize(hipStream_t s, const FinalizeParams &p) {
  if (p.B == 0) return hipSuccess;
  hipLaunchKernelGGL(finalize_kernel, dim3((unsigned)p.B), dim3(64), 0, s, p);
  return hipGetLastError();
}

hipError_t launch_lse(hipStream_t s, const LseParams &p) {
  if (p.B == 0) return hipSuccess;
  const int kd = p.per_k ? p.K : 1;
  const unsigned grid = (unsigned)(p.B * ((p.with_drafts ? kd : 0) + (p.with_target ? 1 : 0)));
  if (grid == 0) return hipSuccess;
  if (p.dtype == LLC_F32)
    hipLaunchKernelGGL(lse_kernel<float>, dim3(grid), dim3(256), 0, s, p);
  else
    hipLaunchKernelGGL(lse_kernel<uint16_t>, dim3(grid), dim3(256), 0, s, p);
  return hipGetLastError();
}

}  // namespace llc
