// The list matching lemma's lower bound on the matching probability (paper Theorem 1,
// eq. (1)), its relaxed form (the display that follows the theorem's proof sketch) and the total
// variation distance behind the two-party bound of the introduction, evaluated per row on the
// device so that a serving stack can choose the list size K from the distributions it has.
//
// Eq. (1) for K drafts drawn from p and a target q:
//   sum_j K / sum_i ( max{q_i/q_j, p_i/p_j} + (K - 1) q_i/q_j ).
// max{q_i/q_j, p_i/p_j} is q_i/q_j exactly when q_i/p_i >= q_j/p_j, so with the indices sorted by
// r = q/p the inner sum is (the q-mass from j on)/q_j + (the p-mass before j)/p_j + (K-1) Q/q_j:
// one sort and one running sum per row.  One workgroup does a whole row: normalisers, sort keys,
// four passes of a stable 8-bit radix sort on the fp32 image of ln r through two buffers in the
// workspace, and the running sums in fp64.  Indices whose r agree to fp32 precision may come out
// in either order, which moves their contribution by a relative 2^-23 at most.
// Entries without mass on one side follow the limits: p_j = 0 or q_j = 0 gives term j = 0; as a
// summand i such an entry still counts with the mass it has on the other side.
#include "common.hpp"

namespace llc {
namespace {

constexpr int kThreads = 1024;        // sixteen wavefronts share a row: each owns a sixteenth of it
constexpr int kWaves = kThreads / 64;

template <typename E>
__device__ __forceinline__ float elem(const E *row, int i);
template <>
__device__ __forceinline__ float elem<float>(const float *row, int i) { return row[i]; }
template <>
__device__ __forceinline__ float elem<uint16_t>(const uint16_t *row, int i) {
  return __uint_as_float((uint32_t)row[i] << 16);
}

// Sum / maximum over the workgroup; every thread gets the result.  `scratch` holds kWaves doubles.
__device__ double block_sum(double v, double *scratch) {
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) v += __shfl_xor(v, d);
  __syncthreads();  // scratch may still be read from the previous reduction
  if ((threadIdx.x & 63) == 0) scratch[threadIdx.x >> 6] = v;
  __syncthreads();
  double r = 0.0;
#pragma unroll
  for (int w = 0; w < kWaves; ++w) r += scratch[w];  // a fixed order
  return r;
}
__device__ double block_max(double v, double *scratch) {
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) v = fmax(v, __shfl_xor(v, d));
  __syncthreads();
  if ((threadIdx.x & 63) == 0) scratch[threadIdx.x >> 6] = v;
  __syncthreads();
  double r = scratch[0];
#pragma unroll
  for (int w = 1; w < kWaves; ++w) r = fmax(r, scratch[w]);
  return r;
}

// ln of the normalised mass of one entry.  Logits and log-weights: (x - m)/T - ln z with m the
// row's largest finite value; probabilities: ln x - ln z.  NaN, +inf (and for probabilities
// anything not > 0) carry no mass.
struct Side {
  double m, inv_t, ln_z;
  int probs;
  __device__ __forceinline__ double log_mass(float x) const {
    const double ninf = -__builtin_huge_val();
    if (probs) return (x > 0.0f && x < __builtin_huge_valf()) ? log((double)x) - ln_z : ninf;
    return (x < __builtin_huge_valf() && x > -__builtin_huge_valf()) ? ((double)x - m) * inv_t - ln_z : ninf;
  }
};

template <typename E>
__device__ Side normalise(const E *row, int V, int probs, float temp, double *scratch) {
  Side s;
  s.probs = probs;
  s.inv_t = 1.0 / (double)temp;
  double m = -__builtin_huge_val();
  if (!probs) {
    for (int i = threadIdx.x; i < V; i += kThreads) {
      const float x = elem<E>(row, i);
      if (x < __builtin_huge_valf()) m = fmax(m, (double)x);  // (NaN compares false)
    }
    m = block_max(m, scratch);
  }
  s.m = m;
  double z = 0.0;
  for (int i = threadIdx.x; i < V; i += kThreads) {
    const float x = elem<E>(row, i);
    if (probs) {
      if (x > 0.0f && x < __builtin_huge_valf()) z += (double)x;
    } else if (x < __builtin_huge_valf() && x > -__builtin_huge_valf()) {
      z += exp(((double)x - m) * s.inv_t);
    }
  }
  z = block_sum(z, scratch);
  s.ln_z = log(z);  // z == 0: no mass at all, every log_mass is -inf or NaN-free below
  return s;
}

// order-preserving image of a float in the unsigned integers
__device__ __forceinline__ uint32_t sort_key(float f) {
  const uint32_t u = __float_as_uint(f);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

template <typename E>
__global__ void __launch_bounds__(kThreads) lml_kernel(const LmlParams p) {
  __shared__ double s_red[kWaves];
  __shared__ int s_bins[kWaves][256];
  __shared__ int s_wave_total[4];
  __shared__ double s_seg[kWaves][2];

  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const long long b = blockIdx.x;
  const int V = p.V;
  const E *prow = reinterpret_cast<const E *>(p.draft) + b * p.draft_stride_b;
  const E *qrow = reinterpret_cast<const E *>(p.target) + b * p.target_stride_b;
  // (key, index) pairs travel together: one 8-byte store per element and pass
  uint2 *buf_a = p.pairs + (size_t)b * 2 * V, *buf_b = buf_a + V;

  const Side sp = normalise<E>(prow, V, p.probs, p.temp_draft, s_red);
  const Side sq = normalise<E>(qrow, V, p.probs, p.temp_target, s_red);

  // ---- sort keys, and the sums that need no order
  double tv = 0.0, relaxed[kLmlMaxK];
#pragma unroll
  for (int kk = 0; kk < kLmlMaxK; ++kk) relaxed[kk] = 0.0;
  for (int i = tid; i < V; i += kThreads) {
    const double lp = sp.log_mass(elem<E>(prow, i)), lq = sq.log_mass(elem<E>(qrow, i));
    const bool hp = lp > -__builtin_huge_val(), hq = lq > -__builtin_huge_val();
    float lr = -__builtin_huge_valf();           // no target mass (or none at all): sorts first
    if (hq) lr = hp ? (float)(lq - lp) : __builtin_huge_valf();
    buf_a[i] = make_uint2(sort_key(lr), (uint32_t)i);
    const double pm = hp ? exp(lp) : 0.0, qm = hq ? exp(lq) : 0.0;
    tv += fabs(pm - qm);
    if (hp && hq) {
#pragma unroll
      for (int kk = 0; kk < kLmlMaxK; ++kk)
        if (kk < p.n_k) relaxed[kk] += qm / (1.0 + qm / ((double)p.k[kk] * pm));
    }
  }
  tv = block_sum(tv, s_red);
#pragma unroll
  for (int kk = 0; kk < kLmlMaxK; ++kk)
    if (kk < p.n_k) {  // uniform
      const double r = block_sum(relaxed[kk], s_red);
      if (tid == 0 && p.relaxed != nullptr) p.relaxed[b * p.n_k + kk] = r;
    }
  if (tid == 0 && p.tv != nullptr) p.tv[b] = 0.5 * tv;

  // ---- stable radix sort, 8 bits a pass.  Wavefront w owns the w-th part of the row: it counts
  // its digits, gets its own start inside every digit's range (after the parts before it), and
  // then moves its part tile by tile in order, so equal digits keep their order.
  const int seg = (V + kWaves - 1) / kWaves;
  const int seg_begin = min(wv * seg, V), seg_end = min(seg_begin + seg, V);
  uint2 *in = buf_a, *out = buf_b;
#pragma unroll 1
  for (int pass = 0; pass < 4; ++pass) {
    const int shift = 8 * pass;
    __syncthreads();  // the previous pass's (or the key loop's) stores are done and visible
    for (int j = tid; j < kWaves * 256; j += kThreads) (&s_bins[0][0])[j] = 0;
    __syncthreads();
    for (int i = seg_begin + lane; i < seg_end; i += 64) atomicAdd(&s_bins[wv][(in[i].x >> shift) & 255u], 1);
    __syncthreads();
    {
      // thread t < 256 = digit t: where the digit's range starts, then every part's start inside it
      int total = 0;
      if (tid < 256) {
#pragma unroll
        for (int w = 0; w < kWaves; ++w) total += s_bins[w][tid];
      }
      int incl = total;
#pragma unroll
      for (int d = 1; d < 64; d <<= 1) {
        const int up = __shfl_up(incl, d);
        if (lane >= d) incl += up;
      }
      if (tid < 256 && lane == 63) s_wave_total[wv] = incl;
      __syncthreads();
      if (tid < 256) {
        int start = incl - total;
        for (int w = 0; w < wv; ++w) start += s_wave_total[w];
#pragma unroll
        for (int w = 0; w < kWaves; ++w) {
          const int c = s_bins[w][tid];
          s_bins[w][tid] = start;
          start += c;
        }
      }
    }
    __syncthreads();
    // (the next tile is fetched before this one is placed)
    uint2 next = make_uint2(0u, 0u);
    if (seg_begin + lane < seg_end) next = in[seg_begin + lane];
    for (int i0 = seg_begin; i0 < seg_end; i0 += 64) {
      const int i = i0 + lane;
      const bool valid = i < seg_end;
      const uint2 cur = next;
      if (i + 64 < seg_end) next = in[i + 64];
      const uint32_t d = (cur.x >> shift) & 255u;
      // lanes of this tile with the same digit
      unsigned long long peers = __ballot(valid);
#pragma unroll
      for (int bit = 0; bit < 8; ++bit) {
        const bool set = (d >> bit) & 1u;
        const unsigned long long have = __ballot(set);
        peers &= set ? have : ~have;
      }
      if (valid) {
        const int rank = __popcll(peers & ((1ull << lane) - 1ull));
        const int start = s_bins[wv][d];
        if (rank == 0) s_bins[wv][d] = start + __popcll(peers);
        out[start + rank] = cur;
      }
      __builtin_amdgcn_wave_barrier();
    }
    uint2 *t = in; in = out; out = t;
  }
  __syncthreads();
  // after four passes the sorted order is back in the first buffer (in == buf_a)

  // ---- running sums over the sorted order.  One pass gathers the masses by sorted index, leaves
  // them in sorted order in the spare buffer (as fp32: a relative 2^-24 per mass) and adds up each
  // part's masses; then every wavefront walks its part, reading the masses back in order, with
  // the masses of the parts before it as the carry.
  float2 *mass = reinterpret_cast<float2 *>(out);
  double seg_p = 0.0, seg_q = 0.0;
  for (int j = seg_begin + lane; j < seg_end; j += 64) {
    const int i = (int)in[j].y;
    const double lp = sp.log_mass(elem<E>(prow, i)), lq = sq.log_mass(elem<E>(qrow, i));
    const float pf = lp > -__builtin_huge_val() ? (float)exp(lp) : 0.0f;
    const float qf = lq > -__builtin_huge_val() ? (float)exp(lq) : 0.0f;
    mass[j] = make_float2(pf, qf);
    seg_p += (double)pf;
    seg_q += (double)qf;
  }
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) { seg_p += __shfl_xor(seg_p, d); seg_q += __shfl_xor(seg_q, d); }
  if (lane == 0) { s_seg[wv][0] = seg_p; s_seg[wv][1] = seg_q; }
  __syncthreads();
  double p_before = 0.0, q_before = 0.0, q_total = 0.0;
  for (int w = 0; w < kWaves; ++w) {
    if (w < wv) { p_before += s_seg[w][0]; q_before += s_seg[w][1]; }
    q_total += s_seg[w][1];
  }
  double acc[kLmlMaxK];
#pragma unroll
  for (int kk = 0; kk < kLmlMaxK; ++kk) acc[kk] = 0.0;
  for (int j0 = seg_begin; j0 < seg_end; j0 += 64) {
    const int j = j0 + lane;
    double pm = 0.0, qm = 0.0;
    if (j < seg_end) {
      const float2 m = mass[j];  // written by this lane in the pass above
      pm = (double)m.x;
      qm = (double)m.y;
    }
    double pin = pm, qin = qm;  // inclusive sums over the lanes of this tile
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
      const double up_p = __shfl_up(pin, d), up_q = __shfl_up(qin, d);
      if (lane >= d) { pin += up_p; qin += up_q; }
    }
    if (pm > 0.0 && qm > 0.0) {
      const double p_pre = p_before + (pin - pm);             // mass of p strictly before j
      const double q_suf = q_total - (q_before + (qin - qm));  // mass of q from j on
      const double common = q_suf / qm + p_pre / pm;
#pragma unroll
      for (int kk = 0; kk < kLmlMaxK; ++kk)
        if (kk < p.n_k) {
          const double K = (double)p.k[kk];
          acc[kk] += K / (common + (K - 1.0) * q_total / qm);
        }
    }
    p_before += __shfl(pin, 63);
    q_before += __shfl(qin, 63);
  }
#pragma unroll
  for (int kk = 0; kk < kLmlMaxK; ++kk)
    if (kk < p.n_k) {  // uniform
      const double r = block_sum(acc[kk], s_red);
      if (tid == 0) p.bound[b * p.n_k + kk] = r;
    }
}

}  // namespace

hipError_t launch_lml(hipStream_t s, const LmlParams &p) {
  if (p.B == 0) return hipSuccess;
  if (p.dtype == LLC_F32)
    hipLaunchKernelGGL(lml_kernel<float>, dim3((unsigned)p.B), dim3(kThreads), 0, s, p);
  else
    hipLaunchKernelGGL(lml_kernel<uint16_t>, dim3((unsigned)p.B), dim3(kThreads), 0, s, p);
  return hipGetLastError();
}

}  // namespace llc
