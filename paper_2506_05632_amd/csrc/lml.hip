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
// four passes of a stable 8-bit radix sort on the fp32 image of ln r, in which the two masses of
// an entry (rounded to fp32) travel with its key through two buffers in the workspace, and the
// running sums in fp64.  Indices whose r agree to fp32 precision may come out in either order,
// which together with the rounding of the masses moves a result by a relative 2^-22 at most.
// Entries without mass on one side follow the limits: p_j = 0 or q_j = 0 gives term j = 0; as a
// summand i such an entry still counts with the mass it has on the other side.
#include "common.hpp"

#include <type_traits>

namespace llc {
namespace {

constexpr int kThreads = 512;         // eight wavefronts share a row
constexpr int kWaves = kThreads / 64;
constexpr int kRounds = 8;            // elements a thread holds per tile of the sort
constexpr int kTile = kThreads * kRounds;

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
  __shared__ unsigned short s_cnt[kWaves][256];  // per wavefront and digit of a tile: counts, then starts
  __shared__ int s_goff[256];          // where a digit's run continues in the output
  __shared__ int s_tstart[256];        // where a digit's run starts inside the tile
  __shared__ int s_gbase[256];         // s_goff - s_tstart of the tile at hand
  __shared__ uint32_t st_key[kTile];   // the tile in digit order, on its way out
  __shared__ float2 st_mass[kTile];
  __shared__ double s_seg[kWaves][2];
  __shared__ int s_total[4][256];      // how often every digit of every pass occurs in the row
  // while the keys are made the staging area holds the counters: per pass, wavefront and digit
  static_assert(sizeof(st_mass) >= 4 * kWaves * 256 * sizeof(int), "the counters do not fit");
  int (*hist)[kWaves][256] = reinterpret_cast<int (*)[kWaves][256]>(st_mass);

  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const long long b = p.row0 + blockIdx.x;
  const int V = p.V;
  const E *prow = reinterpret_cast<const E *>(p.draft) + b * p.draft_stride_b;
  const E *qrow = reinterpret_cast<const E *>(p.target) + b * p.target_stride_b;
  // A launch takes as many rows as the workspace has slots (two key buffers, then two buffers of
  // (p-mass, q-mass) each); the launches of one call follow each other on the stream, so the
  // workspace is as large as the workgroups that can be resident need, not as the batch.
  char *work = p.work + (size_t)blockIdx.x * 24u * (size_t)V;
  uint32_t *key_a = reinterpret_cast<uint32_t *>(work), *key_b = key_a + V;
  float2 *mass_a = reinterpret_cast<float2 *>(work + 8u * (size_t)V), *mass_b = mass_a + V;

  const Side sp = normalise<E>(prow, V, p.probs, p.temp_draft, s_red);
  const Side sq = normalise<E>(qrow, V, p.probs, p.temp_target, s_red);

  // ---- sort keys with the masses that travel with them, how often every digit occurs (the
  // arithmetic around them hides the counters' collisions), and the sums that need no order
  for (int j = tid; j < 4 * kWaves * 256; j += kThreads) (&hist[0][0][0])[j] = 0;
  __syncthreads();
  double tv = 0.0, relaxed[kLmlMaxK];
#pragma unroll
  for (int kk = 0; kk < kLmlMaxK; ++kk) relaxed[kk] = 0.0;
  for (int i = tid; i < V; i += kThreads) {
    const double lp = sp.log_mass(elem<E>(prow, i)), lq = sq.log_mass(elem<E>(qrow, i));
    const bool hp = lp > -__builtin_huge_val(), hq = lq > -__builtin_huge_val();
    float lr = -__builtin_huge_valf();           // no target mass (or none at all): sorts first
    if (hq) lr = hp ? (float)(lq - lp) : __builtin_huge_valf();
    const double pm = hp ? exp(lp) : 0.0, qm = hq ? exp(lq) : 0.0;
    const uint32_t key = sort_key(lr);
    key_a[i] = key;
#pragma unroll
    for (int pass = 0; pass < 4; ++pass) atomicAdd(&hist[pass][wv][(key >> (8 * pass)) & 255u], 1);
    mass_a[i] = make_float2((float)pm, (float)qm);
    tv += fabs(pm - qm);
    if (hp && hq) {
#pragma unroll
      for (int kk = 0; kk < kLmlMaxK; ++kk)
        if (kk < p.n_k) {  // q / (1 + q / (K p)) with one division
          const double kp = (double)p.k[kk] * pm;
          relaxed[kk] += kp * qm / (kp + qm);
        }
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
  // (block_sum has synchronised since the last counter was bumped)
  for (int j = tid; j < 4 * 256; j += kThreads) {
    int total = 0;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) total += hist[j >> 8][w][j & 255];
    s_total[j >> 8][j & 255] = total;
  }

  // ---- stable radix sort, 8 bits a pass.  A pass takes the row a tile of kTile entries at a
  // time: wavefront w holds the w-th part of the tile,
  // ranks them among the tile's entries of the same digit (within the wavefront by ballots, in
  // order; across wavefronts by a prefix over their counts), the tile is laid out in digit order
  // in LDS, and is written from there so that neighbouring threads write neighbouring addresses
  // (a digit's entries of one tile are contiguous in the output).
  uint32_t *kin = key_a, *kout = key_b;
  float2 *min_ = mass_a, *mout = mass_b;
#pragma unroll 1
  for (int pass = 0; pass < 4; ++pass) {
    const int shift = 8 * pass;
    __syncthreads();  // the previous pass's (or the key loop's) stores are done and visible
    if (wv == 0) {
      // lane l takes digits l, 64 + l, 128 + l, 192 + l: the start of every digit's run
      int carry = 0;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int d = q * 64 + lane;
        const int total = s_total[pass][d];
        int incl = total;
#pragma unroll
        for (int dd = 1; dd < 64; dd <<= 1) {
          const int up = __shfl_up(incl, dd);
          if (lane >= dd) incl += up;
        }
        s_goff[d] = carry + incl - total;
        carry += __shfl(incl, 63);
      }
    }
    // (FULL: every entry of the tile exists, nothing is checked)
    auto sort_tile = [&](auto full_tag, const int t0) {
      constexpr bool FULL = decltype(full_tag)::value;
      __syncthreads();  // the tile before is on its way out of LDS; s_goff is in place
      for (int j = tid; j < kWaves * 256; j += kThreads) (&s_cnt[0][0])[j] = 0;
      __syncthreads();
      uint32_t key[kRounds];
      float2 mass[kRounds];
      int where[kRounds];  // rank among the wavefront's entries of the same digit
#pragma unroll
      for (int e = 0; e < kRounds; ++e) {
        const int i = t0 + wv * (64 * kRounds) + e * 64 + lane;
        const bool valid = FULL || i < V;
        key[e] = valid ? kin[i] : 0u;
        mass[e] = valid ? min_[i] : make_float2(0.0f, 0.0f);
      }
#pragma unroll
      for (int e = 0; e < kRounds; ++e) {
        const bool valid = FULL || t0 + wv * (64 * kRounds) + e * 64 + lane < V;
        const uint32_t d = (key[e] >> shift) & 255u;
        // lanes of this round with the same digit: bit by bit, keep those whose bit is like mine
        const unsigned long long live = __ballot(valid);
        uint32_t peers_lo = (uint32_t)live, peers_hi = (uint32_t)(live >> 32);
#pragma unroll
        for (int bit = 0; bit < 8; ++bit) {
          const uint32_t mine = (uint32_t)__builtin_amdgcn_sbfe((int)d, bit, 1);  // all ones if the bit is set
          const unsigned long long have = __ballot(mine != 0u);
          peers_lo &= ~((uint32_t)have ^ mine);
          peers_hi &= ~((uint32_t)(have >> 32) ^ mine);
        }
        where[e] = 0;
        if (valid) {
          const int rank = (int)__builtin_amdgcn_mbcnt_hi(peers_hi, __builtin_amdgcn_mbcnt_lo(peers_lo, 0u));
          const int seen = s_cnt[wv][d];
          if (rank == 0) s_cnt[wv][d] = (unsigned short)(seen + __popc(peers_lo) + __popc(peers_hi));
          where[e] = seen + rank;
        }
        __builtin_amdgcn_wave_barrier();
      }
      __syncthreads();
      if (wv == 0) {
        // per digit: every wavefront's start inside the digit's part of the tile, the part's start
        // inside the tile, and where the part goes in the output
        int carry = 0;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int d = q * 64 + lane;
          int total = 0;
#pragma unroll
          for (int w = 0; w < kWaves; ++w) {
            const int c = s_cnt[w][d];
            s_cnt[w][d] = (unsigned short)total;
            total += c;
          }
          int incl = total;
#pragma unroll
          for (int dd = 1; dd < 64; dd <<= 1) {
            const int up = __shfl_up(incl, dd);
            if (lane >= dd) incl += up;
          }
          const int start = carry + incl - total;
          carry += __shfl(incl, 63);
          const int g = s_goff[d];
          s_tstart[d] = start;
          s_gbase[d] = g - start;
          s_goff[d] = g + total;
        }
      }
      __syncthreads();
#pragma unroll
      for (int e = 0; e < kRounds; ++e) {
        if (FULL || t0 + wv * (64 * kRounds) + e * 64 + lane < V) {
          const uint32_t d = (key[e] >> shift) & 255u;
          const int pos = s_tstart[d] + s_cnt[wv][d] + where[e];
          st_key[pos] = key[e];
          st_mass[pos] = mass[e];
        }
      }
      __syncthreads();
      const int n_tile = FULL ? kTile : min(kTile, V - t0);
#pragma unroll
      for (int e = 0; e < kRounds; ++e) {
        const int pos = e * kThreads + tid;
        if (FULL || pos < n_tile) {
          const uint32_t k = st_key[pos];
          const int g = s_gbase[(k >> shift) & 255u] + pos;
          kout[g] = k;
          mout[g] = st_mass[pos];
        }
      }
    };
    int t0 = 0;
#pragma unroll 1
    for (; t0 + kTile <= V; t0 += kTile) sort_tile(std::true_type(), t0);
    if (t0 < V) sort_tile(std::false_type(), t0);
    { uint32_t *t = kin; kin = kout; kout = t; }
    { float2 *t = min_; min_ = mout; mout = t; }
  }
  __syncthreads();
  // after four passes the sorted order is back in the first buffers (min_ == mass_a)

  // ---- running sums over the sorted order.  Wavefront w takes the w-th part of the row: first
  // every part's masses are added up, then every wavefront walks its part with the masses of the
  // parts before it as the carry.
  const int seg = (V + kWaves - 1) / kWaves;
  const int seg_begin = min(wv * seg, V), seg_end = min(seg_begin + seg, V);
  const float2 *mass = min_;
  double seg_p = 0.0, seg_q = 0.0;
  for (int j = seg_begin + lane; j < seg_end; j += 64) {
    const float2 m = mass[j];
    seg_p += (double)m.x;
    seg_q += (double)m.y;
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
      const float2 m = mass[j];
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
      // K / (q_suf/q_j + p_pre/p_j + (K - 1) Q/q_j), numerator and denominator times q_j
      const double common = q_suf + p_pre * (qm / pm);
#pragma unroll
      for (int kk = 0; kk < kLmlMaxK; ++kk)
        if (kk < p.n_k) {
          const double K = (double)p.k[kk];
          acc[kk] += K * qm / (common + (K - 1.0) * q_total);
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

hipError_t launch_lml(hipStream_t s, const LmlParams &params) {
  LmlParams p = params;
  for (p.row0 = 0; p.row0 < p.B; p.row0 += p.slots) {
    const long long left = p.B - p.row0;
    const unsigned grid = (unsigned)(left < (long long)p.slots ? left : (long long)p.slots);
    if (p.dtype == LLC_F32)
      hipLaunchKernelGGL(lml_kernel<float>, dim3(grid), dim3(kThreads), 0, s, p);
    else
      hipLaunchKernelGGL(lml_kernel<uint16_t>, dim3(grid), dim3(kThreads), 0, s, p);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

}  // namespace llc
