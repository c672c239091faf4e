// Finalize: merge the per-chunk partial argmins of a row and take Algorithm 1's
// last step, accept = [Y in {X^(1..K)}] (paper Section 3).  Also the row
// normalisers ln sum exp(x/T) that turn log-domain keys into S/p with p
// normalised (Section 3 defines p and q as distributions; Appendix C normalises
// the importance weights the same way).
#include "common.hpp"

namespace llc {

namespace {

// Smaller key wins; equal keys: smaller index, then smaller k.
__device__ __forceinline__ bool beats(double key, int idx, int k, double bkey, int bidx, int bk) {
  if (idx < 0) return false;
  if (bidx < 0) return true;
  if (key != bkey) return key < bkey;
  if (idx != bidx) return idx < bidx;
  return k < bk;
}

__global__ void __launch_bounds__(64) finalize_kernel(const FinalizeParams p) {
  __shared__ int s_match;
  __shared__ int s_y;
  const long long b = blockIdx.x;
  const int tid = threadIdx.x;
  if (tid == 0) s_match = 0x7FFFFFFF;

  // draft side: one thread per k merges the chunks
  unsigned long long degenerate = 0;
  for (int k = tid; k < p.K; k += 64) {
    const long long o = (b * p.K + k) * p.n_chunks;
    double bkey = __builtin_huge_val();
    int bidx = -1;
    for (int c = 0; c < p.n_chunks; ++c) {
      const double key = p.in.keyX[o + c];
      const int idx = p.in.idxX[o + c];
      if (beats(key, idx, 0, bkey, bidx, 0)) { bkey = key; bidx = idx; }
    }
    p.X[b * p.K + k] = bidx;
    if (bidx < 0) ++degenerate;
    if (p.keyX != nullptr) {
      double out = __builtin_huge_val();
      if (bidx >= 0) out = p.log_kind ? exp(bkey + p.in.lse[b * (p.K + 1) + k]) : bkey;
      p.keyX[b * p.K + k] = (float)out;
    }
  }
  // target side: the pool over draft groups and chunks
  if (tid == 0) {
    const long long o = b * p.n_kgroups * p.n_chunks;
    double bkey = __builtin_huge_val();
    int bidx = -1, bk = -1;
    for (int c = 0; c < p.n_kgroups * p.n_chunks; ++c) {
      const double key = p.in.keyY[o + c];
      const int idx = p.in.idxY[o + c];
      const int k = p.in.kY[o + c];
      if (beats(key, idx, k, bkey, bidx, bk)) { bkey = key; bidx = idx; bk = k; }
    }
    p.Y[b] = bidx;
    s_y = bidx;
    if (bidx < 0) ++degenerate;
    if (p.keyY != nullptr) {
      double out = __builtin_huge_val();
      if (bidx >= 0) out = p.log_kind ? exp(bkey + p.in.lse[b * (p.K + 1) + p.K]) : bkey;
      p.keyY[b] = (float)out;
    }
  }
  __syncthreads();
  const int y = s_y;
  if (y >= 0) {
    for (int k = tid; k < p.K; k += 64)
      if (p.X[b * p.K + k] == y) atomicMin(&s_match, k);
  }
  __syncthreads();
  if (tid == 0) {
    const bool hit = s_match != 0x7FFFFFFF;
    p.accept[b] = hit ? 1 : 0;
    if (p.match_k != nullptr) p.match_k[b] = hit ? s_match : -1;
  }
  if (p.stats != nullptr && degenerate) atomicAdd(&p.stats->degenerate, degenerate);
}

// ln sum_i exp(x_i / T) of one input row; fp32 terms relative to the row maximum,
// fp64 accumulation.  NaN and +inf entries carry no mass.
template <typename E>
__device__ __forceinline__ float widen(const E *row, int i);
template <>
__device__ __forceinline__ float widen<float>(const float *row, int i) { return row[i]; }
template <>
__device__ __forceinline__ float widen<uint16_t>(const uint16_t *row, int i) {
  return __uint_as_float((uint32_t)row[i] << 16);
}

template <typename E>
__global__ void __launch_bounds__(256) lse_kernel(const LseParams p) {
  __shared__ float s_max[4];
  __shared__ double s_sum[4];
  const int kd = p.draft_stride_k == 0 && p.temp_draft == nullptr ? 1 : p.K;  // distinct draft rows
  const long long b = blockIdx.x / (unsigned)(kd + 1);
  const int which = (int)(blockIdx.x % (unsigned)(kd + 1));  // kd = the target row
  const int tid = threadIdx.x;
  const E *row;
  float T;
  if (which == kd) {
    row = reinterpret_cast<const E *>(p.target) + b * p.target_stride_b;
    T = p.temp_target;
  } else {
    row = reinterpret_cast<const E *>(p.draft) + b * p.draft_stride_b + (long long)which * p.draft_stride_k;
    T = p.temp_draft != nullptr ? p.temp_draft[which] : p.temp_draft_all;
  }
  if (!p.is_logits) T = 1.0f;
  const float inf = __builtin_huge_valf();

  float m = -inf;
  for (int i = tid; i < p.V; i += 256) {
    const float v = widen<E>(row, i);
    if (v < inf) m = fmaxf(m, v);
  }
  for (int d = 32; d >= 1; d >>= 1) m = fmaxf(m, __shfl_xor(m, d));
  if ((tid & 63) == 0) s_max[tid >> 6] = m;
  __syncthreads();
  m = fmaxf(fmaxf(s_max[0], s_max[1]), fmaxf(s_max[2], s_max[3]));

  double sum = 0.0;
  if (m > -inf) {
    const float c = 1.4426950408889634f / T;
    for (int i0 = tid; i0 < p.V; i0 += 256 * 8) {
      float part = 0.0f;  // eight terms in fp32, then into the fp64 running sum
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const int i = i0 + u * 256;
        if (i < p.V) {
          const float v = widen<E>(row, i);
          if (v < inf) part += exp2f((v - m) * c);
        }
      }
      sum += (double)part;
    }
  }
  for (int d = 32; d >= 1; d >>= 1) sum += __shfl_xor(sum, d);
  if ((tid & 63) == 0) s_sum[tid >> 6] = sum;
  __syncthreads();
  if (tid == 0) {
    sum = (s_sum[0] + s_sum[1]) + (s_sum[2] + s_sum[3]);
    const bool ok = (m > -inf) && (T > 0.0f) && (T < inf);
    const double lse = ok ? (double)m / (double)T + log(sum) : -__builtin_huge_val();
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

}  // namespace

hipError_t launch_finalize(hipStream_t s, const FinalizeParams &p) {
  if (p.B == 0) return hipSuccess;
  hipLaunchKernelGGL(finalize_kernel, dim3((unsigned)p.B), dim3(64), 0, s, p);
  return hipGetLastError();
}

hipError_t launch_lse(hipStream_t s, const LseParams &p) {
  if (p.B == 0) return hipSuccess;
  const int kd = p.draft_stride_k == 0 && p.temp_draft == nullptr ? 1 : p.K;
  const unsigned grid = (unsigned)(p.B * (kd + 1));
  if (p.dtype == LLC_F32)
    hipLaunchKernelGGL(lse_kernel<float>, dim3(grid), dim3(256), 0, s, p);
  else
    hipLaunchKernelGGL(lse_kernel<uint16_t>, dim3(grid), dim3(256), 0, s, p);
  return hipGetLastError();
}

}  // namespace llc
