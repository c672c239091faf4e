// The finalize step of one row: merge the per-chunk partial argmins and take Algorithm 1's last
// step, accept = [Y in {X^(1..K)}] (paper Section 3).  Shared by the finalize kernel and by the
// scan kernel's variant that finishes its row itself (rows that are one workgroup each).
#pragma once

#include "common.hpp"

namespace llc {

// Smaller key wins; equal keys: smaller index, then smaller k.
__device__ __forceinline__ bool beats(double key, int idx, int k, double bkey, int bidx, int bk) {
  if (idx < 0) return false;
  if (bidx < 0) return true;
  if (key != bkey) return key < bkey;
  if (idx != bidx) return idx < bidx;
  return k < bk;
}

// A winner within this relative distance (in S/p) of the best key at another index is a near-tie.
constexpr double kNearTie = 1e-6;

// Whether the runner-up key is that close.  Log-domain keys are ln(S/p) up to a constant that both
// share, so the relative distance is expm1 of their difference.
__device__ __forceinline__ bool near_tie(double best, double second, int log_kind) {
  if (!(second < __builtin_huge_val())) return false;
  if (log_kind) return expm1(second - best) < kNearTie;
  return best > 0.0 ? (second - best) / best < kNearTie : !(second > 0.0);
}

// One row of the finalize step, by the NT threads of a workgroup (all of them must call it: it
// holds barriers).  `fs` is the workgroup's scratch in LDS.
struct FinalizeShared {
  int match;
  int y;
  unsigned long long err;  // ordered image of the smallest squared error among the decoders
};
template <int NT>
__device__ __forceinline__ void finalize_row(const FinalizeParams &p, const long long b, const int tid, FinalizeShared &fs) {
  int &s_match = fs.match;
  int &s_y = fs.y;
  unsigned long long &s_err = fs.err;
  if (tid == 0) { s_match = 0x7FFFFFFF; s_err = 0x7FF0000000000000ull; }  // (+inf; squared errors are >= 0)
  if (p.cand != nullptr) __syncthreads();
  if (p.in.lse_part != nullptr) {
    // the scan left every chunk's share of the normalisers: ln sum_chunks exp(share)
    // (without lse_part_target the target's normaliser is already in place)
    for (int k = tid; k < p.K + (p.in.lse_part_target ? 1 : 0); k += NT) {
      const double *sh = p.in.lse_part + (b * (p.K + 1) + k) * p.n_chunks;
      double m = -__builtin_huge_val();
      for (int c = 0; c < p.n_chunks; ++c) m = fmax(m, sh[c]);
      double sum = 0.0;
      if (m > -__builtin_huge_val())
        for (int c = 0; c < p.n_chunks; ++c) sum += exp(sh[c] - m);
      p.in.lse[b * (p.K + 1) + k] = m > -__builtin_huge_val() ? m + log(sum) : -__builtin_huge_val();
    }
    __syncthreads();
  }

  // draft side: one thread per k merges the chunks.  The runner-up of the merged reduction is the
  // smallest of the other chunks' winners and of the winning chunk's own runner-up (a draft meets
  // every index in one chunk only).
  unsigned long long degenerate = 0, near = 0;
  for (int k = tid; k < p.K; k += NT) {
    const long long o = (b * p.K + k) * p.n_chunks;
    double bkey = __builtin_huge_val(), sec = __builtin_huge_val();
    int bidx = -1;
    for (int c = 0; c < p.n_chunks; ++c) {
      const double key = p.in.keyX[o + c];
      const int idx = p.in.idxX[o + c];
      if (beats(key, idx, 0, bkey, bidx, 0)) {
        if (bidx >= 0) sec = fmin(sec, bkey);
        bkey = key; bidx = idx;
      } else if (idx >= 0) {
        sec = fmin(sec, key);
      }
      sec = fmin(sec, p.in.secX[o + c]);
    }
    p.X[b * p.K + k] = bidx;
    if (bidx < 0) ++degenerate;
    else if (near_tie(bkey, sec, p.log_kind)) ++near;
    if (p.log_keyX != nullptr)
      p.log_keyX[b * p.K + k] = bidx >= 0 ? bkey + p.in.lse[b * (p.K + 1) + k] : __builtin_huge_val();
    if (p.log_secX != nullptr)
      p.log_secX[b * p.K + k] = (bidx >= 0 && sec < __builtin_huge_val()) ? sec + p.in.lse[b * (p.K + 1) + k]
                                                                          : __builtin_huge_val();
    if (p.keyX != nullptr) {
      double out = __builtin_huge_val();
      if (bidx >= 0) out = p.log_kind ? exp(bkey + p.in.lse[b * (p.K + 1) + k]) : bkey;
      p.keyX[b * p.K + k] = (float)out;
    }
    if (p.cand != nullptr) {
      // the decoder's output W_k = U_{X^(k)} (Appendix C) and its MMSE estimate of the source
      // (Appendix D.2), in fp64 from the fp32 inputs; NaN where the decoder found no candidate
      double w = __builtin_nan(""), est = __builtin_nan("");
      if (bidx >= 0) {
        w = (double)p.cand[b * p.cand_stride_b + bidx];
        if (p.side != nullptr) {
          const double t = (double)p.side[b * p.side_stride_b + k];
          est = (p.var_z * w + p.var_e * t) / (p.var_e + p.var_z + p.var_e * p.var_z);
        }
        if (p.sq_err != nullptr) {
          const double d = est - (double)p.source[b];
          const double e2 = d * d;
          if (e2 == e2) atomicMin(&s_err, (unsigned long long)__double_as_longlong(e2));
        }
      }
      if (p.W != nullptr) p.W[b * p.K + k] = (float)w;
      if (p.A_hat != nullptr) p.A_hat[b * p.K + k] = (float)est;
    }
  }
  if (!p.count_draft) { degenerate = 0; near = 0; }
  if (p.Y == nullptr) {  // draft side only
    if (p.stats != nullptr && degenerate) atomicAdd(&p.stats->degenerate, degenerate);
    if (p.stats != nullptr && near && p.count_near) atomicAdd(&p.stats->near_ties, near);
    return;
  }
  if (p.y_given) {
    // the pool's index was settled by an earlier pass (binned selection): announce its bin
    if (tid == 0) {
      const int y = p.Y[b];
      s_y = y;
      if (p.message != nullptr) p.message[b] = (y >= 0 && p.bins != nullptr) ? (int)p.bins[b * p.bins_stride_b + y] : -1;
    }
  } else if (tid == 0) {
    // target side: the pool over draft groups and chunks
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
    if (bidx < 0) {
      if (p.count_pool) ++degenerate;
    } else if (p.count_pool) {
      // the runner-up at another index: a part whose winner sits at the same index (another draft
      // group met it under other race times) contributes its own runner-up instead
      double sec = __builtin_huge_val();
      for (int c = 0; c < p.n_kgroups * p.n_chunks; ++c) {
        const int idx = p.in.idxY[o + c];
        if (idx < 0) continue;
        sec = fmin(sec, idx != bidx ? p.in.keyY[o + c] : p.in.secY[o + c]);
      }
      if (near_tie(bkey, sec, p.log_kind)) ++near;
    }
    if (p.keyY != nullptr) {
      double out = __builtin_huge_val();
      if (bidx >= 0) out = p.log_kind ? exp(bkey + p.in.lse[b * (p.K + 1) + p.K]) : bkey;
      p.keyY[b] = (float)out;
    }
  }
  __syncthreads();
  const int y = s_y;
  if (y >= 0) {
    for (int k = tid; k < p.K; k += NT)
      if (p.X[b * p.K + k] == y) atomicMin(&s_match, k);
  }
  __syncthreads();
  if (tid == 0) {
    const bool hit = s_match != 0x7FFFFFFF;
    p.accept[b] = hit ? 1 : 0;
    if (p.match_k != nullptr) p.match_k[b] = hit ? s_match : -1;
    // (the barriers above order the decoders' offers before this read)
    if (p.cand != nullptr && p.sq_err != nullptr) p.sq_err[b] = (float)__longlong_as_double((long long)s_err);
  }
  if (p.stats != nullptr && degenerate) atomicAdd(&p.stats->degenerate, degenerate);
  if (p.stats != nullptr && near && p.count_near) atomicAdd(&p.stats->near_ties, near);
}


}  // namespace llc
