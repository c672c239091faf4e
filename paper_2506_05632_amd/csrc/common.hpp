// Shared declarations of the HIP implementation (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/llc.h"

namespace llc {

constexpr int kBlock = 256;        // threads per workgroup: four 64-wide wavefronts
constexpr int kListCap = 1024;     // candidate records a workgroup can hold in LDS

// Partial result of one reduction: the smallest exact key and where it sits.
// Keys are fp64; for the logit / log-weight kinds they are ln(S) - x/T (a
// monotone image of S/p that cannot overflow), for the probability kind S/p.
struct Partials {
  double *keyX;   // [B][K][n_chunks]
  int32_t *idxX;  // [B][K][n_chunks]
  double *keyY;   // [B][n_kgroups][n_chunks]
  int32_t *idxY;  // [B][n_kgroups][n_chunks]
  int32_t *kY;    // [B][n_kgroups][n_chunks]
  double *lse;    // [B][K+1]: ln sum exp(x/T) of draft k (k < K) and of the target (k == K)
};

struct ScanParams {
  const void *draft;
  const void *target;
  long long draft_stride_b, draft_stride_k, target_stride_b;  // elements
  long long B;
  int K, V;
  int n_chunks;          // workgroups a row's V is split over
  int groups_per_chunk;  // 4-element groups per chunk (a multiple of kBlock)
  int n_kgroups;         // ceil(K / KT)
  unsigned seed_lo, seed_hi;
  unsigned long long row_offset;
  float temp_target, temp_draft_all;
  const float *temp_draft;  // device, K entries, or nullptr
  int vector_loads;         // rows are aligned for 4-element vector loads
  int force_exact;
  Partials out;
  llc_stats *stats;
};

struct FinalizeParams {
  long long B;
  int K, n_chunks, n_kgroups;
  int log_kind;        // keys are in the log domain and need the normaliser
  Partials in;
  int32_t *X, *Y, *match_k;
  uint8_t *accept;
  float *keyX, *keyY;  // optional
  llc_stats *stats;
};

struct LseParams {
  const void *draft;
  const void *target;
  long long draft_stride_b, draft_stride_k, target_stride_b;
  long long B;
  int K, V;
  int dtype;
  float temp_target, temp_draft_all;
  const float *temp_draft;
  int is_logits;  // divide by the temperature
  double *lse;    // [B][K+1]
};

// One launcher per (element type, draft layout); defined in scan_*.hip.
// kt: drafts per workgroup pass (1, 2, 4, 8); probs: inputs are probabilities.
hipError_t launch_scan_f32_shared(int kt, bool probs, unsigned grid, hipStream_t s, const ScanParams &p);
hipError_t launch_scan_f32_perk(int kt, bool probs, unsigned grid, hipStream_t s, const ScanParams &p);
hipError_t launch_scan_bf16_shared(int kt, bool probs, unsigned grid, hipStream_t s, const ScanParams &p);
hipError_t launch_scan_bf16_perk(int kt, bool probs, unsigned grid, hipStream_t s, const ScanParams &p);

hipError_t launch_finalize(hipStream_t s, const FinalizeParams &p);
hipError_t launch_lse(hipStream_t s, const LseParams &p);

}  // namespace llc
