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
  double *secX;   // [B][K][n_chunks] runner-up keys: the smallest key at an index other than the
  double *secY;   // [B][n_kgroups][n_chunks] winner's (+inf if none was seen within the band)
  double *lse;    // [B][K+1]: ln sum exp(x/T) of draft k (k < K) and of the target (k == K)
  double *lse_part;  // [B][K+1][n_chunks] per-chunk shares to merge into lse first, or nullptr
  int lse_part_target;  // the shares include the target row's (slot K); else lse[.][K] is in place
};

// Rows may be a two-level index b = outer * inner_count + inner (sequences x positions in
// the verifier); plain batches have inner_count = 1.
struct RowMap {
  long long inner_count;
  long long draft_outer, draft_inner;    // element strides of the draft tensor
  long long target_outer, target_inner;  // element strides of the target tensor
  long long row_outer, row_inner;        // strides of the random stream's row number
  __host__ __device__ long long draft_off(long long b) const {
    return (b / inner_count) * draft_outer + (b % inner_count) * draft_inner;
  }
  __host__ __device__ long long target_off(long long b) const {
    return (b / inner_count) * target_outer + (b % inner_count) * target_inner;
  }
  __host__ __device__ unsigned long long row_of(long long b) const {
    return (unsigned long long)((b / inner_count) * row_outer + (b % inner_count) * row_inner);
  }
};

struct FinalizeParams {
  long long B;
  int K, n_chunks, n_kgroups;
  int log_kind;        // keys are in the log domain and need the normaliser
  Partials in;
  int32_t *X, *Y, *match_k;  // Y, accept may be null (draft side only)
  int y_given;               // Y holds the pool's index already: only the accept test is taken
  const uint8_t *bins;       // optional: message[b] = bin of candidate Y[b]
  long long bins_stride_b;
  int32_t *message;
  uint8_t *accept;
  float *keyX, *keyY;  // optional
  double *log_keyX;    // optional [B][K]: ln of the normalised winning key (log kinds)
  double *log_secX;    // optional [B][K]: the same for the runner-up (another index) of that reduction
  // optional decoder outputs of the compression scheme (Appendix C, Appendix D.2): W_k = cand[X_k],
  // the estimate g(W_k, T_k) = (vz W_k + ve T_k) / (ve + vz + ve vz), the best squared error
  const float *cand;         // [B][V'] candidates U_i, or nullptr
  long long cand_stride_b;
  const float *side;         // [B][K] side information T_k
  long long side_stride_b;
  const float *source;       // [B] the source sample A (known to an evaluation only), or nullptr
  double var_e, var_z;       // variance of W given A, of T given A
  float *W, *A_hat;          // [B][K] optional
  float *sq_err;             // [B] optional: min_k (g(W_k, T_k) - A)^2
  int count_draft;     // count the draft side's reductions in stats->degenerate
  int count_pool;      // count the pool's
  int count_near;      // also count the near-ties of the sides that are counted
  llc_stats *stats;
};

struct ScanParams {
  const void *draft;
  const void *target;
  RowMap map;
  long long draft_stride_k;  // elements
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
  int no_pool;              // draft-side reductions only: the target is never read
  int no_draft;             // pool only: the draft rows are never read, X comes out as -1
  int same_race;            // every draft uses draft 0's race times (binned / pool-only variant only)
  const uint8_t *bins;      // optional [B][V] bins of the candidates (bins_stride_b bytes per row):
  long long bins_stride_b;  // on the draft side only candidates in the bin of index bin_of[b] count
  const int32_t *bin_of;    // [B]
  double *lse_part;         // [B][K+1][n_chunks] or nullptr: the scan also forms the rows' normalisers,
                            // ln of every chunk's sum of exp(x/T) (merged by the finalize kernel)
  const long long *draft_row_off;  // optional [B]: elements added to row b's draft offset; a negative
                            // entry means the row is not wanted (its partial results come out empty)
  int *shared_tau;          // [B][K+1] running bests shared by a row's workgroups, preset to
                            // the ordered image of +inf; nullptr when a row is one workgroup
  Partials out;
  llc_stats *stats;
  // The variant for rows that are one workgroup each also takes the finalize step, so that no
  // finalize launch follows.
  FinalizeParams fin;       // used by that variant only
};


// Algorithm 2's sequential epilogue over the per-(position, draft) target-side argmins.
struct VerifyParams {
  long long S;
  int L, K;
  const int32_t *cand;       // [S][L+1][K] argmin_i S_i^(j,k) / q_i^(j,k)
  const double *cand_key;    // [S][L+1][K] ln of its normalised key
  const double *cand_sec;    // [S][L+1][K] ln of the normalised runner-up key of the same reduction
  const int32_t *tokens;     // draft tokens
  long long tok_stride_s, tok_stride_j;
  int32_t *Y;                // [S][L+1]
  int32_t *n_out;            // [S]
  uint8_t *active;           // [S][K] optional
  float *keyY;               // [S][L+1] optional
  llc_stats *stats;          // optional: near_ties of the emitted positions
};

struct LseParams {
  const void *draft;
  const void *target;
  RowMap map;
  long long draft_stride_k;
  long long B;
  int K, V;
  int dtype;
  float temp_target, temp_draft_all;
  const float *temp_draft;
  int is_logits;  // divide by the temperature
  int per_k;      // every draft has its own row (else one row serves the K drafts)
  int with_target;  // also the target row's normaliser
  int with_drafts;  // the draft rows' normalisers (0: the scan kernel forms them itself)
  int vector_loads; // rows are aligned for 4-element vector loads
  const uint8_t *bins;      // as in ScanParams: masks the draft rows
  long long bins_stride_b;
  const int32_t *bin_of;
  const long long *draft_row_off;  // as in ScanParams (rows that are not wanted are skipped)
  double *lse;    // [B][K+1]
};

// One position of Algorithm 2's loop in its strongly drafter-invariant form (Appendix B): the pool
// runs over all K drafts' race times; a viable draft is priced with its own target row, a dropped
// one with the row of the first viable draft.
struct StrongStepParams {
  long long S;
  int L, K, j;               // position j of 0..L
  const int32_t *cand;       // [S][L+1][K] own-row argmins (viable drafts)
  const double *cand_key;    // [S][L+1][K] ln of their normalised keys
  const double *cand_sec;    // [S][L+1][K] ln of the normalised runner-up keys
  // this position priced with the first viable draft's row, as the scan left it: per-chunk
  // partial argmins (only read for dropped drafts; unused at j == 0)
  const double *part_key;    // [S][K][n_chunks] ln-domain keys before the normaliser is added
  const int32_t *part_idx;   // [S][K][n_chunks]
  const double *part_sec;    // [S][K][n_chunks] runner-up keys of the same partial reductions
  int n_chunks;
  int32_t *tau_all;          // [L][S][K+1] the later positions' shared running bests: reset at j == 0
  const int32_t *tokens;
  long long tok_stride_s, tok_stride_j;
  long long stride_k;        // of the target tensor, for the next position's row offsets
  uint8_t *viable;           // [S][K] state, set up at j == 0
  int32_t *running;          // [S] state
  long long *next_off;       // [S] out: stride_k * (first viable draft) if the next position needs
                             // dropped drafts priced, else -1
  const double *lse;         // [S][L+1][K+1] normalisers of every (position, draft) row
  double *lse_sel;           // [S][K+1] out: the normaliser of the row that prices the next position
  int32_t *Y;                // [S][L+1]
  int32_t *n_out;            // [S]
  uint8_t *active;           // [S][K] optional
  float *keyY;               // [S][L+1] optional
  llc_stats *stats;          // optional: near_ties of the emitted positions
};

// Algorithm 1 on candidate lists: one workgroup per row, every key exact.
struct TopmParams {
  long long B;
  int K, Md, Mt;
  int dtype, kind;
  const int32_t *draft_ids;
  const void *draft_val;
  long long draft_stride_b, draft_stride_k;
  const int32_t *target_ids;
  const void *target_val;
  long long target_stride_b;
  float temp_target, temp_draft_all;
  const float *temp_draft;
  unsigned seed_lo, seed_hi;
  unsigned long long row_offset;
  int32_t *X, *Y, *match_k;
  uint8_t *accept;
  float *keyX, *keyY;
  llc_stats *stats;
};

// Theorem 1's bound per row (diagnostics): one workgroup sorts a row by q/p and sums.
constexpr int kLmlMaxK = LLC_LML_MAX_K;
constexpr int kLmlSlots = 512;  // two 512-thread workgroups on each of 256 CUs: more cannot be resident
struct LmlParams {
  long long B;
  int V;
  int dtype;
  int probs;        // inputs are probabilities (else logits / log-weights)
  const void *draft;
  const void *target;
  long long draft_stride_b, target_stride_b;
  float temp_draft, temp_target;  // 1 for log-weights and probabilities
  int n_k;
  int k[kLmlMaxK];  // list sizes
  double *bound;    // [B][n_k]
  double *relaxed;  // [B][n_k] or nullptr
  double *tv;       // [B] or nullptr
  char *work;       // workspace: per slot two buffers of V sort keys, then two of V (p-mass, q-mass) pairs
  int slots;        // rows the workspace holds at a time (= rows per launch; a call is ceil(B / slots) launches)
  long long row0;   // first row of this launch (set by the launcher)
};

// One launcher per (element type, draft layout); defined in scan_*.hip.
// kt: drafts per workgroup pass (1, 2, 4, 8); probs: inputs are probabilities; finish: the
// variant that also takes the finalize step (plain scans only: no bins, no fused normalisers).
hipError_t launch_scan_f32_shared(int kt, bool probs, bool finish, unsigned grid, hipStream_t s, const ScanParams &p);
hipError_t launch_scan_f32_perk(int kt, bool probs, bool finish, unsigned grid, hipStream_t s, const ScanParams &p);
hipError_t launch_scan_bf16_shared(int kt, bool probs, bool finish, unsigned grid, hipStream_t s, const ScanParams &p);
hipError_t launch_scan_bf16_perk(int kt, bool probs, bool finish, unsigned grid, hipStream_t s, const ScanParams &p);
// the same with the race times drawn min-first (no binned or pool-only passes)
hipError_t launch_scan_f32_shared_minf(int kt, bool probs, bool finish, unsigned grid, hipStream_t s, const ScanParams &p);
hipError_t launch_scan_f32_perk_minf(int kt, bool probs, bool finish, unsigned grid, hipStream_t s, const ScanParams &p);
hipError_t launch_scan_bf16_shared_minf(int kt, bool probs, bool finish, unsigned grid, hipStream_t s, const ScanParams &p);
hipError_t launch_scan_bf16_perk_minf(int kt, bool probs, bool finish, unsigned grid, hipStream_t s, const ScanParams &p);

// llc_couple on a given workspace (api.hip).
int couple_on(const llc_couple_args *a, void *workspace, size_t workspace_bytes);

hipError_t launch_finalize(hipStream_t s, const FinalizeParams &p);
hipError_t launch_lse(hipStream_t s, const LseParams &p);
hipError_t launch_verify(hipStream_t s, const VerifyParams &p);
hipError_t launch_strong_step(hipStream_t s, const StrongStepParams &p);
hipError_t launch_fill(hipStream_t s, int32_t *dst, long long n, int32_t value);
hipError_t launch_topm(hipStream_t s, const TopmParams &p);
hipError_t launch_lml(hipStream_t s, const LmlParams &p);

}  // namespace llc
