/* llc.h -- list-level Gumbel-max coupling (Gumbel-max list sampling, GLS) on MI355X.
 *
 * C ABI of libllc_hip.so.  All data pointers are DEVICE pointers owned by the
 * caller (allocated by whatever the caller likes, e.g. torch); the library
 * allocates nothing, keeps no state between calls, enqueues its kernels on
 * `stream` and never synchronises.  Every entry point returns 0 (LLC_OK) or a
 * negative LLC_E_* code and never throws or aborts; argument errors are found
 * on the host before anything is launched.  Data-dependent conditions are not
 * errors: a reduction in which no entry has positive probability returns index
 * -1 (and accept = 0 for the row).
 *
 * Shared randomness (a reading, the paper only asks for i.i.d. uniforms):
 * Philox4x32 with 10 rounds, key = (lo32(seed), hi32(seed)), row = row_offset + b.
 * The 32-bit word x of element (row, k, i) is two 16-bit halves from two blocks:
 * counter (lo32(row), i >> 2, hi32(row), k >> 1) gives the upper half, the same
 * counter with bit 31 of its fourth word set gives the lower half; both read
 * output word (i & 3), its lower 16 bits for even k, its upper 16 bits for odd k.
 * U = (x + 1/2) / 2^32 and S = -ln U.
 * Ties in an argmin go to the smaller index, then (pool) to the smaller k.
 */
#ifndef LLC_H_
#define LLC_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define LLC_VERSION 110

enum {
  LLC_OK = 0,
  LLC_E_NULL = -1,      /* a required pointer is NULL                                   */
  LLC_E_SHAPE = -2,     /* B < 0, K < 1, V < 1, V >= 2^31 - 4, K > 65535, bad strides, or
                           more than 2^24 - 1 workgroups in one launch (B * ceil(K / k_tile)
                           * v_chunks: split such a batch over several calls)            */
  LLC_E_TEMP = -3,      /* a host-visible temperature is not finite and > 0             */
  LLC_E_DTYPE = -4,     /* unknown dtype / kind, or a combination that is not built     */
  LLC_E_ALIGN = -5,     /* an input base pointer is not aligned to its element size     */
  LLC_E_WORKSPACE = -6, /* workspace missing, misaligned (256 B) or too small           */
  LLC_E_LAUNCH = -7,    /* the HIP runtime refused a launch (hipGetLastError)           */
  LLC_E_OPTION = -8,    /* v_chunks / k_tile / flags out of range                       */
  LLC_E_SCRATCH = -9    /* llc_couple_static: the call needs more than LLC_STATIC_SCRATCH_BYTES */
};

enum { LLC_F32 = 0, LLC_BF16 = 1 };

/* How an input row denotes a distribution. */
enum {
  LLC_LOGITS = 0, /* p = softmax(x / T)                                              */
  LLC_PROBS = 1,  /* p = x as given (>= 0; need not sum to 1); temperatures ignored   */
  LLC_LOGW = 2    /* p = exp(x) / sum exp(x) (log-weights); temperatures ignored      */
};

enum {
  LLC_FLAG_EXACT_SCAN = 1, /* debugging: evaluate every key in fp64, no prefilter     */
  LLC_FLAG_STRONG = 2,     /* llc_verify only: the strongly drafter-invariant loop    */
  LLC_FLAG_SHARED_RACE = 8,/* llc_compress_select only: the baseline scheme of Section 5.3, in
                              which all decoders share one set of random numbers: the encoder's
                              pool and every decoder use the race times of the first set    */
  LLC_FLAG_DRY_RUN = 4,    /* llc_couple, llc_couple_is, llc_compress_select, llc_verify: check
                              the arguments, plan every launch of the call and check the
                              workspace against the plan, then return without launching
                              anything (no pointer is dereferenced)                    */
  LLC_FLAG_DRAFT_ONLY = 32,/* llc_couple, llc_couple_static, llc_couple_is: the draft side alone, i.e. the
                              drafters' step of Algorithm 2 (Section 4.2: every draft k samples its
                              next token X^(k) = argmin_i S_i^(k) / p_i^(k) with the randomness that
                              the verification of the same position will use).  No target is read
                              and nothing is written to Y, accept, match_k, keyY: those pointers,
                              `target` and its stride may be NULL / 0.  X and keyX are as without
                              the flag                                                  */
  LLC_FLAG_MIN_FIRST = 16  /* llc_couple, llc_couple_static, llc_couple_is, llc_verify: how Algorithm 1's
                              first step draws its K N independent Exp(1) race times from the row's
                              stream.  Default: one 32-bit word per (k, i), S = -ln U.  With this flag
                              the K times of an index are drawn through their minimum: M = -ln(U0) / K
                              (U0 from the index's own word) is the smallest, the draft kappa =
                              floor(K r / 2^32) (r: the index's second word) holds it, and every other
                              draft's time is M - ln U_i^(k), U_i^(k) its word as above.  The K times
                              are again independent Exp(1) variables (the minimum of K of them is
                              Exp(K), sits at a uniform position, and the others exceed it by
                              independent Exp(1) amounts), so every statement of Section 3 holds
                              unchanged; the samples differ from the default's for the same seed.
                              The scan then tests one word per index instead of one per (k, i).  All
                              calls that are to be coupled (the drafters' and the verifier's) must
                              agree on the flag.  LLC_E_OPTION in llc_compress_select, llc_couple_topm */
};

/* Optional device counters, accumulated with atomics (zero them yourself). */
typedef struct llc_stats {
  unsigned long long survivors;   /* elements that passed the integer prefilter              */
  unsigned long long exact_evals; /* keys evaluated in fp64                                  */
  unsigned long long slow_blocks; /* workgroups that fell back to the all-fp64 scan          */
  unsigned long long degenerate;  /* reductions that found no entry with positive probability */
  unsigned long long near_ties;   /* reductions whose winner is within 1e-6 (relative, in S/p) of
                                     the best key at another index: there the exact fp64 argmin
                                     returned here and an argmin taken in other arithmetic may
                                     differ (the paper's own caveat on floating-point determinism,
                                     Section 5.3).  llc_couple, llc_couple_is, llc_compress_select:
                                     every draft's reduction and the pool's; llc_verify: the pool
                                     of every emitted position; llc_couple_topm: both sides        */
} llc_stats;

/* Arguments of llc_couple: one call runs Algorithm 1 of the paper on B rows.
 *
 * Inputs.  draft is [B,K,V] addressed as draft[b*draft_stride_b + k*draft_stride_k + i]
 * (strides in elements, last dimension contiguous); draft_stride_k == 0 means the K
 * drafts of a row are i.i.d. from one proposal p_X (Section 4.1: a single draft model),
 * otherwise draft k has its own p^(k) (Appendix A.3).  target is [B,V].  Rows should
 * start on 16-byte boundaries for full-width loads; other layouts are read element-wise.
 *
 * Outputs.  X[b,k] = argmin_i S_i^(k) / p_i^(k);  Y[b] = argmin_i min_k S_i^(k) / q_i;
 * accept[b] = 1 iff Y[b] is one of X[b,0..K) (Section 3, Algorithm 1).
 * match_k[b] = the first k with X[b,k] == Y[b], else -1 (Section 4.1).
 * keyX / keyY = the winning values of S/p and S/q, with p, q normalised for the logit
 * and log-weight kinds and as given for the probability kind (+inf where the index is -1).
 */
typedef struct llc_couple_args {
  int64_t B, K, V;
  int32_t dtype;            /* LLC_F32 | LLC_BF16 (both inputs)                          */
  int32_t kind;             /* LLC_LOGITS | LLC_PROBS | LLC_LOGW (both inputs)           */
  const void *draft;        /* device */
  int64_t draft_stride_b, draft_stride_k;
  const void *target;       /* device */
  int64_t target_stride_b;
  float temp_target;        /* > 0; LLC_LOGITS only                                      */
  float temp_draft_all;     /* > 0; used when temp_draft == NULL                         */
  const float *temp_draft;  /* device, K entries, or NULL.  Entries must be finite and
                               > 0; they are not checked on the host, a bad entry makes
                               that draft's X equal -1.                                  */
  uint64_t seed;
  uint64_t row_offset;      /* global row of b = 0 (sharding, successive steps)          */
  int32_t *X;               /* [B,K] required                                            */
  int32_t *Y;               /* [B]   required                                            */
  uint8_t *accept;          /* [B]   required                                            */
  int32_t *match_k;         /* [B]   optional                                            */
  float *keyX;              /* [B,K] optional                                            */
  float *keyY;              /* [B]   optional                                            */
  llc_stats *stats;         /* optional device counters                                  */
  void *workspace;          /* device, 256-byte aligned, >= llc_couple_workspace_size()  */
  size_t workspace_bytes;
  void *stream;             /* hipStream_t; NULL = the default stream                    */
  int32_t flags;            /* LLC_FLAG_EXACT_SCAN | _DRY_RUN | _MIN_FIRST | _DRAFT_ONLY        */
  int32_t v_chunks;         /* 0 = choose; else split V over this many workgroups (1..4096).
                               Results do not depend on it.                              */
  int32_t k_tile;           /* 0 = choose; else drafts per workgroup pass: 2, 4 or 8 (1 is
                               accepted and runs as 2).  Results do not depend on it.    */
  void *ev_scan_begin;      /* optional hipEvent_t pair, recorded on `stream` right before */
  void *ev_scan_end;        /* and right after the scan kernel (for timing it alone)      */
} llc_couple_args;

/* Importance-weight form (Appendix C: lossy compression with K decoders, here L).
 * logw_enc[b,i] = ln of the encoder's unnormalised weight of candidate i (lambda~_q),
 * logw_dec[b,l,i] = ln of decoder l's (lambda~_p^(l)); fp32; -inf marks a candidate a
 * party has excluded.  Y[b] = the encoder's index (pool argmin under lambda_q),
 * X[b,l] = decoder l's index, accept[b] = 1 iff some decoder recovers Y[b].
 * Equivalent to llc_couple with kind = LLC_LOGW, draft = logw_dec, target = logw_enc.
 */
typedef struct llc_couple_is_args {
  int64_t B, L, N;
  const float *logw_enc;    /* device [B,N]   */
  int64_t enc_stride_b;
  const float *logw_dec;    /* device [B,L,N] */
  int64_t dec_stride_b, dec_stride_l;
  uint64_t seed, row_offset;
  int32_t *X;               /* [B,L] required */
  int32_t *Y;               /* [B]   required */
  uint8_t *accept;          /* [B]   required */
  int32_t *match_l;         /* [B]   optional */
  float *keyX;              /* [B,L] optional */
  float *keyY;              /* [B]   optional */
  llc_stats *stats;
  void *workspace;          /* >= llc_couple_workspace_size(B, L, N) */
  size_t workspace_bytes;
  void *stream;
  int32_t flags, v_chunks, k_tile;   /* as in llc_couple_args */
  void *ev_scan_begin, *ev_scan_end; /* as in llc_couple_args */
} llc_couple_is_args;

/* Arguments of llc_compress_select: the index selection of the list-decoding compression
 * scheme with bins (Section 5.1; Appendix C for importance weights).  Candidate i of row b
 * carries the bin bins[b*bins_stride_b + i] (one byte, so L_max <= 256).  The encoder draws
 * Y[b] = argmin_i min_l S_i^(l) / lambda_q,i over all N candidates and announces
 * message[b] = the bin of Y[b]; decoder l draws X[b,l] = argmin_i S_i^(l) / lambda_p,i^(l)
 * over the candidates of that bin only (its weights hold the indicator 1{l_i = message} and
 * are normalised over that bin).  accept[b] = 1 iff some decoder recovers Y[b].  Two passes
 * over the inputs (encoder, then decoders) on the same stream; otherwise as llc_couple_is,
 * with which it coincides when all candidates share one bin.
 *
 * Decoder outputs (optional; Appendix C and, for the Gaussian source, Appendix D.2).  Given the
 * candidates cand[b,i] = U_i (the prior samples the weights were computed on) the call returns
 * decoder l's output W[b,l] = U_{X[b,l]}.  Given also its side information side[b,l] = T_l and
 * the two variances of the Gaussian model (W = A + eta, T = A + zeta), it returns the MMSE
 * estimate A_hat[b,l] = (var_t_given_a * W + var_w_given_a * T_l) /
 * (var_w_given_a + var_t_given_a + var_w_given_a * var_t_given_a), and, given the source sample
 * source[b] = A (which only an evaluation knows), the trial's distortion sq_err[b] =
 * min_l (A_hat[b,l] - A)^2, the estimate with the least error among the decoders (Section 5.3).
 * A decoder that found no candidate (X = -1) gives NaN and takes no part in the minimum
 * (+inf if none did).  Arithmetic in fp64 on the fp32 inputs, results rounded to fp32.
 */
typedef struct llc_compress_select_args {
  int64_t B, L, N;
  const float *logw_enc;    /* device [B,N]   */
  int64_t enc_stride_b;
  const float *logw_dec;    /* device [B,L,N] */
  int64_t dec_stride_b, dec_stride_l;
  const uint8_t *bins;      /* device [B,N]   */
  int64_t bins_stride_b;
  uint64_t seed, row_offset;
  int32_t *X;               /* [B,L] required */
  int32_t *Y;               /* [B]   required */
  uint8_t *accept;          /* [B]   required */
  int32_t *message;         /* [B]   optional */
  int32_t *match_l;         /* [B]   optional */
  float *keyX;              /* [B,L] optional: S / lambda_p with lambda_p normalised over the bin */
  float *keyY;              /* [B]   optional */
  llc_stats *stats;
  void *workspace;          /* >= llc_couple_workspace_size(B, L, N) */
  size_t workspace_bytes;
  void *stream;
  int32_t flags, v_chunks, k_tile;   /* LLC_FLAG_SHARED_RACE is taken here                   */
  void *ev_scan_begin, *ev_scan_end; /* recorded around the decoders' scan */
  /* decoder outputs: all optional; W needs cand, A_hat also side and the variances, sq_err also source */
  const float *cand;        /* device [B,N] candidates U_i                                  */
  int64_t cand_stride_b;
  const float *side;        /* device [B,L] side information T_l                            */
  int64_t side_stride_b;
  const float *source;      /* device [B] source samples A                                  */
  float var_w_given_a;      /* finite and > 0 when any of the outputs below is asked for     */
  float var_t_given_a;
  float *W;                 /* [B,L] */
  float *A_hat;             /* [B,L] */
  float *sq_err;            /* [B]   */
} llc_compress_select_args;

/* Arguments of llc_verify: the verification loop of Algorithm 2 (Section 4.2,
 * drafter-invariant multi-draft speculative decoding) for S independent sequences, each
 * with K drafts of L tokens.
 *
 * Inputs.  target[s,j,k,:] denotes q^(j,k), the target model's next-token distribution
 * after draft k's first j tokens, j = 0..L (j = L is the bonus position); addressed as
 * target[s*stride_s + j*stride_j + k*stride_k + i], last dimension contiguous, kind
 * LLC_LOGITS (with temp_target) or LLC_LOGW (the keys of different rows are compared, so
 * rows must be normalisable: LLC_PROBS is refused).  tokens[s*tok_stride_s + j*tok_stride_j
 * + k] = X_j^(k), j = 0..L-1, the draft tokens (from llc_couple's X, or anywhere else).
 * Randomness: position j of sequence s uses the stream of row
 * row_offset + s*row_stride_s + j*row_stride_j, draft k uses counter word k, exactly as
 * llc_couple does, so a drafting call on the same row and this call are coupled.
 *
 * Outputs.  Position by position, Y[s,j] = argmin_i min_{k viable} S_i^(j,k) / q_i^(j,k)
 * with q normalised; every draft whose token differs from Y[s,j] stops being viable; the
 * loop ends after the first position at which no draft is viable, or after the bonus
 * position.  n_out[s] = number of tokens emitted (accepted + 1), Y[s,j] = -1 for
 * j >= n_out[s].  active[s,k] = 1 iff draft k is still viable at the end (all L tokens
 * accepted).  keyY[s,j] = the winning S/q.  Yk / keyYk[s,j,k] = draft k's own
 * argmin_i S_i^(j,k)/q_i^(j,k) and its key, whether or not k was viable.
 *
 * flags & LLC_FLAG_STRONG: the strongly drafter-invariant form (Appendix B).  The minimum of a
 * position runs over all K drafts' race times: a viable draft is priced with its own row as
 * above, a draft that has been dropped with the row of the first draft that is still viable
 * (whose prefix is the output so far).  The viability rule and every output are as above.  The
 * positions are then processed one after the other (L extra, small, passes over one row per
 * sequence).
 */
typedef struct llc_verify_args {
  int64_t S, L, K, V;       /* S >= 0, L >= 0, K in 1..64, V >= 1                       */
  int32_t dtype;            /* LLC_F32 | LLC_BF16                                        */
  int32_t kind;             /* LLC_LOGITS | LLC_LOGW                                     */
  const void *target;       /* device [S, L+1, K, V]                                     */
  int64_t stride_s, stride_j, stride_k;
  float temp_target;        /* > 0; LLC_LOGITS only                                      */
  const int32_t *tokens;    /* device [S, L, K]; may be NULL when L == 0                 */
  int64_t tok_stride_s, tok_stride_j;
  uint64_t seed, row_offset;
  int64_t row_stride_s, row_stride_j; /* >= 0                                            */
  int32_t *Y;               /* [S, L+1] required                                         */
  int32_t *n_out;           /* [S]      required                                         */
  uint8_t *active;          /* [S, K]   optional                                         */
  float *keyY;              /* [S, L+1] optional                                         */
  int32_t *Yk;              /* [S, L+1, K] optional                                      */
  float *keyYk;             /* [S, L+1, K] optional                                      */
  llc_stats *stats;
  void *workspace;          /* device, 256-byte aligned, >= llc_verify_workspace_size()  */
  size_t workspace_bytes;
  void *stream;
  int32_t flags, v_chunks, k_tile;   /* as in llc_couple_args, and LLC_FLAG_STRONG       */
  void *ev_scan_begin, *ev_scan_end; /* as in llc_couple_args                            */
} llc_verify_args;

/* Arguments of llc_couple_topm: Algorithm 1 on candidate lists (Section 4.4: with top-K
 * sampling all but M << N high-probability tokens are thrown away before the coupling).
 *
 * Inputs.  Each distribution is a list of (token id, value) pairs: draft k of row b has
 * entries e = 0..Md-1 at draft_ids / draft_val[b*draft_stride_b + k*draft_stride_k + e]
 * (draft_stride_k == 0: the K drafts are i.i.d. from one list), the target has Mt entries
 * at target_ids / target_val[b*target_stride_b + e].  Values denote the distribution
 * restricted to the list (softmax over the list for logits, normalised over the list for
 * log-weights, as given for probabilities).  Ids must lie in [0, 2^31 - 4); an entry with a
 * negative id is an empty slot.  An id that occurs twice in a list competes twice with the
 * same race time (the larger probability wins).  The lists of the two sides need not hold
 * the same ids: the uniforms are keyed by the token id, exactly as in llc_couple, so the
 * result equals llc_couple on the dense rows that carry no mass outside the lists.
 *
 * Outputs are token ids: X[b,k] = id of argmin_e S_id^(k) / p_e^(k), Y[b] = id of the pool
 * argmin over (k, target entry); ties go to the smaller id, then the smaller k; accept,
 * match_k, keyX, keyY as in llc_couple.  No workspace is needed.
 */
typedef struct llc_couple_topm_args {
  int64_t B, K, Md, Mt;     /* B >= 0, K in 1..1024, Md, Mt in 1..65536                   */
  int32_t dtype;            /* LLC_F32 | LLC_BF16 (both value arrays)                     */
  int32_t kind;             /* LLC_LOGITS | LLC_PROBS | LLC_LOGW                          */
  const int32_t *draft_ids; /* device */
  const void *draft_val;    /* device */
  int64_t draft_stride_b, draft_stride_k;   /* elements, shared by ids and values         */
  const int32_t *target_ids;/* device */
  const void *target_val;   /* device */
  int64_t target_stride_b;
  float temp_target;        /* > 0; LLC_LOGITS only                                       */
  float temp_draft_all;     /* > 0; used when temp_draft == NULL                          */
  const float *temp_draft;  /* device, K entries, or NULL                                 */
  uint64_t seed, row_offset;
  int32_t *X;               /* [B,K] required */
  int32_t *Y;               /* [B]   required */
  uint8_t *accept;          /* [B]   required */
  int32_t *match_k;         /* [B]   optional */
  float *keyX;              /* [B,K] optional */
  float *keyY;              /* [B]   optional */
  llc_stats *stats;         /* optional: exact_evals and degenerate are counted           */
  void *stream;
  void *ev_begin, *ev_end;  /* optional hipEvent_t pair recorded around the kernel        */
} llc_couple_topm_args;

/* Arguments of llc_lml_bound: the list matching lemma's lower bound on the probability that the
 * target's sample is in the list (Theorem 1, eq. (1)), per row and for several list sizes K at
 * once, for K drafts drawn i.i.d. from the row's proposal p against the row's target q:
 *   bound[b,n] = sum_j K_n / sum_i ( max{q_i/q_j, p_i/p_j} + (K_n - 1) q_i/q_j ).
 * Also, on request, the relaxed form stated after the theorem,
 *   relaxed[b,n] = sum_j q_j / (1 + q_j / (K_n p_j)),
 * and the total variation distance tv[b] = (1/2) sum_j |p_j - q_j| (the introduction's two-party
 * bound is (1 - tv)/(1 + tv)).  A diagnostic: it draws no randomness.
 *
 * Inputs as in llc_couple with one proposal row per batch row (draft is [B,V]); p and q are the
 * softmax of logits / temperature, the normalised exp of log-weights, or the given probabilities
 * divided by their sum.  An entry without mass on one side (logit -inf, probability 0) adds no
 * term j but still counts as a summand i with the mass it has on the other side (the limit of the
 * formula); NaN and +inf entries carry no mass.  Results are fp64; indices whose q/p agree to fp32
 * precision are ordered arbitrarily and the masses enter the running sums rounded to fp32, which
 * together move a result by a relative 2^-22 at most.
 * The workspace (256-byte aligned, device) belongs to the call until it has finished: 24 V bytes
 * serve one row at a time, llc_lml_workspace_size gives what keeps the whole GPU busy (at most 512
 * rows' worth, whatever B is); a smaller one, down to one row's, is accepted and only costs time. */
#define LLC_LML_MAX_K 8
typedef struct llc_lml_args {
  int64_t B, V;             /* 0 <= B < 2^31, 1 <= V <= 2^28                              */
  int32_t dtype;            /* LLC_F32 | LLC_BF16 (both inputs)                           */
  int32_t kind;             /* LLC_LOGITS | LLC_PROBS | LLC_LOGW                          */
  const void *draft;        /* device, [B,V]                                              */
  int64_t draft_stride_b;   /* elements                                                   */
  const void *target;       /* device, [B,V]                                              */
  int64_t target_stride_b;
  float temp_target;        /* > 0; LLC_LOGITS only                                       */
  float temp_draft;         /* > 0; LLC_LOGITS only                                       */
  int32_t n_k;              /* 1..LLC_LML_MAX_K list sizes                                */
  int32_t k[LLC_LML_MAX_K]; /* each >= 1                                                  */
  double *bound;            /* device [B,n_k] required */
  double *relaxed;          /* device [B,n_k] optional */
  double *tv;               /* device [B]     optional */
  void *workspace;
  size_t workspace_bytes;
  void *stream;
  void *ev_begin, *ev_end;  /* optional hipEvent_t pair recorded around the kernel        */
} llc_lml_args;

/* Algorithm 1 on a batch (Section 3).  Asynchronous on a->stream. */
int llc_couple(const llc_couple_args *a);

/* llc_couple for callers that cannot allocate device memory or pass a workspace: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments,
 * same kernels and same results as llc_couple, but a->workspace and a->workspace_bytes are
 * ignored: the partial results live in an array of LLC_STATIC_SCRATCH_BYTES that is part of
 * the library's device code (each GPU the library runs on holds its copy until the process
 * ends).  The call allocates and frees nothing.  The device that a->stream belongs to must be
 * the current device.  A shape whose partial results do not fit (roughly B * K * chunks above
 * 2^19) returns LLC_E_SCRATCH before anything is launched.  All calls on one GPU share the
 * array: calls that may overlap in time (different streams, different threads) race; order
 * them on one stream.  Nothing is carried over between calls. */
#define LLC_STATIC_SCRATCH_BYTES (16u << 20)
int llc_couple_static(const llc_couple_args *a);

/* Appendix C's index selection at the encoder and the L decoders.  Asynchronous. */
int llc_couple_is(const llc_couple_is_args *a);

/* Binned index selection of the compression scheme (Section 5.1, Appendix C).  Asynchronous. */
int llc_compress_select(const llc_compress_select_args *a);

/* Algorithm 1 on top-M candidate lists (Section 4.4).  Asynchronous. */
int llc_couple_topm(const llc_couple_topm_args *a);

/* Algorithm 2's verification loop (Section 4.2) on S sequences.  Asynchronous. */
int llc_verify(const llc_verify_args *a);

/* Theorem 1's lower bound on the matching probability, per row (Section 3).  Asynchronous. */
int llc_lml_bound(const llc_lml_args *a);

/* Bytes of device scratch with which llc_lml_bound runs at full speed (min(B, 512) x 24 V + 256);
 * 0 on bad shapes. */
size_t llc_lml_workspace_size(int64_t B, int64_t V);

/* Bytes of device scratch llc_couple, llc_couple_is and llc_compress_select need for this shape:
 * enough for any k_tile and for v_chunks = 0 (the library's choice) or up to 16; an explicit
 * v_chunks = c above 16 needs ceil(c / 16) times as much.  0 on bad shapes. */
size_t llc_couple_workspace_size(int64_t B, int64_t K, int64_t V);

/* Bytes of device scratch llc_verify needs for this shape, either form of the loop (same rule
 * for v_chunks and k_tile); 0 on bad shapes. */
size_t llc_verify_workspace_size(int64_t S, int64_t L, int64_t K, int64_t V);

/* Text for a return code (static storage). */
const char *llc_status_string(int code);

/* LLC_VERSION of the built library. */
int llc_version(void);

#ifdef __cplusplus
}
#endif
#endif /* LLC_H_ */
