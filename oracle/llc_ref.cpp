// CPU oracle for Gumbel-max list sampling (GLS).  TEST INFRASTRUCTURE ONLY.
//
// This file is the slow, literal, scalar fp64 statement of what the sampler
// computes.  Only the test-suite, the smoke check and the benchmark's
// cpu_baseline leg may load it; the product (the HIP library) never does, and
// shares no source, header, table or helper with it.
//
// What is computed, per row (paper Section 3, Algorithm 1):
//   * shared uniforms U_i^(k), race times S_i^(k) = -ln U_i^(k)      (Alg. 1, step 2)
//   * Y       = argmin_i min_k S_i^(k) / q_i                          (Alg. 1, step 3)
//   * X^(k)   = argmin_i S_i^(k) / p_i^(k)                            (Alg. 1, step 4;
//               distinct proposals p^(k): Appendix A.3)
//   * accept  = [ Y in {X^(1..K)} ]                                   (Alg. 1, step 5)
// llc_verify_ref is Algorithm 2's verification loop (Section 4.2): position by
// position the target token is the pool argmin over the drafts that are still
// viable, and drafts whose token differs are dropped.
// llc_couple_topm_ref is Algorithm 1 on candidate lists (Section 4.4: top-K sampling
// keeps M << N tokens): every distribution is a list of (token id, value) pairs,
// normalised over the list, and the uniforms are keyed by the token id.
// The importance-weight form (Appendix C, the normalised weights lambda_q,
// lambda_p^(k) and the selection rule below them) is the same computation with
// p, q proportional to exp(log-weight).
//
// Readings the paper leaves open (each is also listed in the design notes):
//   * generator: Philox4x32 with 10 rounds (Salmon et al., SC'11); key = the
//     two halves of `seed`; the 32-bit word of element (row, k, i) is made of two
//     16-bit halves taken from two blocks (see shared_word).  row = row_offset + b.
//   * U on the open interval: U = (x + 1/2) / 2^32 for the 32-bit word x.
//   * how step 1's K N independent uniforms come out of the stream: one word per (k, i), or
//     (min_first) the K race times of an index drawn through their minimum (see row_race_time).
//   * argmin ties: smallest key, then smallest i, then (pool only) smallest k.
//   * entries that are NaN or +inf (logit kinds) / NaN, +inf or negative
//     (probability kind) carry zero probability.  A reduction with no finite
//     key returns index -1.
//   * temperature: p = softmax(logit / T), T the fp32 value widened to fp64.
//
// Build: g++ -O2 -fno-fast-math -fopenmp -shared -fPIC (see build.py).

#include <cmath>
#include <cstdint>
#include <cstring>
#include <limits>
#include <vector>

#ifdef _OPENMP
#include <omp.h>
#endif

namespace {

const double kInf = std::numeric_limits<double>::infinity();

// ---- Philox4x32-10 ---------------------------------------------------------
// One round: two 32x32->64 products, the high halves are mixed with the other
// counter words and the round key, the low halves pass through.
void philox_round(uint32_t c[4], const uint32_t k[2]) {
  const uint64_t prod0 = (uint64_t)0xD2511F53u * (uint64_t)c[0];
  const uint64_t prod1 = (uint64_t)0xCD9E8D57u * (uint64_t)c[2];
  const uint32_t hi0 = (uint32_t)(prod0 >> 32), lo0 = (uint32_t)prod0;
  const uint32_t hi1 = (uint32_t)(prod1 >> 32), lo1 = (uint32_t)prod1;
  const uint32_t n0 = hi1 ^ c[1] ^ k[0];
  const uint32_t n1 = lo1;
  const uint32_t n2 = hi0 ^ c[3] ^ k[1];
  const uint32_t n3 = lo0;
  c[0] = n0; c[1] = n1; c[2] = n2; c[3] = n3;
}

void philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]) {
  uint32_t c[4] = {ctr[0], ctr[1], ctr[2], ctr[3]};
  uint32_t k[2] = {key[0], key[1]};
  for (int r = 0; r < 10; ++r) {
    if (r > 0) {  // Weyl key schedule: bump before every round but the first
      k[0] += 0x9E3779B9u;
      k[1] += 0xBB67AE85u;
    }
    philox_round(c, k);
  }
  for (int j = 0; j < 4; ++j) out[j] = c[j];
}

// 32-bit word for element (row, k, i): two 16-bit halves from two Philox blocks.
// Four consecutive indices and two consecutive drafts share a block: counter
// (lo32(row), i >> 2, hi32(row), k >> 1) gives the high halves, the same counter with bit 31
// of its fourth word set gives the low halves; element (k, i) reads output word (i & 3) of
// each, its lower 16 bits for even k and its upper 16 bits for odd k.
uint32_t shared_word(uint64_t seed, uint64_t row, uint32_t k, uint64_t i) {
  const uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
  const uint32_t ctr_hi[4] = {(uint32_t)row, (uint32_t)(i >> 2), (uint32_t)(row >> 32), k >> 1};
  const uint32_t ctr_lo[4] = {(uint32_t)row, (uint32_t)(i >> 2), (uint32_t)(row >> 32), (k >> 1) | 0x80000000u};
  uint32_t out_hi[4], out_lo[4];
  philox4x32_10(ctr_hi, key, out_hi);
  philox4x32_10(ctr_lo, key, out_lo);
  const unsigned shift = (k & 1u) ? 16u : 0u;
  const uint32_t hi16 = (out_hi[i & 3] >> shift) & 0xFFFFu;
  const uint32_t lo16 = (out_lo[i & 3] >> shift) & 0xFFFFu;
  return (hi16 << 16) | lo16;
}

// S = -ln U with U = (x + 1/2) 2^-32 (exact in fp64).  Section 3: S_i^(k) = -ln U_i^(k).
double race_time(uint32_t x) {
  const double U = ((double)x + 0.5) * (1.0 / 4294967296.0);
  return -std::log(U);
}

// Auxiliary 32-bit word of (row, i): output word (i & 3) of the block with counter
// (lo32(row), i >> 2, hi32(row), 0x40000000 | which).  Bit 30 of the fourth counter word keeps
// these blocks apart from the per-draft ones.  which = 0: the word of the smallest race time of
// index i; which = 1: the word that picks the draft holding it.
uint32_t aux_word(uint64_t seed, uint64_t row, uint64_t i, uint32_t which) {
  const uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
  const uint32_t ctr[4] = {(uint32_t)row, (uint32_t)(i >> 2), (uint32_t)(row >> 32), 0x40000000u | which};
  uint32_t out[4];
  philox4x32_10(ctr, key, out);
  return out[i & 3];
}

// Race time S_i^(k) of a row with K drafts.  Algorithm 1's first step asks for K N independent
// uniforms U_i^(k), i.e. independent Exp(1) race times S = -ln U; it does not say how to draw them.
//   min_first == 0: one word per (k, i), S = -ln U of that word.
//   min_first != 0: the K race times of index i are drawn through their minimum.  The smallest of
//     K independent Exp(1) variables is Exp(K), it sits at a uniformly random draft, and the
//     others exceed it by independent Exp(1) amounts (memorylessness): with M = -ln(U0) / K from
//     the index's first auxiliary word and kappa = floor(K r / 2^32) from its second, S^(kappa) = M
//     and S^(k) = M - ln U_i^(k) for k != kappa, U_i^(k) from the word of (k, i) as above.  The K
//     times are again independent Exp(1) (so the U = exp(-S) are the independent uniforms of step
//     1), and the pool's key of index i, min_k S_i^(k) / q_i, is M / q_i.
double row_race_time(int min_first, uint64_t seed, uint64_t row, uint32_t k, uint64_t i, int64_t K) {
  if (!min_first) return race_time(shared_word(seed, row, k, i));
  const double M = race_time(aux_word(seed, row, i, 0)) / (double)K;
  const uint32_t kappa = (uint32_t)(((uint64_t)aux_word(seed, row, i, 1) * (uint64_t)K) >> 32);
  if (k == kappa) return M;
  return M + race_time(shared_word(seed, row, k, i));
}

// ---- inputs ---------------------------------------------------------------
enum { DT_F32 = 0, DT_BF16 = 1 };
enum { KIND_LOGITS = 0, KIND_PROBS = 1, KIND_LOGW = 2 };

double load_elem(const void *base, int dtype, int64_t off) {
  if (dtype == DT_F32) {
    return (double)((const float *)base)[off];
  }
  // bfloat16 = the top 16 bits of an fp32
  const uint16_t h = ((const uint16_t *)base)[off];
  const uint32_t w = (uint32_t)h << 16;
  float f;
  std::memcpy(&f, &w, 4);
  return (double)f;
}

// Fill prob[0..V) with the distribution one input row denotes; return the
// normaliser's log (0 for the probability kind, which is used as given).
// logit kinds: p = softmax(x / T).  log-weight kind: p = exp(x) / sum exp(x).
void row_distribution(const void *base, int dtype, int64_t off, int64_t V, int kind,
                      double T, std::vector<double> &prob) {
  prob.resize((size_t)V);
  if (kind == KIND_PROBS) {
    for (int64_t i = 0; i < V; ++i) {
      const double v = load_elem(base, dtype, off + i);
      prob[i] = (std::isfinite(v) && v > 0.0) ? v : 0.0;
    }
    return;
  }
  const double temp = (kind == KIND_LOGITS) ? T : 1.0;
  double zmax = -kInf;
  for (int64_t i = 0; i < V; ++i) {
    double z = load_elem(base, dtype, off + i) / temp;
    if (std::isnan(z) || z == kInf) z = -kInf;
    prob[i] = z;
    if (z > zmax) zmax = z;
  }
  if (zmax == -kInf) {
    for (int64_t i = 0; i < V; ++i) prob[i] = 0.0;
    return;
  }
  double sum = 0.0;
  for (int64_t i = 0; i < V; ++i) sum += std::exp(prob[i] - zmax);
  const double lse = zmax + std::log(sum);
  for (int64_t i = 0; i < V; ++i) prob[i] = std::exp(prob[i] - lse);
}

// The distribution a candidate list denotes, on its own entries (Section 4.4: all but the M listed
// tokens are thrown away).  An entry with a negative id is an empty slot and carries nothing.
void list_distribution(const int32_t *ids, const void *val, int dtype, int64_t off, int64_t M,
                       int kind, double T, std::vector<double> &prob) {
  prob.assign((size_t)M, 0.0);
  if (kind == KIND_PROBS) {
    for (int64_t e = 0; e < M; ++e) {
      const double v = load_elem(val, dtype, off + e);
      prob[e] = (ids[e] >= 0 && std::isfinite(v) && v > 0.0) ? v : 0.0;
    }
    return;
  }
  const double temp = (kind == KIND_LOGITS) ? T : 1.0;
  double zmax = -kInf;
  for (int64_t e = 0; e < M; ++e) {
    double z = load_elem(val, dtype, off + e) / temp;
    if (ids[e] < 0 || std::isnan(z) || z == kInf) z = -kInf;
    prob[e] = z;
    if (z > zmax) zmax = z;
  }
  if (zmax == -kInf) {
    for (int64_t e = 0; e < M; ++e) prob[e] = 0.0;
    return;
  }
  double sum = 0.0;
  for (int64_t e = 0; e < M; ++e) sum += std::exp(prob[e] - zmax);
  const double lse = zmax + std::log(sum);
  for (int64_t e = 0; e < M; ++e) prob[e] = std::exp(prob[e] - lse);
}

// Running (smallest, runner-up) of a race; `second` is the smallest key among
// entries whose index differs from the leader's index.
struct Race {
  double best = kInf;
  int64_t idx = -1;
  int64_t k = -1;
  double second = kInf;
  void offer(double key, int64_t i, int64_t kk) {
    if (!(key < kInf)) return;
    bool wins = false;
    if (idx < 0) wins = true;
    else if (key < best) wins = true;
    else if (key == best) {
      if (i < idx) wins = true;
      else if (i == idx && kk < k) wins = true;
    }
    if (wins) {
      if (idx >= 0 && idx != i) {
        if (best < second) second = best;
      }
      best = key; idx = i; k = kk;
    } else if (i != idx) {
      if (key < second) second = key;
    }
  }
  double rel_gap() const {
    if (idx < 0) return kInf;
    if (!(second < kInf)) return kInf;
    if (best == 0.0) return second > 0.0 ? kInf : 0.0;
    return (second - best) / best;
  }
};

}  // namespace

extern "C" {

struct llc_ref_args {
  int64_t B, K, V;
  int32_t dtype, kind;
  const void *draft;   // host
  int64_t draft_stride_b, draft_stride_k;  // elements; stride_k == 0: one p per row
  const void *target;  // host
  int64_t target_stride_b;
  float temp_target;
  const float *temp_draft;  // K entries or NULL
  float temp_draft_all;
  uint64_t seed, row_offset;
  // outputs (host); any of the optional ones may be NULL
  int32_t *X;        // [B,K]
  int32_t *Y;        // [B]
  uint8_t *accept;   // [B]
  int32_t *match_k;  // [B]   optional
  double *keyX;      // [B,K] optional: winning S/p
  double *keyY;      // [B]   optional: winning S/q over the pool
  int32_t *Yk;       // [B,K] optional: argmin_i S_i^(k)/q_i
  double *keyYk;     // [B,K] optional
  double *gapX;      // [B,K] optional: (runner-up - best)/best on the draft side
  double *gapY;      // [B]   optional: same for the pool, runner-up with index != Y
  double *gapYk;     // [B,K] optional
  int32_t threads;   // <=0: all
  int32_t min_first; // how the race times are drawn from the stream (see row_race_time)
};

void llc_ref_philox4x32_10(const uint32_t *ctr, const uint32_t *key, uint32_t *out) {
  philox4x32_10(ctr, key, out);
}

uint32_t llc_ref_shared_word(uint64_t seed, uint64_t row, uint32_t k, uint64_t i) {
  return shared_word(seed, row, k, i);
}

double llc_ref_race_time(uint32_t x) { return race_time(x); }

uint32_t llc_ref_aux_word(uint64_t seed, uint64_t row, uint64_t i, uint32_t which) {
  return aux_word(seed, row, i, which);
}

// out[r * K + k] = S_i^(k) of row row0 + r, for r = 0..n_rows-1.
void llc_ref_race_times(int32_t min_first, uint64_t seed, uint64_t row0, int64_t n_rows, uint64_t i,
                        int64_t K, double *out) {
  for (int64_t r = 0; r < n_rows; ++r)
    for (int64_t k = 0; k < K; ++k)
      out[r * K + k] = row_race_time(min_first, seed, row0 + (uint64_t)r, (uint32_t)k, i, K);
}

int llc_ref_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

// Algorithm 1 over a batch of rows.  Returns 0, or -1 on a malformed call.
int llc_couple_ref(const llc_ref_args *a) {
  if (!a || !a->draft || !a->target || !a->X || !a->Y || !a->accept) return -1;
  if (a->B < 0 || a->K < 1 || a->V < 1) return -1;
  const int64_t B = a->B, K = a->K, V = a->V;
  int nthreads = a->threads;
#ifdef _OPENMP
  if (nthreads <= 0) nthreads = omp_get_max_threads();
#else
  nthreads = 1;
#endif

#pragma omp parallel for schedule(dynamic, 1) num_threads(nthreads)
  for (int64_t b = 0; b < B; ++b) {
    const uint64_t row = a->row_offset + (uint64_t)b;
    std::vector<double> q, p;
    row_distribution(a->target, a->dtype, b * a->target_stride_b, V, a->kind,
                     (double)a->temp_target, q);
    Race pool;                 // over all (k, i): the flattened K*V race of Theorem 1's proof
    int64_t match = -1;
    std::vector<int64_t> xs((size_t)K);
    for (int64_t k = 0; k < K; ++k) {
      if (k == 0 || a->draft_stride_k != 0 || a->temp_draft) {
        const double Tk = a->temp_draft ? (double)a->temp_draft[k] : (double)a->temp_draft_all;
        row_distribution(a->draft, a->dtype, b * a->draft_stride_b + k * a->draft_stride_k,
                         V, a->kind, Tk, p);
      }
      Race draft, tk;
      for (int64_t i = 0; i < V; ++i) {
        const double S = row_race_time(a->min_first, a->seed, row, (uint32_t)k, (uint64_t)i, K);
        const double kx = p[i] > 0.0 ? S / p[i] : kInf;
        const double ky = q[i] > 0.0 ? S / q[i] : kInf;
        draft.offer(kx, i, k);
        tk.offer(ky, i, k);
        pool.offer(ky, i, k);
      }
      xs[k] = draft.idx;
      a->X[b * K + k] = (int32_t)draft.idx;
      if (a->keyX) a->keyX[b * K + k] = draft.best;
      if (a->gapX) a->gapX[b * K + k] = draft.rel_gap();
      if (a->Yk) a->Yk[b * K + k] = (int32_t)tk.idx;
      if (a->keyYk) a->keyYk[b * K + k] = tk.best;
      if (a->gapYk) a->gapYk[b * K + k] = tk.rel_gap();
    }
    a->Y[b] = (int32_t)pool.idx;
    if (a->keyY) a->keyY[b] = pool.best;
    if (a->gapY) a->gapY[b] = pool.rel_gap();
    if (pool.idx >= 0) {
      for (int64_t k = 0; k < K; ++k) {
        if (xs[k] == pool.idx) { match = k; break; }
      }
    }
    a->accept[b] = (uint8_t)(match >= 0);
    if (a->match_k) a->match_k[b] = (int32_t)match;
  }
  return 0;
}

// Importance-weight form (Appendix C): the encoder's index is the pool argmin
// under lambda_q, decoder l's index is the argmin under lambda_p^(l); weights
// are given as logs and normalised over the N candidates.
int llc_couple_is_ref(int64_t B, int64_t L, int64_t N,
                      const float *logw_enc, int64_t enc_stride_b,
                      const float *logw_dec, int64_t dec_stride_b, int64_t dec_stride_l,
                      uint64_t seed, uint64_t row_offset,
                      int32_t *X, int32_t *Y, uint8_t *accept, int32_t *match_l,
                      double *keyX, double *keyY, double *gapX, double *gapY, int32_t threads,
                      int32_t min_first) {
  llc_ref_args a;
  std::memset(&a, 0, sizeof(a));
  a.B = B; a.K = L; a.V = N;
  a.dtype = DT_F32; a.kind = KIND_LOGW;
  a.draft = logw_dec; a.draft_stride_b = dec_stride_b; a.draft_stride_k = dec_stride_l;
  a.target = logw_enc; a.target_stride_b = enc_stride_b;
  a.temp_target = 1.0f; a.temp_draft = nullptr; a.temp_draft_all = 1.0f;
  a.seed = seed; a.row_offset = row_offset;
  a.X = X; a.Y = Y; a.accept = accept; a.match_k = match_l;
  a.keyX = keyX; a.keyY = keyY; a.gapX = gapX; a.gapY = gapY;
  a.threads = threads;
  a.min_first = min_first;
  return llc_couple_ref(&a);
}

// Index selection of the list-decoding compression scheme with bins (Section 5.1; Appendix C for
// importance weights).  Candidate i carries a bin l_i.  The encoder draws Y = argmin_i min_l
// S_i^(l) / lambda_q,i over all candidates and sends the message M = l_Y; decoder l draws
// X^(l) = argmin_i S_i^(l) / lambda_p,i^(l) over the candidates with l_i = M only (its weights
// carry the indicator 1{l_i = M} and are normalised over those candidates).  bins: [B,N] uint8.
// shared_race != 0 is the baseline scheme that Section 5.3 compares with: all decoders share the
// same set of random numbers, i.e. every decoder (and the encoder's pool) uses the race times of
// the first set, S_i^(1).
int llc_compress_select_ref(int64_t B, int64_t L, int64_t N,
                            const float *logw_enc, int64_t enc_stride_b,
                            const float *logw_dec, int64_t dec_stride_b, int64_t dec_stride_l,
                            const uint8_t *bins, int64_t bins_stride_b,
                            uint64_t seed, uint64_t row_offset,
                            int32_t *X, int32_t *Y, int32_t *message, uint8_t *accept, int32_t *match_l,
                            double *keyX, double *keyY, double *gapX, double *gapY, int32_t threads,
                            int32_t shared_race) {
  if (!logw_enc || !logw_dec || !bins || !X || !Y || !accept) return -1;
  if (B < 0 || L < 1 || N < 1) return -1;
  int nthreads = threads;
#ifdef _OPENMP
  if (nthreads <= 0) nthreads = omp_get_max_threads();
#else
  nthreads = 1;
#endif
#pragma omp parallel for schedule(dynamic, 1) num_threads(nthreads)
  for (int64_t b = 0; b < B; ++b) {
    const uint64_t row = row_offset + (uint64_t)b;
    const uint8_t *bin = bins + b * bins_stride_b;
    std::vector<double> q, p;
    // encoder: lambda_q over all N candidates, pool over the L sets of race times
    row_distribution(logw_enc, DT_F32, b * enc_stride_b, N, KIND_LOGW, 1.0, q);
    Race pool;
    for (int64_t l = 0; l < (shared_race ? 1 : L); ++l)
      for (int64_t i = 0; i < N; ++i) {
        const double S = race_time(shared_word(seed, row, (uint32_t)l, (uint64_t)i));
        pool.offer(q[i] > 0.0 ? S / q[i] : kInf, i, l);
      }
    Y[b] = (int32_t)pool.idx;
    if (keyY) keyY[b] = pool.best;
    if (gapY) gapY[b] = pool.rel_gap();
    const int msg = pool.idx >= 0 ? (int)bin[pool.idx] : -1;
    if (message) message[b] = msg;
    // decoders: lambda_p^(l) lives on the candidates of the announced bin
    int64_t match = -1;
    for (int64_t l = 0; l < L; ++l) {
      p.assign((size_t)N, 0.0);
      double zmax = -kInf;
      for (int64_t i = 0; i < N; ++i) {
        double z = (double)logw_dec[b * dec_stride_b + l * dec_stride_l + i];
        if (msg < 0 || (int)bin[i] != msg || std::isnan(z) || z == kInf) z = -kInf;
        p[i] = z;
        if (z > zmax) zmax = z;
      }
      double sum = 0.0;
      if (zmax > -kInf)
        for (int64_t i = 0; i < N; ++i) sum += std::exp(p[i] - zmax);
      Race dec;
      for (int64_t i = 0; i < N; ++i) {
        const double w = zmax > -kInf ? std::exp(p[i] - zmax - std::log(sum)) : 0.0;
        if (!(w > 0.0)) continue;
        const double S = race_time(shared_word(seed, row, (uint32_t)(shared_race ? 0 : l), (uint64_t)i));
        dec.offer(S / w, i, l);
      }
      X[b * L + l] = (int32_t)dec.idx;
      if (keyX) keyX[b * L + l] = dec.best;
      if (gapX) gapX[b * L + l] = dec.rel_gap();
      if (match < 0 && dec.idx >= 0 && dec.idx == pool.idx) match = l;
    }
    accept[b] = (uint8_t)(match >= 0);
    if (match_l) match_l[b] = (int32_t)match;
  }
  return 0;
}

// Algorithm 1 on candidate lists (Section 4.4).  draft_ids / draft_val: [B,K,Md] (stride_k == 0:
// one list per row), target_ids / target_val: [B,Mt].  A negative id marks an empty slot.  The
// distribution a list denotes lives on its entries only: softmax of the listed logits, the
// listed log-weights normalised, or the listed probabilities as given.  Outputs are token ids.
struct llc_topm_ref_args {
  int64_t B, K, Md, Mt;
  int32_t dtype, kind;
  const int32_t *draft_ids;
  const void *draft_val;
  int64_t draft_stride_b, draft_stride_k;
  const int32_t *target_ids;
  const void *target_val;
  int64_t target_stride_b;
  float temp_target;
  const float *temp_draft;
  float temp_draft_all;
  uint64_t seed, row_offset;
  int32_t *X;        // [B,K] token ids
  int32_t *Y;        // [B]
  uint8_t *accept;   // [B]
  int32_t *match_k;  // [B]   optional
  double *keyX;      // [B,K] optional
  double *keyY;      // [B]   optional
  double *gapX;      // [B,K] optional: relative gap to the best entry with another id
  double *gapY;      // [B]   optional
  int32_t threads;
};

int llc_couple_topm_ref(const llc_topm_ref_args *a) {
  if (!a || !a->draft_ids || !a->draft_val || !a->target_ids || !a->target_val || !a->X || !a->Y ||
      !a->accept)
    return -1;
  if (a->B < 0 || a->K < 1 || a->Md < 1 || a->Mt < 1) return -1;
  const int64_t B = a->B, K = a->K, Md = a->Md, Mt = a->Mt;
  int nthreads = a->threads;
#ifdef _OPENMP
  if (nthreads <= 0) nthreads = omp_get_max_threads();
#else
  nthreads = 1;
#endif
#pragma omp parallel for schedule(dynamic, 4) num_threads(nthreads)
  for (int64_t b = 0; b < B; ++b) {
    const uint64_t row = a->row_offset + (uint64_t)b;
    std::vector<double> q, p;
    const int32_t *tid = a->target_ids + b * a->target_stride_b;
    list_distribution(tid, a->target_val, a->dtype, b * a->target_stride_b, Mt, a->kind,
                      (double)a->temp_target, q);
    Race pool;
    std::vector<int64_t> xs((size_t)K);
    for (int64_t k = 0; k < K; ++k) {
      const int64_t off = b * a->draft_stride_b + k * a->draft_stride_k;
      const int32_t *did = a->draft_ids + off;
      const double Tk = a->temp_draft ? (double)a->temp_draft[k] : (double)a->temp_draft_all;
      list_distribution(did, a->draft_val, a->dtype, off, Md, a->kind, Tk, p);
      Race draft;
      for (int64_t e = 0; e < Md; ++e) {
        if (did[e] < 0) continue;
        const double S = race_time(shared_word(a->seed, row, (uint32_t)k, (uint64_t)did[e]));
        draft.offer(p[e] > 0.0 ? S / p[e] : kInf, did[e], k);
      }
      for (int64_t e = 0; e < Mt; ++e) {
        if (tid[e] < 0) continue;
        const double S = race_time(shared_word(a->seed, row, (uint32_t)k, (uint64_t)tid[e]));
        pool.offer(q[e] > 0.0 ? S / q[e] : kInf, tid[e], k);
      }
      xs[k] = draft.idx;
      a->X[b * K + k] = (int32_t)draft.idx;
      if (a->keyX) a->keyX[b * K + k] = draft.best;
      if (a->gapX) a->gapX[b * K + k] = draft.rel_gap();
    }
    a->Y[b] = (int32_t)pool.idx;
    if (a->keyY) a->keyY[b] = pool.best;
    if (a->gapY) a->gapY[b] = pool.rel_gap();
    int64_t match = -1;
    if (pool.idx >= 0)
      for (int64_t k = 0; k < K; ++k)
        if (xs[k] == pool.idx) { match = k; break; }
    a->accept[b] = (uint8_t)(match >= 0);
    if (a->match_k) a->match_k[b] = (int32_t)match;
  }
  return 0;
}

// Algorithm 2 (Section 4.2), the verification loop, for S independent sequences.
// target[s, j, k, :] denotes q^(j,k) = M_b(. | X_{1:j-1}^(k), c) for j = 0..L (L is the
// bonus position), tokens[s, j, k] = X_j^(k) for j = 0..L-1.  Randomness of position j of
// sequence s is the stream of row  row_offset + s*row_stride_s + j*row_stride_j.
// strong != 0: the pool runs over all K drafts' randomness, viable or not (Appendix B, strong
// drafter invariance); dropped drafts are priced with a viable draft's target row.  Y[s, j] = -1 for positions that are not reached.
struct llc_verify_ref_args {
  int64_t S, L, K, V;
  int32_t dtype, kind;
  const void *target;
  int64_t stride_s, stride_j, stride_k;
  float temp_target;
  const int32_t *tokens;
  int64_t tok_stride_s, tok_stride_j;
  uint64_t seed, row_offset;
  int64_t row_stride_s, row_stride_j;
  int32_t strong;
  int32_t *Y;        // [S, L+1]
  int32_t *n_out;    // [S]
  uint8_t *active;   // [S, K] optional: drafts still viable when the loop ends
  double *key;       // [S, L+1] optional: winning S/q (normalised q)
  double *gap;       // [S, L+1] optional: relative gap to the best entry with another index
  int32_t threads;
  int32_t min_first; // how the race times are drawn from the stream (see row_race_time)
};

int llc_verify_ref(const llc_verify_ref_args *a) {
  if (!a || !a->target || !a->Y || !a->n_out) return -1;
  if (a->S < 0 || a->L < 0 || a->K < 1 || a->V < 1) return -1;
  if (a->L > 0 && !a->tokens) return -1;
  if (a->kind == KIND_PROBS) return -1;  // keys of different drafts are compared: needs normalised q
  const int64_t S = a->S, L = a->L, K = a->K, V = a->V;
  int nthreads = a->threads;
#ifdef _OPENMP
  if (nthreads <= 0) nthreads = omp_get_max_threads();
#else
  nthreads = 1;
#endif
#pragma omp parallel for schedule(dynamic, 1) num_threads(nthreads)
  for (int64_t s = 0; s < S; ++s) {
    std::vector<uint8_t> viable((size_t)K, 1);
    std::vector<double> q;
    int32_t n = 0;
    for (int64_t j = 0; j <= L; ++j) {
      a->Y[s * (L + 1) + j] = -1;
      if (a->key) a->key[s * (L + 1) + j] = kInf;
      if (a->gap) a->gap[s * (L + 1) + j] = kInf;
    }
    for (int64_t j = 0; j <= L; ++j) {
      const uint64_t row = a->row_offset + (uint64_t)(s * a->row_stride_s + j * a->row_stride_j);
      Race pool;
      int64_t kref = 0;  // the first viable draft: its prefix equals the output so far
      while (kref < K && !viable[kref]) ++kref;
      for (int64_t k = 0; k < K; ++k) {
        if (!a->strong && !viable[k]) continue;
        // A dropped draft's own row is conditioned on a prefix that is not the output; the
        // strong variant keeps its randomness in the pool but prices it with the target
        // distribution given the output prefix, i.e. the row of a viable draft.
        const int64_t krow = viable[k] ? k : kref;
        row_distribution(a->target, a->dtype, s * a->stride_s + j * a->stride_j + krow * a->stride_k, V,
                         a->kind, (double)a->temp_target, q);
        for (int64_t i = 0; i < V; ++i) {
          const double St = row_race_time(a->min_first, a->seed, row, (uint32_t)k, (uint64_t)i, K);
          pool.offer(q[i] > 0.0 ? St / q[i] : kInf, i, k);
        }
      }
      a->Y[s * (L + 1) + j] = (int32_t)pool.idx;
      if (a->key) a->key[s * (L + 1) + j] = pool.best;
      if (a->gap) a->gap[s * (L + 1) + j] = pool.rel_gap();
      n = (int32_t)(j + 1);
      if (j == L) break;
      bool any = false;
      for (int64_t k = 0; k < K; ++k) {
        if (viable[k] && a->tokens[s * a->tok_stride_s + j * a->tok_stride_j + k] != (int32_t)pool.idx)
          viable[k] = 0;
        any = any || viable[k];
      }
      if (!any) break;
    }
    a->n_out[s] = n;
    if (a->active) for (int64_t k = 0; k < K; ++k) a->active[s * K + k] = viable[k];
  }
  return 0;
}

}  // extern "C"
