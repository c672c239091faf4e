// The scan kernel: one pass over a row's (draft k, index i) pairs that finds, for
// each of the K drafts, argmin_i S_i^(k)/p_i^(k) and, for the target, the argmin
// over the K x V pool of S_i^(k)/q_i (paper Section 3, Algorithm 1, steps 2-4).
//
// Work per element is dominated by the random word itself, so the kernel is
// organised to do nothing else for almost every element:
//
//  level 1 (every element, integer): a race time S = -ln U can only beat the
//    best key seen so far, 2^tau, if 1 - U <= S <= 2^tau * p.  With the 32-bit
//    word x and xt = ~x, 1 - U = (xt + 1/2) 2^-32, so the test is xt <= t with an
//    integer threshold t >= 2^(32 + tau) p.  t is built from the raw input by one
//    fused multiply-add into the exponent/mantissa field of a float (a
//    piecewise-linear 2^y that never under-estimates) and two conversions.
//    The draft-side and target-side thresholds are merged by a median-of-three.
//    The word's upper and lower 16 bits come from two different Philox blocks, and
//    the upper half alone decides almost every element (x >= ~t needs
//    hi16(x) >= hi16(~t)): only the "upper" block is generated in the main loop,
//    its eight half-words (four indices x two drafts) are tested two at a time
//    with packed 16-bit operations, and the "lower" block is generated only for
//    the few lanes whose upper half passes.
//  level 2 (survivors, fp32): an approximate key a = log2 S - log2 p; survivors
//    within a band of the running best are recorded in an LDS list and lower tau.
//  level 3 (end of the scan, fp64): records still within the band of the final
//    tau are evaluated exactly -- ln(-ln U) - x/T in fp64 -- and reduced with
//    64-bit LDS atomics; ties go to the smaller index, then the smaller k.
//
// Because every element whose exact key could be the minimum passes levels 1
// and 2 (the margins below bound the fp32 error of both), the result is the
// exact fp64 argmin, independent of grid shape and of the order of arrival.
//
// MINF (the min-first way of drawing Algorithm 1's race times): the K race times of an index are
// drawn through their minimum M = -ln(U0) / K, which sits at draft kappa = floor(K r / 2^32); every
// other draft's time is M - ln U_i^(k).  No draft's time is below M, so level 1 tests M alone: one
// 32-bit word per index instead of one half-word per (index, draft), against the loosest of the
// bounds (raised by log2 K).  The survivors' path draws kappa, hands M to the draft that holds it
// (and to the pool, whose key of the index is M / q_i), and for the other drafts runs the old
// half-word test on their own word: M - ln U can only win if -ln U alone is below the bound.
#pragma once

#include "common.hpp"
#include "finalize_row.hpp"

namespace llc {

// raw: four consecutive elements as they sit in memory (what a prefetched tile keeps per lane)
struct F32In { using elem = float; using raw = float4; };
struct BF16In { using elem = uint16_t; using raw = uint2; };

// ---- margins (log2 units) ---------------------------------------------------
// |tau| <= kTauLimit is enforced (else the workgroup redoes its chunk in fp64).
// Level-2 keys then carry an error below 3.4e-4, level-1 exponents below 1.4e-4.
constexpr float kEps2 = 0x1p-9f;       // band around tau for "may be the minimum"
constexpr float kEps1 = 0x1p-7f;       // slack of the integer prefilter
constexpr float kPseudoLog = 0.0861f;  // max of log2(1+f) - f: slack when log2 p is read off the bits
constexpr float kTauLimit = 1024.0f;
constexpr float kTwo23 = 8388608.0f;
// Cap of the scaled exponent where thresholds are formed in full (the candidates' path): the
// bit pattern of the float 0xFFFE8000.  An element whose exponent reaches the cap is "hot": it
// goes to level 2 whatever its random word is.
constexpr float kCapHot = 1333788288.0f;
// The main loop lowers its exponents by 32, so that the float an exponent stands for is t / 2^32
// in [0, 1] and one conversion to a normalised 16-bit integer (round(f * 65535), measured: to
// nearest) yields hi16(t) for two thresholds at once.  The conversion must not come out below
// floor(f * 65536): 1024 units of the scaled exponent raise f by a factor >= 1 + 2^-14 > 65536/65535.
// The lowered exponent is capped at the bit pattern of 1.0f: a hot element (and a few just below)
// gets the half-word threshold 0xFFFF, which every half-word passes.
constexpr float kShift32 = 268435456.0f - 1024.0f;       // 32 * 2^23, less the raise
constexpr float kCapOne32 = 1065353216.0f;               // 0x3F800000 read as an integer
constexpr uint32_t kLowBlock = 0x80000000u;  // bit 31 of counter word 3 marks the lower-half block
// min-first: counter word 3 of the block with the smallest race times of four indices (one 32-bit
// word each) and of the block whose words pick the drafts that hold them
constexpr uint32_t kMinBlock = 0x40000000u;
constexpr uint32_t kHolderBlock = 0x40000001u;
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLog2Ln2 = -0.5287663729448977f;  // log2(ln 2)

// a ^ b ^ c in one instruction (gfx950's three-input bitwise op, truth table 0x96).
__device__ __forceinline__ uint32_t xor3(uint32_t a, uint32_t b, uint32_t c) {
  return __builtin_amdgcn_bitop3_b32(a, b, c, 0x96);
}

// ---- Philox4x32, ten rounds (Salmon et al., SC'11) ----------------------------
__device__ __forceinline__ void philox_block(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                             uint32_t k0, uint32_t k1, uint32_t (&out)[4]) {
#pragma unroll
  for (int r = 0; r < 10; ++r) {
    const uint64_t pa = (uint64_t)c0 * 0xD2511F53ull;
    const uint64_t pb = (uint64_t)c2 * 0xCD9E8D57ull;
    const uint32_t n0 = xor3((uint32_t)(pb >> 32), c1, k0);
    const uint32_t n2 = xor3((uint32_t)(pa >> 32), c3, k1);
    c1 = (uint32_t)pb;
    c3 = (uint32_t)pa;
    c0 = n0;
    c2 = n2;
    k0 += 0x9E3779B9u;
    k1 += 0xBB67AE85u;
  }
  out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

// KB blocks that differ only in counter word 3 (the draft pair), advanced round by round so
// that the KB dependency chains interleave.  The counter is (row, index group, row, pair): the
// index group and the pair sit in the words that a round only xors in, so the first round is
// uniform over the wave, the second and third have one vector multiplication each that all KB
// blocks share, and only from the fourth round on does every block cost its two multiplications
// (the compiler finds this by itself: common subexpressions and uniform values).
template <int KB>
__device__ __forceinline__ void philox_blocks(uint32_t g, uint32_t pair_base, uint32_t row_lo,
                                              uint32_t row_hi, uint32_t k0, uint32_t k1,
                                              uint32_t (&out)[KB][4]) {
  uint32_t c0[KB], c1[KB], c2[KB], c3[KB];
#pragma unroll
  for (int m = 0; m < KB; ++m) { c0[m] = row_lo; c1[m] = g; c2[m] = row_hi; c3[m] = pair_base + m; }
#pragma unroll
  for (int r = 0; r < 10; ++r) {
#pragma unroll
    for (int m = 0; m < KB; ++m) {
      const uint64_t pa = (uint64_t)c0[m] * 0xD2511F53ull;
      const uint64_t pb = (uint64_t)c2[m] * 0xCD9E8D57ull;
      const uint32_t n0 = xor3((uint32_t)(pb >> 32), c1[m], k0);
      const uint32_t n2 = xor3((uint32_t)(pa >> 32), c3[m], k1);
      c1[m] = (uint32_t)pb;
      c3[m] = (uint32_t)pa;
      c0[m] = n0;
      c2[m] = n2;
    }
    k0 += 0x9E3779B9u;
    k1 += 0xBB67AE85u;
  }
#pragma unroll
  for (int m = 0; m < KB; ++m) { out[m][0] = c0[m]; out[m][1] = c1[m]; out[m][2] = c2[m]; out[m][3] = c3[m]; }
}

// The 32-bit word of one element from the words its index selects in the upper-half and the
// lower-half block of its draft pair: even drafts read the lower 16 bits, odd drafts the upper.
__device__ __forceinline__ uint32_t element_word(uint32_t upper_word, uint32_t lower_word, int odd) {
  const uint32_t hi = odd ? (upper_word >> 16) : (upper_word & 0xFFFFu);
  const uint32_t lo = odd ? (lower_word >> 16) : (lower_word & 0xFFFFu);
  return (hi << 16) | lo;
}

// Packed unsigned 16-bit maximum and saturating difference of two half-word pairs.
typedef unsigned short ushort2v __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pk_max_u16(uint32_t a, uint32_t b) {
  return __builtin_bit_cast(uint32_t, __builtin_elementwise_max(__builtin_bit_cast(ushort2v, a),
                                                                __builtin_bit_cast(ushort2v, b)));
}
__device__ __forceinline__ uint32_t pk_add_sat_u16(uint32_t a, uint32_t b) {
  return __builtin_bit_cast(uint32_t, __builtin_elementwise_add_sat(__builtin_bit_cast(ushort2v, a),
                                                                    __builtin_bit_cast(ushort2v, b)));
}

// ---- small helpers ------------------------------------------------------------
__device__ __forceinline__ int ord32(float f) {  // order-preserving float -> int
  const int b = __float_as_int(f);
  return b ^ ((b >> 31) & 0x7FFFFFFF);
}
__device__ __forceinline__ float unord32(int o) {
  return __int_as_float(o ^ ((o >> 31) & 0x7FFFFFFF));
}
__device__ __forceinline__ unsigned long long ord64(double d) {  // order-preserving double -> u64
  const unsigned long long b = (unsigned long long)__double_as_longlong(d);
  return (b >> 63) ? ~b : (b | 0x8000000000000000ull);
}
__device__ __forceinline__ double unord64(unsigned long long o) {
  const unsigned long long b = (o >> 63) ? (o & 0x7FFFFFFFFFFFFFFFull) : ~o;
  return __longlong_as_double((long long)b);
}
constexpr unsigned long long kOrdInf64 = 0xFFF0000000000000ull;  // ord64(+inf)

__device__ __forceinline__ uint32_t cvt_u32_saturating(float f) {
  uint32_t r;  // hardware conversion: clamps to [0, 2^32 - 1], NaN -> 0
  asm("v_cvt_u32_f32 %0, %1" : "=v"(r) : "v"(f));
  return r;
}

template <typename T>
__device__ __forceinline__ void load4(const typename T::elem *row, int i0, int V, bool vec,
                                      float fill, float (&v)[4]);

template <>
__device__ __forceinline__ void load4<F32In>(const float *row, int i0, int V, bool vec, float fill,
                                             float (&v)[4]) {
  if (vec && i0 + 3 < V) {
    const float4 t = *reinterpret_cast<const float4 *>(row + i0);
    v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w;
  } else {
#pragma unroll
    for (int j = 0; j < 4; ++j) v[j] = (i0 + j < V) ? row[i0 + j] : fill;
  }
}

template <>
__device__ __forceinline__ void load4<BF16In>(const uint16_t *row, int i0, int V, bool vec,
                                              float fill, float (&v)[4]) {
  if (vec && i0 + 3 < V) {
    const uint2 t = *reinterpret_cast<const uint2 *>(row + i0);
    v[0] = __uint_as_float(t.x << 16);
    v[1] = __uint_as_float(t.x & 0xFFFF0000u);
    v[2] = __uint_as_float(t.y << 16);
    v[3] = __uint_as_float(t.y & 0xFFFF0000u);
  } else {
#pragma unroll
    for (int j = 0; j < 4; ++j)
      v[j] = (i0 + j < V) ? __uint_as_float((uint32_t)row[i0 + j] << 16) : fill;
  }
}

// Four in-range elements of an aligned row, kept as loaded; unpack() widens them to fp32.
template <typename T>
__device__ __forceinline__ typename T::raw load_raw(const typename T::elem *row, int i0) {
  return *reinterpret_cast<const typename T::raw *>(row + i0);
}
// The same four elements with bounds checks (ragged tails, unaligned rows); `fill` stands for
// elements past the end.
template <typename T>
__device__ __forceinline__ typename T::raw load_raw_checked(const typename T::elem *row, int i0, int V, bool vec, float fill);
template <>
__device__ __forceinline__ float4 load_raw_checked<F32In>(const float *row, int i0, int V, bool vec, float fill) {
  if (vec && i0 + 3 < V) return *reinterpret_cast<const float4 *>(row + i0);
  float4 r;
  r.x = (i0 + 0 < V) ? row[i0 + 0] : fill;
  r.y = (i0 + 1 < V) ? row[i0 + 1] : fill;
  r.z = (i0 + 2 < V) ? row[i0 + 2] : fill;
  r.w = (i0 + 3 < V) ? row[i0 + 3] : fill;
  return r;
}
template <>
__device__ __forceinline__ uint2 load_raw_checked<BF16In>(const uint16_t *row, int i0, int V, bool vec, float fill) {
  if (vec && i0 + 3 < V) return *reinterpret_cast<const uint2 *>(row + i0);
  const uint32_t f = __float_as_uint(fill) >> 16;  // 0 and -inf are exact in bf16
  const uint32_t e0 = (i0 + 0 < V) ? row[i0 + 0] : f, e1 = (i0 + 1 < V) ? row[i0 + 1] : f;
  const uint32_t e2 = (i0 + 2 < V) ? row[i0 + 2] : f, e3 = (i0 + 3 < V) ? row[i0 + 3] : f;
  return make_uint2(e0 | (e1 << 16), e2 | (e3 << 16));
}
__device__ __forceinline__ void unpack(const float4 &r, float (&v)[4]) {
  v[0] = r.x; v[1] = r.y; v[2] = r.z; v[3] = r.w;
}
__device__ __forceinline__ void unpack(const uint2 &r, float (&v)[4]) {
  v[0] = __uint_as_float(r.x << 16);
  v[1] = __uint_as_float(r.x & 0xFFFF0000u);
  v[2] = __uint_as_float(r.y << 16);
  v[3] = __uint_as_float(r.y & 0xFFFF0000u);
}

// Bins of four consecutive candidates (one byte each) and the mask they imply: a candidate whose
// bin differs from the announced one carries no mass on the draft (decoder) side (paper Section
// 5.1: the decoder's target distribution holds the indicator 1{l_i = l_j}).
__device__ __forceinline__ uint32_t load_bins4(const uint8_t *row, int i0, int V, bool aligned) {
  if (aligned && i0 + 3 < V) return *reinterpret_cast<const uint32_t *>(row + i0);
  uint32_t w = 0;
#pragma unroll
  for (int j = 0; j < 4; ++j)
    if (i0 + j < V) w |= (uint32_t)row[i0 + j] << (8 * j);
  return w;
}
__device__ __forceinline__ void mask_bins(uint32_t bins4, int announced, float fill, float (&v)[4]) {
#pragma unroll
  for (int j = 0; j < 4; ++j)
    if ((int)((bins4 >> (8 * j)) & 0xFFu) != announced) v[j] = fill;
}

template <typename T>
__device__ __forceinline__ float load1(const typename T::elem *row, int i);
template <>
__device__ __forceinline__ float load1<F32In>(const float *row, int i) { return row[i]; }
template <>
__device__ __forceinline__ float load1<BF16In>(const uint16_t *row, int i) {
  return __uint_as_float((uint32_t)row[i] << 16);
}

// log2 of the race time S = -ln U, U = (x + 1/2) 2^-32, in fp32 (relative error of S
// below 2^-16).  Near U = 1 the series of -ln(1 - W), W = 1 - U = (~x + 1/2) 2^-32.
__device__ __forceinline__ float approx_log2_race_time(uint32_t x) {
  const uint32_t xt = ~x;
  if (xt < (1u << 25)) {
    const float W = ((float)xt + 0.5f) * 0x1p-32f;
    const float S = W * fmaf(W, fmaf(W, 0.33333334f, 0.5f), 1.0f);
    return __log2f(S);  // arguments here are never subnormal: the bare hardware log2 suffices
  }
  const float U = ((float)x + 0.5f) * 0x1p-32f;
  return __log2f(-__log2f(U)) + kLog2Ln2;
}

// The race time itself in fp32 (relative error below 2^-16).
__device__ __forceinline__ float approx_race_time(uint32_t x) {
  const uint32_t xt = ~x;
  if (xt < (1u << 25)) {
    const float W = ((float)xt + 0.5f) * 0x1p-32f;
    return W * fmaf(W, fmaf(W, 0.33333334f, 0.5f), 1.0f);
  }
  const float U = ((float)x + 0.5f) * 0x1p-32f;
  return -__log2f(U) * 0.6931471805599453f;
}
// min-first: the draft that holds an index's smallest race time, from the index's second word.
__device__ __forceinline__ int holder_of(uint32_t r, int K) { return (int)__umulhi(r, (uint32_t)K); }

// The race time S = -ln U in fp64.
__device__ __forceinline__ double exact_race_time(uint32_t x) {
  const double U = ((double)x + 0.5) * 0x1p-32;
  return -log(U);
}

// What an input value contributes to the level-1 exponent: the logit itself, or for
// probabilities the float's own bits (a piecewise-linear log2 that never over-estimates).
template <bool PROBS>
__device__ __forceinline__ float level1_value(float v) {
  return PROBS ? (float)__float_as_int(v) : v;
}

// The largest of four values' contributions to the level-1 exponent (NaN entries are ignored:
// they carry no mass; for probabilities the integer images are compared, a NaN's is large and only
// sends the lane to the survivors' path, which drops it).
template <bool PROBS>
__device__ __forceinline__ float level1_max4(const float (&v)[4]) {
  if (PROBS) {
    const int a = max(__float_as_int(v[0]), __float_as_int(v[1]));
    const int b = max(__float_as_int(v[2]), __float_as_int(v[3]));
    return (float)max(a, b);
  }
  return fmaxf(fmaxf(fmaxf(v[0], v[1]), v[2]), v[3]);
}

// log2 of the unnormalised probability an input value stands for; false if it carries no mass.
template <bool PROBS>
__device__ __forceinline__ bool approx_log2_mass(float v, float c, float &ell) {
  if (PROBS) {
    if (!(v > 0.0f && v < __builtin_huge_valf())) return false;
    ell = log2f(v);
    return true;
  }
  if (!(v < __builtin_huge_valf())) return false;  // NaN or +inf
  ell = v * c;
  return true;
}

// Exact key in fp64: ln S - x/T for logits and log-weights, S/p for probabilities.
template <bool PROBS>
__device__ __forceinline__ double exact_key(double S, float v, double T) {
  if (PROBS) {
    if (!(v > 0.0f && v < __builtin_huge_valf())) return __builtin_huge_val();
    return S / (double)v;
  }
  if (!(v < __builtin_huge_valf())) return __builtin_huge_val();
  return log(S) - (double)v / T;
}

// LSE with one shared proposal: the lanes' two running sums, kept in LDS (the other variants carry
// an empty stand-in).
template <bool ON, int N>
struct LaneSums { double v[N][kBlock]; };
template <int N>
struct LaneSums<false, N> { double v[1][1]; };

// Min-first survivors' path: words of a wavefront's staging area (eight lanes' tiles of 4 words, 4 target
// values, the group's number (padded) and up to 32 draft values) and of its queue (up to 8 + 32
// indices of 3 words and up to 8 draft values).
constexpr int kStageWords = 8 * 44;
constexpr int kQueueWords = 40 * 11;

struct Lds {
  int tau[9];            // ordered-int log2 keys: drafts 0..KT-1, pool at [KT]
  int O[9];              // bits of the level-1 offsets (tau + slack + bias) 2^23; shared layout: [0] = max over drafts
  int OL[9];             // the same lowered for the main loop (see kShift32); -inf for a reduction that is not taken
  float lgK;             // min-first: log2 K, by which the level-1 bounds on the smallest time are raised (else 0)
  int count;             // records appended (may exceed kListCap)
  int unsafe;            // chunk must be redone in fp64
  unsigned long long best[9];
  unsigned long long where[9];
  unsigned long long second[9];  // smallest exact key among entries whose index differs from the winner's
  unsigned long long n_survivors, n_exact;
  float cd23[8];         // per draft of this pass: log2(e) / T_k scaled by 2^23 ...
  int kok[8];            // ... and whether its temperature is usable (for lanes that pick a draft at run time)
  struct Stage {         // one lane's tile, laid out for the wave (survivors' path)
    uint32_t up[16];
    float vq[4];
    float vd[32];
  } stage[4];
  int qn[4];             // min-first: candidates in each wavefront's queue
  int lse_redo;          // LSE: the running sums were not formed (the main loop was skipped) or are not finite
  float lse_wmax[4][9];  // LSE: per-wave references (whole numbers, in powers of two) ...
  double lse_wave[4][9]; // ... and per-wave sums relative to them, merged in a fixed order
  int *shared_tau;       // the row's running bests shared by all its workgroups (or null)
  int shared_base, shared_pool;  // where this workgroup's draft 0 and the pool sit in it
  float rec_a[kListCap];
  int rec_i[kListCap];
  int rec_tag[kListCap];
};

template <bool PROBS>
__device__ __forceinline__ float make_offset(float tau, float lgK = 0.0f) {
  // logits: exponent bias 127 plus the 2^32 scale of the integer word; probabilities: the
  // bias is already in the float's own bits
  return (tau + lgK + ((PROBS ? 32.0f + kPseudoLog : 159.0f) + kEps1)) * kTwo23;
}
__device__ __forceinline__ void store_offset(int *slot, float O) {
  __atomic_store_n(slot, __float_as_int(O), __ATOMIC_RELAXED);
}
__device__ __forceinline__ float load_offset(const int *slot) {
  return __int_as_float(__atomic_load_n(slot, __ATOMIC_RELAXED));
}
// An offset is kept in both forms: as it is (candidates' path) and lowered for the main loop
// (min-first: the main loop tests whole words, its copy is not lowered).
template <bool MINF>
__device__ __forceinline__ void store_offsets(Lds &s, int slot, float O) {
  store_offset(&s.O[slot], O);
  store_offset(&s.OL[slot], MINF ? O : O - kShift32);
}
// Scaled exponent of one element's threshold, merged with the target side's (FY) and capped.
template <bool PROBS>
__device__ __forceinline__ float merged_exponent(float v, float c23, float O, float FY) {
  return __builtin_amdgcn_fmed3f(fmaf(level1_value<PROBS>(v), c23, O), FY, kCapHot);
}
// The threshold t on ~x that a scaled exponent stands for (t <= 0xFFFE8000).
__device__ __forceinline__ uint32_t threshold_of(float F) {
  return cvt_u32_saturating(__int_as_float((int)F));
}
// hi16 of the thresholds that two scaled exponents lowered by 32 stand for (never below the true
// value; 0xFFFF at the cap), packed: the first in the lower half.
__device__ __forceinline__ uint32_t packed_hi16(float F0, float F1) {
  return __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pknorm_u16(__int_as_float((int)F0), __int_as_float((int)F1)));
}
// Lower tau[slot] to `a` and refresh the level-1 offset that depends on it.  When the row is
// spread over several workgroups the new best is also posted to the row's shared array, from
// which the others pick it up (a bound found in one chunk prunes all of them).
template <int KT, bool SHARED, bool PROBS, bool MINF>
__device__ __forceinline__ void publish(Lds &s, int slot, float a, bool post = true) {
  atomicMin(&s.tau[slot], ord32(a));
  if (post && s.shared_tau != nullptr)
    atomicMin(&s.shared_tau[slot < KT ? s.shared_base + slot : s.shared_pool], ord32(a));
  if (!(fabsf(a) <= kTauLimit)) s.unsafe = 1;
  if (SHARED && slot < KT) {
    int m = s.tau[0];
#pragma unroll
    for (int kk = 1; kk < KT; ++kk) m = max(m, __atomic_load_n(&s.tau[kk], __ATOMIC_RELAXED));
    store_offsets<MINF>(s, 0, make_offset<PROBS>(unord32(m), s.lgK));
  } else {
    store_offsets<MINF>(s, slot, make_offset<PROBS>(unord32(__atomic_load_n(&s.tau[slot], __ATOMIC_RELAXED)), s.lgK));
  }
}

// Level 2 for one survivor of level 1.  tau_d / tau_p: the draft's and the pool's running best
// as read a little earlier (a stale, larger value only lets more candidates through).
template <int KT, bool SHARED, bool PROBS, bool MINF>
__device__ __forceinline__ void level2(Lds &s, float l2S, float vd, float vq, int i, int kk,
                                       bool draft_ok, bool pool_ok, float cd, float cq,
                                       float tau_d, float tau_p) {
  float ell;
  if (draft_ok && approx_log2_mass<PROBS>(vd, cd, ell)) {
    const float a = l2S - ell;
    if (a <= tau_d + kEps2) {
      const int pos = atomicAdd(&s.count, 1);
      if (pos < kListCap) { s.rec_a[pos] = a; s.rec_i[pos] = i; s.rec_tag[pos] = kk; }
      if (a < tau_d) publish<KT, SHARED, PROBS, MINF>(s, kk, a);
    }
  }
  if (pool_ok && approx_log2_mass<PROBS>(vq, cq, ell)) {
    const float a = l2S - ell;
    if (a <= tau_p + kEps2) {
      const int pos = atomicAdd(&s.count, 1);
      if (pos < kListCap) { s.rec_a[pos] = a; s.rec_i[pos] = i; s.rec_tag[pos] = KT + kk; }
      if (a < tau_p) publish<KT, SHARED, PROBS, MINF>(s, KT, a);
    }
  }
}

// Offer an exact key to reduction `slot` (phase 1: smallest key).
__device__ __forceinline__ void offer_key(Lds &s, int slot, double key) {
  if (key < __builtin_huge_val()) atomicMin(&s.best[slot], ord64(key));
}
// Phase 2: among the holders of the smallest key, the smallest (index, k).
__device__ __forceinline__ void offer_where(Lds &s, int slot, double key, int i, int k) {
  if (key < __builtin_huge_val() && ord64(key) == s.best[slot])
    atomicMin(&s.where[slot], ((unsigned long long)(uint32_t)i << 32) | (uint32_t)k);
}
// Phase 3: the runner-up, i.e. the smallest key at an index other than the winner's (what the
// near-tie count compares the winner with; the same index under another draft does not count).
__device__ __forceinline__ void offer_second(Lds &s, int slot, double key, int i) {
  if (key < __builtin_huge_val() && (uint32_t)i != (uint32_t)(s.where[slot] >> 32))
    atomicMin(&s.second[slot], ord64(key));
}

// ln sum exp(x/T) over one chunk of a row by the whole workgroup, exactly: maximum first, then
// fp64 exponentials, sums added in a fixed order.  The cold companion of the running sums of the
// LSE variant (used when those overflowed or were never formed).  Every thread gets the result.
template <typename T>
__device__ double chunk_lse_exact(const typename T::elem *row, int g_begin, int g_end, int V, double temp,
                                  float *s_max, double *s_sum) {
  const int tid = threadIdx.x;
  const float inf = __builtin_huge_valf();
  float m = -inf;
  for (int g = g_begin + tid; g < g_end; g += kBlock) {
    float v[4];
    load4<T>(row, g * 4, V, false, -inf, v);
#pragma unroll
    for (int j = 0; j < 4; ++j)
      if (v[j] < inf) m = fmaxf(m, v[j]);
  }
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) m = fmaxf(m, __shfl_xor(m, d));
  __syncthreads();  // the scratch arrays may still be read from a previous call
  if ((tid & 63) == 0) s_max[tid >> 6] = m;
  __syncthreads();
  m = fmaxf(fmaxf(s_max[0], s_max[1]), fmaxf(s_max[2], s_max[3]));
  double sum = 0.0;
  if (m > -inf) {
    for (int g = g_begin + tid; g < g_end; g += kBlock) {
      float v[4];
      load4<T>(row, g * 4, V, false, -inf, v);
#pragma unroll
      for (int j = 0; j < 4; ++j)
        if (v[j] < inf && v[j] > -inf) sum += exp(((double)v[j] - (double)m) / temp);
    }
  }
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) sum += __shfl_xor(sum, d);
  if ((tid & 63) == 0) s_sum[tid >> 6] = sum;
  __syncthreads();
  sum = (s_sum[0] + s_sum[1]) + (s_sum[2] + s_sum[3]);
  const bool ok = m > -inf && temp > 0.0 && temp < (double)inf;
  return ok ? (double)m / temp + log(sum) : -__builtin_huge_val();
}

// One workgroup scans one (row, draft group, chunk).  KB = draft pairs per pass (KT = 2 KB
// drafts): each pair of drafts shares its Philox blocks.
// MASKED: the variant that knows binned candidates and the pool-only mode (built for fp32
// log-weights only, which is what the compression scheme uses).
// LSE: the variant that also accumulates the rows' normalisers ln sum exp(x/T) while it scans
// them (logit kinds), so that no second pass over the inputs is needed.
// FIN: the variant for rows that are one workgroup each: it also takes the finalize step (Algorithm
// 1's accept test and the outputs), so that no finalize launch follows.
// MINF: the race times are drawn min-first (see the top of the file).
// Registers: four workgroups per CU (128 registers) where a workgroup reads one shared proposal or
// at most four drafts' rows, except for the variants that read per-draft rows and form their
// normalisers: held to 128 registers those reload spilled values inside the main loop, each reload
// waiting for the next tile's loads as well.  (One such build also returned wrong target-side
// results, which the parity tests caught: the compiler had put the spill store of a value that
// every lane needs into a stretch of code that runs with the exec mask narrowed to a few lanes.
// The build's audit looks for that in the assembly of every kernel.)  They are allowed more
// and take about 150: three workgroups per CU.
template <typename T, int KB, bool SHARED, bool PROBS, bool MASKED, bool LSE, bool FIN, bool MINF>
__global__ void __launch_bounds__(kBlock, ((SHARED || KB <= 2) && !(LSE && !SHARED)) ? 4 : 2) scan_kernel(const ScanParams p) {
  using elem = typename T::elem;
  constexpr int KT = 2 * KB;
  static_assert(!(MINF && MASKED), "the binned and pool-only passes draw one word per (index, draft)");
  __shared__ Lds s;
  __shared__ __align__(16) uint32_t s_minf[MINF ? 4 * (kStageWords + kQueueWords) : 4];  // (see the main loop)
  // (with per-draft rows the sums stay in registers: in LDS they measured slower there)
  constexpr bool kSumsInLds = LSE && SHARED;
  __shared__ LaneSums<kSumsInLds, 2> sums;

  const int tid = threadIdx.x;
  // Workgroups are handed to the 8 XCDs round-robin by index.  Renumber them so that the
  // workgroups of one row (its draft groups and chunks, which share the target row and, in the
  // shared layout, the draft row) get indices that are congruent modulo 8: they then run on one
  // XCD, close in time, and the second reader finds the row in that XCD's L2.
  unsigned bid = blockIdx.x;
  {
    const unsigned per_xcd = gridDim.x >> 3;
    if (bid < (per_xcd << 3)) bid = (bid & 7u) * per_xcd + (bid >> 3);
  }
  const int chunk = (int)(bid % (unsigned)p.n_chunks);
  const int kg = (int)((bid / (unsigned)p.n_chunks) % (unsigned)p.n_kgroups);
  const long long b = (long long)(bid / ((unsigned)p.n_chunks * (unsigned)p.n_kgroups));
  const int kbase = kg * KT;
  // same_race: every draft of the row uses the race times of draft 0 (the compression scheme's
  // baseline, in which all decoders share one set of random numbers; paper Section 5.3)
  const bool same_race = MASKED && p.same_race != 0;
  const uint32_t pair_base = same_race ? 0u : (uint32_t)(kg * KB);
  const int V = p.V;
  const int G = (V + 3) >> 2;
  const int g_begin = chunk * p.groups_per_chunk;
  const int g_end = min(g_begin + p.groups_per_chunk, G);
  const int iters = (g_end - g_begin + kBlock - 1) / kBlock;
  const bool vec = p.vector_loads != 0;
  const bool with_pool = p.no_pool == 0;  // false: draft-side reductions only, the target is not read
  const float fill = PROBS ? 0.0f : -__builtin_huge_valf();

  const unsigned long long row = p.row_offset + p.map.row_of(b);
  const uint32_t row_lo = (uint32_t)row, row_hi = (uint32_t)(row >> 32);

  const elem *trow = reinterpret_cast<const elem *>(p.target) + p.map.target_off(b);
  const elem *drow0 = reinterpret_cast<const elem *>(p.draft) + p.map.draft_off(b);
  if (p.draft_row_off != nullptr) {
    const long long off = p.draft_row_off[b];
    if (off < 0) {
      // the row is not wanted: empty partial results (uniform over the workgroup, before any barrier)
      if (tid < KT) {
        if (kbase + tid < p.K) {
          const long long o = (b * p.K + kbase + tid) * p.n_chunks + chunk;
          p.out.keyX[o] = __builtin_huge_val();
          p.out.idxX[o] = -1;
          p.out.secX[o] = __builtin_huge_val();
          if (LSE) p.lse_part[(b * (p.K + 1) + kbase + tid) * p.n_chunks + chunk] = -__builtin_huge_val();
        }
      } else if (tid == KT) {
        const long long o = (b * p.n_kgroups + kg) * p.n_chunks + chunk;
        p.out.keyY[o] = __builtin_huge_val();
        p.out.idxY[o] = -1;
        p.out.kY[o] = -1;
        p.out.secY[o] = __builtin_huge_val();
      }
      return;
    }
    drow0 += off;
  }
  // binned candidates: only those in the announced bin (the bin of the index in bin_of[b]) count
  // on the draft side
  const bool binned = MASKED && p.bins != nullptr;
  const uint8_t *brow = binned ? p.bins + b * p.bins_stride_b : nullptr;
  int announced = -1;
  if (binned) {
    const int y = p.bin_of[b];
    if (y >= 0 && y < V) announced = (int)brow[y];
  }
  const bool bins_aligned = binned && (((uintptr_t)p.bins | (uintptr_t)p.bins_stride_b) & 3u) == 0;
  // pool only (the encoder's pass of the binned selection): the draft rows are not read and no
  // candidate counts on the draft side, as if every bin differed from the announced one
  const bool no_draft = MASKED && p.no_draft != 0;
  const bool draft_masked = binned || no_draft;
  if (no_draft) announced = -2;

  // per-draft constants (wave-uniform)
  float cd23[KT];  // log2(e) / T_k scaled by 2^23 (an exact scaling: the plain factor is cd23 * 2^-23)
  bool kok[KT];
#pragma unroll
  for (int kk = 0; kk < KT; ++kk) {
    const int k = kbase + kk;
    float t = p.temp_draft_all;
    if (p.temp_draft != nullptr && k < p.K) t = p.temp_draft[k];
    kok[kk] = (k < p.K) && (t > 0.0f) && (t < __builtin_huge_valf());
    cd23[kk] = PROBS ? 1.0f : (kLog2e / t) * kTwo23;
  }
  // min-first: the smallest of an index's K times is (-ln U0) / K
  const float lgK = MINF ? log2f((float)p.K) : 0.0f;
  const float invK = MINF ? 1.0f / (float)p.K : 1.0f;
  const float Tq = p.temp_target;
  const float cq = PROBS ? 1.0f : kLog2e / Tq;
  const float cq23 = PROBS ? 1.0f : cq * kTwo23;
  // LSE: log2(e)/T of every slot as a two-float sum (no systematic rounding of 1/T in the exponent)
  float lse_hi[KT + 1], lse_lo[KT + 1];
  // With one shared proposal the scan also forms the target row's normaliser (two rows per
  // workgroup in all); with per-draft rows it is left to the normaliser kernel.
  const bool lse_target = SHARED && with_pool;
  if (LSE) {
#pragma unroll
    for (int kk = 0; kk <= KT; ++kk) {
      float t = kk == KT ? Tq : p.temp_draft_all;
      if (kk < KT && p.temp_draft != nullptr && kbase + kk < p.K) t = p.temp_draft[kbase + kk];
      const double c64 = 1.4426950408889634 / (double)t;
      // (hi rounded towards zero and lo kept above zero, so that lo has hi's sign and is not 0: an
      // entry of -inf then gives -inf in both products, never NaN)
      float hi = (float)c64;
      if (fabs((double)hi) > fabs(c64)) hi = __uint_as_float(__float_as_uint(hi) - 1u);
      lse_hi[kk] = hi;
      lse_lo[kk] = fmaxf((float)(c64 - (double)hi), 1e-30f);
    }
  }
  bool lse_ran = false;  // the main loop (which feeds the sums) was executed
  // LSE: per slot a whole number n that is the same in all lanes of a wavefront (about the largest
  // x log2(e)/T the wavefront has seen) and per lane the sum of 2^(x log2(e)/T - n): the terms that
  // matter then have small exponents, where fp32 arithmetic is accurate enough, and moving n
  // rescales a sum by a power of two, exactly
  // (with one shared proposal only two rows are summed: slot 0 for the drafts, slot KT for the target)
  constexpr int NL = LSE ? (SHARED ? 2 : KT + 1) : 1;
  auto lidx = [](const int slot) { return LSE ? (SHARED ? (slot == KT ? 1 : 0) : slot) : 0; };
  double lse_acc[NL];
  float lse_n[NL];
#pragma unroll
  for (int kk = 0; kk < NL; ++kk) { lse_acc[kk] = 0.0; lse_n[kk] = -__builtin_huge_valf(); }
  // With one shared proposal the two running sums live in LDS: the kernel has no two registers to
  // spare for them across the main loop, and the compiler's own choice, scratch memory, costs a
  // round trip through the memory system per tile.
  if (kSumsInLds) {
#pragma unroll
    for (int kk = 0; kk < NL; ++kk) sums.v[kSumsInLds ? kk : 0][tid] = 0.0;
  }

  if (tid < 9) {
    // unused draft slots sit at -inf so the shared layout's max over drafts ignores them
    const bool used = (tid == KT) || (tid < KT && kbase + tid < p.K);
    s.tau[tid] = used ? 0x7F800000 : (int)0x80800000;  // ord32(+inf) : ord32(-inf)
    s.O[tid] = 0x7F800000;
    bool live = tid == KT && with_pool;
    if (tid < KT && kbase + tid < p.K) {
      float t = p.temp_draft_all;
      if (p.temp_draft != nullptr) t = p.temp_draft[kbase + tid];
      live = (t > 0.0f) && (t < __builtin_huge_valf());
    }
    s.OL[tid] = live ? 0x7F800000 : (int)0xFF800000;  // +inf until the warm-up has a bound : -inf
    s.best[tid] = kOrdInf64;
    s.where[tid] = ~0ull;
    s.second[tid] = kOrdInf64;
  }
  if (tid == 0) {
#pragma unroll
    for (int kk = 0; kk < KT; ++kk) { s.cd23[kk] = cd23[kk]; s.kok[kk] = kok[kk] ? 1 : 0; }
    s.lgK = lgK;
    s.count = 0; s.unsafe = p.force_exact ? 1 : 0; s.n_survivors = 0; s.n_exact = 0;
    s.shared_tau = p.shared_tau != nullptr ? p.shared_tau + b * (p.K + 1) : nullptr;
    s.shared_base = kbase;
    s.shared_pool = p.K;
    s.lse_redo = 0;
    s.qn[0] = 0; s.qn[1] = 0; s.qn[2] = 0; s.qn[3] = 0;
  }
  __syncthreads();

  unsigned long long my_survivors = 0;

  if (!p.force_exact) {
    // ---- warm-up: approximate keys of a few hundred elements give every reduction a finite
    // tau.  Each wave takes one draft pair (wave w: pair w mod KB) and 64 groups of the chunk's
    // first tile, so a lane evaluates 8 elements on both sides.
    {
      const int wv = tid >> 6;
      const int m = wv % KB;
      const int g = g_begin + (wv / KB) * 64 + (tid & 63);
      float a_even = __builtin_huge_valf(), a_odd = __builtin_huge_valf(), a_pool = __builtin_huge_valf();
      if (g < g_end && kbase + 2 * m < p.K) {
        float vq[4] = {fill, fill, fill, fill};
        if (with_pool) load4<T>(trow, g * 4, V, vec, fill, vq);
        uint32_t up[4], lo[4];
        const uint32_t pair = same_race ? 0u : pair_base + m;
        philox_block(row_lo, (uint32_t)g, row_hi, pair, p.seed_lo, p.seed_hi, up);
        philox_block(row_lo, (uint32_t)g, row_hi, pair | kLowBlock, p.seed_lo, p.seed_hi, lo);
        float Mj[4] = {0.0f, 0.0f, 0.0f, 0.0f};  // min-first: the indices' smallest times ...
        int holder[4] = {-1, -1, -1, -1};        // ... and the drafts that hold them
        if (MINF) {
          uint32_t mn[4], hd[4];
          philox_block(row_lo, (uint32_t)g, row_hi, kMinBlock, p.seed_lo, p.seed_hi, mn);
          philox_block(row_lo, (uint32_t)g, row_hi, kHolderBlock, p.seed_lo, p.seed_hi, hd);
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            Mj[j] = approx_race_time(mn[j]) * invK;
            holder[j] = holder_of(hd[j], p.K);
            float ell;
            if (with_pool && approx_log2_mass<PROBS>(vq[j], cq, ell)) a_pool = fminf(a_pool, __log2f(Mj[j]) - ell);
          }
        }
#pragma unroll
        for (int h = 0; h < 2; ++h) {
          const int k = kbase + 2 * m + h;
          if (k < p.K) {
            float tk = p.temp_draft_all;
            if (p.temp_draft != nullptr) tk = p.temp_draft[k];
            const bool ok = (tk > 0.0f) && (tk < __builtin_huge_valf());
            const float ck = PROBS ? 1.0f : kLog2e / tk;
            float vd[4];
            load4<T>(drow0 + (SHARED ? 0 : (long long)k * p.draft_stride_k), g * 4, V, vec, fill, vd);
            if (draft_masked) mask_bins(no_draft ? 0u : load_bins4(brow, g * 4, V, bins_aligned), announced, fill, vd);
            float a_k = __builtin_huge_valf();
#pragma unroll
            for (int j = 0; j < 4; ++j) {
              const uint32_t x = element_word(up[j], lo[j], same_race ? 0 : h);
              const float l2S = MINF ? __log2f(holder[j] == k ? Mj[j] : Mj[j] + approx_race_time(x))
                                     : approx_log2_race_time(x);
              float ell;
              if (ok && approx_log2_mass<PROBS>(vd[j], ck, ell)) a_k = fminf(a_k, l2S - ell);
              if (!MINF && with_pool && approx_log2_mass<PROBS>(vq[j], cq, ell)) a_pool = fminf(a_pool, l2S - ell);
            }
            if (h == 0) a_even = a_k; else a_odd = a_k;
          }
        }
      }
      int oe = ord32(a_even), oo = ord32(a_odd), op = ord32(a_pool);
#pragma unroll
      for (int d = 32; d >= 1; d >>= 1) {
        oe = min(oe, __shfl_xor(oe, d));
        oo = min(oo, __shfl_xor(oo, d));
        op = min(op, __shfl_xor(op, d));
      }
      if ((tid & 63) == 0) {
        if (oe < 0x7F800000) atomicMin(&s.tau[2 * m], oe);
        if (oo < 0x7F800000) atomicMin(&s.tau[2 * m + 1], oo);
        if (op < 0x7F800000) atomicMin(&s.tau[KT], op);
      }
      __syncthreads();
      if (tid <= KT) {
        const bool used = tid == KT ? with_pool : (kbase + tid < p.K);
        if (used && p.shared_tau != nullptr) {
          // post this chunk's first bound and take what the row's other workgroups have posted
          int *slot = p.shared_tau + b * (p.K + 1) + (tid < KT ? kbase + tid : p.K);
          const int mine = s.tau[tid];
          const int theirs = mine < 0x7F800000 ? atomicMin(slot, mine)
                                               : __hip_atomic_load(slot, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          if (theirs < mine) s.tau[tid] = theirs;
        }
        const float tau = unord32(s.tau[tid]);
        if (used && tau < __builtin_huge_valf() && !(fabsf(tau) <= kTauLimit)) s.unsafe = 1;
      }
      __syncthreads();
      if (tid == 0) {
        if (SHARED) {
          int m = s.tau[0];
#pragma unroll
          for (int kk = 1; kk < KT; ++kk) m = max(m, s.tau[kk]);
          if (kok[0]) store_offsets<MINF>(s, 0, make_offset<PROBS>(unord32(m), lgK));
        } else {
#pragma unroll
          for (int kk = 0; kk < KT; ++kk)
            if (kok[kk]) store_offsets<MINF>(s, kk, make_offset<PROBS>(unord32(s.tau[kk]), lgK));
        }
        if (with_pool) store_offsets<MINF>(s, KT, make_offset<PROBS>(unord32(s.tau[KT]), lgK));
      }
      __syncthreads();
    }

    // ---- main loop: level 1 on the upper half-words of every element, the rest on survivors.
    // No branch depends on the draft index: a padded draft (kbase + kk >= K) reads the last
    // real row and its half-words are tested like the others; only its hits are masked off.
    if (!s.unsafe) {
      lse_ran = true;
      constexpr int KD = SHARED ? 1 : KT;
      const elem *drow[KD];
#pragma unroll
      for (int kk = 0; kk < KD; ++kk)
        drow[kk] = drow0 + (SHARED ? 0 : (long long)min(kbase + kk, p.K - 1) * p.draft_stride_k);
      // One tile (kBlock groups).  The next tile's loads are issued before this tile's Philox
      // chains, thresholds and compares, so they have a whole tile of arithmetic to arrive.
      // Without a pool the target-side exponent is pinned at 0 (threshold 0: never a hit).
      using raw = typename T::raw;
      auto load_tile = [&](const int g, const bool interior, raw &rq, raw (&rd)[KD], uint32_t &rb) {
        if (binned && !no_draft) rb = load_bins4(brow, g * 4, V, bins_aligned);
        if (interior) {
          if (with_pool) rq = load_raw<T>(trow, g * 4);
          if (!no_draft) {
#pragma unroll
            for (int kk = 0; kk < KD; ++kk) rd[kk] = load_raw<T>(drow[kk], g * 4);
          }
        } else {
          if (with_pool) rq = load_raw_checked<T>(trow, g * 4, V, vec, fill);
          if (!no_draft) {
#pragma unroll
            for (int kk = 0; kk < KD; ++kk) rd[kk] = load_raw_checked<T>(drow[kk], g * 4, V, vec, fill);
          }
        }
      };
      // The tile is kept in its raw form and widened where it is used, so that few registers
      // are live across the (rare) branch to the survivors' path, which widens it again.
      // LSE: four more terms of one slot's sum of exp(x/T), as 2^(x c - n) with c = log2(e)/T a
      // two-float sum and n the wavefront's whole-number reference: x c_hi - n in one fused step (the
      // product is not rounded before n is taken off), then x c_lo on top; fp32 terms, four at a
      // time, into the lane's fp64 sum.  When some lane meets an exponent above 1 (a few times per
      // row; always at the first entry with mass, n starting at -inf), n moves to the wavefront's
      // largest x c, rounded, and the lanes' sums move with it by a power of two.  An entry of -inf
      // adds an exact 0; a NaN or +inf entry makes the sum NaN or +inf, which sends the workgroup
      // to the exact two-pass form at the end (there such entries carry no mass).
      auto lse_add = [&](const int slot, const float (&v)[4]) {
        const int sl = lidx(slot);
        float e[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) e[j] = fmaf(v[j], lse_lo[slot], fmaf(v[j], lse_hi[slot], -lse_n[sl]));
        const float em = fmaxf(fmaxf(e[0], e[1]), fmaxf(e[2], e[3]));  // (a NaN among them is passed over)
        if (__ballot(em > 1.0f) != 0ull) {
          float wm = -__builtin_huge_valf();
#pragma unroll
          for (int j = 0; j < 4; ++j)
            if (v[j] < __builtin_huge_valf()) wm = fmaxf(wm, v[j]);
#pragma unroll
          for (int d = 32; d >= 1; d >>= 1) wm = fmaxf(wm, __shfl_xor(wm, d));
          const float nn = rintf(__builtin_amdgcn_fmed3f(wm * lse_hi[slot], -1e9f, 1e9f));
          if (nn > lse_n[sl]) {  // (not so if only a +inf entry brought us here)
            if (lse_n[sl] > -__builtin_huge_valf()) {
              const int down = (int)fmaxf(lse_n[sl] - nn, -4000.0f);
              if (kSumsInLds) sums.v[kSumsInLds ? sl : 0][tid] = ldexp(sums.v[kSumsInLds ? sl : 0][tid], down);
              else lse_acc[sl] = ldexp(lse_acc[sl], down);
            }
            lse_n[sl] = nn;
#pragma unroll
            for (int j = 0; j < 4; ++j) e[j] = fmaf(v[j], lse_lo[slot], fmaf(v[j], lse_hi[slot], -nn));
          }
        }
        if (lse_n[sl] > -__builtin_huge_valf()) {
          // (the bare hardware exp2: a term below 2^-126 may flush to 0)
          const float part = (__builtin_amdgcn_exp2f(e[0]) + __builtin_amdgcn_exp2f(e[1])) +
                             (__builtin_amdgcn_exp2f(e[2]) + __builtin_amdgcn_exp2f(e[3]));
          if (kSumsInLds) sums.v[kSumsInLds ? sl : 0][tid] += (double)part;
          else lse_acc[sl] += (double)part;
        }
      };
      // min-first, survivors of the main loop's test.  The lanes whose tile passed lay it out in LDS,
      // eight lanes at a time, and a lane per laid-out index tests it against the index's own
      // exponent (the main loop's threshold is that of the tile's largest value).  What still passes
      // is not finished on the spot but put into the wavefront's queue: when enough indices have
      // gathered, and after the last tile, one lane per queued index and draft redoes the test with
      // its draft's bound as it stands by then (bounds only ever tighten, and a tighter bound is
      // still valid), draws the holder where that passes, and hands survivors to level 2.  One pass
      // serves the indices of many tiles: its Philox blocks and its level 2 cost a wavefront the
      // same whether one lane or all of them have work.
      const int wv = tid >> 6, lane = tid & 63;
      uint32_t *const stg = s_minf + wv * (kStageWords + kQueueWords);
      uint32_t *const que = stg + kStageWords;
      constexpr int kEntry = 3 + KD;  // index, word, target value, draft values
      constexpr int kPerPass = 64 / KT;
      constexpr int kQueueFlush = 8;
      static_assert((kQueueFlush + 32) * kEntry <= kQueueWords, "queue too small");
      auto drain = [&]() {
        __builtin_amdgcn_wave_barrier();
        const int n = __atomic_load_n(&s.qn[wv], __ATOMIC_RELAXED);
        for (int base = 0; base < n; base += kPerPass) {
          const int e = base + lane / KT;
          const int kk = lane % KT;
          if (e < n && kbase + kk < p.K) {
            const uint32_t *q = que + e * kEntry;
            const int i = (int)q[0];
            const uint32_t w = q[1];
            const float qs = __uint_as_float(q[2]);
            const float ds = __uint_as_float(q[3 + (SHARED ? 0 : kk)]);
            const int m = kk >> 1, h = kk & 1, j = i & 3;
            const uint32_t gs = (uint32_t)(i >> 2);
            const float c23 = s.cd23[kk];
            const bool okk = s.kok[kk] != 0;
            const float tau_d = unord32(__atomic_load_n(&s.tau[kk], __ATOMIC_RELAXED));
            const float tau_y = unord32(__atomic_load_n(&s.tau[KT], __ATOMIC_RELAXED));
            const float OYs = with_pool ? load_offset(&s.O[KT]) : -__builtin_huge_valf();
            const float fy = __builtin_amdgcn_fmed3f(fmaf(level1_value<PROBS>(qs), cq23, OYs), 0.0f, kCapHot);
            const float cdk = PROBS ? 1.0f : c23 * (1.0f / kTwo23);
            // w is the index's smallest time.  The test is redone with the draft's own bound (merged
            // with the pool's); where it passes the holder is drawn: if this draft holds the smallest
            // time, that time goes to level 2 for the draft and the pool; if not, the draft's time is
            // the smallest plus that of its own word, which can only matter if the word alone passes
            // the draft's bound (half-word first, as in the other variant).
            const float OX = okk ? make_offset<PROBS>(tau_d, lgK) : -__builtin_huge_valf();
            const float Fs = merged_exponent<PROBS>(ds, c23, OX, fy);
            if (Fs >= kCapHot || w >= ~threshold_of(Fs)) {
              uint32_t hd[4];
              philox_block(row_lo, gs, row_hi, kHolderBlock, p.seed_lo, p.seed_hi, hd);
              const uint32_t r = j == 0 ? hd[0] : j == 1 ? hd[1] : j == 2 ? hd[2] : hd[3];
              if (holder_of(r, p.K) == kbase + kk) {
                ++my_survivors;
                level2<KT, SHARED, PROBS, MINF>(s, approx_log2_race_time(w) - lgK, ds, qs, i, kk, okk, with_pool,
                                                cdk, cq, tau_d, tau_y);
              } else if (okk) {
                const float Fd = __builtin_amdgcn_fmed3f(fmaf(level1_value<PROBS>(ds), c23, make_offset<PROBS>(tau_d)),
                                                         0.0f, kCapHot);
                const uint32_t t = threshold_of(Fd);
                uint32_t up[4];
                philox_block(row_lo, gs, row_hi, pair_base + m, p.seed_lo, p.seed_hi, up);
                const uint32_t uw = j == 0 ? up[0] : j == 1 ? up[1] : j == 2 ? up[2] : up[3];
                const uint32_t hw = h ? (uw >> 16) : (uw & 0xFFFFu);
                if (Fd >= kCapHot || hw >= 0xFFFFu - (t >> 16)) {
                  uint32_t lo[4];
                  philox_block(row_lo, gs, row_hi, (pair_base + m) | kLowBlock, p.seed_lo, p.seed_hi, lo);
                  const uint32_t lw = j == 0 ? lo[0] : j == 1 ? lo[1] : j == 2 ? lo[2] : lo[3];
                  const uint32_t x = element_word(uw, lw, h);
                  if (Fd >= kCapHot || x >= ~t) {
                    ++my_survivors;
                    const float S = approx_race_time(w) * invK + approx_race_time(x);
                    level2<KT, SHARED, PROBS, MINF>(s, __log2f(S), ds, qs, i, kk, true, false, cdk, cq, tau_d, tau_y);
                  }
                }
              }
            }
          }
        }
        __builtin_amdgcn_wave_barrier();
        if (lane == 0) __atomic_store_n(&s.qn[wv], 0, __ATOMIC_RELAXED);
        __builtin_amdgcn_wave_barrier();
      };
      // min-first: one block holds the four indices' smallest race times, one word each; the tile's
      // largest word is tested against the loosest bound (every draft's and the pool's, each raised
      // by log2 K in its offset), and the survivors' path sorts out which draft the time belongs to.
      auto process_tile_minf = [&](const int g, const raw &rq, const raw (&rd)[KD], const uint32_t rb) {
        uint32_t mn[1][4];
        philox_blocks<1>((uint32_t)g, kMinBlock, row_lo, row_hi, p.seed_lo, p.seed_hi, mn);
        float F;
        {
          float vq[4];
          unpack(rq, vq);  // (without a pool the tile's target part keeps its initial zeros, and the offset is -inf)
          F = fmaf(level1_max4<PROBS>(vq), cq23, load_offset(&s.OL[KT]));
          if (LSE && lse_target) lse_add(KT, vq);
        }
#pragma unroll
        for (int kk = 0; kk < KD; ++kk) {
          float vd[4];
          unpack(rd[kk], vd);
          if (LSE) lse_add(kk, vd);  // (one shared row stands for all drafts: slot 0)
          F = fmaxf(F, fmaf(level1_max4<PROBS>(vd), cd23[kk], load_offset(&s.OL[kk])));
        }
        F = __builtin_amdgcn_fmed3f(F, 0.0f, kCapHot);
        const uint32_t mx = max(max(mn[0][0], mn[0][1]), max(mn[0][2], mn[0][3]));
        // Rare: some lane's largest word passed, or it holds a hot element.  The tile's one threshold
        // is that of its largest value, so most hits are another index's word under it.  Up to eight
        // such lanes at a time lay their tiles out; a lane per laid-out index tests it against the
        // index's own exponent (still the loosest over the drafts, merged with the pool's) and
        // queues it if it passes.
        const bool hit = F >= kCapHot || mx >= ~threshold_of(F);
        unsigned long long todo = __ballot(hit);
        if (todo != 0ull) {
          constexpr int kSlot = 12 + 4 * KD;  // words, target values, the group's number (padded), draft values
          static_assert(8 * kSlot <= kStageWords, "staging area too small");
          while (todo != 0ull) {
            const int rank = __builtin_amdgcn_mbcnt_hi((uint32_t)(todo >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)todo, 0u));
            const bool mine = ((todo >> lane) & 1ull) != 0ull && rank < 8;
            const unsigned long long taken = __ballot(mine);
            todo &= ~taken;
            if (mine) {
              uint32_t *o = stg + rank * kSlot;
              *reinterpret_cast<uint4 *>(o) = make_uint4(mn[0][0], mn[0][1], mn[0][2], mn[0][3]);
              float vq[4] = {0.0f, 0.0f, 0.0f, 0.0f};
              if (with_pool) unpack(rq, vq);
              *reinterpret_cast<float4 *>(o + 4) = make_float4(vq[0], vq[1], vq[2], vq[3]);
              o[8] = (uint32_t)g;
#pragma unroll
              for (int kk = 0; kk < KD; ++kk) {
                float vd[4];
                unpack(rd[kk], vd);
                *reinterpret_cast<float4 *>(o + 12 + 4 * kk) = make_float4(vd[0], vd[1], vd[2], vd[3]);
              }
            }
            __builtin_amdgcn_wave_barrier();
            const int n_taken = __popcll(taken);
            if (lane < 4 * n_taken) {
              const uint32_t *o = stg + (lane >> 2) * kSlot;
              const int j = lane & 3;
              const uint32_t x0 = o[j];
              const float qs = __uint_as_float(o[4 + j]);
              const int i = (int)o[8] * 4 + j;
              float Fj = fmaf(level1_value<PROBS>(qs), cq23, load_offset(&s.OL[KT]));
#pragma unroll
              for (int kk = 0; kk < KD; ++kk)
                Fj = fmaxf(Fj, fmaf(level1_value<PROBS>(__uint_as_float(o[12 + 4 * kk + j])), cd23[kk], load_offset(&s.OL[kk])));
              Fj = __builtin_amdgcn_fmed3f(Fj, 0.0f, kCapHot);
              if ((Fj >= kCapHot || x0 >= ~threshold_of(Fj)) && i < V) {
                uint32_t *q = que + atomicAdd(&s.qn[wv], 1) * kEntry;
                q[0] = (uint32_t)i; q[1] = x0; q[2] = o[4 + j];
#pragma unroll
                for (int kk = 0; kk < KD; ++kk) q[3 + kk] = o[12 + 4 * kk + j];
              }
            }
            __builtin_amdgcn_wave_barrier();
            if (__atomic_load_n(&s.qn[wv], __ATOMIC_RELAXED) >= kQueueFlush) drain();
          }
        }
        (void)rb;
      };
      auto process_tile_words = [&](const int g, const raw &rq, const raw (&rd)[KD], const uint32_t rb) {
        uint32_t up[KB][4];  // upper half-words: word j of block m = (index 4g+j, drafts 2m | 2m+1)
        if (same_race) {
          // one block for all drafts: draft 0's half-word of every index, in both halves of every pair
          uint32_t one[1][4];
          philox_blocks<1>((uint32_t)g, 0u, row_lo, row_hi, p.seed_lo, p.seed_hi, one);
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            const uint32_t w = (one[0][j] & 0xFFFFu) * 0x10001u;
#pragma unroll
            for (int m = 0; m < KB; ++m) up[m][j] = w;
          }
        } else {
          philox_blocks<KB>((uint32_t)g, pair_base, row_lo, row_hi, p.seed_lo, p.seed_hi, up);
        }

        // The main loop works with exponents lowered by 32 (kShift32): see packed_hi16.
        // One threshold serves the lane's four indices: that of the largest of the four values (the
        // exponent grows with the value), so a half-word that passes its own index's threshold also
        // passes this one; the survivors' path below tests every element against its own.
        const float OY = load_offset(&s.OL[KT]);  // (-inf without a pool)
        float FY;
        {
          float vq[4];
          unpack(rq, vq);  // (without a pool the tile's target part keeps its initial zeros, and OY is -inf)
          FY = fmaf(level1_max4<PROBS>(vq), cq23, OY);
          if (LSE && lse_target) lse_add(KT, vq);
        }

        // A half-word h passes the threshold th iff h + th >= 0xFFFF, i.e. iff the saturating sum
        // is 0xFFFF: the largest half-words of the tile are found first, then tested once.
        uint32_t most = 0u;
        if (SHARED) {
          // the threshold also serves every draft (it is built from the loosest of their bounds):
          // any (h > c) == (max h > c) over the tile's 8 KB half-words
          const float OX = load_offset(&s.OL[0]);
          float vd[4];
          unpack(rd[0], vd);
          if (draft_masked) mask_bins(rb, announced, fill, vd);
          if (LSE) lse_add(0, vd);  // (one row stands for all drafts: slot 0)
          const float FX = fmaf(level1_max4<PROBS>(vd), cd23[0], OX);
          const float F = __builtin_amdgcn_fmed3f(fmaxf(FX, FY), 0.0f, kCapOne32);
          uint32_t mx = up[0][0];
#pragma unroll
          for (int m = 0; m < KB; ++m)
#pragma unroll
            for (int j = 0; j < 4; ++j)
              if (m + j > 0) mx = pk_max_u16(mx, up[m][j]);
          most = pk_add_sat_u16(mx, packed_hi16(F, F));
        } else {
          const float FYc = __builtin_amdgcn_fmed3f(FY, 0.0f, kCapOne32);
#pragma unroll
          for (int m = 0; m < KB; ++m) {
            const float OX0 = load_offset(&s.OL[2 * m]);  // (-inf for a draft that is not taken)
            const float OX1 = load_offset(&s.OL[2 * m + 1]);
            float v0[4], v1[4];
            unpack(rd[SHARED ? 0 : 2 * m], v0);
            unpack(rd[SHARED ? 0 : 2 * m + 1], v1);
            if (draft_masked) { mask_bins(rb, announced, fill, v0); mask_bins(rb, announced, fill, v1); }
            if (LSE) { lse_add(2 * m, v0); lse_add(2 * m + 1, v1); }
            const float F0 = __builtin_amdgcn_fmed3f(fmaf(level1_max4<PROBS>(v0), cd23[2 * m], OX0), FYc, kCapOne32);
            const float F1 = __builtin_amdgcn_fmed3f(fmaf(level1_max4<PROBS>(v1), cd23[2 * m + 1], OX1), FYc, kCapOne32);
            const uint32_t mx = pk_max_u16(pk_max_u16(up[m][0], up[m][1]), pk_max_u16(up[m][2], up[m][3]));
            most = pk_max_u16(most, pk_add_sat_u16(mx, packed_hi16(F0, F1)));
          }
        }
        // Rare (about one wave and tile in ten): some lane has a half-word that passed, or a hot
        // element.  The wave takes such lanes one at a time: the lane lays its tile out in LDS and
        // the first 8 KB lanes each take one of its elements (index j of draft 2m + h), redo the
        // test with that draft's own bound (the shared layout's main loop used the loosest one),
        // draw the lower half-word where it still passes, and run the full-word test.  Bounds are
        // read again here: they only ever tighten, and a tighter bound is still valid.
        unsigned long long todo = __ballot((most & 0xFFFFu) == 0xFFFFu || (most >> 16) == 0xFFFFu);
        if (todo != 0ull) {
          const int lane = tid & 63;
          Lds::Stage &st = s.stage[tid >> 6];
          while (todo != 0ull) {
            const int src = __ffsll((long long)todo) - 1;
            todo &= todo - 1ull;
            if (lane == src) {
#pragma unroll
              for (int m = 0; m < KB; ++m)
#pragma unroll
                for (int j = 0; j < 4; ++j) st.up[m * 4 + j] = up[m][j];
              float vq[4] = {0.0f, 0.0f, 0.0f, 0.0f};
              if (with_pool) unpack(rq, vq);
#pragma unroll
              for (int j = 0; j < 4; ++j) st.vq[j] = vq[j];
#pragma unroll
              for (int kk = 0; kk < KD; ++kk) {
                float vd[4];
                unpack(rd[kk], vd);
                if (draft_masked) mask_bins(rb, announced, fill, vd);
#pragma unroll
                for (int j = 0; j < 4; ++j) st.vd[kk * 4 + j] = vd[j];
              }
            }
            __builtin_amdgcn_wave_barrier();
            const int gs = g - lane + src;  // the lanes of a wave hold consecutive groups
            if (lane < 8 * KB) {
              const int m = lane >> 3, j = (lane >> 1) & 3, h = lane & 1;
              const int kk = 2 * m + h;
              const int i = gs * 4 + j;
              if (kbase + kk < p.K && i < V) {
                const uint32_t uw = st.up[m * 4 + j];
                const float ds = st.vd[(SHARED ? 0 : kk) * 4 + j], qs = st.vq[j];
                const float c23 = s.cd23[kk];
                const bool okk = s.kok[kk] != 0;
                const float tau_d = unord32(__atomic_load_n(&s.tau[kk], __ATOMIC_RELAXED));
                const float tau_y = unord32(__atomic_load_n(&s.tau[KT], __ATOMIC_RELAXED));
                const float OYs = with_pool ? load_offset(&s.O[KT]) : -__builtin_huge_valf();
                const float fy = __builtin_amdgcn_fmed3f(fmaf(level1_value<PROBS>(qs), cq23, OYs), 0.0f, kCapHot);
                const float OX = SHARED ? make_offset<PROBS>(tau_d)
                                        : (okk ? load_offset(&s.O[kk]) : -__builtin_huge_valf());
                const float F = merged_exponent<PROBS>(ds, c23, OX, fy);
                const uint32_t t = threshold_of(F);
                const uint32_t hw = h ? (uw >> 16) : (uw & 0xFFFFu);
                if (F >= kCapHot || hw >= 0xFFFFu - (t >> 16)) {
                  uint32_t lo[4];
                  philox_block(row_lo, (uint32_t)gs, row_hi, (same_race ? 0u : pair_base + m) | kLowBlock, p.seed_lo, p.seed_hi, lo);
                  const uint32_t lw = j == 0 ? lo[0] : j == 1 ? lo[1] : j == 2 ? lo[2] : lo[3];
                  const uint32_t x = element_word(uw, lw, same_race ? 0 : h);
                  if (F >= kCapHot || x >= ~t) {
                    ++my_survivors;
                    level2<KT, SHARED, PROBS, MINF>(s, approx_log2_race_time(x), ds, qs, i, kk, okk, with_pool,
                                                    PROBS ? 1.0f : c23 * (1.0f / kTwo23), cq, tau_d, tau_y);
                  }
                }
              }
            }
            __builtin_amdgcn_wave_barrier();
          }
        }
      };
      auto process_tile = [&](const int g, const raw &rq, const raw (&rd)[KD], const uint32_t rb) {
        if constexpr (MINF) process_tile_minf(g, rq, rd, rb);
        else process_tile_words(g, rq, rd, rb);
      };
      // A tile is interior when every lane's group is complete and inside the chunk: all rows
      // are then read with unconditional vector loads.
      const int interior_end = vec ? min(g_end, V >> 2) : g_begin;
      const int n_interior = max(0, (interior_end - g_begin) / kBlock);
      int it = 0;
      if (n_interior > 0) {
        // the next tile's loads are issued one tile of arithmetic before they are used (two
        // register sets that swap roles in a loop unrolled twice, instead of the copies below,
        // measured slower in both layouts)
        raw aq = raw(), ad[KD], bq = raw(), bd[KD];
        uint32_t ab = 0, bb = 0;
        const int g0 = g_begin + tid;
        load_tile(g0, true, aq, ad, ab);
        // lanes 0..KT of the first wave follow the row's shared bounds: read every fourth
        // iteration, merged four iterations later (the load never has to be waited for)
        const bool follows = p.shared_tau != nullptr && tid <= KT &&
                             (tid == KT ? with_pool : (kbase + tid < p.K));
        // (the slot is kept as an index: the row's base is wave-uniform)
        const int *row_tau = p.shared_tau != nullptr ? p.shared_tau + b * (p.K + 1) : nullptr;
        const int follow_idx = tid < KT ? kbase + tid : p.K;
        int seen = 0x7F800000;
        int prio_step = -1;
        for (; it < n_interior; ++it) {
          // A SIMD serves its wavefronts oldest first, so the workgroups of a CU drift apart and the
          // last one finishes on a nearly empty machine.  The wave's own priority therefore falls as
          // it advances, in steps at 1/2, 3/4 and 7/8 of its tiles: whoever is behind a step is
          // served first and the waves meet again at every step, the last time close to the end.
          {
            const int left = n_interior - it;
            const int step = left * 2 > n_interior ? 0 : left * 4 > n_interior ? 1 : left * 8 > n_interior ? 2 : 3;
            if (step != prio_step) {  // uniform
              prio_step = step;
              switch (step) {
                case 0: __builtin_amdgcn_s_setprio(3); break;
                case 1: __builtin_amdgcn_s_setprio(2); break;
                case 2: __builtin_amdgcn_s_setprio(1); break;
                default: __builtin_amdgcn_s_setprio(0); break;
              }
            }
          }
          if (follows && (it & 3) == 0) {
            if (seen < __atomic_load_n(&s.tau[tid], __ATOMIC_RELAXED))
              publish<KT, SHARED, PROBS, MINF>(s, tid, unord32(seen), false);
            seen = __hip_atomic_load(row_tau + follow_idx, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          }
          load_tile(g0 + min(it + 1, n_interior - 1) * kBlock, true, bq, bd, bb);
          process_tile(g0 + it * kBlock, aq, ad, ab);
          aq = bq; ab = bb;
#pragma unroll
          for (int kk = 0; kk < KD; ++kk) ad[kk] = bd[kk];
        }
      }
      for (; it < iters; ++it) {
        // every lane takes part (the survivors' path works wave-wide); a group past the end of the
        // row reads as entries without mass
        const int g = g_begin + it * kBlock + tid;
        raw rq = raw(), rd[KD];
        uint32_t rb = 0;
        load_tile(g, false, rq, rd, rb);
        process_tile(g, rq, rd, rb);
      }
      if constexpr (MINF) drain();  // what is still queued
    }
    __syncthreads();
    if (tid == 0 && s.count > kListCap) s.unsafe = 1;
    __syncthreads();
  }

  // ---- LSE: the lanes' running sums become per-wave sums in LDS right away (they are merged after
  // level 3), so that the registers that carried them through the main loop are free from here on
  if (LSE) {
    const int wv = tid >> 6;
#pragma unroll
    for (int kk = 0; kk <= KT; ++kk) {
      if (SHARED && kk != 0 && kk != KT) continue;
      // the lanes of a wave share the reference: their sums add up as they are
      const float wm = lse_n[lidx(kk)];
      double v = lse_acc[lidx(kk)];
      if (kSumsInLds) v = sums.v[kSumsInLds ? lidx(kk) : 0][tid];
      if (!(wm > -__builtin_huge_valf())) v = 0.0;
#pragma unroll
      for (int d = 32; d >= 1; d >>= 1) v += __shfl_xor(v, d);
      if ((tid & 63) == 0) { s.lse_wave[wv][kk] = v; s.lse_wmax[wv][kk] = wm; }
    }
  }

  unsigned long long my_exact = 0;
  const bool exact_all = s.unsafe != 0;  // uniform: read after the barrier

  if (!exact_all) {
    // ---- level 3: exact keys of the records that are still within the band
    const int n = s.count;
    constexpr int kPer = kListCap / kBlock;
    double key[kPer];
    int ri[kPer], rslot[kPer], rk[kPer];
#pragma unroll
    for (int e = 0; e < kPer; ++e) {
      key[e] = __builtin_huge_val();
      ri[e] = 0; rslot[e] = 0; rk[e] = 0;
      const int r = e * kBlock + tid;
      if (r < n) {
        const int tag = s.rec_tag[r];
        const bool pool = tag >= KT;
        const int kk = pool ? tag - KT : tag;
        const int slot = pool ? KT : kk;
        const float tau = unord32(s.tau[slot]);
        if (s.rec_a[r] <= tau + kEps2) {
          const int i = s.rec_i[r];
          const int k = kbase + kk;
          uint32_t up[4], lo[4];
          const int kr = same_race ? 0 : k;  // the draft whose race times this one uses
          philox_block(row_lo, (uint32_t)(i >> 2), row_hi, (uint32_t)(kr >> 1), p.seed_lo, p.seed_hi, up);
          philox_block(row_lo, (uint32_t)(i >> 2), row_hi, (uint32_t)(kr >> 1) | kLowBlock, p.seed_lo, p.seed_hi, lo);
          const int j = i & 3;
          const uint32_t uw = j == 0 ? up[0] : j == 1 ? up[1] : j == 2 ? up[2] : up[3];
          const uint32_t lw = j == 0 ? lo[0] : j == 1 ? lo[1] : j == 2 ? lo[2] : lo[3];
          double S = exact_race_time(element_word(uw, lw, kr & 1));
          if (MINF) {
            uint32_t mn[4], hd[4];
            philox_block(row_lo, (uint32_t)(i >> 2), row_hi, kMinBlock, p.seed_lo, p.seed_hi, mn);
            philox_block(row_lo, (uint32_t)(i >> 2), row_hi, kHolderBlock, p.seed_lo, p.seed_hi, hd);
            const double M = exact_race_time(j == 0 ? mn[0] : j == 1 ? mn[1] : j == 2 ? mn[2] : mn[3]) / (double)p.K;
            const int holder = holder_of(j == 0 ? hd[0] : j == 1 ? hd[1] : j == 2 ? hd[2] : hd[3], p.K);
            S = (pool || holder == k) ? M : M + S;  // (a pool record is the holder's: the index's smallest time)
          }
          float temp = Tq;
          float v;
          if (pool) {
            v = load1<T>(trow, i);
          } else {
            v = load1<T>(drow0 + (SHARED ? 0 : (long long)k * p.draft_stride_k), i);
            temp = p.temp_draft != nullptr ? p.temp_draft[k] : p.temp_draft_all;
          }
          key[e] = exact_key<PROBS>(S, v, (double)temp);
          ri[e] = i; rslot[e] = slot; rk[e] = pool ? k : 0;
          ++my_exact;
          offer_key(s, slot, key[e]);
        }
      }
    }
    __syncthreads();
#pragma unroll
    for (int e = 0; e < kPer; ++e) offer_where(s, rslot[e], key[e], ri[e], rk[e]);
    __syncthreads();
#pragma unroll
    for (int e = 0; e < kPer; ++e) offer_second(s, rslot[e], key[e], ri[e]);
  } else {
    // ---- fallback: every element of the chunk in fp64 (debug flag, out-of-range tau, list overflow)
    if (tid < 9) { s.best[tid] = kOrdInf64; s.where[tid] = ~0ull; s.second[tid] = kOrdInf64; }
    __syncthreads();
    // A lane keeps its own best per reduction; every key that loses against it (or that it
    // displaces) goes straight to the reduction's runner-up in LDS.  For the pool a lane meets an
    // index once per draft: a loser at the lane's current index is dropped (the lane's best at
    // that index stands for it), and one that was offered earlier and now shares the winner's
    // index is always dominated by a smaller key at another index that was offered as well.
    auto offer_loser = [&](const int slot, const double key) {
      if (key < __builtin_huge_val() && ord64(key) < __atomic_load_n(&s.second[slot], __ATOMIC_RELAXED))
        atomicMin(&s.second[slot], ord64(key));
    };
    double best[KT + 1];
    int bi[KT + 1], bk = 0;
#pragma unroll
    for (int kk = 0; kk <= KT; ++kk) { best[kk] = __builtin_huge_val(); bi[kk] = -1; }
    for (int it = 0; it < iters; ++it) {
      const int g = g_begin + it * kBlock + tid;
      if (g >= g_end) continue;
      float vq[4] = {fill, fill, fill, fill};
      if (with_pool) load4<T>(trow, g * 4, V, false, fill, vq);
#pragma unroll 1
      for (int kk = 0; kk < KT; ++kk) {
        const int k = kbase + kk;
        if (k >= p.K) break;
        float vd[4];
        load4<T>(drow0 + (SHARED ? 0 : (long long)k * p.draft_stride_k), g * 4, V, false, fill, vd);
        if (draft_masked) mask_bins(no_draft ? 0u : load_bins4(brow, g * 4, V, bins_aligned), announced, fill, vd);
        uint32_t up[4], lo[4];
        const int kr = same_race ? 0 : k;
        philox_block(row_lo, (uint32_t)g, row_hi, (uint32_t)(kr >> 1), p.seed_lo, p.seed_hi, up);
        philox_block(row_lo, (uint32_t)g, row_hi, (uint32_t)(kr >> 1) | kLowBlock, p.seed_lo, p.seed_hi, lo);
        uint32_t mn[4] = {0u, 0u, 0u, 0u}, hd[4] = {0u, 0u, 0u, 0u};
        if (MINF) {  // (drawn again for every draft: this path is cold, and fewer registers stay live)
          philox_block(row_lo, (uint32_t)g, row_hi, kMinBlock, p.seed_lo, p.seed_hi, mn);
          philox_block(row_lo, (uint32_t)g, row_hi, kHolderBlock, p.seed_lo, p.seed_hi, hd);
        }
        const float tk = p.temp_draft != nullptr ? p.temp_draft[k] : p.temp_draft_all;
        const bool ok = (tk > 0.0f) && (tk < __builtin_huge_valf());
        double bx = __builtin_huge_val();
        int bxi = -1;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const int i = g * 4 + j;
          if (i >= V) continue;
          double S = exact_race_time(element_word(up[j], lo[j], kr & 1));
          if (MINF) {
            const double M = exact_race_time(mn[j]) / (double)p.K;
            S = holder_of(hd[j], p.K) == k ? M : M + S;
          }
          const double kx = ok ? exact_key<PROBS>(S, vd[j], (double)tk) : __builtin_huge_val();
          const double ky = with_pool ? exact_key<PROBS>(S, vq[j], (double)Tq) : __builtin_huge_val();
          my_exact += 2;
          if (kx < bx) { offer_loser(kk, bx); bx = kx; bxi = i; }
          else offer_loser(kk, kx);
          if (ky < best[KT] || (ky == best[KT] && ky < __builtin_huge_val() &&
                                (i < bi[KT] || (i == bi[KT] && k < bk)))) {
            if (bi[KT] != i) offer_loser(KT, best[KT]);
            best[KT] = ky; bi[KT] = i; bk = k;
          } else if (i != bi[KT]) {
            offer_loser(KT, ky);
          }
        }
        // fold (bx, bxi) into draft kk's running best without dynamic register indexing
#pragma unroll
        for (int q = 0; q < KT; ++q)
          if (q == kk) {
            if (bx < best[q] || (bx == best[q] && bx < __builtin_huge_val() && bxi < bi[q])) {
              offer_loser(q, best[q]);
              best[q] = bx; bi[q] = bxi;
            } else {
              offer_loser(q, bx);
            }
          }
      }
    }
    // Lanes own disjoint indices, so a lane's best that does not become the workgroup's is a
    // runner-up candidate, and so is the best it displaces.
#pragma unroll
    for (int kk = 0; kk <= KT; ++kk) {
      if (best[kk] < __builtin_huge_val()) {
        const unsigned long long mine = ord64(best[kk]);
        const unsigned long long old = atomicMin(&s.best[kk], mine);
        const unsigned long long loser = mine < old ? old : mine;
        if (loser != kOrdInf64) atomicMin(&s.second[kk], loser);
      }
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk <= KT; ++kk) offer_where(s, kk, best[kk], bi[kk], kk == KT ? bk : 0);
  }
  __syncthreads();

  // ---- LSE: this chunk's share of every slot's normaliser, ln of (sum of exp(x/T) over the chunk)
  if (LSE) {
    __syncthreads();
    const bool slot_used = tid < KT ? (kbase + tid < p.K) : (tid == KT && lse_target);
    // the slot whose sums this thread reports: with one shared proposal slot 0 stands for every draft
    const int from = SHARED ? (tid < KT ? 0 : KT) : tid;
    double share = -__builtin_huge_val();
    if (tid <= KT && slot_used) {
      float tk = tid == KT ? Tq : p.temp_draft_all;
      if (tid < KT && p.temp_draft != nullptr) tk = p.temp_draft[kbase + tid];
      const bool t_ok = tk > 0.0f && tk < __builtin_huge_valf();
      if (!t_ok) {
        share = -__builtin_huge_val();
      } else if (!lse_ran) {
        s.lse_redo = 1;
      } else {
        // the waves' sums, each relative to 2^(its reference), brought to the largest reference
        float gm = -__builtin_huge_valf();
        for (int w = 0; w < 4; ++w) gm = fmaxf(gm, s.lse_wmax[w][from]);
        double tot = 0.0;
        for (int w = 0; w < 4; ++w)
          if (s.lse_wmax[w][from] > -__builtin_huge_valf())
            tot += ldexp(s.lse_wave[w][from], (int)fmaxf(s.lse_wmax[w][from] - gm, -4000.0f));
        if (!(gm > -__builtin_huge_valf())) {
          share = -__builtin_huge_val();   // no entry of the chunk carries mass
        } else if (!(tot >= 0.5 && tot < __builtin_huge_val())) {
          s.lse_redo = 1;                  // not finite, or the largest entry's own term (>= 2^-1/2) is missing
        } else {
          share = (double)gm * 0.6931471805599453 + log(tot);
        }
      }
    }
    __syncthreads();
    if (s.lse_redo) {  // uniform
      float *s_max = reinterpret_cast<float *>(&s.lse_wmax[0][0]);
      double *s_sum = &s.lse_wave[0][0];
#pragma unroll 1
      for (int kk = 0; kk <= KT; ++kk) {
        const bool used = kk < KT ? (SHARED ? kk == 0 : kbase + kk < p.K) : lse_target;
        if (!used) continue;  // uniform
        float tk = kk == KT ? Tq : p.temp_draft_all;
        if (kk < KT && p.temp_draft != nullptr) tk = p.temp_draft[kbase + kk];
        const elem *rowp = kk == KT ? trow : drow0 + (SHARED ? 0 : (long long)(kbase + kk) * p.draft_stride_k);
        const double v = chunk_lse_exact<T>(rowp, g_begin, g_end, V, (double)tk, s_max, s_sum);
        if (from == kk) share = v;
      }
    }
    if (tid <= KT && slot_used) {
      const long long slot = tid < KT ? kbase + tid : p.K;
      p.lse_part[(b * (p.K + 1) + slot) * p.n_chunks + chunk] = share;
    }
  }

  // ---- partial results of this (row, draft group, chunk)
  if (tid <= KT) {
    const bool has = s.where[tid] != ~0ull;
    const double key = has ? unord64(s.best[tid]) : __builtin_huge_val();
    const int idx = has ? (int)(s.where[tid] >> 32) : -1;
    if (tid < KT) {
      const int k = kbase + tid;
      if (k < p.K) {
        const long long o = (b * p.K + k) * p.n_chunks + chunk;
        p.out.keyX[o] = key;
        p.out.idxX[o] = idx;
        p.out.secX[o] = unord64(s.second[tid]);
      }
    } else {
      const long long o = (b * p.n_kgroups + kg) * p.n_chunks + chunk;
      p.out.keyY[o] = key;
      p.out.idxY[o] = idx;
      p.out.kY[o] = has ? (int)(uint32_t)s.where[tid] : -1;
      p.out.secY[o] = unord64(s.second[tid]);
    }
  }
  if (p.stats != nullptr) {
    if (my_survivors) atomicAdd(&s.n_survivors, my_survivors);
    if (my_exact) atomicAdd(&s.n_exact, my_exact);
    __syncthreads();
    if (tid == 0) {
      if (s.n_survivors) atomicAdd(&p.stats->survivors, s.n_survivors);
      if (s.n_exact) atomicAdd(&p.stats->exact_evals, s.n_exact);
      if (exact_all && !p.force_exact) atomicAdd(&p.stats->slow_blocks, 1ull);
    }
  }
  if (FIN) {
    // the row is this workgroup's alone (the host launches this variant only then): its partial
    // results are complete, written by this workgroup's own threads
    __shared__ FinalizeShared s_fin;
    __syncthreads();
    finalize_row<kBlock>(p.fin, b, tid, s_fin);
  }
}

// kt: drafts per workgroup pass (2, 4 or 8; 1 runs as 2: a draft pair shares its blocks).
template <typename T, bool SHARED, bool MINF>
hipError_t launch_scan(int kt, bool probs, bool finish, unsigned grid, hipStream_t st, const ScanParams &p) {
#define LLC_LAUNCH(KB_, PR_, MK_, LS_, FN_)                                                                        \
  hipLaunchKernelGGL((scan_kernel<T, KB_, SHARED, PR_, MK_, LS_, FN_, MINF>), dim3(grid), dim3(kBlock), 0, st, p); \
  return hipGetLastError();
  const bool masked = p.bins != nullptr || p.no_draft != 0 || p.same_race != 0;
  if (p.lse_part != nullptr) {
    // fused normalisers: logit kinds, no bins
    if (probs || masked || finish) return hipErrorInvalidValue;
    switch (kt) {
      case 2: LLC_LAUNCH(1, false, false, true, false)
      case 4: LLC_LAUNCH(2, false, false, true, false)
      case 8: LLC_LAUNCH(4, false, false, true, false)
    }
    return hipErrorInvalidValue;
  }
  if (masked) {
    // binned candidates / pool-only passes exist for fp32 log-weights, one word per (index, draft)
    if constexpr (sizeof(typename T::elem) == 4 && !MINF) {
      if (probs || finish) return hipErrorInvalidValue;
      switch (kt) {
        case 2: LLC_LAUNCH(1, false, true, false, false)
        case 4: LLC_LAUNCH(2, false, true, false, false)
        case 8: LLC_LAUNCH(4, false, true, false, false)
      }
    }
    return hipErrorInvalidValue;
  }
  if (!probs) {
    if (finish) {
      switch (kt) {
        case 2: LLC_LAUNCH(1, false, false, false, true)
        case 4: LLC_LAUNCH(2, false, false, false, true)
        case 8: LLC_LAUNCH(4, false, false, false, true)
      }
    } else {
      switch (kt) {
        case 2: LLC_LAUNCH(1, false, false, false, false)
        case 4: LLC_LAUNCH(2, false, false, false, false)
        case 8: LLC_LAUNCH(4, false, false, false, false)
      }
    }
  } else {
    if (finish) {
      switch (kt) {
        case 2: LLC_LAUNCH(1, true, false, false, true)
        case 4: LLC_LAUNCH(2, true, false, false, true)
        case 8: LLC_LAUNCH(4, true, false, false, true)
      }
    } else {
      switch (kt) {
        case 2: LLC_LAUNCH(1, true, false, false, false)
        case 4: LLC_LAUNCH(2, true, false, false, false)
        case 8: LLC_LAUNCH(4, true, false, false, false)
      }
    }
  }
#undef LLC_LAUNCH
  return hipErrorInvalidValue;
}

}  // namespace llc
