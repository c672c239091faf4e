// Sanitizer harness for the CPU oracle (test infrastructure): the oracle's source compiled into one
// executable with -fsanitize=address,undefined and run on the tiny configuration and on the edge
// rows the parity tests use (rows without mass, NaN and infinite entries, ragged and one-entry
// rows, empty list slots, every variant of the calls).  It checks nothing but that the run is
// clean: tests/test_oracle_sanitizers.py builds it, runs it and looks at the exit status.
#include "../oracle/llc_ref.cpp"

#include <cstdio>
#include <cstdlib>

namespace {

struct Lcg {  // inputs only: any fixed sequence will do
  uint64_t s;
  double next() { s = s * 6364136223846793005ull + 1442695040888963407ull; return (double)(s >> 11) / 9007199254740992.0; }
  float normal() { double a = 0; for (int i = 0; i < 12; ++i) a += next(); return (float)(a - 6.0); }
};

uint16_t bf16_of(float f) { uint32_t w; std::memcpy(&w, &f, 4); return (uint16_t)(w >> 16); }

void couple_case(int64_t B, int64_t K, int64_t V, int kind, bool per_k, bool bf16, bool edge, Lcg &g, int min_first = 0) {
  const int64_t rows_d = per_k ? B * K : B;
  std::vector<float> d((size_t)(rows_d * V)), t((size_t)(B * V)), temps((size_t)K);
  for (auto &v : d) v = kind == KIND_PROBS ? (float)g.next() : 2.0f * g.normal();
  for (auto &v : t) v = kind == KIND_PROBS ? (float)g.next() : 2.0f * g.normal();
  for (auto &v : temps) v = 0.5f + (float)g.next();
  if (edge && B >= 4) {
    const float ninf = -std::numeric_limits<float>::infinity();
    for (int64_t i = 0; i < V; ++i) t[(size_t)i] = kind == KIND_PROBS ? 0.0f : ninf;             // target without mass
    for (int64_t i = 0; i < V; ++i) d[(size_t)((per_k ? K : 1) * V + i)] = kind == KIND_PROBS ? 0.0f : ninf;  // a draft without mass
    t[(size_t)(2 * V)] = std::numeric_limits<float>::quiet_NaN();
    d[(size_t)((per_k ? 2 * K : 2) * V + V - 1)] = std::numeric_limits<float>::infinity();
    if (kind == KIND_PROBS) t[(size_t)(3 * V)] = -1.0f;
  }
  std::vector<uint16_t> dh, th;
  if (bf16) {
    for (float v : d) dh.push_back(bf16_of(v));
    for (float v : t) th.push_back(bf16_of(v));
  }
  std::vector<int32_t> X((size_t)(B * K)), Y((size_t)B), match((size_t)B), Yk((size_t)(B * K));
  std::vector<uint8_t> acc((size_t)B);
  std::vector<double> keyX((size_t)(B * K)), keyY((size_t)B), keyYk((size_t)(B * K)), gapX((size_t)(B * K)), gapY((size_t)B),
      gapYk((size_t)(B * K));
  llc_ref_args a;
  std::memset(&a, 0, sizeof(a));
  a.B = B; a.K = K; a.V = V; a.dtype = bf16 ? DT_BF16 : DT_F32; a.kind = kind;
  a.draft = bf16 ? (const void *)dh.data() : (const void *)d.data();
  a.draft_stride_b = per_k ? K * V : V; a.draft_stride_k = per_k ? V : 0;
  a.target = bf16 ? (const void *)th.data() : (const void *)t.data(); a.target_stride_b = V;
  a.temp_target = 0.8f; a.temp_draft = per_k ? temps.data() : nullptr; a.temp_draft_all = 1.2f;
  a.seed = 0x5EED0001ull; a.row_offset = (1ull << 35) + 7;
  a.X = X.data(); a.Y = Y.data(); a.accept = acc.data(); a.match_k = match.data();
  a.keyX = keyX.data(); a.keyY = keyY.data(); a.Yk = Yk.data(); a.keyYk = keyYk.data();
  a.gapX = gapX.data(); a.gapY = gapY.data(); a.gapYk = gapYk.data();
  a.threads = 2;
  a.min_first = min_first;
  if (llc_couple_ref(&a) != 0) { std::puts("llc_couple_ref rejected its arguments"); std::exit(2); }
}

}  // namespace

int main() {
  Lcg g{12345};
  // the tiny configuration (B=64, V=1024, K=4, one shared proposal, fp32 logits)
  couple_case(64, 4, 1024, KIND_LOGITS, false, false, false, g);
  couple_case(64, 4, 1024, KIND_LOGITS, false, false, false, g, 1);
  // edge rows, every kind and layout, ragged and one-entry rows
  for (int kind : {KIND_LOGITS, KIND_PROBS, KIND_LOGW})
    for (int per_k = 0; per_k < 2; ++per_k)
      for (int bf = 0; bf < 2; ++bf)
        for (int64_t V : {1, 3, 5, 255, 1001})
          for (int mf = 0; mf < 2; ++mf) couple_case(5, 3, V, kind, per_k != 0, bf != 0, true, g, mf);
  // importance weights, binned selection (own race times and the shared-race baseline)
  {
    const int64_t B = 6, L = 3, N = 777;
    std::vector<float> enc((size_t)(B * N)), dec((size_t)(B * L * N));
    std::vector<uint8_t> bins((size_t)(B * N));
    for (auto &v : enc) v = 2.0f * g.normal();
    for (auto &v : dec) v = 2.0f * g.normal();
    for (auto &v : bins) v = (uint8_t)(g.next() * 8);
    for (int64_t i = 0; i < N; ++i) enc[(size_t)i] = -std::numeric_limits<float>::infinity();
    for (int64_t i = 0; i < N; ++i) dec[(size_t)(L * N + i)] = -std::numeric_limits<float>::infinity();
    std::vector<int32_t> X((size_t)(B * L)), Y((size_t)B), msg((size_t)B), match((size_t)B);
    std::vector<uint8_t> acc((size_t)B);
    std::vector<double> keyX((size_t)(B * L)), keyY((size_t)B), gapX((size_t)(B * L)), gapY((size_t)B);
    if (llc_couple_is_ref(B, L, N, enc.data(), N, dec.data(), L * N, N, 9, 1, X.data(), Y.data(), acc.data(), match.data(),
                          keyX.data(), keyY.data(), gapX.data(), gapY.data(), 2, 0) != 0) return 2;
    if (llc_couple_is_ref(B, L, N, enc.data(), N, dec.data(), L * N, N, 9, 1, X.data(), Y.data(), acc.data(), match.data(),
                          keyX.data(), keyY.data(), gapX.data(), gapY.data(), 2, 1) != 0) return 2;
    for (int shared = 0; shared < 2; ++shared)
      if (llc_compress_select_ref(B, L, N, enc.data(), N, dec.data(), L * N, N, bins.data(), N, 9, 1, X.data(), Y.data(),
                                  msg.data(), acc.data(), match.data(), keyX.data(), keyY.data(), gapX.data(), gapY.data(),
                                  2, shared) != 0)
        return 2;
  }
  // candidate lists: empty slots, repeated ids, a list without mass
  {
    const int64_t B = 4, K = 3, Md = 9, Mt = 7;
    std::vector<int32_t> did((size_t)(B * K * Md)), tid((size_t)(B * Mt));
    std::vector<float> dv((size_t)(B * K * Md)), tv((size_t)(B * Mt));
    for (auto &v : did) v = (int32_t)(g.next() * 50) - 3;
    for (auto &v : tid) v = (int32_t)(g.next() * 50) - 3;
    for (auto &v : dv) v = g.normal();
    for (auto &v : tv) v = g.normal();
    for (int64_t e = 0; e < Mt; ++e) tv[(size_t)e] = -std::numeric_limits<float>::infinity();
    std::vector<int32_t> X((size_t)(B * K)), Y((size_t)B), match((size_t)B);
    std::vector<uint8_t> acc((size_t)B);
    std::vector<double> keyX((size_t)(B * K)), keyY((size_t)B), gapX((size_t)(B * K)), gapY((size_t)B);
    llc_topm_ref_args a;
    std::memset(&a, 0, sizeof(a));
    a.B = B; a.K = K; a.Md = Md; a.Mt = Mt; a.dtype = DT_F32; a.kind = KIND_LOGITS;
    a.draft_ids = did.data(); a.draft_val = dv.data(); a.draft_stride_b = K * Md; a.draft_stride_k = Md;
    a.target_ids = tid.data(); a.target_val = tv.data(); a.target_stride_b = Mt;
    a.temp_target = 1.0f; a.temp_draft_all = 1.0f; a.seed = 3;
    a.X = X.data(); a.Y = Y.data(); a.accept = acc.data(); a.match_k = match.data();
    a.keyX = keyX.data(); a.keyY = keyY.data(); a.gapX = gapX.data(); a.gapY = gapY.data(); a.threads = 2;
    if (llc_couple_topm_ref(&a) != 0) return 2;
  }
  // Algorithm 2's loop, both forms, with a position without mass
  for (int strong = 0; strong < 2; ++strong) {
    const int64_t S = 5, L = 3, K = 4, V = 333;
    std::vector<float> t((size_t)(S * (L + 1) * K * V));
    for (auto &v : t) v = 3.0f * g.normal();
    for (int64_t i = 0; i < K * V; ++i) t[(size_t)((L + 1) * K * V + i)] = -std::numeric_limits<float>::infinity();
    std::vector<int32_t> tok((size_t)(S * L * K)), Y((size_t)(S * (L + 1))), n((size_t)S);
    for (auto &v : tok) v = (int32_t)(g.next() * V);
    std::vector<uint8_t> active((size_t)(S * K));
    std::vector<double> key((size_t)(S * (L + 1))), gap((size_t)(S * (L + 1)));
    llc_verify_ref_args a;
    std::memset(&a, 0, sizeof(a));
    a.S = S; a.L = L; a.K = K; a.V = V; a.dtype = DT_F32; a.kind = KIND_LOGITS; a.target = t.data();
    a.stride_s = (L + 1) * K * V; a.stride_j = K * V; a.stride_k = V; a.temp_target = 0.7f;
    a.tokens = tok.data(); a.tok_stride_s = L * K; a.tok_stride_j = K;
    a.seed = 5; a.row_offset = 11; a.row_stride_s = L + 1; a.row_stride_j = 1; a.strong = strong;
    a.Y = Y.data(); a.n_out = n.data(); a.active = active.data(); a.key = key.data(); a.gap = gap.data(); a.threads = 2;
    for (int mf = 0; mf < 2; ++mf) {
      a.min_first = mf;
      if (llc_verify_ref(&a) != 0) return 2;
    }
  }
  std::puts("sanitizer run clean");
  return 0;
}
