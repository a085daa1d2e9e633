// Host-only driver that runs every oracle function on small inputs with the edge cases the tests care about
// (empty sequences, no nuggets, one token, NaN / infinite scores, rows that see nothing, both layouts, both
// element types), for a build with AddressSanitizer and UndefinedBehaviorSanitizer:
//   g++ -std=c++17 -O1 -g -fsanitize=address,undefined -fno-sanitize-recover=all -static-libasan sanitize_main.cpp
// Exit status 0 means no report.  TEST INFRASTRUCTURE, like the oracle itself.
#include "dodo_oracle.cpp"

#include <cstdio>

namespace {
uint64_t state = 0x9e3779b97f4a7c15ull;
double uniform() {  // small deterministic generator in (-1, 1)
  state ^= state << 13;
  state ^= state >> 7;
  state ^= state << 17;
  return static_cast<double>(state >> 11) / 9007199254740992.0 * 2.0 - 1.0;
}
std::vector<float> randf(size_t n) {
  std::vector<float> v(n);
  for (auto& x : v) x = static_cast<float>(uniform());
  return v;
}
std::vector<uint16_t> randbf(size_t n) {
  std::vector<uint16_t> v(n);
  for (auto& x : v) {
    const float f = static_cast<float>(uniform());
    uint32_t b;
    std::memcpy(&b, &f, 4);
    x = static_cast<uint16_t>(b >> 16);
  }
  return v;
}
std::vector<int32_t> cumulative(const std::vector<int32_t>& lens) {
  std::vector<int32_t> cu(lens.size() + 1, 0);
  for (size_t i = 0; i < lens.size(); ++i) cu[i + 1] = cu[i] + lens[i];
  return cu;
}

template <typename T>
void run(int dtype, std::vector<T> (*gen)(size_t)) {
  const int32_t H = 4, H_kv = 2, d_h = 8, d = 16;
  const std::vector<int32_t> n_lens = {9, 1, 0, 30}, q_lens = {3, 1, 0, 5}, tau = {2, 0, 0, 1};
  const int32_t B = static_cast<int32_t>(n_lens.size());
  std::vector<int32_t> k_lens, m_lens;
  for (int32_t b = 0; b < B; ++b) {
    k_lens.push_back(static_cast<int32_t>(oracle_nugget_count(n_lens[b], 1, 4)));
    m_lens.push_back(b == 3 ? 2 : q_lens[b] + tau[b]);  // the last text's local buffer is shorter than its query block
  }
  const auto cu_s = cumulative(n_lens), cu_k = cumulative(k_lens), cu_q = cumulative(q_lens), cu_m = cumulative(m_lens);
  const int64_t N = cu_s[B], Kt = cu_k[B], Sq = cu_q[B], Sm = cu_m[B];
  auto hidden = gen(N * d), w = gen(d), K = gen(N * H_kv * d_h), V = gen(N * H_kv * d_h);
  std::vector<float> scores(N);
  oracle_score(hidden.data(), w.data(), 0.25f, dtype, N, d, d, scores.data());
  auto W1 = gen(12 * d), w2 = gen(12);
  std::vector<float> b1 = randf(12), s2(N);
  for (int act = 0; act < 3; ++act)
    oracle_score_mlp(hidden.data(), W1.data(), b1.data(), w2.data(), 0.5f, act, dtype, N, d, 12, d, s2.data());
  scores[2] = std::numeric_limits<float>::quiet_NaN();
  scores[4] = std::numeric_limits<float>::infinity();
  scores[5] = -std::numeric_limits<float>::infinity();
  scores[6] = -0.0f;
  std::vector<int32_t> idx(Kt);
  for (uint32_t flags = 0; flags < 2; ++flags)
    if (oracle_select_topk(scores.data(), cu_s.data(), cu_k.data(), B, flags, idx.data()) != 0) std::abort();
  std::vector<uint8_t> alpha(N);
  std::vector<int32_t> counts(B), cu_t(B + 1), idx_t(N);
  const float lam = oracle_threshold_from_sample(scores.data(), N, 1, 4);
  oracle_select_threshold(scores.data(), cu_s.data(), B, lam, alpha.data(), counts.data());
  oracle_select_threshold_indices(scores.data(), cu_s.data(), B, lam, counts.data(), cu_t.data(), idx_t.data());
  for (int layout = 0; layout < 2; ++layout) {
    std::vector<T> Kn(Kt * H_kv * d_h), Vn(Kt * H_kv * d_h), Kp(Kt * H_kv * d_h), Vp(Kt * H_kv * d_h);
    oracle_gather(K.data(), V.data(), dtype, idx.data(), cu_s.data(), cu_k.data(), B, Kt, H_kv, d_h, H_kv * d_h, Kn.data(),
                  Vn.data(), layout);
    oracle_meanpool(K.data(), V.data(), dtype, cu_s.data(), cu_k.data(), B, Kt, H_kv, d_h, H_kv * d_h, Kp.data(), Vp.data(),
                    layout);
    auto Q = gen(Sq * H * d_h), Kl = gen(Sm * H_kv * d_h), Vl = gen(Sm * H_kv * d_h), dO = gen(Sq * H * d_h);
    std::vector<double> O(Sq * H * d_h), lse(Sq * H);
    oracle_attention(Q.data(), Kn.data(), Vn.data(), Kl.data(), Vl.data(), cu_q.data(), cu_k.data(), cu_m.data(), B, H, H_kv,
                     d_h, 0.35, dtype, layout, Kt, O.data(), lse.data());
    const int32_t rb[2] = {0, 3}, rh[2] = {1, 3}, ri[2] = {2, 0};
    std::vector<double> Or(2 * d_h), lr(2);
    oracle_attention_rows(Q.data(), Kn.data(), Vn.data(), Kl.data(), Vl.data(), cu_q.data(), cu_k.data(), cu_m.data(), H,
                          H_kv, d_h, 0.35, dtype, layout, Kt, 2, rb, rh, ri, Or.data(), lr.data());
    if (layout == 0) {
      std::vector<double> grad(Kt);
      oracle_ste_score_grad(Q.data(), Kn.data(), Vn.data(), Kl.data(), Vl.data(), dO.data(), cu_q.data(), cu_k.data(),
                            cu_m.data(), B, H, H_kv, d_h, 0.35, 0.35, dtype, Kt, grad.data());
      // segment form: every token of the texts is a query row
      auto Qs = gen(N * H * d_h);
      std::vector<double> Os(N * H * d_h), ls(N * H);
      oracle_attention_segment_mask(Qs.data(), Kn.data(), Vn.data(), K.data(), V.data(), idx.data(), cu_s.data(), cu_k.data(),
                                    B, H, H_kv, d_h, 4, 3, 0.35, dtype, Os.data(), ls.data());
      int64_t E = 0;
      for (int32_t b = 0; b < B; ++b) E += (n_lens[b] + 3) / 4;
      std::vector<int32_t> scq(E + 1), ns(E), nl(E), lo(E), ll(E);
      if (oracle_segment_plan(idx.data(), cu_s.data(), cu_k.data(), B, 4, 3, E, scq.data(), ns.data(), nl.data(), lo.data(),
                              ll.data()) != E)
        std::abort();
    }
  }
  // one decode step of the autoregressive mode on caches with room for two rows per sequence
  auto Kr = gen(B * H_kv * d_h), Vr = gen(B * H_kv * d_h);
  std::vector<T> Kc(B * 2 * H_kv * d_h), Vc(B * 2 * H_kv * d_h);
  std::vector<int32_t> cnt = {0, 2, 1, 0};
  std::vector<float> sc = {1.f, 1.f, -1.f, std::numeric_limits<float>::quiet_NaN()};
  oracle_stream_append(sc.data(), 0.f, Kr.data(), Vr.data(), dtype, B, H_kv, d_h, H_kv * d_h, 2, cnt.data(), Kc.data(),
                       Vc.data());
}
}  // namespace

int main() {
  run<float>(kF32, randf);
  run<uint16_t>(kBF16, randbf);
  std::puts("oracle sanitizer driver: ok");
  return 0;
}
