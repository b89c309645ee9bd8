// Drives the CPU oracle through its whole C interface on seeded synthetic inputs; built with
// -fsanitize=address,undefined by tests/test_sanitizers.py (CPU only).  Exit status 0 = no finding
// (the sanitizers abort the process on one).  Checks no values: the pins in tests/test_oracle_*.py do that.
#include "../../oracle/c2t_oracle.cpp"

#include <cstdio>
#include <random>

static uint16_t to_bf16(float f) {
  uint32_t u; std::memcpy(&u, &f, 4);
  if ((u & 0x7f800000u) == 0x7f800000u) return (uint16_t)(u >> 16);      // inf / nan as they are
  u += 0x7fffu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

int main() {
  std::mt19937 rng(12345);
  std::normal_distribution<float> g(0.f, 2.f);
  const float inf = std::numeric_limits<float>::infinity();
  long checks = 0;
  for (int dtype = 0; dtype < 2; ++dtype) {
    for (int trial = 0; trial < 6; ++trial) {
      const int B = 1 + trial % 3, V = trial == 0 ? 1 : 5 + 37 * trial, F = 1 + trial % 4, K = std::min(V, 1 + (trial * 2) % 5),
                D = 1 + trial % 4, N = 1 + 3 * trial, h = 1 + trial;
      const int stride = V + (trial % 2 ? 3 : 0);
      void* t = c2t_ref_create(B, V, F, K, D, N, h, dtype, trial % 2 ? 0.0f : 0.4f);
      if (!t) return 2;
      std::vector<float> W1(3 * h), b1(h), w2(h);
      for (auto& x : W1) x = 0.3f * g(rng);
      for (auto& x : b1) x = 0.3f * g(rng);
      for (auto& x : w2) x = 0.3f * g(rng);
      c2t_ref_set_classifier(t, W1.data(), b1.data(), w2.data(), 0.7f);
      if (trial % 3 == 2) c2t_ref_set_entropy_top_m(t, 1 + trial);
      for (int round = 0; round < 2; ++round) {
        c2t_ref_reset(t);
        for (int l = 0; l < D; ++l) {
          std::vector<float> x((size_t)B * F * stride);
          for (auto& v : x) v = g(rng);
          if (trial == 3) x[0] = -inf;                              // masked logit
          if (trial == 4 && l == 1) x[1] = std::nanf("");           // bad row
          if (trial == 5) for (size_t i = 0; i < x.size(); i += 2) x[i] = 1.5f;   // ties
          int rc;
          if (dtype == DT_BF16) {
            std::vector<uint16_t> xb(x.size());
            for (size_t i = 0; i < x.size(); ++i) xb[i] = to_bf16(x[i]);
            rc = c2t_ref_expand_layer(t, xb.data(), stride);
          } else {
            rc = c2t_ref_expand_layer_range(t, x.data(), stride, 0, B);
            c2t_ref_end_layer(t);
          }
          if (rc) return 3;
          std::vector<int32_t> tok((size_t)B * F), slot((size_t)B * F), nf(B);
          c2t_ref_get_frontier(t, tok.data(), slot.data(), nf.data());
          const size_t FK = (size_t)F * K;
          std::vector<int32_t> nc(B), ct(B * FK), cs(B * FK), kept(B * FK);
          std::vector<float> p(B * FK), P(B * FK), H(B * FK), z(B * FK);
          c2t_ref_get_candidates(t, nc.data(), ct.data(), cs.data(), p.data(), P.data(), H.data(), z.data(), kept.data());
          checks += nc[0];
        }
        if (c2t_ref_layer(t) != D) return 4;
        if (c2t_ref_expand_layer(t, nullptr, stride) == 0) return 5;   // beyond max_depth: refused before anything is read
        std::vector<double> a(B), gp(B); std::vector<int64_t> sc(B);
        c2t_ref_get_audit(t, a.data(), gp.data(), sc.data());
        std::vector<int32_t> tokens((size_t)B * N), parent((size_t)B * N), pos((size_t)B * N), nn(B);
        std::vector<float> conf((size_t)B * N), jp((size_t)B * N), ent((size_t)B * N), ex1((size_t)B * N), ex2((size_t)B * N);
        std::vector<uint8_t> mask((size_t)B * N * N); std::vector<uint32_t> st(B);
        c2t_ref_finalize(t, tokens.data(), parent.data(), pos.data(), conf.data(), jp.data(), ent.data(), nn.data(), mask.data(), st.data());
        c2t_ref_get_node_extras(t, ex1.data(), ex2.data());
        for (int n_out : {1, 3, (int)sc[0] + 2}) {
          std::vector<int32_t> rt((size_t)B * n_out), rp((size_t)B * n_out), rq((size_t)B * n_out), rn(B);
          std::vector<float> rc1((size_t)B * n_out), rc2((size_t)B * n_out), rc3((size_t)B * n_out), rc4((size_t)B * n_out);
          std::vector<uint8_t> rm((size_t)B * n_out * n_out); std::vector<uint32_t> rs(B);
          c2t_ref_finalize_rerank(t, n_out, rt.data(), rp.data(), rq.data(), rc1.data(), rc2.data(), rc3.data(), rc4.data(), rn.data(), rm.data(), rs.data());
          checks += rn[0];
        }
      }
      c2t_ref_destroy(t);
    }
  }
  // single-row entry points
  for (int V : {1, 2, 33}) {
    std::vector<float> row(V);
    for (auto& v : row) v = g(rng);
    double m, Z, S, H; std::vector<int32_t> ids(V); std::vector<double> xs(V), ps(V);
    if (c2t_ref_row(row.data(), DT_F32, V, V, &m, &Z, &S, &H, ids.data(), xs.data(), ps.data())) return 6;
    (void)c2t_ref_entropy_top_m(row.data(), DT_F32, V, 1);
    (void)c2t_ref_entropy_top_m(row.data(), DT_F32, V, V + 5);
    row[0] = inf;
    if (!c2t_ref_row(row.data(), DT_F32, V, 1, &m, &Z, &S, &H, ids.data(), nullptr, nullptr)) return 7;
  }
  (void)c2t_ref_mlp_logit(0, nullptr, nullptr, nullptr, 0.5f, 0.1f, 1.f, 2.f);
  (void)c2t_ref_logit_of_beta(0.f); (void)c2t_ref_logit_of_beta(0.999f);
  if (c2t_ref_create(0, 1, 1, 1, 1, 1, 1, 0, 0.5f) || c2t_ref_create(1, 1, 1, 1, 1, 1, 1, 0, 1.0f) || c2t_ref_create(1, 1, 1, 1, 1, 1, 1, 5, 0.5f)) return 8;
  std::printf("oracle driver ok (%ld)\n", checks);
  return 0;
}
