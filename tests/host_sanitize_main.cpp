// Driver of the host-only sanitizer build (AddressSanitizer + UndefinedBehaviorSanitizer, CPU only): walks the
// library's host code -- argument validation and canonicalisation, the variant table, legality, workspace
// arithmetic, the compiled selector with its memo, the default dispatch, status strings -- and the C oracle over
// tight buffers, so that an out-of-bounds access, a signed overflow or a misaligned read anywhere in them ends the
// run.  Test infrastructure; built and run by tests/test_host_sanitizers.py.  No GPU runtime is linked.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "../paper_1806_07060_amd/csrc/mdg_host.h"

extern "C" {
int oracle_sgemm(int, int, int, int64_t, int64_t, int64_t, float, const float*, int64_t, const float*, int64_t, float, float*,
                 int64_t);
int oracle_sgemm_ijk(int, int, int, int64_t, int64_t, int64_t, float, const float*, int64_t, const float*, int64_t, float,
                     float*, int64_t);
int oracle_sgemm_elements(int, int, int, int64_t, int64_t, int64_t, float, const float*, int64_t, const float*, int64_t,
                          float, const float*, int64_t, int64_t, const int64_t*, const int64_t*, float*);
}

#define CHECK(cond)                                                     \
  do {                                                                  \
    if (!(cond)) {                                                      \
      std::fprintf(stderr, "%s:%d: check failed: %s\n", __FILE__, __LINE__, #cond); \
      return 1;                                                         \
    }                                                                   \
  } while (0)

static uint64_t rng_state = 0x9E3779B97F4A7C15ull;
static uint64_t rnd() {
  rng_state ^= rng_state << 13, rng_state ^= rng_state >> 7, rng_state ^= rng_state << 17;
  return rng_state;
}

int main() {
  using namespace mdg;
  const int n = mdg_variant_count();
  CHECK(n > 20);
  // ---- variant table, fallback chains, names
  for (int v = -2; v < n + 2; ++v) {
    mdg_variant_desc d;
    const int st = mdg_variant_info(v, &d);
    CHECK((st == MDG_OK) == (v >= 0 && v < n));
    if (st != MDG_OK) continue;
    CHECK(d.id == v && d.fallback >= 0 && d.fallback < n && std::strlen(d.name) > 0 && std::strlen(d.name) < sizeof(d.name));
    int x = v, hops = 0;
    while (x != 0 && hops <= n) {
      mdg_variant_desc e;
      CHECK(mdg_variant_info(x, &e) == MDG_OK);
      x = e.fallback, ++hops;
    }
    CHECK(x == 0);
  }
  CHECK(mdg_variant_info(0, nullptr) == MDG_ERR_NULL);
  // ---- selectors over ordinary, extreme and nonsensical sizes (products must saturate, not overflow)
  const int64_t sizes[] = {0, 1, 2, 3, 15, 16, 17, 31, 32, 33, 63, 64, 65, 127, 128, 129, 255, 256, 257, 1000, 4096, 8191,
                           8192, 50176, 65536, 1 << 20, (int64_t)MDG_MAX_DIM - 1, (int64_t)MDG_MAX_DIM};
  const int ns = (int)(sizeof(sizes) / sizeof(sizes[0]));
  long checked = 0;
  for (int a = 0; a < ns; ++a)
    for (int b = 0; b < ns; ++b)
      for (int c = 0; c < ns; ++c)
        for (int t = 0; t < 4; ++t) {
          const int v = mdg_select(t & 1, t >> 1, sizes[a], sizes[b], sizes[c]);
          CHECK(v >= 0 && v < n);
          CHECK(mdg_select_memo(t & 1, t >> 1, sizes[a], sizes[b], sizes[c]) == v);
          CHECK(mdg_select_memo(t & 1, t >> 1, sizes[a], sizes[b], sizes[c]) == v);  // and from the memo
          const int dv = mdg_select_default(t & 1, t >> 1, sizes[a], sizes[b], sizes[c]);
          CHECK(dv >= 0 && dv < n);
          ++checked;
        }
  for (int i = 0; i < 200000; ++i) {  // random shapes: more memo sets than entries, evictions included
    const int64_t M = 1 + (int64_t)(rnd() % 9000), N = 1 + (int64_t)(rnd() % 9000), K = 1 + (int64_t)(rnd() % 9000);
    const int t = (int)(rnd() & 3);
    CHECK(mdg_select_memo(t & 1, t >> 1, M, N, K) == mdg_select(t & 1, t >> 1, M, N, K));
  }
  // ---- legality and workspace arithmetic for every variant, with and without a registered workspace
  for (int pass = 0; pass < 3; ++pass) {
    if (pass == 0) CHECK(mdg_set_workspace(nullptr, 0) == MDG_OK);
    if (pass == 1) CHECK(mdg_set_workspace(reinterpret_cast<void*>(uintptr_t(1) << 20), size_t(1) << 20) == MDG_OK);
    if (pass == 2) CHECK(mdg_set_workspace(reinterpret_cast<void*>(uintptr_t(1) << 20), ~size_t(0)) == MDG_OK);
    for (int v = 0; v < n; ++v)
      for (int a = 0; a < ns; a += 2)
        for (int b = 1; b < ns; b += 3)
          for (int c = 0; c < ns; c += 2)
            for (int t = 0; t < 4; ++t) {
              const int64_t M = sizes[a], N = sizes[b], K = sizes[c];
              const int ok = mdg_variant_legal(v, t & 1, t >> 1, M, N, K, (t & 1) ? K : M, (t >> 1) ? N : K, M, nullptr,
                                               nullptr, nullptr);
              CHECK(ok == 0 || ok == 1);
              // variant 0 runs everything whose 64 x 64 tiles can be counted in 31 bits (anything that fits in memory)
              if (v == 0 && ((M + 63) / 64) * ((N + 63) / 64) <= 0x7fffffffLL) CHECK(ok == 1);
              (void)mdg_workspace_bytes(v, M, N, K);
            }
  }
  CHECK(mdg_set_workspace(reinterpret_cast<void*>(uintptr_t(4100)), 64) == MDG_ERR_ALIGNMENT);
  CHECK(mdg_set_workspace(nullptr, 0) == MDG_OK);
  CHECK(mdg_variant_legal(n, 0, 0, 1, 1, 1, 1, 1, 1, nullptr, nullptr, nullptr) == MDG_ERR_BAD_VARIANT);
  // ---- validation / canonicalisation: every argument position, both layouts
  {
    float a = 0, b = 0, c = 0;
    GemmArgs g;
    CHECK(canonicalise(MDG_COL_MAJOR, MDG_NO_TRANS, MDG_TRANS, 5, 6, 7, 1.f, &a, 5, &b, 6, 0.f, &c, 5, nullptr, nullptr, 0, &g) == MDG_OK);
    CHECK(g.tA == 0 && g.tB == 1 && g.M == 5 && g.N == 6 && g.K == 7 && g.lda == 5 && g.ldb == 6);
    CHECK(canonicalise(MDG_ROW_MAJOR, MDG_NO_TRANS, MDG_TRANS, 5, 6, 7, 1.f, &a, 7, &b, 7, 0.f, &c, 6, nullptr, nullptr, 0, &g) == MDG_OK);
    CHECK(g.tA == 1 && g.tB == 0 && g.M == 6 && g.N == 5 && g.A == &b && g.B == &a && g.lda == 7 && g.ldb == 7);
    CHECK(canonicalise(7, MDG_NO_TRANS, MDG_TRANS, 5, 6, 7, 1.f, &a, 5, &b, 6, 0.f, &c, 5, nullptr, nullptr, 0, &g) == -1);
    CHECK(canonicalise(MDG_COL_MAJOR, 0, MDG_TRANS, 5, 6, 7, 1.f, &a, 5, &b, 6, 0.f, &c, 5, nullptr, nullptr, 0, &g) == -2);
    CHECK(canonicalise(MDG_COL_MAJOR, MDG_NO_TRANS, 9, 5, 6, 7, 1.f, &a, 5, &b, 6, 0.f, &c, 5, nullptr, nullptr, 0, &g) == -3);
    CHECK(canonicalise(MDG_COL_MAJOR, MDG_NO_TRANS, MDG_TRANS, -1, 6, 7, 1.f, &a, 5, &b, 6, 0.f, &c, 5, nullptr, nullptr, 0, &g) == -4);
    CHECK(canonicalise(MDG_COL_MAJOR, MDG_NO_TRANS, MDG_TRANS, 5, (int64_t)MDG_MAX_DIM + 1, 7, 1.f, &a, 5, &b, (int64_t)MDG_MAX_DIM + 1, 0.f, &c, 5, nullptr, nullptr, 0, &g) == -5);
    CHECK(canonicalise(MDG_COL_MAJOR, MDG_NO_TRANS, MDG_TRANS, 5, 6, -7, 1.f, &a, 5, &b, 6, 0.f, &c, 5, nullptr, nullptr, 0, &g) == -6);
    CHECK(canonicalise(MDG_COL_MAJOR, MDG_NO_TRANS, MDG_TRANS, 5, 6, 7, 1.f, nullptr, 5, &b, 6, 0.f, &c, 5, nullptr, nullptr, 0, &g) == -8);
    CHECK(canonicalise(MDG_COL_MAJOR, MDG_NO_TRANS, MDG_TRANS, 5, 6, 7, 1.f, &a, 4, &b, 6, 0.f, &c, 5, nullptr, nullptr, 0, &g) == -9);
    CHECK(canonicalise(MDG_COL_MAJOR, MDG_NO_TRANS, MDG_TRANS, 5, 6, 7, 1.f, &a, 5, nullptr, 6, 0.f, &c, 5, nullptr, nullptr, 0, &g) == -10);
    CHECK(canonicalise(MDG_COL_MAJOR, MDG_NO_TRANS, MDG_TRANS, 5, 6, 7, 1.f, &a, 5, &b, 5, 0.f, &c, 5, nullptr, nullptr, 0, &g) == -11);
    CHECK(canonicalise(MDG_COL_MAJOR, MDG_NO_TRANS, MDG_TRANS, 5, 6, 7, 1.f, &a, 5, &b, 6, 0.f, nullptr, 5, nullptr, nullptr, 0, &g) == -13);
    CHECK(canonicalise(MDG_COL_MAJOR, MDG_NO_TRANS, MDG_TRANS, 5, 6, 7, 1.f, &a, 5, &b, 6, 0.f, &c, 4, nullptr, nullptr, 0, &g) == -14);
    CHECK(canonicalise(MDG_COL_MAJOR, MDG_NO_TRANS, MDG_TRANS, 5, 6, 7, 0.f, nullptr, 5, nullptr, 6, 0.f, &c, 5, nullptr, nullptr, 0, &g) == MDG_OK);  // alpha = 0: A, B unread
    // the variant a call would run, with and without workspace
    for (int t = 0; t < 4; ++t) {
      CHECK(canonicalise(MDG_COL_MAJOR, (t & 1) ? MDG_TRANS : MDG_NO_TRANS, (t >> 1) ? MDG_CONJ_TRANS : MDG_NO_TRANS, 300, 40,
                         5000, 1.f, &a, 5000, &b, 5000, 0.f, &c, 300, nullptr, nullptr, 0, &g) == MDG_OK);
      const int v0 = choose_variant(g, SEL_TREE), d0 = choose_variant(g, SEL_DEFAULT);
      CHECK(v0 >= 0 && v0 < n && d0 >= 0 && d0 < n && legal(variant_table(nullptr)[v0], g));
      g.ws = &c, g.ws_bytes = ~size_t(0);
      const int v1 = choose_variant(g, SEL_TREE);
      CHECK(v1 >= 0 && v1 < n && legal(variant_table(nullptr)[v1], g));
    }
  }
  for (int s = -120; s <= 1; ++s) CHECK(mdg_status_string(s) != nullptr && std::strlen(mdg_status_string(s)) > 0);
  CHECK(std::strlen(mdg_selector_name()) > 0);
  // ---- the oracle on tight buffers: every transpose, both layouts, padded and tight leading dimensions
  int cases = 0;
  for (int layout = 101; layout <= 102; ++layout)
    for (int t = 0; t < 4; ++t)
      for (int M = 0; M <= 9; M += 3)
        for (int N = 0; N <= 7; N += 7)
          for (int K = 0; K <= 5; K += 5)
            for (int pad = 0; pad <= 2; pad += 2) {
              const int tA = (t & 1) ? 112 : 111, tB = (t >> 1) ? 113 : 111;
              const bool col = layout == 102;
              const int a_rows = (t & 1) ? K : M, a_cols = (t & 1) ? M : K;
              const int b_rows = (t >> 1) ? N : K, b_cols = (t >> 1) ? K : N;
              const int64_t lda = (col ? a_rows : a_cols) + pad + (((col ? a_rows : a_cols) + pad) == 0);
              const int64_t ldb = (col ? b_rows : b_cols) + pad + (((col ? b_rows : b_cols) + pad) == 0);
              const int64_t ldc = (col ? M : N) + pad + (((col ? M : N) + pad) == 0);
              // buffers end exactly at the last logical element: reading a byte further is an error ASan reports
              auto len = [&](int rows, int cols, int64_t ld) -> size_t {
                const int outer = col ? cols : rows, inner = col ? rows : cols;
                return outer == 0 || inner == 0 ? 0 : (size_t)(ld * (outer - 1) + inner);
              };
              std::vector<float> A(len(a_rows, a_cols, lda)), B(len(b_rows, b_cols, ldb)), C(len(M, N, ldc)), C2, out;
              for (auto& x : A) x = (float)((int)(rnd() % 17) - 8);
              for (auto& x : B) x = (float)((int)(rnd() % 17) - 8);
              for (auto& x : C) x = (float)((int)(rnd() % 17) - 8);
              C2 = C;
              std::vector<float> C0 = C;
              CHECK(oracle_sgemm(layout, tA, tB, M, N, K, 1.5f, A.data(), lda, B.data(), ldb, -0.5f, C.data(), ldc) == 0);
              CHECK(oracle_sgemm_ijk(layout, tA, tB, M, N, K, 1.5f, A.data(), lda, B.data(), ldb, -0.5f, C2.data(), ldc) == 0);
              CHECK(C == C2);
              std::vector<int64_t> ii, jj;
              for (int i = 0; i < M; ++i)
                for (int j = 0; j < N; ++j) ii.push_back(i), jj.push_back(j);
              out.resize(ii.size());
              CHECK(oracle_sgemm_elements(layout, tA, tB, M, N, K, 1.5f, A.data(), lda, B.data(), ldb, -0.5f, C0.data(), ldc,
                                          (int64_t)ii.size(), ii.data(), jj.data(), out.data()) == 0);
              for (size_t e = 0; e < ii.size(); ++e)
                CHECK(out[e] == C[col ? ii[e] + jj[e] * ldc : ii[e] * ldc + jj[e]]);
              ++cases;
            }
  std::printf("ok: %d variants, %ld selector probes, %d oracle cases\n", n, checked, cases);
  return 0;
}
