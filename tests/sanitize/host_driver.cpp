// Sanitizer driver for the host-side code: built by tests/test_host_sanitizers.py with
// -fsanitize=address,undefined together with oracle/tva_oracle.c (the CPU oracle) and
// paper_2510_26577_amd/csrc/cast.cpp (the tree-size selection and the host mask builder), and run once.
// Every buffer is a heap allocation of exactly the documented size, so a read or write one element past
// it is a sanitizer report; a few results are cross-checked so that the calls cannot be optimised away
// and the run also fails on a wrong answer.  Exit status 0 = clean.
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <memory>
#include <vector>

#include "tva.h"
#include "tva_cast.h"

extern "C" {
// the oracle's C interface (oracle/tva_oracle.c; it has no header of its own: tests bind it by name)
typedef struct {
  int32_t B, Hq, Hkv, D;
  double scale;
  const int32_t *cu_T, *L, *parent;
  const uint16_t *q, *k_tree, *v_tree, *k_cache, *v_cache;
  const int32_t *cu_L, *page_table;
  int32_t page_size, max_pages;
  int64_t key_lo, key_hi;
} tvo_problem;
int64_t tvo_ancestor_mask(const int32_t *parent, const int32_t *cu_T, int32_t B, int32_t W, uint64_t *mask);
int tvo_attention(const tvo_problem *p, double *out, double *lse);
int tvo_attention_rows(const tvo_problem *p, const int32_t *rows, int64_t n, double *out, double *lse);
void tvo_set_num_threads(int n);
}

static int failures = 0;
#define CHECK(cond) do { if (!(cond)) { std::fprintf(stderr, "CHECK failed line %d: %s\n", __LINE__, #cond); ++failures; } } while (0)

template <typename T>
static std::unique_ptr<T[]> exact(size_t n) { return std::unique_ptr<T[]>(new T[n ? n : 1]); }

static uint64_t rng_state = 0x2510265770001ull;
static uint32_t rnd() {  // xorshift64*
  rng_state ^= rng_state >> 12; rng_state ^= rng_state << 25; rng_state ^= rng_state >> 27;
  return (uint32_t)((rng_state * 0x2545F4914F6CDD1Dull) >> 32);
}
static uint16_t rnd_bf16() {  // a finite bf16 of modest size
  const float f = ((int)(rnd() % 2001) - 1000) / 500.0f;
  uint32_t u; std::memcpy(&u, &f, 4);
  return (uint16_t)(u >> 16);
}

static void masks_and_attention() {
  // three trees: 128 nodes (two mask words), a forest of 70, a single node; ragged caches incl. an empty one
  const int B = 3, Hq = 4, Hkv = 2, D = 64, page = 16;
  const int T[B] = {128, 70, 1}, L[B] = {37, 0, 65};
  auto cu_T = exact<int32_t>(B + 1), cu_L = exact<int32_t>(B + 1), Lb = exact<int32_t>(B);
  cu_T[0] = cu_L[0] = 0;
  for (int b = 0; b < B; ++b) cu_T[b + 1] = cu_T[b] + T[b], cu_L[b + 1] = cu_L[b] + L[b], Lb[b] = L[b];
  const int sum_T = cu_T[B], sum_L = cu_L[B];
  auto parent = exact<int32_t>(sum_T);
  for (int b = 0; b < B; ++b)
    for (int i = 0; i < T[b]; ++i) parent[cu_T[b] + i] = i == 0 ? -1 : (int32_t)(rnd() % i);
  parent[cu_T[1] + 17] = parent[cu_T[1] + 40] = -1;  // several roots
  const int W = 2;
  auto m_oracle = exact<uint64_t>((size_t)sum_T * W), m_host = exact<uint64_t>((size_t)sum_T * W);
  CHECK(tvo_ancestor_mask(parent.get(), cu_T.get(), B, W, m_oracle.get()) == 0);
  int32_t bad = -7;
  CHECK(tva_build_ancestor_mask_host(parent.get(), cu_T.get(), B, 128, W, m_host.get(), &bad) == TVA_OK);
  CHECK(std::memcmp(m_oracle.get(), m_host.get(), sizeof(uint64_t) * sum_T * W) == 0);
  // a malformed tree is reported, by both
  const int32_t keep = parent[cu_T[1] + 5];
  parent[cu_T[1] + 5] = 9;
  CHECK(tvo_ancestor_mask(parent.get(), cu_T.get(), B, W, m_oracle.get()) == cu_T[1] + 5 + 1);
  CHECK(tva_build_ancestor_mask_host(parent.get(), cu_T.get(), B, 128, W, m_host.get(), &bad) == TVA_BAD_TREE && bad == cu_T[1] + 5);
  parent[cu_T[1] + 5] = keep;

  auto q = exact<uint16_t>((size_t)sum_T * Hq * D), kt = exact<uint16_t>((size_t)sum_T * Hkv * D), vt = exact<uint16_t>((size_t)sum_T * Hkv * D);
  auto kc = exact<uint16_t>((size_t)sum_L * Hkv * D), vc = exact<uint16_t>((size_t)sum_L * Hkv * D);
  for (size_t i = 0; i < (size_t)sum_T * Hq * D; ++i) q[i] = rnd_bf16();
  for (size_t i = 0; i < (size_t)sum_T * Hkv * D; ++i) kt[i] = rnd_bf16(), vt[i] = rnd_bf16();
  for (size_t i = 0; i < (size_t)sum_L * Hkv * D; ++i) kc[i] = rnd_bf16(), vc[i] = rnd_bf16();
  tvo_problem p{};
  p.B = B, p.Hq = Hq, p.Hkv = Hkv, p.D = D, p.scale = 0.125;
  p.cu_T = cu_T.get(), p.L = Lb.get(), p.parent = parent.get();
  p.q = q.get(), p.k_tree = kt.get(), p.v_tree = vt.get(), p.k_cache = kc.get(), p.v_cache = vc.get();
  p.cu_L = cu_L.get(), p.page_table = nullptr, p.key_lo = 0, p.key_hi = -1;
  tvo_set_num_threads(2);
  auto out = exact<double>((size_t)sum_T * Hq * D), lse = exact<double>((size_t)sum_T * Hq);
  CHECK(tvo_attention(&p, out.get(), lse.get()) == 0);
  for (size_t i = 0; i < (size_t)sum_T * Hq; ++i) CHECK(std::isfinite(lse[i]));
  // the single-node tree with 65 cached keys: lse of the zero-score case is ln(66) when q = 0 (checked in pytest);
  // here: sampled rows equal the full computation
  const int n_rows = 5;
  auto rows = exact<int32_t>(3 * n_rows);
  const int32_t pick[n_rows][3] = {{0, 0, 0}, {0, 127, 3}, {1, 69, 1}, {2, 0, 2}, {1, 17, 0}};
  std::memcpy(rows.get(), pick, sizeof(pick));
  auto ro = exact<double>((size_t)n_rows * D), rl = exact<double>(n_rows);
  CHECK(tvo_attention_rows(&p, rows.get(), n_rows, ro.get(), rl.get()) == 0);
  for (int r = 0; r < n_rows; ++r) {
    const size_t g = ((size_t)cu_T[pick[r][0]] + pick[r][1]) * Hq + pick[r][2];
    CHECK(rl[r] == lse[g]);
    CHECK(std::memcmp(ro.get() + (size_t)r * D, out.get() + g * D, sizeof(double) * D) == 0);
  }
  // the same cache scattered into 16-token pages, table rows of exactly the pages each sequence needs at most
  int max_pages = 0;
  for (int b = 0; b < B; ++b) max_pages = std::max(max_pages, (L[b] + page - 1) / page);
  int n_pages = 0;
  auto table = exact<int32_t>((size_t)B * max_pages);
  for (int b = 0; b < B; ++b)
    for (int j = 0; j < max_pages; ++j) table[b * max_pages + j] = j < (L[b] + page - 1) / page ? n_pages++ : 0;
  auto kp = exact<uint16_t>((size_t)n_pages * page * Hkv * D), vp = exact<uint16_t>((size_t)n_pages * page * Hkv * D);
  std::memset(kp.get(), 0x7f, sizeof(uint16_t) * n_pages * page * Hkv * D);  // tails hold NaN patterns: never read
  std::memset(vp.get(), 0x7f, sizeof(uint16_t) * n_pages * page * Hkv * D);
  for (int b = 0; b < B; ++b)
    for (int t = 0; t < L[b]; ++t) {
      const size_t dst = ((size_t)table[b * max_pages + t / page] * page + t % page) * Hkv * D, src = ((size_t)cu_L[b] + t) * Hkv * D;
      std::memcpy(kp.get() + dst, kc.get() + src, sizeof(uint16_t) * Hkv * D);
      std::memcpy(vp.get() + dst, vc.get() + src, sizeof(uint16_t) * Hkv * D);
    }
  p.k_cache = kp.get(), p.v_cache = vp.get(), p.cu_L = nullptr, p.page_table = table.get(), p.page_size = page, p.max_pages = max_pages;
  auto out2 = exact<double>((size_t)sum_T * Hq * D), lse2 = exact<double>((size_t)sum_T * Hq);
  CHECK(tvo_attention(&p, out2.get(), lse2.get()) == 0);
  CHECK(std::memcmp(out.get(), out2.get(), sizeof(double) * sum_T * Hq * D) == 0);
  CHECK(std::memcmp(lse.get(), lse2.get(), sizeof(double) * sum_T * Hq) == 0);
}

static void tree_size_selection() {
  // the hand-worked two-step case of tests/cast_cases.py, every buffer at its documented size
  const int L = 4, M = 3, N = 4, n0 = 2, R = 2;
  const double C1 = 0.24, C2 = 0.48;
  auto S_D = exact<double>(M * N), S_T = exact<double>(M * N);
  const double st0[3] = {1.0, 2.0, 4.0};
  for (int r = 0; r < M; ++r)
    for (int k = 0; k < N; ++k) S_D[r * N + k] = k + 1.0, S_T[r * N + k] = st0[r] + 0.5 * k;
  const float step1[3][4] = {{0.8f, 0.4f, 0.3f, 0.1f}, {0.5f, 0.25f, 0.125f, 0.1f}, {0.6f, 0.2f, 0.04f, 0.02f}};
  const float step2[3][4] = {{0.9f, 0.6f, 0.5f, 0.1f}, {0.3f, 0.19f, 0.01f, 0.01f}, {0.6f, 0.2f, 0.04f, 0.02f}};
  auto N_i = exact<int32_t>(3);
  N_i[0] = N_i[1] = N_i[2] = N;
  const int max_layers = 3;
  const size_t state_bytes = tva_cast_depth_bytes(max_layers, R);
  CHECK(state_bytes > 0);
  auto state = exact<double>((state_bytes + 7) / 8);  // exactly the bytes asked for, 8-byte aligned
  CHECK(tva_cast_depth_init(state.get(), max_layers, R, C2) == TVA_OK);
  auto kept = exact<int32_t>(3);
  auto work = exact<double>(2 * N);
  auto flat = exact<float>(3 * N);
  std::memcpy(flat.get(), step1, sizeof(step1));
  CHECK(tva_cast_expansion_plan(flat.get(), N_i.get(), 3, 1, S_D.get(), S_T.get(), M, N, L, n0, C1, state.get(), kept.get(), work.get()) == 3);
  CHECK(kept[0] == 3 && kept[1] == 3 && kept[2] == 2);
  CHECK(std::fabs(tva_cast_depth_alpha(state.get(), 1) - 19.0 / 24.0) < 1e-6);
  std::memcpy(flat.get(), step2, sizeof(step2));
  CHECK(tva_cast_expansion_plan(flat.get(), N_i.get(), 3, 1, S_D.get(), S_T.get(), M, N, L, n0, C1, state.get(), kept.get(), work.get()) == 2);
  CHECK(kept[0] == 3 && kept[1] == 2);
  // the buffers: many updates of every layer (the FIFO wraps many times), alpha stays a mean of R values
  for (int it = 0; it < 1000; ++it) {
    const int layer = 1 + (int)(rnd() % max_layers);
    tva_cast_depth_update(state.get(), layer, 0.5 + (rnd() % 100) / 100.0, 1.0);
    const double a = tva_cast_depth_alpha(state.get(), layer);
    CHECK(a >= 0.5 - 1e-12 && a <= 1.5 + 1e-12);
  }
  CHECK(std::isnan(tva_cast_depth_alpha(state.get(), max_layers + 1)));
  // Algorithm 1, Eq. 1, Eq. 2 on their own, buffers of exactly n
  auto u = exact<double>(N), c = exact<double>(N);
  CHECK(tva_cast_layer_utility(flat.get(), 1, N, u.get()) == TVA_OK);
  CHECK(tva_cast_layer_cost(S_D.get(), S_T.get(), M, N, L, 5, N, c.get()) == TVA_OK);
  CHECK(tva_cast_select_max_valid_index(u.get(), c.get(), N, C1) == 3);  // (.9 .6 .5 .1 against costs .5 1 1.5 2: only the chord 3 -> 4 is flat)
  c[2] = c[1];  // not strictly increasing: refused, nothing read past the end
  CHECK(tva_cast_select_max_valid_index(u.get(), c.get(), N, C1) < 0);
  // reranking count and subtree selection
  const int B = 3, N_tot = 23, m = 10;
  auto tree = exact<float>(B * N_tot);
  for (int i = 0; i < B * N_tot; ++i) tree[i] = (rnd() % 1000) / 1000.0f;
  const int N_table = 12;
  auto S_T2 = exact<double>(M * N_table);
  for (int r = 0; r < M; ++r)
    for (int k = 0; k < N_table; ++k) S_T2[r * N_table + k] = 10.0 + r + 0.7 * k;
  auto work2 = exact<double>(B * N_tot + 2 * std::min(N_tot, m));
  const int32_t cnt = tva_cast_rerank_count(tree.get(), B, N_tot, S_T2.get(), M, N_table, L, 7, m, 3.0, work2.get());
  CHECK(cnt >= 1 && cnt <= m);
  const int n = 40, keepn = 17;
  auto score = exact<float>(n);
  auto par = exact<int32_t>(n);
  par[0] = -1, score[0] = 1.f;
  for (int i = 1; i < n; ++i) par[i] = (int32_t)(rnd() % i), score[i] = score[par[i]] * (0.3f + (rnd() % 60) / 100.0f);
  auto old_index = exact<int32_t>(keepn), new_parent = exact<int32_t>(keepn), work3 = exact<int32_t>(n);
  CHECK(tva_cast_select_subtree(score.get(), par.get(), n, keepn, old_index.get(), new_parent.get(), work3.get()) == TVA_OK);
  for (int k = 0; k < keepn; ++k) CHECK(new_parent[k] < k && (k == 0 || old_index[k] > old_index[k - 1]));
}

int main() {
  masks_and_attention();
  tree_size_selection();
  std::printf("host sanitizer driver: %d failure(s)\n", failures);
  return failures ? 1 : 0;
}
