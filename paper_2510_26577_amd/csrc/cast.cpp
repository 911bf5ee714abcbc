// Host part of libtva: the cost-aware choice of draft-tree sizes (paper, section "Method";
// declared in include/tva_cast.h) and the host variant of the ancestor-mask builder with its
// synchronous tree validation (include/tva.h).  Plain C++ on host memory; the caller owns every
// buffer.
#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstring>
#include <limits>

#include "tva.h"
#include "tva_cast.h"

namespace {

// State block of the depth-pruning buffers: a header, then per layer a ring of R values.
struct DepthHeader {
  int32_t max_layers, R;
  double C2;
};
struct DepthRing {
  int32_t count, head;  // values held, position of the oldest
};
inline size_t ring_stride(int32_t R) { return sizeof(DepthRing) + sizeof(double) * (size_t)R; }
inline DepthRing *ring_of(void *state, int32_t layer) {
  auto *h = static_cast<DepthHeader *>(state);
  return reinterpret_cast<DepthRing *>(static_cast<char *>(state) + sizeof(DepthHeader) + ring_stride(h->R) * (size_t)(layer - 1));
}
inline double *values_of(DepthRing *r) { return reinterpret_cast<double *>(r + 1); }
inline bool layer_ok(const void *state, int32_t layer) {
  return state && layer >= 1 && layer <= static_cast<const DepthHeader *>(state)->max_layers;
}

inline int32_t table_row(int32_t c, int32_t L, int32_t M) { return std::min(c / L, M - 1); }  // 0-based

}  // namespace

extern "C" {

// Host variant of the ancestor-mask builder: one pass per tree, a node's mask is its own bit OR its
// parent's mask (parents come first in the order the interface requires).
int tva_build_ancestor_mask_host(const int32_t *parent, const int32_t *cu_T, int32_t B, int32_t max_T,
                                 int32_t mask_words, uint64_t *mask, int32_t *bad_node) {
  if (B < 0 || max_T < 0 || mask_words < 1 || (int64_t)mask_words * 64 < max_T) return TVA_INVALID_ARG;
  if (B == 0) return TVA_OK;
  if (!parent || !cu_T || !mask) return TVA_INVALID_ARG;
  for (int32_t b = 0; b < B; ++b) {
    const int32_t t0 = cu_T[b], T = cu_T[b + 1] - t0;
    if (T < 0 || T > (int64_t)mask_words * 64) return TVA_INVALID_ARG;
    for (int32_t i = 0; i < T; ++i) {
      const int32_t p = parent[t0 + i];
      if (p < -1 || p >= i) {
        if (bad_node) *bad_node = t0 + i;
        return TVA_BAD_TREE;
      }
      uint64_t *row = mask + (size_t)(t0 + i) * mask_words;
      if (p < 0) std::memset(row, 0, sizeof(uint64_t) * mask_words);
      else std::memcpy(row, mask + (size_t)(t0 + p) * mask_words, sizeof(uint64_t) * mask_words);
      row[i / 64] |= 1ull << (i % 64);
    }
  }
  return TVA_OK;
}

int32_t tva_cast_select_context(int32_t c, int32_t L, int32_t M) {
  if (c < 0 || L < 1 || M < 1) return TVA_INVALID_ARG;
  return (table_row(c, L, M) + 1) * L;
}

// Algorithm 1.  Index j survives iff the smallest chord from any earlier point reaches C, so one
// pass per j with an early exit does the marking of the printed double loop.
int32_t tva_cast_select_max_valid_index(const double *u, const double *c, int32_t n, double C) {
  if (!u || !c || n < 1) return TVA_INVALID_ARG;
  for (int32_t j = 1; j < n; ++j)
    if (!(c[j] > c[j - 1])) return TVA_INVALID_ARG;
  for (int32_t j = n - 1; j >= 1; --j) {
    bool valid = true;
    for (int32_t i = 0; i < j && valid; ++i) valid = !((u[j] - u[i]) / (c[j] - c[i]) < C);
    if (valid) return j + 1;
  }
  return 1;
}

// Eq. 1 through per-rank column sums: u_k = u_{k-1} + mean over samples of their k-th best score.
int tva_cast_layer_utility(const float *scores, int32_t B, int32_t N, double *u) {
  if (!scores || !u || B < 1 || N < 1) return TVA_INVALID_ARG;
  double run = 0.0;
  for (int32_t s = 0; s < N; ++s) {
    double col = 0.0;
    for (int32_t j = 0; j < B; ++j) col += (double)scores[(size_t)j * N + s];
    run += col;
    u[s] = run / B;
  }
  return TVA_OK;
}

int tva_cast_layer_cost(const double *S_D, const double *S_T, int32_t M, int32_t N_table, int32_t L, int32_t ctx,
                        int32_t n_candidates, double *c) {
  if (!S_D || !S_T || !c || M < 1 || N_table < 1 || L < 1 || ctx < 0 || n_candidates < 1 || n_candidates > N_table)
    return TVA_INVALID_ARG;
  const size_t row = (size_t)table_row(ctx, L, M) * N_table;
  const double target_one = S_T[row];
  for (int32_t k = 0; k < n_candidates; ++k) c[k] = S_D[row + k] / target_one;
  return TVA_OK;
}

int32_t tva_cast_breadth_prune(const float *scores, int32_t B, int32_t N, const double *S_D, const double *S_T,
                               int32_t M, int32_t N_table, int32_t L, int32_t ctx, double C1, double *u_at,
                               double *c_at, double *work) {
  if (!work) return TVA_INVALID_ARG;
  double *u = work, *c = work + N;
  int rc = tva_cast_layer_utility(scores, B, N, u);
  if (rc != TVA_OK) return rc;
  rc = tva_cast_layer_cost(S_D, S_T, M, N_table, L, ctx, N, c);
  if (rc != TVA_OK) return rc;
  const int32_t n_i = tva_cast_select_max_valid_index(u, c, N, C1);
  if (n_i < 1) return n_i;
  if (u_at) *u_at = u[n_i - 1];
  if (c_at) *c_at = c[n_i - 1];
  return n_i;
}

size_t tva_cast_depth_bytes(int32_t max_layers, int32_t R) {
  if (max_layers < 1 || R < 1) return 0;
  return sizeof(DepthHeader) + ring_stride(R) * (size_t)max_layers;
}

int tva_cast_depth_init(void *state, int32_t max_layers, int32_t R, double C2) {
  if (!state || max_layers < 1 || R < 1 || (reinterpret_cast<uintptr_t>(state) & 7)) return TVA_INVALID_ARG;
  auto *h = static_cast<DepthHeader *>(state);
  h->max_layers = max_layers;
  h->R = R;
  h->C2 = C2;
  for (int32_t i = 1; i <= max_layers; ++i) {
    DepthRing *r = ring_of(state, i);
    r->count = 1;
    r->head = 0;
    values_of(r)[0] = 1.0;  // every buffer starts as {1}
  }
  return TVA_OK;
}

double tva_cast_depth_alpha(const void *state, int32_t layer) {
  if (!layer_ok(state, layer)) return std::numeric_limits<double>::quiet_NaN();
  DepthRing *r = ring_of(const_cast<void *>(state), layer);
  const int32_t R = static_cast<const DepthHeader *>(state)->R;
  double sum = 0.0;
  for (int32_t k = 0; k < r->count; ++k) sum += values_of(r)[(r->head + k) % R];  // oldest first
  return sum / r->count;
}

int tva_cast_depth_should_expand(const void *state, int32_t layer, double u_ni, double c_ni) {
  if (!layer_ok(state, layer)) return TVA_INVALID_ARG;
  return tva_cast_depth_alpha(state, layer) * u_ni / c_ni >= static_cast<const DepthHeader *>(state)->C2 ? 1 : 0;
}

double tva_cast_depth_update(void *state, int32_t layer, double u_next, double u_cur) {
  if (!layer_ok(state, layer)) return std::numeric_limits<double>::quiet_NaN();
  DepthRing *r = ring_of(state, layer);
  const int32_t R = static_cast<DepthHeader *>(state)->R;
  const double phi = u_next / u_cur;
  if (r->count < R) {
    values_of(r)[(r->head + r->count) % R] = phi;
    ++r->count;
  } else {  // full: the new value takes the oldest one's place
    values_of(r)[r->head] = phi;
    r->head = (r->head + 1) % R;
  }
  return phi;
}

int32_t tva_cast_expansion_plan(const float *scores, const int32_t *N_i, int32_t n_layers, int32_t B,
                                const double *S_D, const double *S_T, int32_t M, int32_t N_table, int32_t L,
                                int32_t n0, double C1, void *depth_state, int32_t *n_kept, double *work) {
  if (!scores || !N_i || !n_kept || !work || n_layers < 1 || B < 1 || n0 < 0) return TVA_INVALID_ARG;
  if (!layer_ok(depth_state, n_layers)) return TVA_INVALID_ARG;
  const float *layer_scores = scores;
  int32_t ctx = n0;
  double u_prev = 0.0;
  for (int32_t i = 1; i <= n_layers; ++i) {
    double u_ni, c_ni;
    const int32_t n_i = tva_cast_breadth_prune(layer_scores, B, N_i[i - 1], S_D, S_T, M, N_table, L, ctx, C1, &u_ni,
                                               &c_ni, work);
    if (n_i < 1) return n_i;
    n_kept[i - 1] = n_i;
    if (i > 1) tva_cast_depth_update(depth_state, i - 1, u_ni, u_prev);  // phi_{i-1}, now that n_i is known
    if (i == n_layers || !tva_cast_depth_should_expand(depth_state, i, u_ni, c_ni)) return i;
    u_prev = u_ni;
    ctx += n_i;
    layer_scores += (size_t)B * N_i[i - 1];
  }
  return n_layers;
}

int32_t tva_cast_rerank_count(const float *tree_scores, int32_t B, int32_t N_tot, const double *S_T, int32_t M,
                              int32_t N_table, int32_t L, int32_t n0, int32_t m, double C3, double *work) {
  if (!tree_scores || !S_T || !work || B < 1 || N_tot < 1 || m < 1 || M < 1 || L < 1 || n0 < 0) return TVA_INVALID_ARG;
  const int32_t N = std::min(N_tot, m);
  if (N > N_table) return TVA_INVALID_ARG;
  double *sorted = work, *u = work + (size_t)B * N_tot, *c = u + N;
  for (int32_t j = 0; j < B; ++j) {
    double *row = sorted + (size_t)j * N_tot;
    for (int32_t s = 0; s < N_tot; ++s) row[s] = (double)tree_scores[(size_t)j * N_tot + s];
    std::sort(row, row + N_tot, [](double a, double b) { return a > b; });
  }
  double run = 0.0;
  for (int32_t s = 0; s < N; ++s) {
    double col = 0.0;
    for (int32_t j = 0; j < B; ++j) col += sorted[(size_t)j * N_tot + s];
    run += col / B;  // v(s+1), the rank-wise batch mean
    u[s] = run;
  }
  const size_t row = (size_t)table_row(n0, L, M) * N_table;
  for (int32_t k = 0; k < N; ++k) c[k] = S_T[row + k] / S_T[row];
  return tva_cast_select_max_valid_index(u, c, N, C3);
}

int tva_cast_select_subtree(const float *score, const int32_t *parent, int32_t n, int32_t keep, int32_t *old_index,
                            int32_t *new_parent, int32_t *work) {
  if (!score || !parent || !old_index || !new_parent || !work || n < 1 || keep < 1 || keep > n) return TVA_INVALID_ARG;
  for (int32_t i = 0; i < n; ++i) {
    if (parent[i] < -1 || parent[i] >= i) return TVA_INVALID_ARG;
    work[i] = i;
  }
  // the `keep` best by (score descending, index ascending), then back to index order
  std::partial_sort(work, work + keep, work + n, [&](int32_t a, int32_t b) {
    return score[a] > score[b] || (score[a] == score[b] && a < b);
  });
  std::sort(work, work + keep);
  for (int32_t k = 0; k < keep; ++k) old_index[k] = work[k];
  // work[] becomes the map old index -> new index (-1 = dropped)
  std::fill(work, work + n, -1);
  for (int32_t k = 0; k < keep; ++k) work[old_index[k]] = k;
  for (int32_t k = 0; k < keep; ++k) {
    const int32_t p = parent[old_index[k]];
    if (p < 0) {
      new_parent[k] = -1;
    } else {
      if (work[p] < 0) return TVA_INVALID_ARG;  // a kept node whose parent was dropped
      new_parent[k] = work[p];
    }
  }
  return TVA_OK;
}

}  // extern "C"
