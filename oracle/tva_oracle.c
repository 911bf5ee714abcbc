/*
 * CPU oracle for tree-masked verification attention.  TEST INFRASTRUCTURE ONLY.
 *
 * This file is the plain definition of what the attention of the target
 * model's verification pass computes (paper: Tree Reranking Phase, last
 * paragraph -- the selected subtree is flattened and its attention mask lets a
 * node see the nodes on its path to the root; Method, first paragraphs -- a batch of B samples, each
 * with a context of length c, verifying n tree tokens).  It is slow on
 * purpose: the full (L+T) boolean mask of every sequence is materialised, all
 * scores of a row are stored, and the softmax is the naive three-pass one.
 * Arithmetic is IEEE double on bf16 inputs widened exactly, so the result does
 * not depend on summation order at the tolerances the tests use.
 *
 * Nothing here is shared with the HIP library: no header, helper, table or
 * constant.  Only tests/, the smoke check and the benchmark's cpu_baseline leg
 * may call it; the product path never does.
 *
 * Readings of points the paper leaves open (each is pinned by a CPU test):
 *   - a node attends to itself as well as to its proper ancestors (otherwise a
 *     chain-shaped tree would not equal causal attention and T=1 would not
 *     equal ordinary decoding);
 *   - the linearised order is topological: parent[i] < i, parent = -1 marks a
 *     root (several roots are accepted);
 *   - query head h reads KV head h / (Hq/Hkv);
 *   - LSE is the natural log of the sum of exponentials of the SCALED scores.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef struct {
  int32_t B, Hq, Hkv, D;
  double scale;
  const int32_t *cu_T;      /* [B+1] */
  const int32_t *L;         /* [B]   */
  const int32_t *parent;    /* [sum_T] local parent index or -1 */
  const uint16_t *q;        /* bf16 [sum_T, Hq, D]  */
  const uint16_t *k_tree;   /* bf16 [sum_T, Hkv, D] */
  const uint16_t *v_tree;
  const uint16_t *k_cache;  /* dense: [sum_L, Hkv, D]; paged: [P, page, Hkv, D] */
  const uint16_t *v_cache;
  const int32_t *cu_L;      /* [B+1] (dense) or NULL */
  const int32_t *page_table;/* [B, max_pages] (paged) or NULL */
  int32_t page_size, max_pages;
  /* keys are numbered 0..L_b-1 (cache) then L_b..L_b+T_b-1 (tree); only keys in
   * [key_lo, key_hi) take part (key_hi < 0: no upper limit).  Used to state
   * what one KV split computes. */
  int64_t key_lo, key_hi;
} tvo_problem;

static double bf16_to_double(uint16_t b) {
  uint32_t u = ((uint32_t)b) << 16;
  float f;
  memcpy(&f, &u, 4);
  return (double)f;
}

int tvo_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

void tvo_set_num_threads(int n) {
#ifdef _OPENMP
  if (n > 0) omp_set_num_threads(n);
#else
  (void)n;
#endif
}

/* Ancestor bitmasks straight from the definition: for every node walk the
 * parent pointers up to a root, setting one bit per visited node (the node
 * itself included).  mask is [sum_T, W] uint64, bit (j % 64) of word (j / 64).
 * Returns 0, or 1 + global index of the first node whose parent is not in
 * [-1, i-1]. */
int64_t tvo_ancestor_mask(const int32_t *parent, const int32_t *cu_T, int32_t B, int32_t W,
                          uint64_t *mask) {
  for (int b = 0; b < B; b++) {
    int t0 = cu_T[b], T = cu_T[b + 1] - cu_T[b];
    for (int i = 0; i < T; i++) {
      int p = parent[t0 + i];
      if (p < -1 || p >= i) return (int64_t)(t0 + i) + 1;
    }
    for (int i = 0; i < T; i++) {
      uint64_t *m = mask + (size_t)(t0 + i) * W;
      for (int w = 0; w < W; w++) m[w] = 0;
      for (int a = i; a >= 0; a = parent[t0 + a]) {
        if (a / 64 < W) m[a / 64] |= (uint64_t)1 << (a % 64);
      }
    }
  }
  return 0;
}

static const uint16_t *key_row(const tvo_problem *p, const uint16_t *cache, const uint16_t *tree,
                               int b, int64_t key, int g) {
  int Lb = p->L[b];
  size_t row = (size_t)p->Hkv * p->D;
  if (key >= Lb) return tree + ((size_t)(p->cu_T[b] + (key - Lb)) * p->Hkv + g) * p->D;
  if (p->page_table) {
    int64_t page = p->page_table[(size_t)b * p->max_pages + key / p->page_size];
    return cache + ((size_t)page * p->page_size + (size_t)(key % p->page_size)) * row + (size_t)g * p->D;
  }
  return cache + ((size_t)p->cu_L[b] + (size_t)key) * row + (size_t)g * p->D;
}

/* One output row (sequence b, tree node i, query head h) given that row of the
 * materialised mask: allowed[k] != 0 iff key k may be attended. */
static void attn_row(const tvo_problem *p, int b, int i, int h, const uint8_t *allowed,
                     double *s, double *out, double *lse) {
  int D = p->D, Lb = p->L[b], Tb = p->cu_T[b + 1] - p->cu_T[b];
  int64_t nk = (int64_t)Lb + Tb;
  int g = h / (p->Hq / p->Hkv);
  const uint16_t *qr = p->q + ((size_t)(p->cu_T[b] + i) * p->Hq + h) * D;
  double M = -INFINITY;
  for (int64_t k = 0; k < nk; k++) {
    int in_range = k >= p->key_lo && (p->key_hi < 0 || k < p->key_hi);
    if (allowed[k] && in_range) {
      const uint16_t *kr = key_row(p, p->k_cache, p->k_tree, b, k, g);
      double dot = 0.0;
      for (int d = 0; d < D; d++) dot += bf16_to_double(qr[d]) * bf16_to_double(kr[d]);
      s[k] = p->scale * dot;
      if (s[k] > M) M = s[k];
    } else {
      s[k] = -INFINITY;
    }
  }
  for (int d = 0; d < D; d++) out[d] = 0.0;
  if (M == -INFINITY) { /* no key at all in this range: empty partial */
    *lse = -INFINITY;
    return;
  }
  double Z = 0.0;
  for (int64_t k = 0; k < nk; k++)
    if (s[k] != -INFINITY) Z += exp(s[k] - M);
  for (int64_t k = 0; k < nk; k++) {
    if (s[k] == -INFINITY) continue;
    double w = exp(s[k] - M) / Z;
    const uint16_t *vr = key_row(p, p->v_cache, p->v_tree, b, k, g);
    for (int d = 0; d < D; d++) out[d] += w * bf16_to_double(vr[d]);
  }
  *lse = M + log(Z);
}

/* Materialise the boolean mask of sequence b: [T_b, L_b + T_b], row i allows
 * every cached key and the tree keys on the path root -> i (i included). */
static uint8_t *build_mask(const tvo_problem *p, int b) {
  int Lb = p->L[b], t0 = p->cu_T[b], Tb = p->cu_T[b + 1] - t0;
  size_t nk = (size_t)Lb + Tb;
  uint8_t *m = (uint8_t *)calloc((size_t)Tb * nk + 1, 1);
  if (!m) return NULL;
  for (int i = 0; i < Tb; i++) {
    uint8_t *r = m + (size_t)i * nk;
    memset(r, 1, (size_t)Lb);
    for (int a = i; a >= 0; a = p->parent[t0 + a]) r[Lb + a] = 1;
  }
  return m;
}

/* Full problem: out double [sum_T, Hq, D], lse double [sum_T, Hq].
 * Parallel over (sequence, head) only.  Returns 0 or -1 (allocation). */
int tvo_attention(const tvo_problem *p, double *out, double *lse) {
  int B = p->B, Hq = p->Hq, D = p->D, fail = 0;
  uint8_t **masks = (uint8_t **)calloc((size_t)B + 1, sizeof(uint8_t *));
  if (!masks) return -1;
  for (int b = 0; b < B; b++) {
    masks[b] = build_mask(p, b);
    if (!masks[b]) fail = 1;
  }
  if (!fail) {
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
    for (int b = 0; b < B; b++) {
      for (int h = 0; h < Hq; h++) {
        int t0 = p->cu_T[b], Tb = p->cu_T[b + 1] - t0;
        size_t nk = (size_t)p->L[b] + Tb;
        double *s = (double *)malloc((nk + 1) * sizeof(double));
        for (int i = 0; i < Tb; i++) {
          size_t r = (size_t)(t0 + i) * Hq + h;
          attn_row(p, b, i, h, masks[b] + (size_t)i * nk, s, out + r * D, lse + r);
        }
        free(s);
      }
    }
  }
  for (int b = 0; b < B; b++) free(masks[b]);
  free(masks);
  return fail ? -1 : 0;
}

/* Selected rows only: rows int32 [n, 3] = (b, i, h); out [n, D], lse [n].
 * The mask row is still materialised in full for each selected row. */
int tvo_attention_rows(const tvo_problem *p, const int32_t *rows, int64_t n, double *out,
                       double *lse) {
  int fail = 0;
#pragma omp parallel for schedule(dynamic, 1)
  for (int64_t r = 0; r < n; r++) {
    int b = rows[3 * r], i = rows[3 * r + 1], h = rows[3 * r + 2];
    int Lb = p->L[b], t0 = p->cu_T[b], Tb = p->cu_T[b + 1] - t0;
    size_t nk = (size_t)Lb + Tb;
    uint8_t *m = (uint8_t *)calloc(nk + 1, 1);
    double *s = (double *)malloc((nk + 1) * sizeof(double));
    if (!m || !s) {
      fail = 1;
    } else {
      memset(m, 1, (size_t)Lb);
      for (int a = i; a >= 0; a = p->parent[t0 + a]) m[Lb + a] = 1;
      attn_row(p, b, i, h, m, s, out + (size_t)r * p->D, lse + r);
    }
    free(m);
    free(s);
  }
  return fail ? -1 : 0;
}

/* Merging the partial results of S disjoint key subsets (what splitting a
 * softmax implies): lse = log sum_s exp(lse_s), O = sum_s exp(lse_s - lse) O_s.
 * part_out [S, n, D], part_lse [S, n]; n_splits_row[n] gives how many leading
 * splits are valid for each row (others ignored).  A partial with lse = -inf
 * contributes nothing. */
void tvo_merge_splits(const double *part_out, const double *part_lse, const int32_t *n_splits_row,
                      int32_t S, int64_t n, int32_t D, double *out, double *lse) {
  for (int64_t r = 0; r < n; r++) {
    int ns = n_splits_row ? n_splits_row[r] : S;
    double M = -INFINITY;
    for (int s = 0; s < ns; s++)
      if (part_lse[(size_t)s * n + r] > M) M = part_lse[(size_t)s * n + r];
    for (int d = 0; d < D; d++) out[(size_t)r * D + d] = 0.0;
    if (M == -INFINITY) {
      lse[r] = -INFINITY;
      continue;
    }
    double Z = 0.0;
    for (int s = 0; s < ns; s++) Z += exp(part_lse[(size_t)s * n + r] - M);
    lse[r] = M + log(Z);
    for (int s = 0; s < ns; s++) {
      double w = exp(part_lse[(size_t)s * n + r] - lse[r]);
      if (w == 0.0) continue;
      for (int d = 0; d < D; d++)
        out[(size_t)r * D + d] += w * part_out[((size_t)s * n + r) * D + d];
    }
  }
}
