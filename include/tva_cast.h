/*
 * libtva, host part -- the cost-aware choice of draft-tree sizes that decides how many tree
 * tokens tva_tree_verify_attn is asked to verify (paper: section "Method").
 *
 * The builder trades the confidence gained by keeping more draft nodes against the measured cost
 * of one more token in the draft / target forward.  Costs come from lookup tables f(B, c, n) kept
 * for contexts c = L, 2L, .., M*L and n = 1..N tokens, one pair of tables (draft S_D, target S_T)
 * per batch size B; this library's own attention kernels supply the attention part of S_T
 * (paper_2510_26577_amd/cost_table.py measures it).
 *
 * Conventions
 *   - EVERY pointer here is HOST memory owned by the caller.  Nothing is allocated, nothing is
 *     kept between calls except in the state block the caller passes to the depth-pruning calls.
 *   - Tables are row-major double [M][N]: row r-1 is context r*L, column n-1 is n tokens.
 *   - Score matrices are row-major float [B][N]: one row per sample, best candidate first.
 *   - Counts and indices that the paper writes 1-based (k, n_i, the result of Algorithm 1) are
 *     returned 1-based.  Negative return values are tva_status codes (tva.h).
 */
#ifndef TVA_CAST_H
#define TVA_CAST_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Table row for a context of c tokens, as a context length (Method, 2nd paragraph: select(c)).
 * Read as the first grid point above c, clamped to the last row: (min(c / L, M - 1) + 1) * L --
 * the printed formula has max(.) there, which would always give M*L.  c >= 0, L >= 1, M >= 1;
 * returns TVA_INVALID_ARG (negative) otherwise.
 */
int32_t tva_cast_select_context(int32_t c, int32_t L, int32_t M);

/*
 * Algorithm 1 ("Select Maximum Valid Index").  u[n], c[n] with c strictly increasing, C > 0.
 * Index j (1-based) is valid unless some i < j has (u[j]-u[i]) / (c[j]-c[i]) < C; returns the
 * largest valid index (index 1 always is).  TVA_INVALID_ARG if n < 1, a pointer is null or c is
 * not strictly increasing.
 */
int32_t tva_cast_select_max_valid_index(const double *u, const double *c, int32_t n, double C);

/*
 * Eq. 1: u[k-1] = (1/B) * sum over samples of the sum of their k best scores, k = 1..N.
 * scores float [B][N], each row in descending order (not checked).
 */
int tva_cast_layer_utility(const float *scores, int32_t B, int32_t N, double *u);

/*
 * Eq. 2: c[k-1] = S_D[select(ctx)][k] / S_T[select(ctx)][1], k = 1..n_candidates <= N_table.
 */
int tva_cast_layer_cost(const double *S_D, const double *S_T, int32_t M, int32_t N_table, int32_t L,
                        int32_t ctx, int32_t n_candidates, double *c);

/*
 * Breadth pruning of one layer (Dynamic Expansion Stage): Algorithm 1 on Eq. 1 / Eq. 2 with
 * threshold C1.  Returns n_i (1-based count of kept nodes); u_at / c_at (may be NULL) receive
 * u_{n_i} and c_{n_i}, which depth pruning needs.  work: 2*N doubles of caller scratch.
 */
int32_t tva_cast_breadth_prune(const float *scores, int32_t B, int32_t N, const double *S_D, const double *S_T,
                               int32_t M, int32_t N_table, int32_t L, int32_t ctx, double C1, double *u_at,
                               double *c_at, double *work);

/*
 * Depth pruning (Dynamic Expansion Stage, last paragraph): one first-in-first-out buffer A_i per
 * layer i = 1..max_layers holding at most R recent gain ratios phi_i, started with the single
 * value 1.  The state lives in caller memory of tva_cast_depth_bytes() bytes (8-byte aligned) and
 * persists across decode steps.
 *   init           fills the state.
 *   alpha          Avg(A_i).
 *   should_expand  1 if alpha_i * u_ni / c_ni >= C2 (generate layer i+1), else 0.
 *   update         pushes phi_i = u_next / u_cur into A_i (dropping the oldest beyond R); returns phi_i.
 * Layer indices outside [1, max_layers] give TVA_INVALID_ARG (alpha / update: NaN).
 */
size_t tva_cast_depth_bytes(int32_t max_layers, int32_t R);
int tva_cast_depth_init(void *state, int32_t max_layers, int32_t R, double C2);
double tva_cast_depth_alpha(const void *state, int32_t layer);
int tva_cast_depth_should_expand(const void *state, int32_t layer, double u_ni, double c_ni);
double tva_cast_depth_update(void *state, int32_t layer, double u_next, double u_cur);

/*
 * Expansion stage over given candidate layers: layer i (1-based) has N_i[i-1] candidates per
 * sample, its scores float [B][N_i[i-1]] stored one layer after the other in `scores`.  The context
 * of layer i is n0 + n_1 + .. + n_{i-1} (n0 = 0 is the printed formula).  Writes the kept counts to
 * n_kept and returns how many layers were generated (>= 1).  work: 2*max(N_i) doubles.
 */
int32_t tva_cast_expansion_plan(const float *scores, const int32_t *N_i, int32_t n_layers, int32_t B,
                                const double *S_D, const double *S_T, int32_t M, int32_t N_table, int32_t L,
                                int32_t n0, double C1, void *depth_state, int32_t *n_kept, double *work);

/*
 * Reranking stage (Dynamic Reranking Stage): number of tree nodes handed to the target model.
 * tree_scores float [B][N_tot]: all node scores of each sample's expanded tree, any order.  The
 * per-sample scores are sorted, averaged rank by rank, truncated to min(N_tot, m) and fed to
 * Algorithm 1 with u_k = v(1)+..+v(k), c_k = S_T[select(n0)][k] / S_T[select(n0)][1], threshold C3.
 * work: B*N_tot + 2*min(N_tot, m) doubles.  Needs min(N_tot, m) <= N_table.
 */
int32_t tva_cast_rerank_count(const float *tree_scores, int32_t B, int32_t N_tot, const double *S_T, int32_t M,
                              int32_t N_table, int32_t L, int32_t n0, int32_t m, double C3, double *work);

/*
 * Tree Reranking Phase: keep the `keep` best-scoring nodes of one tree (ties: lower index first)
 * and relabel them in ascending original index, which keeps parents before children.
 *   score float [n], parent int32 [n] (-1 = root, parent[i] < i)
 *   old_index int32 [keep]: original index of each kept node; new_parent int32 [keep]: parent
 *   array of the kept subtree -- the input tva_build_ancestor_mask takes.  work: n int32.
 * TVA_INVALID_ARG if a kept node's parent is not kept (a child that outscores its parent) or the
 * arguments are malformed; nothing useful is written then.
 */
int tva_cast_select_subtree(const float *score, const int32_t *parent, int32_t n, int32_t keep,
                            int32_t *old_index, int32_t *new_parent, int32_t *work);

#ifdef __cplusplus
}
#endif
#endif /* TVA_CAST_H */
