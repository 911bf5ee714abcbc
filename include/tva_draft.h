/*
 * libtva -- the device side of draft-tree construction: one layer of expansion (the K most probable next
 * tokens of every selected node, the candidates' scores, the candidates in descending order of score), and the
 * cut of a grown tree to its best-scoring nodes.  How many nodes a layer or the final tree keeps is decided by
 * the host logic of tva_cast.h from the sorted scores these calls return.  Same conventions as tva.h: device
 * pointers owned by the caller, work queued on `stream` (hipStream_t as void*), nothing allocated, negative
 * tva_status on rejected arguments (then nothing is queued).
 */
#ifndef TVA_DRAFT_H
#define TVA_DRAFT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define TVA_EXPAND_MAX_K 16           /* children per node */
#define TVA_EXPAND_MAX_CANDIDATES 1024 /* max_N * K: the candidates of one sequence are sorted in LDS */
#define TVA_SUBTREE_MAX_NODES 2048    /* nodes of one grown tree */

/*
 * One layer of draft-tree expansion (paper, "Tree Expansion Phase": a node's value is the product of the draft
 * model's probabilities along its path, the root 1; every selected node is given K children, taken here as its K
 * most probable next tokens; "Dynamic Expansion Stage", Eq. 1: the method looks at the candidates' values in
 * descending order).  Values are carried as scores = log value.
 *
 * Sequence b owns rows cu_N[b] .. cu_N[b+1]-1 (its selected nodes).  For every row r the K largest entries of
 * logp[r, :] are found (among equal ones the lower token first); child j of row r has the score
 * score[r] + logp[r, token] (one float32 addition).  The n_b * K candidates of a sequence are returned in
 * descending order of score (equal scores: earlier row, then lower rank under it, first) at positions
 * cu_N[b] * K ... of the three output arrays.  Exact: no arithmetic but that one addition.  NaNs must not occur;
 * -inf is an ordinary (smallest) value; -0.0 counts as 0.0.
 *   B, V, K          sequences; vocabulary size (K <= V); children per row, 1 <= K <= TVA_EXPAND_MAX_K
 *   sum_N, max_N     cu_N[B] (at most 65535), and the largest n_b (max_N * K <= TVA_EXPAND_MAX_CANDIDATES); host copies
 *   cu_N             device int32 [B+1]
 *   score            device fp32 [sum_N]
 *   logp, ld_logp    device fp32, row r at logp + r * ld_logp (elements; ld_logp >= V)
 *   cand_score       device fp32  [sum_N * K]
 *   cand_parent      device int32 [sum_N * K]  row within the sequence (0 .. n_b-1)
 *   cand_token       device int32 [sum_N * K]
 *   workspace        device, tva_expand_workspace_bytes(args) bytes (the best K of every 8192-token piece of
 *                    every row, and of every row), 8-byte aligned; contents on return unspecified
 * The workspace query reads only B, V, K, sum_N and returns (size_t)-1 for shapes the launch would reject.
 */
typedef struct tva_expand_args {
  int32_t B, V, K, sum_N, max_N;
  const int32_t *cu_N;
  const float *score, *logp;
  int64_t ld_logp;
  float *cand_score;
  int32_t *cand_parent, *cand_token;
  void *workspace;
  size_t workspace_bytes;
  /* Optional, all zero = not asked for: the breadth decision on the sorted candidates in the same call (what
     tva_layer_breadth_count computes, below; its arguments' meaning is the same), on the candidates' VALUES: a
     candidate's utility is exp(cand_score), evaluated in double precision and rounded to float32 (the scores of
     this call are logarithms of the values Eq. 1 adds up).  Every sequence must then have the
     same number of rows (sum_N = B * max_N); max_N * K <= 1024.  For a batch of one sequence of at most 16 rows the
     count rides in the call's last launch (one launch and its wait less: 28 -> 19 us per draft layer at B = 1);
     otherwise the call ends with the launch tva_layer_breadth_count would make.  A call without rows (B = 0 or
     sum_N = 0) writes nothing, the count included. */
  const double *draft_cost_row; /* device fp64 [max_N * K] */
  double target_cost_one, C1;
  int32_t *count;               /* device int32[1]; NULL = no count */
  double *u_c_at;               /* device fp64[2] or NULL */
  int32_t *count_err_flag;      /* device int32[1] or NULL */
} tva_expand_args;

size_t tva_expand_workspace_bytes(const tva_expand_args *shapes);
int tva_expand_layer(const tva_expand_args *a, void *stream);
size_t tva_sizeof_expand_args(void);

/*
 * The cut of a grown tree to its best nodes (paper, "Tree Reranking Phase": the m nodes of highest value are
 * kept; since a node's value never exceeds its parent's they form a subtree).  Sequence b's tree has the nodes
 * cu_M[b] .. cu_M[b+1]-1 (parent[i] < i local, -1 = root) and keeps cu_T[b+1] - cu_T[b] of them: the best by
 * score, among equal scores the lower index first.  The kept nodes are renumbered in ascending old index
 * (which keeps parents before children) and written to positions cu_T[b] ...:
 *   old_index   device int32 [cu_T[B]]  local index the kept node had
 *   new_parent  device int32 [cu_T[B]]  its parent in the new numbering (-1 = root): the `parent` array
 *               tva_tree_verify_attn takes
 *   err_flag    device int32[1] or NULL, zero on entry: stores 1 + b when a kept node's parent is not kept (a
 *               child scored above its parent: not a tree this method grows), or a sequence is asked to keep
 *               more nodes than it has; that sequence's outputs are then unspecified
 * One tree has at most TVA_SUBTREE_MAX_NODES nodes (max_M, a host copy of the largest tree's size, is checked).
 */
int tva_tree_select_subtree(const float *score, const int32_t *parent, const int32_t *cu_M, const int32_t *cu_T,
                            int32_t B, int32_t max_M, int32_t *old_index, int32_t *new_parent, int32_t *err_flag,
                            void *stream);

/*
 * How many nodes the cut keeps (paper, "Dynamic Reranking Stage": the utility of keeping the s best nodes is the
 * running sum of the batch-averaged scores taken rank by rank, the cost the target table's row; Algorithm 1 with
 * threshold C3 gives the count).  The device form of tva_cast_rerank_count (tva_cast.h), with the same arithmetic in
 * the same order -- the scores are on the device when the tree has been grown there, and ranking 64 trees costs a
 * host core more than the verification itself:
 *   tree_scores  device fp32 [B, N_tot]  scores of all nodes of every sample's grown tree, any order, no NaN
 *   cost_row     device fp64 [min(N_tot, m)]  the target cost table's row for the step's context (k tokens at
 *                index k-1; the host picks the row, tva_cast_select_context); strictly increasing
 *   m            the most nodes the cut may keep
 *   count        device int32[1]: the number of nodes to keep, 1 .. min(N_tot, m)
 *   cu_T         device int32 [B+1] or NULL: b * count, what tva_tree_select_subtree takes
 *   err_flag     device int32[1] or NULL, zero on entry: stores 1 when cost_row does not increase strictly (count and
 *                cu_T are then 0)
 *   workspace    device, tva_rerank_workspace_bytes(B, N_tot, m) bytes (every tree's min(N_tot, m) best scores in
 *                order), 4-byte aligned; contents on return unspecified
 * Two launches: one workgroup per tree, then one for the batch.  N_tot <= TVA_SUBTREE_MAX_NODES, min(N_tot, m) <= 1024,
 * else TVA_UNSUPPORTED.
 */
size_t tva_rerank_workspace_bytes(int32_t B, int32_t N_tot, int32_t m);
int tva_tree_rerank_count(const float *tree_scores, int32_t B, int32_t N_tot, const double *cost_row, int32_t m, double C3,
                          int32_t *count, int32_t *cu_T, int32_t *err_flag, void *workspace, size_t workspace_bytes,
                          void *stream);

/*
 * How many candidates of a layer are kept (paper, "Dynamic Expansion Stage": Eq. 1, the utility of the k best
 * candidates averaged over the batch; Eq. 2, their cost under the draft model relative to one token under the target
 * model; Algorithm 1 with threshold C1).  The device form of tva_cast_breadth_prune, same arithmetic in the same order:
 *   cand_score      device fp32 [B, N]  the layer's candidates of every sample in descending order of score --
 *                   tva_expand_layer's cand_score when every sequence has the same number of selected nodes
 *   draft_cost_row  device fp64 [N]  the draft cost table's row for the layer's context (k tokens at index k-1),
 *                   strictly increasing
 *   target_cost_one the target table's cost of one token for that context (host value, > 0)
 *   count           device int32[1]: the number kept, 1 .. N
 *   u_c_at          device fp64[2] or NULL: the utility and the cost at that count (what the depth test reads)
 *   err_flag        device int32[1] or NULL, zero on entry: stores 1 when the cost row does not increase strictly
 * One workgroup, one launch.  N <= 1024, else TVA_UNSUPPORTED.
 */
int tva_layer_breadth_count(const float *cand_score, int32_t B, int32_t N, const double *draft_cost_row, double target_cost_one,
                            double C1, int32_t *count, double *u_c_at, int32_t *err_flag, void *stream);

#ifdef __cplusplus
}
#endif
#endif
