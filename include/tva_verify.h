/*
 * libtva -- the steps that close a verification pass after the attention: acceptance of a root
 * path of each draft tree (greedy, or by speculative sampling), and the commit of the accepted nodes'
 * K/V rows to the end of each sequence's cache.  Same conventions as tva.h: device pointers owned by the
 * caller, work queued on `stream` (hipStream_t as void*), nothing allocated, negative tva_status
 * on rejected arguments (then nothing is queued).
 */
#ifndef TVA_VERIFY_H
#define TVA_VERIFY_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Greedy (temperature 0) acceptance on draft trees (paper, Preliminary: a drafted token is accepted
 * with probability min(1, p/q) and the target's own token replaces the first rejected one; with a
 * tree draft a rejected token leaves its siblings in play.  At temperature 0 the target's
 * distribution is its argmax, so exactly the child that carries that token is accepted).
 *
 * Per sequence b the walk starts at node 0 (always accepted) and moves to the child -- lowest index
 * if several qualify -- whose draft_token equals target_token of the current node, until no child
 * qualifies or max_path nodes are accepted.
 *   parent        device int32 [cu_T[B]]  local parent index per node, -1 = root, parent[i] < i
 *   cu_T          device int32 [B+1]
 *   draft_token   device int32 [cu_T[B]]  token drafted at each node
 *   target_token  device int32 [cu_T[B]]  the target model's argmax for the position after each node
 *   max_path      row length of `path`, >= 1 (tree depth + 1 never truncates)
 *   path          device int32 [B, max_path]: accepted local node indices in path order; entries past
 *                 path_len[b] are not written
 *   path_len      device int32 [B]: accepted nodes (0 for an empty tree)
 *   next_token    device int32 [B]: target_token of the last accepted node (-1 for an empty tree)
 */
int tva_accept_greedy(const int32_t *parent, const int32_t *cu_T, const int32_t *draft_token,
                      const int32_t *target_token, int32_t B, int32_t max_path, int32_t *path,
                      int32_t *path_len, int32_t *next_token, void *stream);

/*
 * Acceptance by speculative sampling on draft trees (paper, Preliminary, "Speculative Decoding": a drafted
 * token x is accepted when a uniform number is at most min(1, p(x) / q(x)), p the target's and q the draft's
 * probability of it; after a rejection the target distribution is replaced by the residual
 * norm(max(0, p - q)) -- the output is then a sample of the target distribution; "EAGLE": with a tree draft a
 * rejected token leaves its siblings in play).
 *
 * Per sequence b the walk starts at node 0 (always accepted).  At the current node its children are tested in
 * index order against the current residual r (r = the node's row of p_target at first, kept unnormalised with
 * Z = sum r):  child c with token x is accepted iff  r[x] > 0  and  u[c] * q[x] * Z <= r[x]  (q = the current
 * node's row of q_draft, the distribution its children were drawn from, independently; a rejection does not
 * change it);  a rejected child replaces r by max(0, r - Z q).  The first accepted child becomes the current
 * node, with a fresh r.  When every child is rejected, or there is none, or max_path nodes are accepted, the
 * step's last token is the smallest v whose cumulative weight r[0] + .. + r[v] exceeds u_final[b] * Z, and the
 * walk ends.  r is held in fp32; sums, products and comparisons are made in fp64.  The random numbers are
 * inputs: the library draws none.
 *   parent, cu_T, draft_token   as for tva_accept_greedy
 *   p_target, q_draft   device fp32 [cu_T[B], V]  rows per node (each a distribution: non-negative, sum 1)
 *   u                   device fp32 [cu_T[B]]     uniform number of each node's test as a child
 *   u_final             device fp32 [B]           uniform number of each sequence's last draw
 *   residual            device fp32 [B, V]        scratch the caller owns; contents on return unspecified
 *   path, path_len, next_token   as for tva_accept_greedy (next_token = the drawn token)
 *   err_flag            device int32[1] or NULL, zero on entry: stores 1 + b when a draft_token is not in
 *                       [0, V) (that child is never accepted) or a residual vanishes (q was not the distribution
 *                       the rejected child came from; the walk ends there with next_token -1)
 *   workspace, workspace_bytes   device memory of tva_sample_workspace_bytes(B) bytes, 8-byte aligned, or NULL.
 *                       With it, the vocabulary of a sequence is spread over several workgroups that wait for one
 *                       another between passes (a sequence's passes are a chain, and one workgroup streams a row at
 *                       what one compute unit can): B = 1, V = 128256 runs three times faster.  The waits are
 *                       bounded (about a second): a sequence whose workgroups do not all arrive -- they are all
 *                       resident at once unless other work holds the compute units that long -- is flagged in
 *                       err_flag like the cases above, and its outputs are unspecified.  Contents unspecified on
 *                       return; calls that share a workspace must not overlap.  Without it: one workgroup per
 *                       sequence, no waits.
 *   sum_T               the number of nodes of the batch, cu_T[B], as the host knows it, or 0.  With it, and a workspace
 *                       of tva_sample_workspace_bytes_rows(B, sum_T, V) bytes, the sums of all target rows of a small
 *                       batch (sum_T * V * 4 bytes up to 40 MB) are made ahead of the walk by a launch that uses the
 *                       whole chip, and the walk passes an accepted node without a pass over its row (V = 128256,
 *                       B = 1 .. 8: 6 to 26 % faster again).  A value that is not cu_T[B] costs time, not correctness:
 *                       rows past cu_T[B] are not read, and a tree that reaches past sum_T is walked as without it.
 *   unit_rows           1: the caller states that every row of p_target sums to one (it is a distribution), and a node
 *                       that has just been reached takes Z = 1 instead of summing its row: its children's tests are
 *                       then u q(x) <= p(x) and the first residual max(0, p - q), as the paper prints them, and an
 *                       accepted node costs two loads instead of a pass over V floats, at any batch size (B = 64,
 *                       V = 128256: 76 -> 54 us; B = 8, 32-node trees: 45 -> 28 us).  The last draw still divides by the sum of the row it draws from.
 *                       With rows that sum to one within float32 rounding the two forms differ only where a test is
 *                       within that rounding of its threshold.  0: rows are summed.
 *   workgroups_per_sequence   0: the library chooses (1 .. 16, so that B times it stays within 256; 1 for
 *                       vocabularies below 48 K tokens, where the waits cost what the slices save -- below 16 K when
 *                       the row sums are made ahead, see sum_T); 1: as without
 *                       a workspace; 2 .. 16: that many (TVA_UNSUPPORTED if B times it exceeds 256).  The results
 *                       do not depend on it beyond the order in which a pass's sum is added up.
 */
typedef struct tva_sample_args {
  int32_t B, V, max_path;
  const int32_t *parent, *cu_T, *draft_token;
  const float *p_target, *q_draft, *u, *u_final;
  float *residual;
  int32_t *path, *path_len, *next_token, *err_flag;
  void *workspace;
  size_t workspace_bytes;
  int32_t workgroups_per_sequence;
  int32_t sum_T;
  int32_t unit_rows;
} tva_sample_args;

int tva_accept_sampling(const tva_sample_args *a, void *stream);
size_t tva_sample_workspace_bytes(int32_t B);
size_t tva_sample_workspace_bytes_rows(int32_t B, int32_t sum_T, int32_t V);  /* the same plus room for the row sums */
/* For tests of the bounded wait: the same call (workspace given, workgroups_per_sequence >= 2), but every wait expects
 * one arrival more than there are workgroups and gives up after `spins` polls (1 .. 2^20).  Every workgroup then
 * leaves at its first wait: err_flag is set, the other outputs are unspecified, and the kernel ends normally. */
int tva_accept_sampling_wait_bound_test(const tva_sample_args *a, int32_t spins, void *stream);
size_t tva_sizeof_sample_args(void);

/*
 * Commit of the accepted path: accepted node j of sequence b (path order) has its K and V rows copied
 * from the tree tensors to cache position L[b] + j.  Cache forms and strides as in tva_args (tva.h):
 *   dense : cu_L != NULL; sequence b owns rows cu_L[b] .. cu_L[b+1]-1 of which the first L[b] are in use
 *   paged : page_table != NULL; position t is slot t % page_size of page page_table[b*max_pages + t/page_size]
 * A position outside the sequence's room (dense: beyond cu_L[b+1]; paged: beyond max_pages pages), or a
 * path entry that is not a node of the sequence's tree, is not written and, if err_flag is given (zero
 * on entry), stores 1 + b there.  The lengths, offsets and page numbers themselves are trusted.
 * L_out[b] = L[b] + path_len[b] is written when L_out is not NULL; it must not alias L.
 *
 * An 8-bit cache (tva_args.kv_fp8) is committed by the same call: only bytes are moved, so pass D / 2 for D
 * and strides counted in two-byte units.
 *
 * k_tree = v_tree = NULL selects the in-cache form: tree node i of sequence b already sits at cache
 * position L[b] + i (the layout tva_tree_verify_attn reads when its k_tree is NULL), and the accepted
 * nodes are moved down in place to L[b], L[b]+1, ...; everything behind them is left as it is.
 *
 * All layers of a model in one call (n_layers > 1): the lengths, the path, the page table and the offsets are the
 * same for every layer, only the tensors differ.  Layer l's caches start layer_stride_cache elements behind layer
 * l-1's (k_cache and v_cache each), its tree tensors layer_stride_tree elements behind (multiples of 8, counted like
 * the other strides); the call is one launch instead of n_layers (32 layers at B = 1: 5 us against 64).
 */
typedef struct tva_commit_args {
  int32_t B, Hkv, D;   /* D * Hkv * 2 bytes per row must be a multiple of 16 */
  int32_t max_path;    /* row length of `path` */
  const int32_t *cu_T; /* device [B+1] */
  const int32_t *L;    /* device [B] */
  const int32_t *path, *path_len;  /* device [B, max_path], [B] (tva_accept_greedy's outputs) */
  const void *k_tree, *v_tree;     /* device bf16 [cu_T[B], Hkv, D]; both NULL = tree rows are in the cache */
  void *k_cache, *v_cache;         /* device bf16, dense or paged */
  const int32_t *cu_L;             /* device [B+1] or NULL */
  const int32_t *page_table;       /* device [B, max_pages] or NULL */
  int32_t page_size, max_pages;
  int64_t stride_page, stride_tok, stride_head; /* elements; 0 = packed default as in tva_args */
  int32_t *L_out;      /* device [B] or NULL */
  int32_t *err_flag;   /* device int32[1] or NULL */
  int32_t n_layers;    /* 0 or 1: one layer */
  int64_t layer_stride_cache, layer_stride_tree; /* elements between consecutive layers' tensors (n_layers > 1) */
} tva_commit_args;

int tva_commit_path(const tva_commit_args *a, void *stream);
size_t tva_sizeof_commit_args(void);

#ifdef __cplusplus
}
#endif
#endif /* TVA_VERIFY_H */
