/*
 * libtva -- tree-masked verification attention for AMD MI355X (gfx950).
 *
 * C ABI of the data-parallel hot path of cost-aware draft-tree speculative
 * decoding: in the target model's verification pass every draft-tree token of
 * every sequence in the batch attends to that sequence's cached context plus
 * its own ancestors in the tree (paper: "Tree Reranking Phase", last paragraph:
 * the selected subtree is linearised and the attention mask lets each token see
 * only its ancestors; "Method", opening paragraphs: a batch of B samples with
 * context length c verifies n tree tokens, at a cost f_T(B, c, n) that the
 * tree builder trades against acceptance).
 *
 * Conventions shared by all entry points
 *   - Every pointer marked "device" is GPU memory the CALLER owns and keeps
 *     alive until the work queued on `stream` has finished.  The library never
 *     allocates, frees or synchronises; inputs are never written.
 *   - `stream` is a hipStream_t passed as void* (NULL = the null stream).  All
 *     work is queued on it and the call returns immediately.
 *   - bf16 tensors are raw 16-bit patterns, innermost dimension contiguous.
 *   - Return value: TVA_OK (0) or a negative tva_status; tva_strerror() names it.
 *     A failing call queues nothing.
 *   - Trees: node indices are local to their tree, parent = -1 marks a root,
 *     and the linearised order must be topological (parent[i] < i).  A node
 *     attends to itself and to its ancestors.
 */
#ifndef TVA_H
#define TVA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  TVA_OK = 0,
  TVA_INVALID_ARG = -1,         /* null pointer, bad sizes, both / neither cache form */
  TVA_UNSUPPORTED = -2,         /* D not in {64,128}, max_T > 128, ... */
  TVA_WORKSPACE_TOO_SMALL = -3, /* see tva_workspace_bytes() */
  TVA_BAD_TREE = -5,            /* tva_build_ancestor_mask_host only: a parent index outside [-1, i-1] */
  TVA_HIP_ERROR = -4            /* a launch failed: the error is left for hipGetLastError (an older
                                   error of the process is cleared before each launch, so the status
                                   is this launch's); TVA_VERBOSE=1 in the environment names it on stderr */
} tva_status;

#define TVA_MAX_TREE 128 /* nodes per tree supported by the attention kernels (2 mask words) */

/* Bytes of scratch memory tva_tree_verify_attn_static owns on every GPU (see there). */
#define TVA_STATIC_SCRATCH_BYTES (32u << 20)

/*
 * Workgroup shapes of the attention kernel, for tva_args.plan_shape: query rows per workgroup
 * (tree nodes x query heads of one KV head) and waves.  TVA_SHAPE_AUTO lets the library choose
 * from the sizes; naming one is a tuning and testing aid (every shape computes the same result
 * for every input; only the speed differs).
 */
typedef enum {
  TVA_SHAPE_AUTO = 0,
  TVA_SHAPE_R32_W2 = 1,       /*  32 rows, 1 x 2 waves (the two waves split each tile's keys) */
  TVA_SHAPE_R64_W4 = 2,       /*  64 rows, 2 x 2 waves, two workgroups per CU */
  TVA_SHAPE_R64_W4_DEEP = 3,  /*  the same with one more tile in flight, one workgroup per CU */
  TVA_SHAPE_R128_W8 = 4,      /* 128 rows, 4 x 2 waves */
  TVA_SHAPE_R256_W8 = 5       /* 256 rows, 8 x 1 waves */
} tva_shape;

/*
 * Arguments of tva_tree_verify_attn.
 *
 * Shapes: B sequences; sequence b verifies T_b = cu_T[b+1]-cu_T[b] tree tokens
 * against L[b] cached tokens.  Hq query heads, Hkv KV heads (Hq % Hkv == 0),
 * query head h reads KV head h / (Hq/Hkv).  Head dimension D is 64 or 128.
 *
 * KV cache, exactly one of two forms:
 *   dense : cu_L != NULL, page_table == NULL.  Token t of sequence b is row
 *           cu_L[b] + t of k_cache / v_cache.
 *   paged : page_table != NULL, cu_L == NULL.  Token t of sequence b is slot
 *           t % page_size of page page_table[b*max_pages + t/page_size].
 *           Entries past ceil(L[b]/page_size) and slots past L[b] in the last
 *           page are never read.
 * In both forms element d of KV head g of a token lives at
 *   base + page*stride_page + slot*stride_tok + g*stride_head + d   (elements),
 * with page = 0 and slot = the row index in the dense form.  A stride given as
 * 0 takes its packed default ([.., Hkv, D] token-major: stride_head = D,
 * stride_tok = Hkv*D, stride_page = page_size*stride_tok).  Addresses of rows
 * must be 16-byte aligned (strides multiples of 8 elements).
 */
typedef struct tva_args {
  int32_t B, Hq, Hkv, D;
  int32_t sum_T;      /* cu_T[B]: total tree tokens */
  int32_t max_T;      /* host-side upper bound of T_b, <= TVA_MAX_TREE */
  int32_t mask_words; /* 64-bit words per ancestor-mask row, >= ceil(max_T/64), <= 2 */
  int32_t max_L;      /* host-side upper bound of L[b] (sizes the launch; a value
                         below some L[b] truncates that sequence's context) */
  float scale;        /* softmax scale applied to q.k, > 0 (1/sqrt(D) usually) */

  const int32_t *cu_T; /* device [B+1] */
  const int32_t *L;    /* device [B], each >= 0 */
  const void *q;       /* device bf16 [sum_T, Hq, D] */
  const void *k_tree;  /* device bf16 [sum_T, Hkv, D]: keys of the tree tokens */
  const void *v_tree;  /* device bf16 [sum_T, Hkv, D]
                          Both NULL: the tree tokens' K/V are in the cache, token i of sequence b at
                          position L[b] + i (dense: row cu_L[b] + L[b] + i, so cu_L leaves that room;
                          paged: through the page table, which then covers L[b] + T_b positions).
                          max_L must then not be below any L[b]. */
  const uint64_t *anc_mask; /* device [sum_T, mask_words]: bit j of row i set iff node j
                               is node i or one of its ancestors (tva_build_ancestor_mask);
                               or NULL, then `parent` below is used */

  const void *k_cache, *v_cache; /* device bf16, dense or paged (above) */
  const int32_t *cu_L;           /* device [B+1] or NULL */
  const int32_t *page_table;     /* device [B, max_pages] or NULL */
  int32_t page_size, max_pages;  /* paged form only */
  int64_t stride_page, stride_tok, stride_head; /* elements; 0 = packed default */

  float *out; /* device fp32 [sum_T, Hq, D]  (sum_Q rows with cu_Q, below) */
  float *lse; /* device fp32 [sum_T, Hq]: natural-log sum-exp of the scaled scores */

  void *workspace;        /* device scratch for the KV splits, may be NULL if 0 bytes */
  size_t workspace_bytes; /* >= tva_workspace_bytes(args) */
  int32_t num_splits;     /* KV splits per sequence; 0 = library chooses */

  const int32_t *parent;  /* device int32 [sum_T] or NULL: local parent index per node (-1 = root,
                             parent[i] < i), read only when anc_mask is NULL.  The attention kernel
                             then derives each row's ancestor set itself (same sets as
                             tva_build_ancestor_mask; no separate launch, nothing written).  A link
                             that does not point backwards is not reported here: it just ends that
                             node's walk -- validate with tva_build_ancestor_mask's err_flag. */

  const int32_t *cu_Q;    /* device int32 [B+1] or NULL.  NULL: every tree node is a query (q, out, lse have
                             sum_T rows).  Else only the LAST cu_Q[b+1]-cu_Q[b] nodes of sequence b's tree
                             are queries -- the keys are still all T_b nodes under the ancestor mask -- and
                             q / out / lse have sum_Q = cu_Q[B] rows, row cu_Q[b] + i being node
                             T_b - Tq_b + i.  This is the draft model's attention while the tree is being
                             grown: the nodes of the newest layer attend to the context and to their
                             ancestors in the layers before (paper, Tree Expansion Phase). */
  int32_t sum_Q, max_Q;   /* with cu_Q: cu_Q[B] and a host-side upper bound of the per-sequence count
                             (<= max_T); ignored otherwise */

  /* 8-bit K/V (a widening of the kernel; the paper keeps the cache in 16 bits).  kv_fp8 = 1: k_cache,
     v_cache and, if given, k_tree, v_tree hold one byte per element in the OCP 8-bit floating point
     format E4M3 (1 sign, 4 exponent, 3 mantissa bits, bias 7, no infinities; the NaN codes 0x7F / 0xFF
     must not occur), with the same shapes, and strides counted in elements (= bytes, multiples of 16).
     K = k_scale * value, V = v_scale * value, one scale per tensor (0 is read as 1).  q, out and lse
     are unchanged; the arithmetic is the bf16 path's on the exactly widened values.  D = 128 only. */
  int32_t kv_fp8;
  float k_scale, v_scale;

  /* Optional planning hint: the sum over the batch of min(L[b], max_L), as the host knows it, or 0.
     The launch plan sizes the KV splits for max_L; with cache lengths that differ a lot some splits
     of the shorter sequences are empty and their workgroups idle.  Given the sum, long splits are
     shortened so that the non-empty ones still fit one round of workgroups.  Results do not depend
     on the value (any number gives a valid plan); tva_workspace_bytes and the tva_plan_* queries
     use it the same way, so pass the same value to them. */
  int64_t sum_L;

  int32_t plan_shape; /* a tva_shape; TVA_SHAPE_AUTO (0) = the library chooses */

  /* Optional planning and placement hint: HOST int32 [B], the cache lengths L[b] as the host knows them, or NULL.
     Read during the call, not kept.  Two uses.  In a launch of one workgroup per (sequence, KV head) that fills the
     chip two workgroups to a CU (8 KV heads, 33 .. 64 sequences, few query rows, no KV split), which sequences share
     a CU decides when the launch ends; given the lengths, the library hands the workgroup slots out so that a long
     and a short sequence share one (a ragged batch of 64: 3 % faster, 17 % with an 8-bit cache).  In a launch with
     KV splits, the split length that sum_L only bounds is found by counting the non-empty splits (lengths of 16 K to
     32 K tokens: 3 % shorter splits).  Results do not depend on the values beyond the split length (any values give
     a valid plan); tva_workspace_bytes and the tva_plan_* queries read it the same way, so pass them the same. */
  const int32_t *L_host;
} tva_args;

/*
 * Ancestor masks from parent arrays (paper: Tree Reranking Phase, last
 * paragraph: the attention mask of the linearised subtree; read here as
 * "a node sees itself and the nodes on its path to the root").
 *   parent   device int32 [cu_T[B]]  local parent index per node, -1 = root
 *   cu_T     device int32 [B+1]
 *   max_T    host upper bound of the tree sizes (any value >= 1)
 *   mask_words  words per mask row, >= ceil(max_T/64)
 *   mask     device uint64 [cu_T[B], mask_words], fully overwritten: bit (j%64) of
 *            word (j/64) of row i is set iff j == i or j is an ancestor of i
 *   err_flag device int32[1] or NULL.  If given it must be zero on entry; a node
 *            whose parent is outside [-1, i-1] makes the kernel store
 *            1 + (smallest such global node index) there, and that node's row
 *            then holds only the bits gathered before the bad link.  The call
 *            itself still returns TVA_OK (detection is asynchronous).
 * One launch per decode step serves all layers of the verification pass.
 */
int tva_build_ancestor_mask(const int32_t *parent, const int32_t *cu_T, int32_t B, int32_t max_T,
                            int32_t mask_words, uint64_t *mask, int32_t *err_flag, void *stream);

/*
 * The same masks on the host, with synchronous validation: every pointer here is HOST memory.
 * Meant for validating trees where they are built (the device variant reports a malformed tree
 * only through err_flag, asynchronously) and for tests; the attention never goes through it.
 * Returns TVA_BAD_TREE if some parent[i] lies outside [-1, i-1] (bad_node, if not NULL, receives the
 * smallest such global node index; mask contents are then unspecified), TVA_INVALID_ARG for
 * malformed arguments, else TVA_OK with mask [cu_T[B], mask_words] fully written.
 */
int tva_build_ancestor_mask_host(const int32_t *parent, const int32_t *cu_T, int32_t B, int32_t max_T,
                                 int32_t mask_words, uint64_t *mask, int32_t *bad_node);

/*
 * Scratch bytes tva_tree_verify_attn needs for these shapes.  Only the shape
 * fields, max_L and num_splits are read (no device memory is touched).
 * Returns 0 when a single split is used, (size_t)-1 on invalid arguments.
 */
size_t tva_workspace_bytes(const tva_args *a);

/*
 * Number of KV splits the library will use for these shapes (>= 1), after
 * applying num_splits (0 = automatic) and rounding; -1 on invalid arguments.
 */
int32_t tva_plan_splits(const tva_args *a);

/*
 * Cached keys per KV split for these shapes: split s of sequence b covers cached keys
 * [s*c, min((s+1)*c, L[b])) with c the returned value; the sequence's last non-empty split
 * (split 0 when L[b] = 0) also covers the tree's own keys.  -1 on invalid arguments.
 */
int32_t tva_plan_chunk_keys(const tva_args *a);

/*
 * Which sequence each workgroup slot of the launch takes when tva_args.L_host is given and the launch is one the
 * placement hint applies to (see L_host): writes slot_seq[0 .. n-1] (HOST int32, room for 64), a permutation of
 * 0 .. n-1 with n = B, and returns n; returns 0 (nothing written) when the sequences keep their order, -1 on
 * invalid arguments.  For tests and tools.
 */
int32_t tva_plan_slot_sequences(const tva_args *a, int32_t *slot_seq);

/*
 * Query rows (tree nodes x query heads of one KV head) one workgroup of the attention kernel
 * covers for these shapes: 32, 64, 128 or 256.  With tva_plan_splits it names the launch
 * (workgroups = B * Hkv * ceil(max_T * Hq / Hkv / rows) * splits); meant for tools that tune
 * or report it.  -1 on invalid arguments.
 */
int32_t tva_plan_workgroup_rows(const tva_args *a);

/*
 * The attention itself.  For sequence b, tree node i, query head h (KV head
 * g = h / (Hq/Hkv)) with keys k = the L[b] cached tokens followed by the tree
 * tokens j for which bit j of anc_mask row i is set:
 *     s_k   = scale * <q[b,i,h,:], K[b,k,g,:]>
 *     lse   = log sum_k exp(s_k)
 *     out   = sum_k exp(s_k - lse) * V[b,k,g,:]
 * computed with bf16 inputs, fp32 accumulation, online softmax over KV splits
 * and a final merge of the splits.  Rows whose mask row is empty and L[b] = 0
 * get out = 0, lse = -inf.
 */
int tva_tree_verify_attn(const tva_args *a, void *stream);

/*
 * tva_tree_verify_attn for callers that cannot allocate device memory or have none to hand over
 * for the KV splits: code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  Same arguments, same kernels, same result as tva_tree_verify_attn, except that
 * a->workspace / a->workspace_bytes are ignored: the partial results of the KV splits go to a
 * device array of TVA_STATIC_SCRATCH_BYTES that is part of the library's code object (every GPU
 * the library runs on holds its own copy until the process ends).  The call allocates and frees
 * nothing; the first call on a device looks up the array's address there (hipGetSymbolAddress).
 *   - Shapes whose plan needs more (tva_workspace_bytes(a) > TVA_STATIC_SCRATCH_BYTES) are
 *     refused with TVA_WORKSPACE_TOO_SMALL and nothing is queued; a smaller num_splits, or
 *     tva_tree_verify_attn with a caller-owned workspace, serves them.
 *   - All calls on one GPU share that GPU's array.  The array keeps whatever the last call
 *     left; nothing in it needs to start at zero (each call writes every slot it later reads).
 *     Calls that overlap on one GPU (different streams, or threads) race on it: serialise them,
 *     or use tva_tree_verify_attn with one workspace per stream.
 */
int tva_tree_verify_attn_static(const tva_args *a, void *stream);
size_t tva_static_scratch_bytes(void); /* = TVA_STATIC_SCRATCH_BYTES */

/*
 * The split-KV part of tva_tree_verify_attn alone: same arguments, but the merge of the KV
 * splits is left to the caller.  With S = tva_plan_splits(a):
 *   S == 1: out / lse hold the final result, the workspace is not touched;
 *   S  > 1: the workspace holds the per-split normalised partial outputs, fp32
 *           [S, sum_T*Hq, D], followed by their natural-log LSE, fp32 [S, sum_T*Hq]
 *           (-inf where a sequence is shorter than the split's first key); out / lse are
 *           not written.  tva_merge_splits(ws, ws + S*sum_T*Hq*D, S, sum_T*Hq, D, out, lse)
 *           completes the computation.
 * This is the piece a context-parallel deployment runs per KV shard before gathering the
 * partials (same definition as above, restricted to the split's keys), and what the benchmark
 * times to price the dominant kernel on its own.
 */
int tva_tree_verify_attn_splits(const tva_args *a, void *stream);

/*
 * Merge of split partial results (the step that follows from splitting a
 * softmax over disjoint key sets; also what a context-parallel deployment
 * would run after gathering per-device partials):
 *     lse = log sum_s exp(lse_s),  out = sum_s exp(lse_s - lse) * out_s.
 *   part_out device fp32 [S, n_rows, D]   normalised partial outputs
 *   part_lse device fp32 [S, n_rows]      natural-log partial LSE (-inf = empty)
 *   out      device fp32 [n_rows, D];  lse device fp32 [n_rows]
 */
int tva_merge_splits(const float *part_out, const float *part_lse, int32_t S, int64_t n_rows,
                     int32_t D, float *out, float *lse, void *stream);

/* Instrumented builds only (the library compiled with -DTVA_TIMELINE; any other build returns
 * TVA_UNSUPPORTED): for profiling tools, not for the hot path.  Copies to the HOST buffer dst the time
 * stamps the kernels of the last tva_tree_verify_attn call left, 8 per workgroup, as counts of the
 * GPU's constant 100 MHz clock: workgroup w (x fastest, then y, then z of the attention launch) at
 * dst[8 w + 0..5] = entry, per-sequence scalars arrived, key loop entered, first tile done, all tiles
 * done, result stores issued; block w of the merge launch at dst[8 w + 6..7] = entry, stores issued.
 * Synchronous; the caller synchronises the stream first.  n_workgroups <= 8192 (workgroups beyond that
 * leave no stamps). */
int tva_timeline_read(uint64_t *dst, int32_t n_workgroups);

const char *tva_strerror(int code);

/* Library version and sizeof(tva_args), for a binding to check that it loaded
 * what it expects and mirrors the struct correctly. */
int tva_version(void);
size_t tva_sizeof_args(void);

#ifdef __cplusplus
}
#endif
#endif /* TVA_H */
