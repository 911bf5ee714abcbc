/*
 * libtva_ubench -- microbenchmarks of the MI355X (gfx950) rates the attention kernels are priced
 * against: matrix-instruction issue rate, how much vector work fits under a matrix instruction,
 * v_exp_f32 / v_fma_f32 rates, LDS read bandwidth, streaming reads, empty launches; and one alternative
 * kernel the attention kernels are compared against (attention for very few query rows on the vector
 * ALUs).  A separate library from libtva (measurement aid, not on the hot path); `bench.py --microbench`
 * runs the probes, paper_2510_26577_amd/small_rows.py the comparison.
 *
 * Conventions: every pointer is DEVICE memory the caller owns; `stream` is a hipStream_t as void*;
 * calls queue one kernel and return 0, -1 for bad arguments, -2 for a combination that has no
 * instantiation.  Timed probes write, per wave, {shader-clock cycles, 100 MHz ticks} of their loop to
 * `out` (uint64 [2 * waves], waves = workgroups * threads / 64); `sink` is a float [512] that is never
 * written in practice (it keeps the probe's arithmetic alive).
 */
#ifndef TVA_UBENCH_H
#define TVA_UBENCH_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Per iteration and accumulator: one v_mfma_f32_32x32x16_bf16 (nacc independent accumulators in turn; 0 = no
 * matrix instruction), then k independent v_fma_f32 and e independent v_exp_f32.  Workgroups of
 * 256 * waves_per_simd threads (1 or 2 waves per SIMD). */
int tva_ubench_mfma_valu(int32_t nacc, int32_t k, int32_t e, int32_t waves_per_simd, int32_t workgroups,
                         int32_t iters, uint64_t *out, float *sink, void *stream);

/* Per iteration: 8 x ds_read_b128 (128 bytes per lane) or, with transpose_reads, 16 x ds_read_b64_tr_b16
 * (128 bytes per lane), conflict-free addresses, then a wait for all of them. */
int tva_ubench_lds(int32_t transpose_reads, int32_t waves_per_simd, int32_t workgroups, int32_t iters, uint64_t *out,
                   float *sink, void *stream);

/* Reads `bytes` of `src` once (16 bytes per lane, 8 loads in flight per lane) with `workgroups` workgroups
 * of 256 threads: into registers with the non-temporal hint (to_lds = 0), or straight into LDS without the
 * hint (1) or with it (2, what the attention kernel's tile loads use).  Timed by the caller. */
int tva_ubench_stream(int32_t to_lds, const void *src, size_t bytes, int32_t workgroups, float *sink, void *stream);

/* Every one of `workgroups` workgroups of 256 threads reads the first `bytes` of `src` (a multiple of 32 KiB, small
 * enough to stay in an L2) `reps` times, 16 bytes per lane: into registers, or with to_lds straight into LDS.
 * Delivered bytes = workgroups * reps * bytes.  Timed by the caller. */
int tva_ubench_reread(int32_t to_lds, const void *src, size_t bytes, int32_t reps, int32_t workgroups, float *sink,
                         void *stream);

/* One empty kernel (one wave).  Timed by the caller, back to back. */
int tva_ubench_empty(void *stream);

/* The alternative for very few query rows that the attention kernels of libtva are compared against:
 * tree-verification attention on the vector ALUs only (no matrix instructions, no LDS staging of K/V).
 * Same operation and layouts as tva_tree_verify_attn (include/tva.h; paper, "Tree Reranking Phase": a tree
 * token attends to its sequence's cache and to its ancestors in the tree and itself), for a dense cache
 * and explicit ancestor masks only, without KV splits.  A workgroup of four waves takes four query rows
 * (token, head of the group) of one (sequence, KV head); a wave takes every fourth 64-key tile: lane =
 * key for the scores (each lane reads its key's row and dots it with the rows' q, which sit in LDS),
 * lane = pair of head dimensions for the output (each key's probability is broadcast from its lane).
 * Cost grows with the number of rows; meant for <= 16.
 *   q [sum_Q, Hq, D] bf16; k_cache / v_cache [sum_L, Hkv, D] bf16 at cu_L; k_tree / v_tree [sum_T, Hkv, D] bf16;
 *   mask [sum_T, mask_words] uint64; cu_T, L, cu_L int32 [B + 1], [B], [B + 1]; cu_Q int32 [B + 1] or null
 *   (null: all T_b nodes are queries, else the last cu_Q[b+1] - cu_Q[b]); out fp32 [sum_Q, Hq, D],
 *   lse fp32 [sum_Q, Hq] (natural log).  D is 64 or 128, max_rows = max_b (query nodes) * Hq / Hkv.
 * Returns 0, -1 for bad arguments. */
typedef struct tva_ubench_attn_args {
  const void *q, *k_cache, *v_cache, *k_tree, *v_tree;
  const uint64_t *mask;
  const int32_t *cu_T, *L, *cu_L, *cu_Q;
  int32_t B, Hq, Hkv, D, mask_words, max_rows;
  float scale;
  float *out, *lse;
} tva_ubench_attn_args;
int tva_ubench_valu_attn(const tva_ubench_attn_args *args, void *stream);

#ifdef __cplusplus
}
#endif
#endif
