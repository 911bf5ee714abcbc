// libtva, device side of draft-tree construction (gfx950): one layer of expansion and the cut of a grown tree to
// its best nodes.  Definitions and argument layout: include/tva_draft.h (paper, "Tree Expansion Phase", "Tree
// Reranking Phase", "Dynamic Expansion Stage").
//
// Kernels:
//   topk_parts_kernel   the HBM-bound part: every row of log-probabilities is cut into pieces of 8192 tokens, one
//                       workgroup of 256 threads per piece holds its 32 tokens per thread in registers (one
//                       coalesced read, nothing read twice) and finds the piece's best K.  Selection without a
//                       sort of the piece: the K-th largest of the 256 thread maxima is a bound that at least K
//                       tokens reach, and almost only the best K do; the few that reach it are gathered in LDS and
//                       put in order by counting, for each, how many are larger.
//   row_merge_kernel    a wave per row merges the pieces' results into the row's best K (skipped when a row is one piece).
//   expand_finish_kernel  one workgroup per sequence: adds the rows' scores and orders the sequence's candidates the
//                       same way.  (expand_finish_small_kernel: both in one launch for sequences of at most 16 rows.)
//   subtree_kernel      one workgroup per tree: rank of every node by (score, index), keep the best, renumber.
//   rank_trees_kernel, rerank_count_kernel   how many nodes the cut keeps: every tree's best scores in order (one
//                       workgroup per tree, by counting), then one workgroup for the batch: the rank-wise means,
//                       their running sums against the cost row, Algorithm 1.
// Everything is compared through one 64-bit key per element: the float mapped to an unsigned integer of the same
// order in the high word, the complement of the index in the low word -- larger key = better, and no two keys of
// one comparison are equal, so every selection below has exactly one answer.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "tva.h"
#include "tva_draft.h"

namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kPieceThreads = 256, kPerThread = 32, kPiece = kPieceThreads * kPerThread;  // 8192 tokens
constexpr int kMaxK = TVA_EXPAND_MAX_K;
constexpr int kMergePerLane = 8;  // a row's pieces x K candidates are merged by one wave: at most 512

// float -> unsigned of the same order (-0.0 first made +0.0, so the two compare equal as numbers do)
__device__ __forceinline__ uint32_t ordered(float x) {
  const uint32_t u = __float_as_uint(x + 0.0f);
  return u ^ ((u >> 31) ? 0xFFFFFFFFu : 0x80000000u);
}
__device__ __forceinline__ float unordered(uint32_t o) {
  return __uint_as_float(o ^ ((o >> 31) ? 0x80000000u : 0xFFFFFFFFu));
}
__device__ __forceinline__ uint64_t make_key(float x, uint32_t index) { return ((uint64_t)ordered(x) << 32) | (uint32_t)~index; }
__device__ __forceinline__ uint64_t max64(uint64_t a, uint64_t b) { return a > b ? a : b; }
__device__ __forceinline__ uint64_t shfl_xor64(uint64_t v, int mask) {
  const uint32_t lo = __shfl_xor((uint32_t)v, mask), hi = __shfl_xor((uint32_t)(v >> 32), mask);
  return ((uint64_t)hi << 32) | lo;
}

__device__ __forceinline__ uint64_t wave_max(uint64_t key) {
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) key = max64(key, shfl_xor64(key, o));
  return key;
}

// Between a wave's LDS writes and its own lanes' reads of what other lanes wrote: the wave's LDS operations run in
// order, so no wait is needed, but the compiler must not move one across the other.
__device__ __forceinline__ void wave_lds_fence() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// rank of `mine` among n keys in LDS = how many of them are larger (every lane reads the same words: broadcasts)
__device__ __forceinline__ int rank_among(const uint64_t *keys, int n, uint64_t mine) {
  int larger = 0;
#pragma unroll 8
  for (int i = 0; i < n; ++i) larger += keys[i] > mine;
  return larger;
}


// ---- Algorithm 1 on a utility and a cost sequence (Dynamic Expansion Stage, Dynamic Reranking Stage) ----
// What a count needs once the per-rank sums are known; called by every thread of a workgroup (a multiple of 64
// threads).  On entry s_u[k] holds, for rank k, the scores of that rank added over the samples in index order (LAYER)
// or their mean (reranking); s_u, s_c: LDS for N doubles each.  The steps and their order are the host routines'
// (tva_cast_breadth_prune, tva_cast_rerank_count): the running sum over k by one thread's additions (LAYER: divided
// by B afterwards), c_k = cost[k] / unit, index j valid unless some chord (u_j - u_i) / (c_j - c_i), i < j, is below C.
struct CountOut {
  int32_t *count;     // [1]
  int32_t *cu_T;      // [B + 1] or NULL: b * count
  double *at;         // [2] or NULL: u and c at the count
  int32_t *err_flag;  // [1] or NULL: 1 when the costs do not increase strictly (count 0)
};

template <bool LAYER>
__device__ __forceinline__ void count_tail(double *s_u, double *s_c, double *s_g, int *s_bad, int *s_keep, int B,
                                           const double *__restrict__ cost, double unit, int N, double C, const CountOut &out) {
  const int tid = threadIdx.x, threads = blockDim.x;
  if (tid == 0) *s_bad = 0, *s_keep = 1;  // (index 1 has no chord: always valid)
  if (tid == 0) reinterpret_cast<unsigned long long *>(s_g + 2 * N)[0] = 0ull;  // (the largest |u| + |C c|, as an ordered integer)
  // (s_u holds room for a multiple of 16: the running sum below reads and writes whole groups)
  for (int k = N + tid; k < ((N + 15) & ~15); k += threads) s_u[k] = 0.0;
  __syncthreads();
  for (int k = tid; k < N; k += threads) {
    s_c[k] = cost[k] / unit;
    if (k > 0 && !(cost[k] / unit > cost[k - 1] / unit)) *s_bad = 1;  // costs must grow with the size
  }
  // the running sum, one addition after the other as the definition has it: one thread, sixteen values fetched from
  // LDS at a time so that only the additions wait for one another
  if (tid == 0) {
    double run = 0.0;
    for (int k0 = 0; k0 < N; k0 += 16) {
      double v[16];
#pragma unroll
      for (int e = 0; e < 16; ++e) v[e] = s_u[k0 + e];
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        run += v[e];
        s_u[k0 + e] = run;  // (past N: the zeros' place, not read again)
      }
    }
  }
  __syncthreads();
  if (LAYER) {  // (Eq. 1 divides the accumulated sums by the number of samples: one division per index, outside the chain)
    for (int k = tid; k < N; k += threads) s_u[k] = s_u[k] / B;
    __syncthreads();
  }
  if (*s_bad) {
    if (tid == 0) {
      if (out.err_flag) atomicCAS(out.err_flag, 0, 1);
      *out.count = 0;
      if (out.at) out.at[0] = out.at[1] = 0.0;
    }
    if (out.cu_T)
      for (int b = tid; b <= B; b += threads) out.cu_T[b] = 0;
    return;
  }
  // Which indices are valid.  The chord from i into j is too flat when (u_j - u_i) / (c_j - c_i) < C; with c rising that
  // is g_j < g_i for g = u - C c, up to rounding.  So j is valid when g_j exceeds the largest g before it by more than
  // a margin that covers every rounding involved (2^-45 of the largest |u| + |C c|: the quotient then clears C by
  // more than 16 units in the last place), invalid when it falls short of it by that margin (that one chord is too
  // flat), and only an index in between -- equal values, a threshold met exactly -- has its chords divided one by
  // one as the definition has them.  s_g: g, then the largest g before each index.
  double *s_G = s_g + N;
  double a_mine = 0.0;
  for (int k = tid; k < N; k += threads) {
    s_g[k] = s_u[k] - C * s_c[k];
    a_mine = fmax(a_mine, fabs(s_u[k]) + fabs(C * s_c[k]));
  }
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) a_mine = fmax(a_mine, __shfl_xor(a_mine, o));
  if ((tid & 63) == 0) atomicMax(reinterpret_cast<unsigned long long *>(s_G + N), (unsigned long long)__double_as_longlong(a_mine));
  __syncthreads();
  if (tid < 64) {
    // the first wave: lane l takes the indices l * per .. l * per + per - 1, the lanes' maxima are scanned, and the
    // lane walks its indices again with what came before them
    const int per = (N + 63) / 64, k0 = tid * per, k1 = k0 + per < N ? k0 + per : N;
    double mine = -INFINITY;
    for (int k = k0; k < k1; ++k) mine = fmax(mine, s_g[k]);
    double before = mine;  // becomes the largest g of the lanes below
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
      const double y = __shfl_up(before, o);
      if (tid >= o) before = fmax(before, y);
    }
    before = __shfl_up(before, 1);
    if (tid == 0) before = -INFINITY;
    for (int k = k0; k < k1; ++k) {
      s_G[k] = before;
      before = fmax(before, s_g[k]);
    }
  }
  __syncthreads();
  const double margin = __longlong_as_double((long long)reinterpret_cast<unsigned long long *>(s_G + N)[0]) * 0x1p-45 + 1e-300;
  for (int j = 1 + tid; j < N; j += threads) {
    const double gap = s_g[j] - s_G[j];
    bool valid = gap > margin;
    if (!valid && !(gap < -margin)) {
      const double uj = s_u[j], cj = s_c[j];
      bool flat = false;
      for (int i = 0; i < j; ++i) flat = flat | ((uj - s_u[i]) / (cj - s_c[i]) < C);
      valid = !flat;
    }
    if (valid) atomicMax(s_keep, j + 1);
  }
  __syncthreads();
  const int keep = *s_keep;
  if (tid == 0) {
    *out.count = keep;
    if (out.at) out.at[0] = s_u[keep - 1], out.at[1] = s_c[keep - 1];
  }
  if (out.cu_T)
    for (int b = tid; b <= B; b += threads) out.cu_T[b] = b * keep;
}

// ---- the best K of every piece of every row ----
// grid (pieces, rows).  part[(row * pieces + piece) * K + j] = key of the piece's j-th best token (0 = none: the
// piece has fewer than K tokens).  Orders are found by counting, for a key, the keys that are larger (keys are unique,
// so the counts of n keys are 0 .. n-1): reads of LDS that all lanes share, no chain of dependent lane exchanges.
template <bool VEC4>
__global__ void __launch_bounds__(kPieceThreads) topk_parts_kernel(const float *__restrict__ logp, int64_t ld, int V, int K,
                                                                  uint64_t *__restrict__ part) {
  __shared__ uint64_t s_max[kPieceThreads];
  __shared__ uint64_t s_top[4 * kMaxK];
  __shared__ uint64_t s_list[64];
  __shared__ uint64_t s_bound, s_wave[4];
  __shared__ int s_count;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int piece = blockIdx.x, row = blockIdx.y;
  const float *src = logp + (size_t)row * ld;
  const int base = piece * kPiece;
  uint64_t key[kPerThread];
  if constexpr (VEC4) {
    // 16 bytes per lane and load: thread t holds tokens base + 1024 i + 4 t + e
    f32x4 x[kPerThread / 4];
#pragma unroll
    for (int i = 0; i < kPerThread / 4; ++i) {
      const int v = base + i * (4 * kPieceThreads) + 4 * tid;
      x[i] = f32x4{0.f, 0.f, 0.f, 0.f};
      if (v < V) x[i] = __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(src + v));  // (V % 4 == 0: no straddling)
    }
#pragma unroll
    for (int i = 0; i < kPerThread / 4; ++i) {
      const int v = base + i * (4 * kPieceThreads) + 4 * tid;
#pragma unroll
      for (int e = 0; e < 4; ++e) key[4 * i + e] = v < V ? make_key(x[i][e], (uint32_t)(v + e)) : 0ull;
    }
  } else {
    float x[kPerThread];
#pragma unroll
    for (int i = 0; i < kPerThread; ++i) {
      const int v = base + i * kPieceThreads + tid;
      x[i] = v < V ? __builtin_nontemporal_load(src + v) : 0.f;
    }
#pragma unroll
    for (int i = 0; i < kPerThread; ++i) {
      const int v = base + i * kPieceThreads + tid;
      key[i] = v < V ? make_key(x[i], (uint32_t)v) : 0ull;
    }
  }
  uint64_t mine = 0;
#pragma unroll
  for (int i = 0; i < kPerThread; ++i) mine = max64(mine, key[i]);
  s_max[tid] = mine;
  if (tid < 4 * kMaxK) s_top[tid] = 0ull;
  if (tid == 0) s_count = 0, s_bound = 0ull;
  __syncthreads();
  // the K-th largest of the 256 thread maxima (0 if fewer than K threads hold a token): the best K of each wave's 64,
  // then the K-th of those 4 K
  if (mine != 0ull) {
    const int r = rank_among(s_max + wave * 64, 64, mine);
    if (r < K) s_top[wave * kMaxK + r] = mine;
  }
  __syncthreads();
  if (tid < 4 * kMaxK) {
    const uint64_t v = s_top[tid];
    if (v != 0ull && rank_among(s_top, 4 * kMaxK, v) == K - 1) s_bound = v;
  }
  __syncthreads();
  // at least K tokens reach the bound (K threads' maxima do) and few more: gather them
  const uint64_t bound = s_bound;
#pragma unroll
  for (int i = 0; i < kPerThread; ++i) {
    if (key[i] >= bound && key[i] != 0ull) {
      const int pos = atomicAdd(&s_count, 1);
      if (pos < 64) s_list[pos] = key[i];
    }
  }
  __syncthreads();
  const int count = s_count;
  uint64_t *dst = part + ((size_t)row * gridDim.x + piece) * K;
  if (count <= 64) {
    if (tid < count) {
      const uint64_t v = s_list[tid];
      const int r = rank_among(s_list, count, v);
      if (r < K) dst[r] = v;
    } else if (tid < K) {
      dst[tid] = 0ull;  // (a piece of fewer than K tokens)
    }
    return;
  }
  // more than 64 tokens reach the bound (a few threads hold most of the piece's large values, as in a row that
  // falls or rises steadily with the token index): K rounds of a search for the maximum over what the threads hold
  for (int j = 0; j < K; ++j) {
    uint64_t best = 0;
#pragma unroll
    for (int i = 0; i < kPerThread; ++i) best = max64(best, key[i]);
    best = wave_max(best);
    if (lane == 0) s_wave[wave] = best;
    __syncthreads();
    const uint64_t top = max64(max64(s_wave[0], s_wave[1]), max64(s_wave[2], s_wave[3]));
    if (tid == 0) dst[j] = top;
#pragma unroll
    for (int i = 0; i < kPerThread; ++i)
      if (key[i] == top) key[i] = 0ull;  // (keys are unique; 0 = nothing left)
    __syncthreads();
  }
}

// ---- per row: its best K out of its pieces' ----
// One wave merges one row: dst[j] = key of the row's j-th best token.  row, surv, tau: the wave's own LDS scratch
// (per_row keys, 64 keys, one key).
__device__ __forceinline__ void merge_row(const uint64_t *__restrict__ src, int pieces, int K, uint64_t *row, uint64_t *surv,
                                          uint64_t *tau_slot, uint64_t *dst) {
  const int lane = threadIdx.x & 63;
  const int per_row = pieces * K;
  uint64_t mine[kMergePerLane];
#pragma unroll
  for (int i = 0; i < kMergePerLane; ++i) {
    mine[i] = lane + 64 * i < per_row ? src[lane + 64 * i] : 0ull;
    if (lane + 64 * i < per_row) row[lane + 64 * i] = mine[i];
  }
  if (lane == 0) *tau_slot = 0ull;
  wave_lds_fence();
  // With K pieces or more, the K-th largest of the pieces' best tokens is a bound that K candidates reach and few
  // more: only those can be among the row's best K.
  if (pieces >= K) {
#pragma unroll
    for (int i = 0; i < kMergePerLane; ++i) {
      const int at = lane + 64 * i;
      if (at < per_row && at % K == 0 && mine[i] != 0ull) {
        int larger = 0;
        for (int q = 0; q < pieces; ++q) larger += row[q * K] > mine[i];
        if (larger == K - 1) *tau_slot = mine[i];
      }
    }
    wave_lds_fence();
  }
  const uint64_t tau = *tau_slot;
  int count = 0;
#pragma unroll
  for (int i = 0; i < kMergePerLane; ++i) {
    const bool in = mine[i] != 0ull && mine[i] >= tau;
    const uint64_t votes = __ballot(in);
    const int pos = count + __popcll(votes & ((1ull << lane) - 1ull));
    if (in && pos < 64) surv[pos] = mine[i];
    count += __popcll(votes);
  }
  wave_lds_fence();
  if (count <= 64) {
    if (lane < count) {
      const uint64_t k = surv[lane];
      const int j = rank_among(surv, count, k);
      if (j < K) dst[j] = k;
    }
  } else {
    // (more than 64 reach the bound: every candidate is ranked among all of the row's)
#pragma unroll
    for (int i = 0; i < kMergePerLane; ++i) {
      if (mine[i] == 0ull) continue;
      const int j = rank_among(row, per_row, mine[i]);
      if (j < K) dst[j] = mine[i];
    }
  }
}

// a wave per row, four rows per workgroup; best[row * K + j]
__global__ void __launch_bounds__(256) row_merge_kernel(const uint64_t *__restrict__ part, int pieces, int K, int rows,
                                                        uint64_t *__restrict__ best) {
  __shared__ uint64_t s_row[4][64 * kMergePerLane];
  __shared__ uint64_t s_surv[4][64];
  __shared__ uint64_t s_tau[4];
  const int wave = threadIdx.x >> 6;
  const int r = blockIdx.x * 4 + wave;
  if (r >= rows) return;  // (no workgroup-wide barrier below: waves are on their own)
  merge_row(part + (size_t)r * pieces * K, pieces, K, s_row[wave], s_surv[wave], &s_tau[wave], best + (size_t)r * K);
}

// ---- per sequence: the candidates' scores, the candidates in order ----
// best: the rows' best K (n * K keys, global memory or LDS); s_key, s_tok: LDS for n * K entries
__device__ __forceinline__ void order_candidates(const uint64_t *best, int n, int K, int r0, const float *__restrict__ score,
                                                 uint64_t *s_key, int32_t *s_tok, float *__restrict__ cand_score,
                                                 int32_t *__restrict__ cand_parent, int32_t *__restrict__ cand_token,
                                                 double *s_sorted = nullptr) {
  const int tid = threadIdx.x, threads = blockDim.x;
  const int total = n * K;
  const size_t out0 = (size_t)r0 * K;
  for (int i = tid; i < total; i += threads) {
    const uint64_t k = best[i];  // (a row has at least K tokens: a real key)
    const float child = score[r0 + i / K] + unordered((uint32_t)(k >> 32));
    s_key[i] = make_key(child, (uint32_t)i);
    s_tok[i] = (int32_t)~(uint32_t)k;
  }
  __syncthreads();
  // the place of a candidate in the sequence's order = the candidates that are better
  for (int i = tid; i < total; i += threads) {
    const uint64_t kx = s_key[i];
    const int place = rank_among(s_key, total, kx);
    cand_score[out0 + place] = unordered((uint32_t)(kx >> 32));
    // (for the count that follows in the same launch: the candidate's value, exp(score) in double precision rounded
    // to float32, as the count's own kernel takes it)
    if (s_sorted) s_sorted[place] = (double)(float)exp((double)unordered((uint32_t)(kx >> 32)));
    cand_parent[out0 + place] = i / K;
    cand_token[out0 + place] = s_tok[i];
  }
}

__global__ void __launch_bounds__(256) expand_finish_kernel(const uint64_t *__restrict__ best, int K,
                                                            const int32_t *__restrict__ cu_N, const float *__restrict__ score,
                                                            float *__restrict__ cand_score, int32_t *__restrict__ cand_parent,
                                                            int32_t *__restrict__ cand_token) {
  __shared__ uint64_t s_key[TVA_EXPAND_MAX_CANDIDATES];
  __shared__ int32_t s_tok[TVA_EXPAND_MAX_CANDIDATES];
  const int b = blockIdx.x;
  const int r0 = cu_N[b], n = cu_N[b + 1] - r0;
  if (n <= 0 || n * K > TVA_EXPAND_MAX_CANDIDATES) return;  // (more rows than the caller's max_N said: nothing written)
  order_candidates(best + (size_t)r0 * K, n, K, r0, score, s_key, s_tok, cand_score, cand_parent, cand_token);
}

// The two steps in one launch for sequences of at most 16 rows of at most 256 piece candidates each (a sequence's
// rows each get a wave of one workgroup of 16): what a single sequence's layer looks like, where a launch more or
// less is a sixth of the call.
constexpr int kSmallRows = 16, kSmallPerRow = 256;
__global__ void __launch_bounds__(64 * kSmallRows) expand_finish_small_kernel(const uint64_t *__restrict__ part, int pieces, int K,
                                                                             const int32_t *__restrict__ cu_N,
                                                                             const float *__restrict__ score,
                                                                             float *__restrict__ cand_score,
                                                                             int32_t *__restrict__ cand_parent,
                                                                             int32_t *__restrict__ cand_token,
                                                                             const double *__restrict__ cost, double unit, double C,
                                                                             CountOut count_out) {
  __shared__ double s_u[kSmallRows * kMaxK], s_c[kSmallRows * kMaxK];
  __shared__ double s_g[2 * kSmallRows * kMaxK + 1];
  __shared__ int s_bad, s_keep;
  __shared__ uint64_t s_row[kSmallRows][kSmallPerRow];
  __shared__ uint64_t s_surv[kSmallRows][64];
  __shared__ uint64_t s_tau[kSmallRows];
  __shared__ uint64_t s_best[kSmallRows * kMaxK];
  __shared__ uint64_t s_key[kSmallRows * kMaxK];
  __shared__ int32_t s_tok[kSmallRows * kMaxK];
  const int wave = threadIdx.x >> 6;
  const int b = blockIdx.x;
  const int r0 = cu_N[b], n = cu_N[b + 1] - r0;
  if (n <= 0 || n > kSmallRows) return;  // (more rows than the caller's max_N said: nothing written)
  if (wave < n)
    merge_row(part + (size_t)(r0 + wave) * pieces * K, pieces, K, s_row[wave], s_surv[wave], &s_tau[wave], s_best + wave * K);
  __syncthreads();
  // a batch of one sequence that also wants the breadth decision: the sorted scores stay in LDS and the count follows
  const bool counted = count_out.count != nullptr;
  order_candidates(s_best, n, K, r0, score, s_key, s_tok, cand_score, cand_parent, cand_token, counted ? s_u : nullptr);
  if (counted) count_tail<true>(s_u, s_c, s_g, &s_bad, &s_keep, 1, cost, unit, n * K, C, count_out);
}

// ---- the best nodes of a grown tree, renumbered ----
__global__ void __launch_bounds__(256) subtree_kernel(const float *__restrict__ score, const int32_t *__restrict__ parent,
                                                      const int32_t *__restrict__ cu_M, const int32_t *__restrict__ cu_T,
                                                      int32_t *__restrict__ old_index, int32_t *__restrict__ new_parent,
                                                      int32_t *__restrict__ err_flag) {
  __shared__ uint64_t s_key[TVA_SUBTREE_MAX_NODES];
  __shared__ int16_t s_new[TVA_SUBTREE_MAX_NODES];  // new index of a kept node, -1 of a dropped one
  const int tid = threadIdx.x, b = blockIdx.x;
  const int m0 = cu_M[b], M = cu_M[b + 1] - m0;
  const int t0 = cu_T[b], keep = cu_T[b + 1] - t0;
  if (keep <= 0) return;
  if (keep > M || M > TVA_SUBTREE_MAX_NODES) {
    if (tid == 0 && err_flag) atomicCAS(err_flag, 0, 1 + b);
    return;
  }
  for (int i = tid; i < M; i += 256) s_key[i] = make_key(score[m0 + i], (uint32_t)i);
  __syncthreads();
  // a node is kept iff fewer than `keep` nodes are better (keys are unique: the ranks are 0 .. M-1)
  for (int i = tid; i < M; i += 256) {
    const uint64_t mine = s_key[i];
    int better = 0;
    for (int j = 0; j < M; ++j) better += s_key[j] > mine;
    s_new[i] = better < keep ? 0 : -1;
  }
  __syncthreads();
  // new index = kept nodes before it
  for (int i = tid; i < M; i += 256) {
    if (s_new[i] < 0) continue;
    int before = 0;
    for (int j = 0; j < i; ++j) before += s_new[j] >= 0;
    old_index[t0 + before] = i;
  }
  __syncthreads();  // (s_new is rewritten below: every thread has finished counting)
  for (int i = tid; i < keep; i += 256) s_new[old_index[t0 + i]] = (int16_t)i;  // (own writes of this workgroup)
  __syncthreads();
  for (int i = tid; i < keep; i += 256) {
    const int old = old_index[t0 + i];
    const int p = parent[m0 + old];
    int np = -1;
    if (p >= 0) {
      np = (p < old && s_new[p] >= 0) ? s_new[p] : -1;
      if (np < 0 && err_flag) atomicCAS(err_flag, 0, 1 + b);
    }
    new_parent[t0 + i] = np;
  }
}

// ---- how many nodes the cut keeps (Dynamic Reranking Stage) ----
// Two launches.  rank_trees_kernel, one workgroup per tree: the tree's N best scores in descending order (place of a
// score = the scores of its tree that come before it: larger, or equal with a lower index), to best[B, N].
// rerank_count_kernel, one workgroup: the arithmetic of the host routine (tva_cast_rerank_count) in its order -- the
// rank-s scores are added over the samples in index order, divided by B, and accumulated over s by one thread;
// c_k = cost[k] / cost[0]; index j stays valid unless some chord (u_j - u_i) / (c_j - c_i), i < j, is below C.
constexpr int kRerankMaxN = 1024;

__global__ void __launch_bounds__(256) rank_trees_kernel(const float *__restrict__ score, int N_tot, int N, float *__restrict__ best) {
  __shared__ float s_x[TVA_SUBTREE_MAX_NODES + 8];
  const int tid = threadIdx.x, j = blockIdx.x;
  const float *row = score + (size_t)j * N_tot;
  const int padded = (N_tot + 7) & ~7;  // (the tail reads as scores that come before nothing)
  for (int i = tid; i < padded; i += 256) s_x[i] = i < N_tot ? row[i] : -INFINITY;
  __syncthreads();
  for (int idx = tid; idx < N_tot; idx += 256) {
    const float mine = s_x[idx];
    int before = 0;
    // (eight reads in flight, and no branches: written with | and &, the compares stay arithmetic)
    for (int i0 = 0; i0 < padded; i0 += 8) {
      float x[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) x[e] = s_x[i0 + e];
#pragma unroll
      for (int e = 0; e < 8; ++e) before += (int)(x[e] > mine) | ((int)(x[e] == mine) & (int)(i0 + e < idx));
    }
    if (before < N) best[(size_t)j * N + before] = mine;
  }
}

constexpr int kCountThreads = 1024;
constexpr int kCountStage = 10240;  // floats of LDS for the trees' best scores (64 samples x 144 candidates fit)

// LAYER = true is the per-layer form (Eq. 1 and Eq. 2 as tva_cast_breadth_prune writes them): best = the layer's
// candidates' scores, already in order; the column sums are accumulated first and the running sum divided by B;
// c_k = cost[k] / unit with the target's cost of one token passed in; at[0], at[1] receive u and c at the kept count.
template <bool LAYER>
__global__ void __launch_bounds__(kCountThreads) rerank_count_kernel(const float *__restrict__ best, int B, const double *__restrict__ cost,
                                                                     double unit, int N, double C, CountOut out, int logs) {
  __shared__ double s_u[kRerankMaxN], s_c[kRerankMaxN];
  __shared__ __align__(8) float s_best[kCountStage];
  __shared__ int s_bad, s_keep;
  const int tid = threadIdx.x;
  // logs: the scores are logarithms of the values the utility adds up (tva_expand_layer's): value = exp(score),
  // evaluated in double precision and rounded to float32
  auto value = [&](float x) { return logs ? (float)exp((double)x) : x; };
  // the trees' best scores, fetched by all threads at once where they fit (one round trip, not one per sample)
  const bool staged = B * N <= kCountStage;
  if (staged)
    for (int e = tid; e < B * N; e += kCountThreads) s_best[e] = value(best[e]);
  __syncthreads();
  for (int k = tid; k < N; k += kCountThreads) {
    double col = 0.0;  // (added in the samples' order)
    if (staged) {
      for (int j = 0; j < B; ++j) col += (double)s_best[j * N + k];
    } else {
      for (int j = 0; j < B; ++j) col += (double)value(best[(size_t)j * N + k]);
    }
    s_u[k] = LAYER ? col : col / B;  // (reranking: the rank-wise batch mean)
  }
  __syncthreads();  // (the staged scores have been added up: their place holds g and its running maximum from here on)
  count_tail<LAYER>(s_u, s_c, reinterpret_cast<double *>(s_best), &s_bad, &s_keep, B, cost, LAYER ? unit : cost[0], N, C, out);
}

int pieces_of(int V) { return (int)(((int64_t)V + kPiece - 1) / kPiece); }

// TVA_OK, or why the shapes are refused (from host values only)
int expand_shapes(const tva_expand_args *a) {
  if (!a || a->B < 0 || a->V < 1 || a->K < 1 || a->K > a->V || a->sum_N < 0) return TVA_INVALID_ARG;
  if (a->K > kMaxK) return TVA_UNSUPPORTED;
  if ((int64_t)pieces_of(a->V) * a->K > 64 * kMergePerLane) return TVA_UNSUPPORTED;  // what one wave merges per row
  if (a->sum_N > 65535) return TVA_UNSUPPORTED;  // rows are the second grid dimension
  return TVA_OK;
}

}  // namespace

extern "C" {

size_t tva_expand_workspace_bytes(const tva_expand_args *a) {
  if (expand_shapes(a) != TVA_OK) return (size_t)-1;
  // the pieces' best K, then the rows' best K
  return (size_t)a->sum_N * (pieces_of(a->V) + 1) * a->K * sizeof(uint64_t);
}

int tva_expand_layer(const tva_expand_args *a, void *stream) {
  if (const int rc = expand_shapes(a)) return rc;
  if (a->max_N < 0 || (int64_t)a->max_N * a->K > TVA_EXPAND_MAX_CANDIDATES) return TVA_UNSUPPORTED;
  if (a->B == 0 || a->sum_N == 0) return TVA_OK;
  if (!a->cu_N || !a->score || !a->logp || !a->cand_score || !a->cand_parent || !a->cand_token || !a->workspace ||
      a->ld_logp < a->V || ((uintptr_t)a->workspace & 7))
    return TVA_INVALID_ARG;
  if (a->workspace_bytes < tva_expand_workspace_bytes(a)) return TVA_WORKSPACE_TOO_SMALL;
  // the breadth decision on the sorted candidates, if asked for: every sequence the same number of rows
  const bool counted = a->count != nullptr;
  const int n_cand = a->max_N * a->K;
  if (counted && (!a->draft_cost_row || !(a->target_cost_one > 0.0) || (int64_t)a->B * a->max_N != a->sum_N)) return TVA_INVALID_ARG;
  if (counted && n_cand > kRerankMaxN) return TVA_UNSUPPORTED;
  const CountOut count_out{a->count, nullptr, a->u_c_at, a->count_err_flag};
  const CountOut no_count{nullptr, nullptr, nullptr, nullptr};
  const int pieces = pieces_of(a->V);
  uint64_t *part = static_cast<uint64_t *>(a->workspace);
  hipStream_t st = (hipStream_t)stream;
  (void)hipGetLastError();  // the status below is these launches'
  const dim3 grid(pieces, a->sum_N);
  // 16-byte loads need every row to start on 16 bytes and no group of four to straddle the row's end
  const bool vec = a->V % 4 == 0 && a->ld_logp % 4 == 0 && ((uintptr_t)a->logp & 15) == 0;
  if (vec) hipLaunchKernelGGL(topk_parts_kernel<true>, grid, dim3(kPieceThreads), 0, st, a->logp, a->ld_logp, a->V, a->K, part);
  else hipLaunchKernelGGL(topk_parts_kernel<false>, grid, dim3(kPieceThreads), 0, st, a->logp, a->ld_logp, a->V, a->K, part);
  uint64_t *best = part;
  if (pieces > 1 && a->max_N <= kSmallRows && pieces * a->K <= kSmallPerRow) {
    // (a batch of one sequence: the count rides in the same launch)
    const bool fused = counted && a->B == 1;
    hipLaunchKernelGGL(expand_finish_small_kernel, dim3(a->B), dim3(64 * kSmallRows), 0, st, part, pieces, a->K, a->cu_N, a->score,
                       a->cand_score, a->cand_parent, a->cand_token, a->draft_cost_row, a->target_cost_one, a->C1,
                       fused ? count_out : no_count);
    if (counted && !fused)
      hipLaunchKernelGGL(rerank_count_kernel<true>, dim3(1), dim3(kCountThreads), 0, st, a->cand_score, a->B, a->draft_cost_row,
                         a->target_cost_one, n_cand, a->C1, count_out, 1);
    return hipPeekAtLastError() == hipSuccess ? TVA_OK : TVA_HIP_ERROR;
  }
  if (pieces > 1) {
    best = part + (size_t)a->sum_N * pieces * a->K;
    hipLaunchKernelGGL(row_merge_kernel, dim3((a->sum_N + 3) / 4), dim3(256), 0, st, part, pieces, a->K, a->sum_N, best);
  }
  hipLaunchKernelGGL(expand_finish_kernel, dim3(a->B), dim3(256), 0, st, best, a->K, a->cu_N, a->score, a->cand_score,
                     a->cand_parent, a->cand_token);
  if (counted)
    hipLaunchKernelGGL(rerank_count_kernel<true>, dim3(1), dim3(kCountThreads), 0, st, a->cand_score, a->B, a->draft_cost_row,
                       a->target_cost_one, n_cand, a->C1, count_out, 1);
  return hipPeekAtLastError() == hipSuccess ? TVA_OK : TVA_HIP_ERROR;
}

size_t tva_sizeof_expand_args(void) { return sizeof(tva_expand_args); }

int tva_tree_select_subtree(const float *score, const int32_t *parent, const int32_t *cu_M, const int32_t *cu_T, int32_t B,
                            int32_t max_M, int32_t *old_index, int32_t *new_parent, int32_t *err_flag, void *stream) {
  if (B < 0 || max_M < 0) return TVA_INVALID_ARG;
  if (max_M > TVA_SUBTREE_MAX_NODES) return TVA_UNSUPPORTED;
  if (B == 0) return TVA_OK;
  if (!score || !parent || !cu_M || !cu_T || !old_index || !new_parent) return TVA_INVALID_ARG;
  (void)hipGetLastError();
  hipLaunchKernelGGL(subtree_kernel, dim3(B), dim3(256), 0, (hipStream_t)stream, score, parent, cu_M, cu_T, old_index,
                     new_parent, err_flag);
  return hipPeekAtLastError() == hipSuccess ? TVA_OK : TVA_HIP_ERROR;
}

size_t tva_rerank_workspace_bytes(int32_t B, int32_t N_tot, int32_t m) {
  if (B < 1 || N_tot < 1 || m < 1) return (size_t)-1;
  return (size_t)B * (N_tot < m ? N_tot : m) * sizeof(float);
}

int tva_tree_rerank_count(const float *tree_scores, int32_t B, int32_t N_tot, const double *cost_row, int32_t m, double C3,
                          int32_t *count, int32_t *cu_T, int32_t *err_flag, void *workspace, size_t workspace_bytes, void *stream) {
  if (B < 1 || N_tot < 1 || m < 1 || !tree_scores || !cost_row || !count || !workspace || ((uintptr_t)workspace & 3))
    return TVA_INVALID_ARG;
  const int N = N_tot < m ? N_tot : m;
  if (N_tot > TVA_SUBTREE_MAX_NODES || N > kRerankMaxN || B > 65535) return TVA_UNSUPPORTED;
  if (workspace_bytes < tva_rerank_workspace_bytes(B, N_tot, m)) return TVA_WORKSPACE_TOO_SMALL;
  float *best = static_cast<float *>(workspace);
  (void)hipGetLastError();
  hipLaunchKernelGGL(rank_trees_kernel, dim3(B), dim3(256), 0, (hipStream_t)stream, tree_scores, N_tot, N, best);
  hipLaunchKernelGGL(rerank_count_kernel<false>, dim3(1), dim3(kCountThreads), 0, (hipStream_t)stream, best, B, cost_row, 0.0, N, C3,
                     CountOut{count, cu_T, nullptr, err_flag}, 0);
  return hipPeekAtLastError() == hipSuccess ? TVA_OK : TVA_HIP_ERROR;
}

int tva_layer_breadth_count(const float *cand_score, int32_t B, int32_t N, const double *draft_cost_row, double target_cost_one,
                            double C1, int32_t *count, double *u_c_at, int32_t *err_flag, void *stream) {
  if (B < 1 || N < 1 || !cand_score || !draft_cost_row || !count || !(target_cost_one > 0.0)) return TVA_INVALID_ARG;
  if (N > kRerankMaxN) return TVA_UNSUPPORTED;
  (void)hipGetLastError();
  hipLaunchKernelGGL(rerank_count_kernel<true>, dim3(1), dim3(kCountThreads), 0, (hipStream_t)stream, cand_score, B, draft_cost_row,
                     target_cost_one, N, C1, CountOut{count, nullptr, u_c_at, err_flag}, 0);
  return hipPeekAtLastError() == hipSuccess ? TVA_OK : TVA_HIP_ERROR;
}

}  // extern "C"
