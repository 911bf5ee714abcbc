// libtva: tree-masked verification attention for gfx950 (MI355X).
//
// Kernels
//   anc_mask_kernel   parent arrays -> ancestor-or-self bitmasks (the attention mask of the
//                     linearised subtree; paper, Tree Reranking Phase, last paragraph)
//   attn_kernel       split-KV attention of all tree tokens of one (sequence, KV head)
//                     against one chunk of that sequence's cache (+ the tree's own
//                     keys under the ancestor mask, folded into the last chunk)
//   merge_kernel      merges the KV splits
//
// attn_kernel in one paragraph.  The T_b*G query rows that share a KV head
// (row = node*G + head-in-group) form the N side of 32x32x16 bf16 MFMAs; keys
// form the M side, so that S^T = K Q^T comes out with one query row per lane
// (row max / row sum need one cross-half exchange, no LDS) and the
// probabilities are already in the B-operand layout of the second product
// O^T = V^T P^T.  K/V tiles are staged once per workgroup in LDS; the V^T
// operand is fetched with the LDS transpose read (ds_read_b64_tr_b16), so V
// stays in its natural [key][d] layout.  Waves of a workgroup are arranged
// WM x WK: WM groups own different query rows, WK groups own different keys of
// each tile and are merged through LDS at the end (used when few rows share a
// KV head, so that the workgroup still has several waves streaming keys).
//
// Every load on the key path is an LDS-writing load the compiler does not track
// (tiles, page-table entries, the tree's parent array), and every wait on them
// is written by hand as a count of the operations queued behind the one waited
// for: left to the compiler, any register it believes pending costs a
// vmcnt(0), which drains the prefetched tiles.
//
// Variants of the inputs handled by the same kernel: dense or paged cache;
// tree K/V in their own tensors or in the cache behind the committed tokens;
// ancestor sets passed as bitmasks or derived here from the parent array; all
// tree nodes as queries or only the last ones of each tree; K/V stored as bf16
// or as 8-bit floating point (E4M3) bytes, which the wave that loaded them
// widens exactly to bf16 inside LDS before the same arithmetic runs.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

#include <algorithm>

#include <atomic>
#include <type_traits>

#include "tva.h"

namespace {

// Instrumented build (-DTVA_TIMELINE, a library of its own): workgroup w of the attention kernel records
// the constant 100 MHz counter at six points of its life, block w of the merge kernel at two; the stamps
// stay in scalar registers until the end of the kernel and lane 0 stores them then, so that the kernel's
// own memory operations are disturbed as little as possible.  tva_timeline_read copies them out.
#ifdef TVA_TIMELINE
constexpr int TL_MAX_WG = 8192, TL_SLOTS = 8;
__device__ unsigned long long timeline[TL_MAX_WG * TL_SLOTS];
#define TL_DECL unsigned long long tl_t[6] = {0, 0, 0, 0, 0, 0}
#define TL_STAMP(i) tl_t[i] = __builtin_amdgcn_s_memrealtime()
#define TL_STORE(wg, first, n)                                                              \
  if (threadIdx.x == 0 && (wg) < TL_MAX_WG)                                                 \
    for (int tl_i = 0; tl_i < (n); ++tl_i) timeline[(size_t)(wg) * TL_SLOTS + (first) + tl_i] = tl_t[tl_i]
#else
#define TL_DECL
#define TL_STAMP(i)
#define TL_STORE(wg, first, n)
#endif

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

#define LDS_PTR(T, p) ((__attribute__((address_space(3))) T *)(p))

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
// A tile takes the low-order P pass when, for some row, (largest probability of the tile) >
// kLoThreshold * (the row's running sum over the keys this wave has seen: both lane halves): then one
// weight can exceed 1/8 of the row's total and its bf16 rounding (2^-8 relative at worst) would be
// visible at the 2e-3 output tolerance.
constexpr float kLoThreshold = 0.125f;
// The reference maximum of a row is only moved (and O, l rescaled) when a tile maximum exceeds it by
// more than 2^kLazy: probabilities then stay below 2^kLazy, harmless in fp32 sums and bf16 operands.
constexpr float kLazy = 8.f;

// ---------------------------------------------------------------------------------------
// ancestor masks
// ---------------------------------------------------------------------------------------
// One workgroup per tree: the parent array is staged in LDS (trees of up to kMaskLds nodes; larger
// ones are walked in global memory), then one thread per node walks its parent chain.  A link that
// does not go strictly downward (or below -1) is reported and ends the walk, so every thread
// finishes in at most T_b steps.
constexpr int kMaskLds = 1024;
__global__ void anc_mask_kernel(const int32_t *__restrict__ parent, const int32_t *__restrict__ cu_T,
                                int B, int W, uint64_t *__restrict__ mask, int32_t *err_flag) {
  __shared__ int32_t spar[kMaskLds];
  const int b = blockIdx.x;
  const int t0 = cu_T[b], T = cu_T[b + 1] - t0;
  const bool in_lds = T <= kMaskLds;
  if (in_lds) {
    for (int i = threadIdx.x; i < T; i += blockDim.x) spar[i] = parent[t0 + i];
    __syncthreads();
  }
  for (int i = threadIdx.x; i < T; i += blockDim.x) {
    uint64_t m[4] = {0, 0, 0, 0};  // W <= 4 handled in registers, larger W goes through memory
    uint64_t *row = mask + (size_t)(t0 + i) * W;
    if (W > 4)
      for (int w = 0; w < W; ++w) row[w] = 0;
    int a = i;
    while (true) {
      if ((a >> 6) < W) {  // a tree larger than the mask row (caller's max_T too small) loses bits, never memory
        if (W <= 4) m[a >> 6] |= 1ull << (a & 63);
        else row[a >> 6] |= 1ull << (a & 63);
      }
      const int p = in_lds ? spar[a] : parent[t0 + a];
      if (p < -1 || p >= a) {
        if (err_flag) {
          // smallest offending global index + 1 (0 = none yet)
          const int code = t0 + a + 1;
          int old = atomicCAS(err_flag, 0, code);
          while (old != 0 && old > code) {
            const int seen = atomicCAS(err_flag, old, code);
            if (seen == old) break;
            old = seen;
          }
        }
        break;
      }
      if (p < 0) break;
      a = p;
    }
    if (W <= 4)
      for (int w = 0; w < W; ++w) row[w] = m[w];
  }
}

// ---------------------------------------------------------------------------------------
// attention
// ---------------------------------------------------------------------------------------
struct AttnParams {
  const __bf16 *q, *k_tree, *v_tree, *k_cache, *v_cache;
  const int32_t *cu_T, *L, *cu_L, *page_table;
  const int32_t *cu_Q;  // null: every tree node is a query; else the last cu_Q[b+1]-cu_Q[b] nodes are
  const uint64_t *mask;
  const int32_t *parent;  // used when mask is null: ancestor masks are derived in the kernel
  float *out, *lse;            // final results
  float *part_out, *part_lse;  // [S, sum_Q, Hq, D], [S, sum_Q, Hq] when S > 1
  int B, Hq, Hkv, G, g_shift, sum_Q, W;  // sum_Q: query rows of the whole batch (= sum_T without cu_Q)
  int chunk_keys, n_chunks, n_row_blocks, max_L;
  int pair_slots;          // > 0: sequences are matched to workgroup slots by length: slot j takes the sequence in
  uint32_t slot_seq[16];   // byte j of this array
  int page_size, page_shift, max_pages;
  int64_t stride_page, stride_tok, stride_head;
  float scale_log2;  // scale * log2(e) (times the K scale of an fp8 cache)
  float v_scale;     // 1, or the V scale of an fp8 cache
};

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// max over the two 32-lane halves (lanes l and l^32 hold the same query row)
__device__ __forceinline__ float half_max(float x) {
  auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float half_sum(float x) {
  auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

template <int D, int WM, int WK, int RB, bool PAGED, int NST, bool KV8 = false>
struct AttnCfg {
  static constexpr int NW = WM * WK;
  static constexpr int NT = NW * 64;
  static constexpr int KBW = (WK == 1) ? (2) : 1;  // 32-key blocks each wave owns in a tile
  static constexpr int TK = WK * KBW * 32;       // keys per tile
  static constexpr int BM = WM * RB * 32;        // query rows per workgroup
  static constexpr int DC = D / 8;               // 16-byte chunks per K/V row
  static constexpr int ROWB = D * 2;             // bytes per K/V row
  static constexpr int RPI = 64 / DC;            // rows one wave-wide 16-byte-per-lane load covers
  // 8-bit K/V: a row is D bytes, a wave-wide load covers twice the rows
  static constexpr int DC8 = D / 16, RPI8 = 64 / DC8;
  static constexpr int NLDK = KV8 ? TK / RPI8 / NW : TK / RPI / NW;  // such loads per wave per tile, for K (same for V)
  static constexpr int NLD = 2 * NLDK;
  // LDS tile layout: NBLK blocks; block n holds rows n, n+NBLK, n+2*NBLK, ... back to back, and
  // blocks are PAD bytes further apart than their size.  Rows that are read together (16
  // consecutive keys, one per lane, by the K operand load; 4 consecutive keys x 32 bytes by one
  // 16-lane group of the V transpose load) then sit in different blocks, PAD apart in bank
  // position, and every read address is one per-lane base plus a compile-time offset.
  static constexpr int NBLK = DC;                // 16 (D=128) or 8 (D=64)
  // 8-bit K/V (see NL below).  Workgroups of up to four waves widen nothing in LDS: the operand reads
  // take the bytes straight from where they landed (8 bytes per lane for K, the 8-bit LDS transpose read
  // for V) and widen them in registers; the ring is four byte tiles, two workgroups fit a CU.  With one
  // row group (WM = 1) every wave reads only the rows it loaded itself and there is no barrier either.
  // (With two row groups each key is widened twice, with eight waves it would be up to eight times:
  // those widen once, cooperatively, through LDS.)
  static constexpr bool KV8_REG = KV8 && NW <= 4;
  static constexpr int SUBS = TK / NBLK;         // rows per block
  static constexpr int BLKB = SUBS * ROWB;       // 1 KiB (TK=64) or 2 KiB (TK=128)
  static constexpr int IPB = BLKB / 1024;        // load instructions per block (16-bit K/V)
  static constexpr int PK = BLKB + 16;           // block pitch of the K tile
  static constexpr int PV = BLKB + 32;           // block pitch of the V tile
  static constexpr int KTILE = NBLK * PK, VTILE = NBLK * PV;
  static constexpr int STAGE_BYTES = KV8_REG ? 2 * TK * D : (KTILE + VTILE + 1023) / 1024 * 1024;
  // NST = stages of the ring (16-bit K/V): NST - 1 tiles are in flight ahead of the one being computed.
  // Two stages of 64-key tiles keep the footprint small enough for two workgroups per CU.
  // 8-bit K/V: the loads land in per-wave zones of NL landing slots (a tile of bytes each); the wave that
  // loaded a piece widens it to bf16 into one of two tiles of the layout above, one tile ahead of
  // the arithmetic.  NL tiles are in flight or being widened.
  static constexpr int NL = KV8_REG ? 0 : KV8 ? NST : 0;
  static constexpr int LAND_SLOT = KV8 ? 2 * TK * D : 0;
  static constexpr int NSTAGE = KV8_REG ? 4 : KV8 ? 2 : NST;
  static constexpr int PD = KV8_REG ? NSTAGE - 1 : KV8 ? NL : NSTAGE - 1;  // tiles in flight ahead of the one being computed (widened)
  static constexpr int WG_PER_CU = KV8 ? (KV8_REG ? 2 : 1) : (NSTAGE == 2 && TK == 64) ? 2 : 1;
  // after the key loop the ring is reused: exchange area of the key-group merge, then (behind it,
  // when the groups are paired; else on top of it, after a barrier) the output transpose patches
  static constexpr bool PAIR = (WK == 2);
  static constexpr int NDW = PAIR ? D / 64 : D / 32;  // 32-wide d blocks of the result each wave writes
  static constexpr int TP = NDW * 32 + 4;             // patch row pitch, floats
  static_assert(WK == 1 || WK == 2, "one key group, or two that are merged pairwise");
  static constexpr int MERGE_BYTES = PAIR ? (2 * WK * WM * RB * 32 * 4 + WM * WK * RB * (D / 64) * 16 * 64 * 4) : 0;
  static constexpr int PATCH_OFF = PAIR ? MERGE_BYTES : 0;
  static constexpr int PATCH_BYTES = (PAIR ? NW : WM) * 32 * TP * 4;
  static constexpr int LAND_OFF = NSTAGE * STAGE_BYTES;
  static constexpr int RING_BYTES = NSTAGE * STAGE_BYTES + NL * LAND_SLOT;
  // paged cache: table entries of the next two tiles, fetched by the same LDS-writing loads as the
  // tiles themselves: [2 slots][wave][load instruction of a tile][lane], behind the ring
  static constexpr int NPG = PAGED ? NLDK : 0;   // table-entry loads per wave and tile
  static constexpr int TILE_OPS = NLD + NPG;     // this wave's memory operations per tile
  static constexpr int PG_SLOT = NW * NLDK * 256;
  static constexpr int PG_BYTES = PAGED ? 2 * PG_SLOT : 0;
  // parent indices of the sequence's tree (used when no ancestor masks are passed), behind those
  static constexpr int PARENT_OFF = RING_BYTES + PG_BYTES;
  static constexpr int PARENT_BYTES = TVA_MAX_TREE * 4;
  static constexpr int TAIL_BYTES = PAIR ? MERGE_BYTES + PATCH_BYTES : (MERGE_BYTES > PATCH_BYTES ? MERGE_BYTES : PATCH_BYTES);
  static constexpr int SMEM = PARENT_OFF + PARENT_BYTES > TAIL_BYTES ? PARENT_OFF + PARENT_BYTES : TAIL_BYTES;
  // load instruction n of a tile (n = wave * NLDK + j): the first tile row it covers
  static constexpr int load_row0(int n) { return KV8 ? n * RPI8 : n / IPB + NBLK * ((n % IPB) * RPI); }
  static_assert(SMEM * WG_PER_CU <= 160 * 1024, "LDS of the workgroups that share a CU");
  static_assert(PD <= 3 && TILE_OPS * (PD > 1 ? PD - 1 : 1) < 64, "the wait counter holds 6 bits");
  static_assert(TK % ((KV8 ? RPI8 : RPI) * NW) == 0, "tile must divide evenly over the waves");
  static_assert(!KV8 || (D == 128 && NLDK >= 1), "8-bit K/V: head dimension 128");
  static_assert(BLKB % 1024 == 0, "a block is a whole number of wave-wide loads");
};

// s_waitcnt immediate that waits for vmcnt <= n only (gfx9 encoding: vmcnt in bits 3:0 and 15:14)
constexpr int vm_cap(int n) { return n > 63 ? 63 : n; }  // the counter holds 6 bits; waiting for less is safe
constexpr int vmcnt_imm(int n) { return (n & 15) | (7 << 4) | (15 << 8) | (((n >> 4) & 3) << 14); }

// Cache policy of the K/V tile loads and of the stores of partial results: the non-temporal hint (the `nt` bit
// of the instruction).  A launch streams K and V through once and its partial rows are read next by another
// kernel; without the hint both displace each other and the rest in the L2s (measured: 3 ... 10 % of the step).
constexpr int kLoadOnce = 2;  // cache-policy operand of the LDS-writing loads: bit 1 = nt
#define GLOBAL_PTR(p) ((const __attribute__((address_space(1))) void *)(p))
typedef __attribute__((address_space(3))) unsigned char lds_byte;

// LDS transpose read of four 16-bit elements per lane (see the V operand comment in attn_kernel),
// issued from inline assembly: the compiler cannot tell these reads apart from the ring stages the
// asynchronous tile loads are still filling and would otherwise drain all outstanding loads
// (vmcnt 0) in front of every one of them.  The matching wait is lds_wait below.
template <int OFF>
__device__ __forceinline__ s16x4 lds_read_tr(uint32_t addr) {
  s16x4 v;
  asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFF));
  return v;
}
// Waits for every outstanding LDS read of this wave; the operands tie the wait to the values.
__device__ __forceinline__ void lds_wait(s16x4 &a, s16x4 &b, s16x4 &c, s16x4 &d) {
  asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(a), "+v"(b), "+v"(c), "+v"(d));
}

// 16-byte LDS read from a landing zone of the 8-bit K/V path (inline assembly for the same reason),
// and its wait.
typedef float f32x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ u32x4 lds_read_b128(uint32_t addr) {
  u32x4 v;
  asm volatile("ds_read_b128 %0, %1" : "=v"(v) : "v"(addr));
  return v;
}
__device__ __forceinline__ void lds_wait(u32x4 &a, u32x4 &b) {
  asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(a), "+v"(b));
}

typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ u32x2 lds_read_b64(uint32_t addr) {
  u32x2 v;
  asm volatile("ds_read_b64 %0, %1" : "=v"(v) : "v"(addr));
  return v;
}
// LDS transpose read of bytes: the 16 lanes of a group pass the addresses of 8 bytes each, rows
// (lane >> 1) of an 8 x 16 byte matrix, columns 8 * (lane & 1) ...; lane j of the group receives
// column j, rows 0 .. 7.
__device__ __forceinline__ u32x2 lds_read_tr8(uint32_t addr) {
  u32x2 v;
  asm volatile("ds_read_b64_tr_b8 %0, %1" : "=v"(v) : "v"(addr));
  return v;
}
__device__ __forceinline__ void lds_wait(u32x2 &a, u32x2 &b, u32x2 &c, u32x2 &d) {
  asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(a), "+v"(b), "+v"(c), "+v"(d));
}
// 8 E4M3 bytes -> 8 bf16
__device__ __forceinline__ bf16x8 widen_e4m3(const u32x2 raw) {
  bf16x8 out;
#pragma unroll
  for (int w = 0; w < 2; ++w) {
    const f32x2 a = __builtin_amdgcn_cvt_pk_f32_fp8((int)raw[w], false);
    const f32x2 b = __builtin_amdgcn_cvt_pk_f32_fp8((int)raw[w], true);
    out[4 * w + 0] = (__bf16)a[0];
    out[4 * w + 1] = (__bf16)a[1];
    out[4 * w + 2] = (__bf16)b[0];
    out[4 * w + 3] = (__bf16)b[1];
  }
  return out;
}
// 16 E4M3 bytes -> 16 bf16 (exact: every E4M3 value is a bf16 value)
__device__ __forceinline__ void widen_e4m3(const u32x4 raw, bf16x8 &lo, bf16x8 &hi) {
#pragma unroll
  for (int w = 0; w < 4; ++w) {
    const f32x2 a = __builtin_amdgcn_cvt_pk_f32_fp8((int)raw[w], false);
    const f32x2 b = __builtin_amdgcn_cvt_pk_f32_fp8((int)raw[w], true);
    bf16x8 &dst = w < 2 ? lo : hi;
    const int o = (w & 1) * 4;
    dst[o + 0] = (__bf16)a[0];
    dst[o + 1] = (__bf16)a[1];
    dst[o + 2] = (__bf16)b[0];
    dst[o + 3] = (__bf16)b[1];
  }
}

template <int D, int WM, int WK, int RB, bool PAGED, int NST, bool KV8>
__global__ void __launch_bounds__(WM *WK * 64, (AttnCfg<D, WM, WK, RB, PAGED, NST, KV8>::WG_PER_CU))
    attn_kernel(const AttnParams p_in) {
  using C = AttnCfg<D, WM, WK, RB, PAGED, NST, KV8>;
  // The arguments the prologue needs, tied together by an empty statement so that they are fetched
  // in one batch at the top rather than one by one, each with its own wait, at their first uses.
  AttnParams p = p_in;
  asm("" : "+s"(p.cu_T), "+s"(p.L), "+s"(p.cu_L), "+s"(p.q), "+s"(p.k_cache), "+s"(p.v_cache), "+s"(p.mask),
      "+s"(p.stride_tok), "+s"(p.stride_head), "+s"(p.G), "+s"(p.g_shift), "+s"(p.Hq), "+s"(p.chunk_keys),
      "+s"(p.n_chunks), "+s"(p.max_L));
  constexpr int TK = C::TK, BM = C::BM, DC = C::DC, ROWB = C::ROWB, RPI = C::RPI, NLDK = C::NLDK, NLD = C::NLD;
  constexpr int KBW = C::KBW, NSTAGE = C::NSTAGE, PD = C::PD, STAGE_BYTES = C::STAGE_BYTES;
  constexpr int NBLK = C::NBLK, IPB = C::IPB, PK = C::PK, PV = C::PV, KTILE = C::KTILE;
  constexpr int NS = D / 16;  // k-steps of the QK product
  constexpr int ND = D / 32;  // 32-wide d blocks of the PV product
  extern __shared__ __align__(1024) unsigned char smem[];
  lds_byte *const lds = (lds_byte *)smem;

  TL_DECL;
  TL_STAMP(0);
  // ---- which (sequence, KV head, row block, chunk) ----
  // grid = (Hkv, row blocks, B * splits): the KV head varies fastest in dispatch order
  const int kvh = blockIdx.x;
  const int rblk = blockIdx.y;
  int b = (int)blockIdx.z / p.n_chunks;
  const int chunk = (int)blockIdx.z - b * p.n_chunks;
  if (p.pair_slots > 0) {
    // (a permutation of the sequences, made on the host: see fill_slots; picked with scalar selects, so that the
    // argument block is never indexed by a register)
    uint32_t word = 0;
#pragma unroll
    for (int i = 0; i < 16; ++i) word = (b >> 2) == i ? p.slot_seq[i] : word;
    b = (int)((word >> (8 * (b & 3))) & 0xFFu);
  }

  // every per-sequence scalar is requested before the first one is needed
  // (read through the constant address space: none of these arrays changes while the kernel
  // runs, and saying so keeps the loads scalar wherever they sit)
  typedef const __attribute__((address_space(4))) int32_t const_i32;
  int t0 = ((const_i32 *)(uintptr_t)p.cu_T)[b];
  int t1 = ((const_i32 *)(uintptr_t)p.cu_T)[b + 1];
  int Lb0 = ((const_i32 *)(uintptr_t)p.L)[b];
  int cuL = PAGED ? 0 : ((const_i32 *)(uintptr_t)p.cu_L)[b];
  // (an empty statement that ties them together: keeps the compiler from moving one of the loads
  // down to its first use, where the wave would wait for it alone)
  int q0 = p.cu_Q ? ((const_i32 *)(uintptr_t)p.cu_Q)[b] : 0;
  int q1 = p.cu_Q ? ((const_i32 *)(uintptr_t)p.cu_Q)[b + 1] : 0;
  asm("" : "+s"(t0), "+s"(t1), "+s"(Lb0), "+s"(cuL), "+s"(q0), "+s"(q1));
#ifdef TVA_TIMELINE
  asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");  // the scalars have arrived
  TL_STAMP(1);
#endif
  const int Tb = t1 - t0;
  // query nodes: all T_b of the tree, or (draft-stage use: one expansion layer attends to the layers
  // before it) only its last Tq; tq0 is the first query row of the sequence in q / out / lse
  const int Tq = p.cu_Q ? (q1 - q0 < Tb ? q1 - q0 : Tb) : Tb;
  const int tq0 = p.cu_Q ? q0 : t0;
  const int node_off = Tb - Tq;
  const int R = Tq * p.G;
  if (rblk * BM >= R) return;
  const int Lb = Lb0 < p.max_L ? Lb0 : p.max_L;
  int nc = (Lb + p.chunk_keys - 1) / p.chunk_keys;
  nc = nc < 1 ? 1 : nc;
  if (chunk >= nc) {
    // this sequence has fewer chunks than the launch provides: mark the slot empty for the merge
    for (int row = rblk * BM + (int)threadIdx.x; row < R && row < (rblk + 1) * BM; row += blockDim.x) {
      const int t = p.g_shift >= 0 ? (row >> p.g_shift) : row / p.G, g = row - t * p.G;
      p.part_lse[(size_t)chunk * p.sum_Q * p.Hq + (size_t)(tq0 + t) * p.Hq + kvh * p.G + g] = -INFINITY;
    }
    return;
  }
  const int k0 = chunk * p.chunk_keys;
  const int k1 = (k0 + p.chunk_keys < Lb) ? k0 + p.chunk_keys : Lb;
  const bool has_tree = (chunk == nc - 1);
  const int n_full = (k1 - k0) / TK;               // cache tiles that need no masking
  const int n_ct = (k1 - k0 + TK - 1) / TK;
  const int n_tt = has_tree ? (Tb + TK - 1) / TK : 0;
  const int n_tiles = n_ct + n_tt;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave % WM, wk = wave / WM;
  const int l32 = lane & 31, hh = lane >> 5;

  const bool wave_has_rows = rblk * BM + wm * RB * 32 < R;  // wave-uniform
  // ---- Q operands (B operand of S^T = K Q^T: lane = query row, 8 consecutive d per k-step) ----
  bf16x8 qreg[RB][NS];
  uint64_t mrow[RB][2];
  bool rvalid[RB];
  int64_t orow[RB];  // (global token * Hq + head) of the lane's row
#pragma unroll
  for (int r = 0; r < RB; ++r) {
    const int row = rblk * BM + (wm * RB + r) * 32 + l32;
    rvalid[r] = row < R;
    // rows past the end compute on a copy of the last row (finite data) and are never stored
    const int rowc = rvalid[r] ? row : R - 1;
    const int t = p.g_shift >= 0 ? (rowc >> p.g_shift) : rowc / p.G;
    const int g = rowc - t * p.G;
    orow[r] = (int64_t)(tq0 + t) * p.Hq + kvh * p.G + g;
    const __bf16 *qp = p.q + orow[r] * D + 8 * hh;
#pragma unroll
    for (int s = 0; s < NS; ++s) {
      qreg[r][s] = *(const __attribute__((address_space(1))) bf16x8 *)(uintptr_t)(qp + 16 * s);
    }
    // mask rows are only requested here (rows past the end read their stand-in's); the first use
    // is in the tree tiles, so nothing waits for them before the key loads have been queued
    mrow[r][0] = mrow[r][1] = 0;
    if (has_tree && p.mask != nullptr) {
      const auto *mp = (const __attribute__((address_space(1))) uint64_t *)(uintptr_t)(p.mask + (size_t)(t0 + node_off + t) * p.W);
      mrow[r][0] = mp[0];
      if (p.W > 1) mrow[r][1] = mp[1];
    }
  }

  // ---- running softmax state (log2 domain; m_run is the reference the exponentials use) ----
  float m_run[RB], l_run[RB];
  f32x16 oacc[RB][ND];
#pragma unroll
  for (int r = 0; r < RB; ++r) {
    m_run[r] = -INFINITY;
    l_run[r] = 0.f;
#pragma unroll
    for (int d = 0; d < ND; ++d)
#pragma unroll
      for (int i = 0; i < 16; ++i) oacc[r][d][i] = 0.f;
  }

  // ---- tile loads: global -> LDS directly (16 bytes per lane, 1 KiB per wave instruction) ----
  // Instruction n of a tile fills part n%IPB of block n/IPB; lane l lands at sub-row
  // (n%IPB)*RPI + l/DC of that block, chunk l%DC.  Rows past the tile's limit re-read the last
  // valid row (finite data; their scores are masked to -inf), so LDS never holds stale values.
  // (8-bit K/V: a row is D bytes, instruction n covers rows n*RPI8 .. n*RPI8 + RPI8 - 1 of the tile and
  // lands in the wave's own zone of a landing slot, from where the same lanes widen it to bf16 into
  // the layout above.)
  constexpr int EB = KV8 ? 1 : 2;                 // bytes per K/V element
  constexpr int LDC = KV8 ? C::DC8 : DC;          // lanes (16-byte chunks) per row of a wave-wide load
  const int lsub = lane / LDC, lpos = lane % LDC;
  const int lrow = KV8 ? lsub : NBLK * lsub;      // the lane's row within its load instruction's rows
  // tile row of (load instruction j of this wave, lane 0), and the LDS byte offsets of that
  // instruction's K and V destinations inside a stage (8-bit: inside the wave's zone of a landing
  // slot): wave-uniform.  (Plain expressions: with calls in their place the host pass of the compiler
  // silently drops the kernel's launch stub.)
  auto row0_of = [&](int j) __attribute__((always_inline)) { return C::load_row0(wave * NLDK + j); };
#define kdst_of(j) (KV8 ? (wave * 2 * NLDK + (j)) * 1024 : ((wave * NLDK + (j)) / IPB) * PK + ((wave * NLDK + (j)) % IPB) * 1024)
#define vdst_of(j) (KV8 ? (wave * 2 * NLDK + NLDK + (j)) * 1024 : KTILE + ((wave * NLDK + (j)) / IPB) * PV + ((wave * NLDK + (j)) % IPB) * 1024)
  const char *const kc_bytes = reinterpret_cast<const char *>(p.k_cache);
  const char *const vc_bytes = reinterpret_cast<const char *>(p.v_cache);
  const char *const kt_bytes = reinterpret_cast<const char *>(p.k_tree);
  const char *const vt_bytes = reinterpret_cast<const char *>(p.v_tree);
  const int64_t cache_base = PAGED ? 0 : (int64_t)cuL * p.stride_tok + (int64_t)kvh * p.stride_head;
  // paged cache: each lane needs the page of the row it loads, one table entry per load
  // instruction of a cache tile.  The entries of tile t + 2 are requested right after the loads of
  // tile t have been queued, by LDS-writing loads like the tiles' own, into one of two slots; the
  // wave's memory operations then come in a fixed order and number per tile (every tile, also a
  // tree tile or the last ones, is followed by a request: past the end it re-reads the entry of the
  // last key), which is what the counted waits below rely on.
  lds_byte *const pg_lds = lds + C::RING_BYTES + wave * (NLDK * 256);
  auto request_pages = [&](int t) __attribute__((always_inline)) {
    if (!PAGED) return;
    // a tree tile whose keys live in the cache (no separate tree tensors): positions L_b + node
    const bool tree_in_cache = t >= n_ct && p.k_tree == nullptr;
    const int base = tree_in_cache ? Lb0 + (t - n_ct) * TK : k0 + t * TK;
    const int last = tree_in_cache ? Lb0 + Tb - 1 : k1 - 1;
#pragma unroll
    for (int j = 0; j < NLDK; ++j) {
      int key = base + row0_of(j) + lrow;
      key = key < last ? key : last;
      key = key < 0 ? 0 : key;
      int pidx = p.page_shift >= 0 ? (key >> p.page_shift) : (key / p.page_size);
      pidx = pidx < p.max_pages ? pidx : p.max_pages - 1;  // never past the sequence's row of the table
      const int32_t *src = p.page_table + (int64_t)b * p.max_pages + pidx;
      __builtin_amdgcn_global_load_lds(GLOBAL_PTR(src), pg_lds + (t & 1) * C::PG_SLOT + j * 256, 4, 0, 0);
    }
  };
  // full tiles of a dense cache: a wave-uniform row pointer plus one tile-independent lane offset
  // (8-bit K/V read in place: inside each 1 KiB piece -- 8 rows of 8 chunks -- the lane that lands in
  // slot (row, c) fetches chunk c ^ row ^ (j & 1) of that row, j the piece's index: the 8-byte operand
  // reads and the byte transpose reads then spread over the LDS banks)
  auto chunk_of = [&](int j) __attribute__((always_inline)) { return C::KV8_REG ? (lpos ^ lsub ^ (j & 1)) : lpos; };
  const uint32_t lane_off2[2] = {(uint32_t)lrow * (uint32_t)p.stride_tok * (uint32_t)EB + (uint32_t)chunk_of(0) * 16u,
                                 (uint32_t)lrow * (uint32_t)p.stride_tok * (uint32_t)EB + (uint32_t)chunk_of(1) * 16u};
  auto issue_impl = [&](int t, auto tree_tag) __attribute__((always_inline)) {
    constexpr bool tree = decltype(tree_tag)::value;
    const int base = tree ? (t - n_ct) * TK : k0 + t * TK;
    const int limit = tree ? Tb : k1;
    lds_byte *stage = (KV8 && !C::KV8_REG) ? lds + C::LAND_OFF + (t % (C::NL > 0 ? C::NL : 1)) * C::LAND_SLOT
                                           : lds + (t % NSTAGE) * STAGE_BYTES;
    if (!PAGED && t < n_full) {
#pragma unroll
      for (int j = 0; j < NLDK; ++j) {
        const int64_t urow = cache_base + (int64_t)(base + row0_of(j)) * p.stride_tok;
        const char *ksrc = kc_bytes + urow * EB + lane_off2[j & 1];
        const char *vsrc = vc_bytes + urow * EB + lane_off2[j & 1];
        __builtin_amdgcn_global_load_lds(GLOBAL_PTR(ksrc), stage + kdst_of(j), 16, 0, kLoadOnce);
        __builtin_amdgcn_global_load_lds(GLOBAL_PTR(vsrc), stage + vdst_of(j), 16, 0, kLoadOnce);
      }
    } else {
#pragma unroll
    for (int j = 0; j < NLDK; ++j) {
      const char *ksrc, *vsrc;
      int key = base + row0_of(j) + lrow;
      key = key < limit ? key : limit - 1;
      const int eoff = chunk_of(j) * (16 / EB);  // first element of the lane's 16-byte chunk
      if (tree && p.k_tree != nullptr) {
        const int64_t off = ((int64_t)(t0 + key) * p.Hkv + kvh) * D + eoff;
        ksrc = kt_bytes + off * EB;
        vsrc = vt_bytes + off * EB;
      } else if (tree) {
        // tree keys stored in the cache behind the sequence's L_b committed tokens
        const int pos = Lb0 + key;
        int64_t off;
        if (PAGED) {
          const int pidx = p.page_shift >= 0 ? (pos >> p.page_shift) : (pos / p.page_size);
          const int page = *reinterpret_cast<const __attribute__((address_space(3))) int *>(pg_lds + (t & 1) * C::PG_SLOT + j * 256 + lane * 4);
          off = (int64_t)page * p.stride_page + (int64_t)(pos - pidx * p.page_size) * p.stride_tok +
                (int64_t)kvh * p.stride_head + eoff;
        } else {
          off = cache_base + (int64_t)pos * p.stride_tok + eoff;
        }
        ksrc = kc_bytes + off * EB;
        vsrc = vc_bytes + off * EB;
      } else if (PAGED) {
        const int pidx = p.page_shift >= 0 ? (key >> p.page_shift) : (key / p.page_size);
        const int page = *reinterpret_cast<const __attribute__((address_space(3))) int *>(pg_lds + (t & 1) * C::PG_SLOT + j * 256 + lane * 4);
        const int64_t off = (int64_t)page * p.stride_page + (int64_t)(key - pidx * p.page_size) * p.stride_tok +
                            (int64_t)kvh * p.stride_head + eoff;
        ksrc = kc_bytes + off * EB;
        vsrc = vc_bytes + off * EB;
      } else {
        const int64_t off = cache_base + (int64_t)key * p.stride_tok + eoff;
        ksrc = kc_bytes + off * EB;
        vsrc = vc_bytes + off * EB;
      }
      __builtin_amdgcn_global_load_lds(GLOBAL_PTR(ksrc), stage + kdst_of(j), 16, 0, kLoadOnce);
      __builtin_amdgcn_global_load_lds(GLOBAL_PTR(vsrc), stage + vdst_of(j), 16, 0, kLoadOnce);
    }
    }
  };

  auto issue_tile = [&](int t) __attribute__((always_inline)) {
    if (t >= n_ct) issue_impl(t, std::true_type{});
    else issue_impl(t, std::false_type{});
    request_pages(t + 2);
  };

  // per-lane LDS read bases (row r of a tile: block r % NBLK, sub-row r / NBLK)
  const int L16 = lane & 15, grp1 = (lane >> 4) & 1;
  const int wave_sub = wk * KBW * (32 / NBLK);  // first sub-row of this wave's keys
  const int kbase_off = (l32 % NBLK) * PK + (wave_sub + l32 / NBLK) * ROWB + hh * 16;
  const int vbase_off = KTILE + (4 * hh + (L16 >> 2)) * PV + wave_sub * ROWB + (2 * grp1 + ((L16 & 3) >> 1)) * 16 +
                        ((L16 & 1) << 3);

  // 8-bit K/V read in place: byte offsets, inside a stage, of the lane's K operand of k-step s (key l32
  // of the wave's 32, bytes 16 s + 8 hh of its row) and of its share of the byte transpose read for
  // d block d (row = L16 >> 1 of the 8 x 16 byte matrix is key 4 hh + (row & 3) + 8 (row >> 2), as the
  // probabilities' operand layout pairs them; columns are bytes 32 d + 16 grp1 ...), with the slot
  // permutation the loads apply inside each 1 KiB piece
  int koff8[NS], voff8[ND];
  if constexpr (C::KV8_REG) {
    // piece n of the tile (keys 8 n .. 8 n + 7) was loaded by wave n / NLDK as its piece n % NLDK: its K bytes
    // sit in that wave's zone, its V bytes NLDK pieces further on
    static_assert(!C::KV8_REG || (NLDK % 2 == 0), "the slot permutation's parity bit is the piece's index in its wave's zone");
    auto piece_off = [&](int n) __attribute__((always_inline)) { return ((n / NLDK) * 2 * NLDK + n % NLDK) * 1024; };
    const int kn = wk * 4 + (l32 >> 3), kr = l32 & 7;
#pragma unroll
    for (int s2 = 0; s2 < NS; ++s2) koff8[s2] = piece_off(kn) + ((kr * 8 + (s2 ^ kr ^ (kn & 1))) << 4) + 8 * hh;
    const int row = L16 >> 1, vn = wk * 4 + (row >> 2), vr = 4 * hh + (row & 3);
#pragma unroll
    for (int d = 0; d < ND; ++d)
      voff8[d] = piece_off(vn) + NLDK * 1024 + ((vr * 8 + ((2 * d + grp1) ^ vr ^ (vn & 1))) << 4) + 8 * (L16 & 1);
  }
  constexpr int V8_SECOND = (NLDK >= 4 ? 2 : 2 * NLDK) * 1024;  // keys 16 .. 31 of the wave: two pieces further on

  // ---- one 32-key block of one tile: S^T = K Q^T, online softmax, O^T += V^T P^T ----
  auto compute_block = [&](const lds_byte *stage, auto kb_tag, int base, int limit, bool tree, auto masked_tag) __attribute__((always_inline)) {
    constexpr bool MASKED = decltype(masked_tag)::value;
    constexpr int kb = decltype(kb_tag)::value;
    constexpr int KBOFF = kb * (32 / NBLK) * ROWB;     // this 32-key block inside the wave's part of the tile
    constexpr int V8 = (NBLK == 16) ? 8 * PV : ROWB;   // V rows 8 keys further on
    const int kofs = (wk * KBW + kb) * 32;
    const lds_byte *kp = stage + kbase_off + KBOFF;
    const uint32_t va = (uint32_t)(uintptr_t)(stage + vbase_off);
    f32x16 sacc[RB];
#pragma unroll
    for (int r = 0; r < RB; ++r)
#pragma unroll
      for (int i = 0; i < 16; ++i) sacc[r][i] = 0.f;
    const uint32_t sb8 = (uint32_t)(uintptr_t)stage;  // (8-bit K/V read in place)
    if constexpr (C::KV8_REG) {
      static_assert(!C::KV8_REG || (NS == 8 && ND == 4 && KBW == 1), "8-bit K/V in place: D = 128, one block per wave and tile");
      u32x2 kraw[NS];
#pragma unroll
      for (int s = 0; s < NS; ++s) kraw[s] = lds_read_b64(sb8 + koff8[s]);
      lds_wait(kraw[0], kraw[1], kraw[2], kraw[3]);
      lds_wait(kraw[NS - 4], kraw[NS - 3], kraw[NS - 2], kraw[NS - 1]);
#pragma unroll
      for (int s = 0; s < NS; ++s) {
        const bf16x8 ka = widen_e4m3(kraw[s]);
#pragma unroll
        for (int r = 0; r < RB; ++r)
          sacc[r] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka, qreg[r][s], sacc[r], 0, 0, 0);
      }
    } else {
#pragma unroll
    for (int s = 0; s < NS; ++s) {
      const bf16x8 ka = *reinterpret_cast<const __attribute__((address_space(3))) bf16x8 *>(kp + s * 32);
#pragma unroll
      for (int r = 0; r < RB; ++r)
        sacc[r] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka, qreg[r][s], sacc[r], 0, 0, 0);
    }
    }
    // V^T operands of the first 16 keys: in flight during the softmax arithmetic
    s16x4 vlo[2][ND], vhi[2][ND];
    u32x2 vraw[2][ND];  // (8-bit K/V read in place: one byte transpose read per operand)
#pragma unroll
    for (int d = 0; d < ND; ++d) {
      if constexpr (C::KV8_REG) {
        vraw[0][d] = lds_read_tr8(sb8 + voff8[d]);
      } else {
        vlo[0][d] = lds_read_tr<KBOFF + 0>(va + d * 64);
        vhi[0][d] = lds_read_tr<KBOFF + V8>(va + d * 64);
      }
    }
    // the V^T operand of the PV product over keys 16 s2 .. 16 s2 + 15, d block d
    auto v_operand = [&](int s2, int d) __attribute__((always_inline)) {
      if constexpr (C::KV8_REG) return widen_e4m3(vraw[s2][d]);
      else return __builtin_bit_cast(bf16x8, __builtin_shufflevector(vlo[s2][d], vhi[s2][d], 0, 1, 2, 3, 4, 5, 6, 7));
    };
    // bit i of ok[r]: element i of this lane (key base+kofs+8*(i/4)+4*hh+i%4) may be attended
    unsigned ok[RB];
#pragma unroll
    for (int r = 0; r < RB; ++r) {
      ok[r] = 0xFFFFu;
      if (MASKED) {
        ok[r] = 0;
#pragma unroll
        for (int qd = 0; qd < 4; ++qd) {
          const int p0 = base + kofs + 8 * qd + 4 * hh;  // first of 4 consecutive keys
          unsigned nib;
          if (tree) {
            // bits at or above T_b can never be keys
            const int nbits = limit - (p0 & ~63);
            const uint64_t trim = nbits >= 64 ? ~0ull : nbits <= 0 ? 0ull : (1ull << nbits) - 1;
            const uint64_t mw = ((p0 < 64) ? mrow[r][0] : mrow[r][1]) & trim;
            nib = (unsigned)(mw >> (p0 & 63)) & 0xFu;
          } else {
            const int left = limit - p0;
            nib = left >= 4 ? 0xFu : (left <= 0 ? 0u : ((1u << left) - 1u));
          }
          ok[r] |= nib << (4 * qd);
        }
      }
    }
    bf16x8 pb[2][RB];
    float m_use[RB];
    bool need_lo = false;
#pragma unroll
    for (int r = 0; r < RB; ++r) {
      float sv[16];
      float mx = -INFINITY;
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        sv[i] = sacc[r][i];
        if (MASKED) sv[i] = ((ok[r] >> i) & 1u) ? sv[i] : -INFINITY;
        mx = fmaxf(mx, sv[i]);
      }
      mx = half_max(mx) * p.scale_log2;
      // lazy reference update: only when some row's tile maximum exceeds its reference by > 2^kLazy
      if (__builtin_amdgcn_ballot_w64(mx > m_run[r] + kLazy) != 0) {
        const float m_new = fmaxf(m_run[r], mx);
        const float alpha = (m_new == -INFINITY) ? 1.f : fast_exp2(m_run[r] - m_new);
        m_run[r] = m_new;
        l_run[r] *= alpha;
#pragma unroll
        for (int d = 0; d < ND; ++d)
#pragma unroll
          for (int i = 0; i < 16; ++i) oacc[r][d][i] *= alpha;
      }
      m_use[r] = (m_run[r] == -INFINITY) ? 0.f : m_run[r];
      const float pmax = fast_exp2(mx - m_use[r]);
      float ls = 0.f;
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const float pv = fast_exp2(fmaf(sv[i], p.scale_log2, -m_use[r]));
        ls += pv;
        pb[i / 8][r][i % 8] = (__bf16)pv;
      }
      l_run[r] += ls;
      need_lo = need_lo || (pmax > kLoThreshold * half_sum(l_run[r]));
    }
    // O^T += V^T P^T: first 16 keys while the operands of the second 16 arrive
    constexpr int S2OFF = (16 / NBLK) * ROWB;
    static_assert(ND == 4 || ND == 2, "head dimension 128 or 64");
    if constexpr (C::KV8_REG) lds_wait(vraw[0][0], vraw[0][1], vraw[0][ND - 2], vraw[0][ND - 1]);
    else if constexpr (ND == 4) lds_wait(vlo[0][0], vlo[0][1], vlo[0][2], vlo[0][3]), lds_wait(vhi[0][0], vhi[0][1], vhi[0][2], vhi[0][3]);
    else lds_wait(vlo[0][0], vlo[0][1], vhi[0][0], vhi[0][1]);
#pragma unroll
    for (int d = 0; d < ND; ++d) {
      if constexpr (C::KV8_REG) {
        vraw[1][d] = lds_read_tr8(sb8 + voff8[d] + V8_SECOND);
      } else {
        vlo[1][d] = lds_read_tr<KBOFF + S2OFF>(va + d * 64);
        vhi[1][d] = lds_read_tr<KBOFF + S2OFF + V8>(va + d * 64);
      }
    }
#pragma unroll
    for (int d = 0; d < ND; ++d) {
      const bf16x8 vop = v_operand(0, d);
#pragma unroll
      for (int r = 0; r < RB; ++r)
        oacc[r][d] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vop, pb[0][r], oacc[r][d], 0, 0, 0);
    }
    if constexpr (C::KV8_REG) lds_wait(vraw[1][0], vraw[1][1], vraw[1][ND - 2], vraw[1][ND - 1]);
    else if constexpr (ND == 4) lds_wait(vlo[1][0], vlo[1][1], vlo[1][2], vlo[1][3]), lds_wait(vhi[1][0], vhi[1][1], vhi[1][2], vhi[1][3]);
    else lds_wait(vlo[1][0], vlo[1][1], vhi[1][0], vhi[1][1]);
#pragma unroll
    for (int d = 0; d < ND; ++d) {
      const bf16x8 vop = v_operand(1, d);
#pragma unroll
      for (int r = 0; r < RB; ++r)
        oacc[r][d] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vop, pb[1][r], oacc[r][d], 0, 0, 0);
    }
    // low-order pass (rare): the bf16 rounding remainder of P, recomputed from the scores
    if (__builtin_amdgcn_ballot_w64(need_lo) != 0) {
      bf16x8 plo[2][RB];
#pragma unroll
      for (int r = 0; r < RB; ++r)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          float sv = sacc[r][i];
          if (MASKED) sv = ((ok[r] >> i) & 1u) ? sv : -INFINITY;
          const float pv = fast_exp2(fmaf(sv, p.scale_log2, -m_use[r]));
          plo[i / 8][r][i % 8] = (__bf16)(pv - (float)pb[i / 8][r][i % 8]);
        }
#pragma unroll
      for (int s2 = 0; s2 < 2; ++s2)
#pragma unroll
        for (int d = 0; d < ND; ++d) {
          const bf16x8 vop = v_operand(s2, d);
#pragma unroll
          for (int r = 0; r < RB; ++r)
            oacc[r][d] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vop, plo[s2][r], oacc[r][d], 0, 0, 0);
        }
    }
  };

  // ---- wait until this wave's loads of tile `it` (and, paged, the table entries the tile queued
  // next needs) have landed: all but the operations queued after them are complete ----
  auto wait_tile = [&](int it) __attribute__((always_inline)) {
    constexpr int OPS = C::TILE_OPS;
    const int later = n_tiles - 1 - it;  // tiles after `it` whose loads are already queued: min(later, PD - 1)
    if constexpr (PAGED) {
      // queued after the loads of tile `it`: entries(it+2), then per later tile its loads and the
      // entries two tiles on.  entries(it+PD) are needed next, so at most one later tile may stay.
      if (PD >= 2 && later >= 1) __builtin_amdgcn_s_waitcnt(vmcnt_imm(OPS));
      else if (PD == 1) __builtin_amdgcn_s_waitcnt(vmcnt_imm(C::NPG));
      else __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
    } else {
      if (PD >= 3 && later >= 2) __builtin_amdgcn_s_waitcnt(vmcnt_imm(NLD * 2));
      else if (PD >= 2 && later >= 1) __builtin_amdgcn_s_waitcnt(vmcnt_imm(NLD * 1));
      else __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
    }
  };

  // ---- 8-bit K/V widened through LDS: this wave's pieces of tile j, once landed, are widened to bf16 into
  // stage j % NSTAGE, and the landing slot they leave takes the loads of tile j + NL.  A lane widens the 16 bytes it
  // loaded itself (row row0_of(jj) + lsub, 16 head-dimension elements from 16 * lpos): 32 bytes of bf16 ----
  auto land_tile = [&](int j) __attribute__((always_inline)) {
    if constexpr (KV8 && !C::KV8_REG) {
      wait_tile(j);
      const uint32_t land = (uint32_t)(uintptr_t)(lds + C::LAND_OFF + (j % C::NL) * C::LAND_SLOT) + lane * 16;
      lds_byte *stage = lds + (j % NSTAGE) * STAGE_BYTES;
#pragma unroll
      for (int jj = 0; jj < NLDK; ++jj) {
        u32x4 kraw = lds_read_b128(land + kdst_of(jj));
        u32x4 vraw = lds_read_b128(land + vdst_of(jj));
        lds_wait(kraw, vraw);
        const int r = row0_of(jj) + lsub;
        const int at = (r / NBLK) * ROWB + lpos * 32;
        bf16x8 lo, hi;
        widen_e4m3(kraw, lo, hi);
        auto *kd = reinterpret_cast<__attribute__((address_space(3))) bf16x8 *>(stage + (r % NBLK) * PK + at);
        kd[0] = lo;
        kd[1] = hi;
        widen_e4m3(vraw, lo, hi);
        auto *vd = reinterpret_cast<__attribute__((address_space(3))) bf16x8 *>(stage + KTILE + (r % NBLK) * PV + at);
        vd[0] = lo;
        vd[1] = hi;
      }
      asm volatile("" ::: "memory");  // the slot is refilled below this line, not above
      if (j + PD < n_tiles) issue_tile(j + PD);
    }
  };

  // ---- one pipeline step: wait for tile `it`, refill the stage tile it-1 used, compute ----
  auto step = [&](int it, auto masked_tag, auto tree_tag) __attribute__((always_inline)) {
    if constexpr (KV8 && !C::KV8_REG) {
      // everyone's widened part of tile `it` is in LDS (the wait covers this wave's LDS writes);
      // everyone is done with tile it-1, whose stage tile it+1 is widened into next
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
      __builtin_amdgcn_s_barrier();
      if (it + 1 < n_tiles) land_tile(it + 1);
    } else {
    // this wave's loads of tile `it` have landed once at most the later tiles' loads are outstanding
    wait_tile(it);
    // everyone's part of tile `it` is in LDS; everyone is done with tile it-1 (no barrier where a wave
    // reads only the bytes it loaded itself)
    if (!(C::KV8_REG && WM == 1)) __builtin_amdgcn_s_barrier();
    if (it + PD < n_tiles) issue_tile(it + PD);
    }
    constexpr bool tree = decltype(tree_tag)::value;
    const int base = tree ? (it - n_ct) * TK : k0 + it * TK;
    const int limit = tree ? Tb : k1;
    const lds_byte *stage = lds + (it % NSTAGE) * STAGE_BYTES;
    {
    // wave-uniform: a block is skipped when none of its keys exists, and all of them by a wave
    // none of whose query rows exists (it still loads its share of every tile)
    if (!wave_has_rows) return;
    if (base + wk * KBW * 32 < limit) compute_block(stage, std::integral_constant<int, 0>{}, base, limit, tree, masked_tag);
    if constexpr (KBW > 1)
      if (base + (wk * KBW + 1) * 32 < limit) compute_block(stage, std::integral_constant<int, 1>{}, base, limit, tree, masked_tag);
    if constexpr (KBW > 2)
      if (base + (wk * KBW + 2) * 32 < limit) compute_block(stage, std::integral_constant<int, 2>{}, base, limit, tree, masked_tag);
    if constexpr (KBW > 3)
      if (base + (wk * KBW + 3) * 32 < limit) compute_block(stage, std::integral_constant<int, 3>{}, base, limit, tree, masked_tag);
    }
  };

  // No ancestor masks passed: the tree's parent array goes to LDS (by the first two waves, with the
  // same LDS-writing loads as everything else here, so it is covered by the counted wait below).
  const bool derive_masks = has_tree && p.mask == nullptr;
  if (derive_masks && wave < 2) {
    int idx = wave * 64 + lane;
    idx = idx < Tb ? idx : Tb - 1;
    __builtin_amdgcn_global_load_lds(GLOBAL_PTR(p.parent + t0 + idx), lds + C::PARENT_OFF + wave * 256, 4, 0, 0);
  }
  request_pages(0);
  request_pages(1);
  // The first PD tiles (fewer if the chunk has fewer).  Q and the mask rows were requested before
  // them and have arrived once no more than the tiles' own operations are outstanding; that wait
  // sits in the same branch as the loads it counts, so that the number is plainly a constant.
  auto issue_first = [&](auto n_tag) __attribute__((always_inline)) {
    constexpr int n = decltype(n_tag)::value;
#pragma unroll
    for (int t = 0; t < n; ++t) {
      if constexpr (PAGED) {
        // entries(t) have landed once only what was queued after them is outstanding
        if (t == 0) __builtin_amdgcn_s_waitcnt(vmcnt_imm(C::NPG));
        else __builtin_amdgcn_s_waitcnt(vmcnt_imm(C::TILE_OPS));
        asm volatile("" ::: "memory");  // the entries are read from LDS below this line, not above
      }
      issue_tile(t);
    }
    __builtin_amdgcn_s_waitcnt(vmcnt_imm(vm_cap(2 * C::NPG + C::TILE_OPS * n)));
  };
  if (PD >= 3 && n_tiles >= 3) issue_first(std::integral_constant<int, PD >= 3 ? 3 : 1>{});
  else if (PD >= 2 && n_tiles >= 2) issue_first(std::integral_constant<int, PD >= 2 ? 2 : 1>{});
  else issue_first(std::integral_constant<int, 1>{});
  if (derive_masks) {
    // Every wave has waited for its own loads queued before the tiles; after the barrier the parent
    // array is complete.  Each lane walks from its node to the root (paper, Tree Reranking Phase:
    // a token attends to its ancestors; and to itself), at most T_b steps whatever the array holds.
    // (A bare barrier: the fenced one would wait for the tiles in flight too.)
    __builtin_amdgcn_s_barrier();
    const auto *par = reinterpret_cast<const __attribute__((address_space(3))) int32_t *>(lds + C::PARENT_OFF);
#pragma unroll
    for (int r = 0; r < RB; ++r) {
      const int row = rblk * BM + (wm * RB + r) * 32 + l32;
      const int rowc = row < R ? row : R - 1;
      int node = node_off + (p.g_shift >= 0 ? (rowc >> p.g_shift) : rowc / p.G);
      uint64_t b0 = 0, b1 = 0;
      for (int step = 0; step < Tb && node >= 0; ++step) {
        if (node < 64) b0 |= 1ull << node;
        else b1 |= 1ull << (node - 64);
        // (read through inline assembly: an ordinary LDS load of memory an LDS-writing load filled
        // makes the compiler drain every outstanding load first, the prefetched tiles included)
        int up;
        asm volatile("ds_read_b32 %0, %1\n\ts_waitcnt lgkmcnt(0)" : "=v"(up) : "v"((uint32_t)(uintptr_t)(par + node)));
        node = up < node ? up : -1;  // a link that does not point backwards ends the walk
      }
      mrow[r][0] = b0;
      mrow[r][1] = b1;
    }
  }
  if constexpr (KV8 && !C::KV8_REG) land_tile(0);
  int it = 0;
  TL_STAMP(2);  // Q and the mask rows have arrived, the first tiles are in flight
#ifdef TVA_TIMELINE
  if (n_full > 0) {
    step(0, std::false_type{}, std::false_type{});
    it = 1;
  }
  TL_STAMP(3);  // first full tile done (a split without one: the same moment as the stamp before)
#endif
  for (; it < n_full; ++it) step(it, std::false_type{}, std::false_type{});
  for (; it < n_ct; ++it) step(it, std::true_type{}, std::false_type{});   // the partial cache tile
  for (; it < n_tiles; ++it) step(it, std::true_type{}, std::true_type{});  // the tree's own keys
  if constexpr (PAGED) __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));  // the last (unused) table entries have landed
  __builtin_amdgcn_s_barrier();  // all waves are done reading the ring before it is reused below
  TL_STAMP(4);  // all tiles done

  // ---- combine the two lane halves' partial sums ----
  float l_tot[RB];
#pragma unroll
  for (int r = 0; r < RB; ++r) l_tot[r] = half_sum(l_run[r]);

  // ---- merge the WK key groups through LDS ----
  // Two key groups: each wave keeps one half of the head dimension and hands the other half to
  // its partner, so both take part in the reduction and in writing the result.
  constexpr bool PAIR = C::PAIR;
  if constexpr (PAIR) {
    constexpr int H = ND / 2;
    float *sm = reinterpret_cast<float *>(smem);            // m then l: [2][WK][WM][RB][32]
    float *sl = sm + WK * WM * RB * 32;
    float *xo = sl + WK * WM * RB * 32;                      // [WM][WK][RB][H][4][64] x 16 bytes
    if (hh == 0) {
#pragma unroll
      for (int r = 0; r < RB; ++r) sm[((wk * WM + wm) * RB + r) * 32 + l32] = m_run[r];
    }
    __syncthreads();
    float a[RB];
#pragma unroll
    for (int r = 0; r < RB; ++r) {
      const float mo = sm[(((1 - wk) * WM + wm) * RB + r) * 32 + l32];
      const float mf = fmaxf(m_run[r], mo);
      a[r] = fast_exp2(m_run[r] - ((mf == -INFINITY) ? 0.f : mf));
      m_run[r] = mf;
      l_tot[r] *= a[r];
      if (hh == 0) sl[((wk * WM + wm) * RB + r) * 32 + l32] = l_tot[r];
    }
    auto swap_halves = [&](auto me_tag) __attribute__((always_inline)) {
      constexpr int me = decltype(me_tag)::value;  // keeps d blocks [me*H, me*H + H), hands over the others
      f32x4 *dst = reinterpret_cast<f32x4 *>(xo) + (size_t)((wm * WK + (1 - me)) * RB * H * 4) * 64;
#pragma unroll
      for (int r = 0; r < RB; ++r)
#pragma unroll
        for (int d = 0; d < H; ++d)
#pragma unroll
          for (int i4 = 0; i4 < 4; ++i4) {
            f32x4 v;
#pragma unroll
            for (int e = 0; e < 4; ++e) v[e] = oacc[r][(1 - me) * H + d][i4 * 4 + e] * a[r];
            dst[((r * H + d) * 4 + i4) * 64 + lane] = v;
          }
      __syncthreads();
      const f32x4 *src = reinterpret_cast<const f32x4 *>(xo) + (size_t)((wm * WK + me) * RB * H * 4) * 64;
#pragma unroll
      for (int r = 0; r < RB; ++r) {
#pragma unroll
        for (int d = 0; d < H; ++d)
#pragma unroll
          for (int i4 = 0; i4 < 4; ++i4) {
            const f32x4 v = src[((r * H + d) * 4 + i4) * 64 + lane];
#pragma unroll
            for (int e = 0; e < 4; ++e)
              oacc[r][me * H + d][i4 * 4 + e] = fmaf(oacc[r][me * H + d][i4 * 4 + e], a[r], v[e]);
          }
        l_tot[r] += sl[(((1 - me) * WM + wm) * RB + r) * 32 + l32];
      }
    };
    if (wk == 0) swap_halves(std::integral_constant<int, 0>{});
    else swap_halves(std::integral_constant<int, 1>{});
  }

  // ---- write (normalised) result: final when there is one split, else the partial ----
  // The accumulators hold O^T (lane = row, registers = 16 scattered d per 32-wide block); each
  // wave transposes one 32-row block at a time through its own LDS patch so that global stores
  // are whole contiguous rows (of the half of the head dimension the wave holds, when paired).
  const bool final_out = (p.n_chunks == 1);
  float *obase = final_out ? p.out : p.part_out + (size_t)chunk * p.sum_Q * p.Hq * D;
  float *lbase = final_out ? p.lse : p.part_lse + (size_t)chunk * p.sum_Q * p.Hq;
  constexpr int NDW = C::NDW;       // 32-wide d blocks this wave writes
  constexpr int TP = C::TP;         // patch row pitch in floats: 16 rows x 16 B apart in bank position
  constexpr int LPR = NDW * 8;      // lanes that cover one row piece with 16 bytes each
  constexpr int RPP = 64 / LPR;     // rows per wave-wide store
  float *tbuf = reinterpret_cast<float *>(smem + C::PATCH_OFF) + (PAIR ? wave : wm) * (32 * TP);
  auto write_out = [&](auto d0_tag, auto once_tag) __attribute__((always_inline)) {
    constexpr int d0 = decltype(d0_tag)::value;  // first d block of this wave's share
    // partial rows (read next by the merge kernel, then dead) are stored with the non-temporal hint; final rows,
    // which the caller's next kernel reads, are left to the caches.  Two copies of the loop: one store whose hint
    // is chosen at run time would lose it.
    constexpr bool ONCE = decltype(once_tag)::value;
#pragma unroll
    for (int r = 0; r < RB; ++r) {
      const float inv = l_tot[r] > 0.f ? p.v_scale / l_tot[r] : 0.f;
#pragma unroll
      for (int d = 0; d < NDW; ++d)
#pragma unroll
        for (int i4 = 0; i4 < 4; ++i4) {
          f32x4 v;
#pragma unroll
          for (int e = 0; e < 4; ++e) v[e] = oacc[r][d0 + d][i4 * 4 + e] * inv;
          *reinterpret_cast<f32x4 *>(tbuf + l32 * TP + 32 * d + 8 * i4 + 4 * hh) = v;
        }
      const int row0 = rblk * BM + (wm * RB + r) * 32;
#pragma unroll
      for (int i = 0; i < 32 / RPP; ++i) {
        const int rl = i * RPP + lane / LPR;
        const int row = row0 + rl;
        const int t = p.g_shift >= 0 ? (row >> p.g_shift) : row / p.G;
        const int64_t og = (int64_t)(tq0 + t) * p.Hq + kvh * p.G + (row - t * p.G);
        const f32x4 v = *reinterpret_cast<const f32x4 *>(tbuf + rl * TP + (lane % LPR) * 4);
        f32x4 *dst = reinterpret_cast<f32x4 *>(obase + og * D + 32 * d0 + (lane % LPR) * 4);
        if (row < R) {
          if constexpr (ONCE) __builtin_nontemporal_store(v, dst);
          else *dst = v;
        }
      }
      if (rvalid[r] && hh == 0 && wk == 0)
        lbase[orow[r]] = l_tot[r] > 0.f ? (m_run[r] + __builtin_amdgcn_logf(l_tot[r])) * kLn2 : -INFINITY;
    }
  };
  auto write_rows = [&](auto d0_tag) __attribute__((always_inline)) {
    if (final_out) write_out(d0_tag, std::false_type{});
    else write_out(d0_tag, std::true_type{});
  };
  if (PAIR && wk == 1) write_rows(std::integral_constant<int, PAIR ? ND / 2 : 0>{});
  else write_rows(std::integral_constant<int, 0>{});
  TL_STAMP(5);  // key groups merged, result stores issued
  TL_STORE(blockIdx.x + gridDim.x * (blockIdx.y + gridDim.y * blockIdx.z), 0, 6);
}
#undef kdst_of
#undef vdst_of

// ---------------------------------------------------------------------------------------
// merge of the KV splits
// ---------------------------------------------------------------------------------------
// One wave per output row (token, head).  The lanes form GROUPS groups of D/4 lanes (16 bytes of
// the row per lane); group g takes the splits g, g + GROUPS, ...  Every load of a block of NI
// splits per group -- the partial rows and their log-sum-exps, clamped to a split that exists --
// is issued before anything is computed from them, so a row costs one memory round trip however
// many splits it has (NI is chosen on the host to cover S where it can).  The groups keep a
// running maximum each and are combined at the end.  Splits whose LSE is -inf (empty, or never
// computed because the sequence is shorter than the launch's split count) get weight zero; their
// O may be uninitialised memory and is dropped by selection, never by multiplication.
template <int D, int NI>
__global__ void __launch_bounds__(256) merge_kernel(const float *__restrict__ part_out,
                                                    const float *__restrict__ part_lse, int S, int64_t n_rows,
                                                    float *__restrict__ out, float *__restrict__ lse) {
  const int lane = threadIdx.x & 63;
  TL_DECL;
  TL_STAMP(0);
  const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= n_rows) return;
  constexpr int LPR = D / 4;        // lanes covering one row with 16 bytes each
  constexpr int GROUPS = 64 / LPR;  // splits processed side by side in one wave
  const int grp = lane / LPR, col = (lane % LPR) * 4;
  float m = -INFINITY, z = 0.f;     // running maximum of the LSEs, sum of weights relative to it
  f32x4 acc = {0.f, 0.f, 0.f, 0.f};
  for (int s0 = grp; s0 < S; s0 += GROUPS * NI) {
    float l[NI];
    f32x4 v[NI];
#pragma unroll
    for (int i = 0; i < NI; ++i) {
      const int s = s0 + i * GROUPS;
      const int sc = s < S ? s : s0;
      l[i] = part_lse[(size_t)sc * n_rows + row];
      v[i] = __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(part_out + ((size_t)sc * n_rows + row) * D + col));
      if (s >= S) l[i] = -INFINITY;
    }
    float mb = m;
#pragma unroll
    for (int i = 0; i < NI; ++i) mb = fmaxf(mb, l[i]);
    if (mb > -INFINITY) {
      const float keep = __expf(m - mb);  // 0 while nothing has been accumulated (m = -inf)
      z *= keep;
#pragma unroll
      for (int e = 0; e < 4; ++e) acc[e] *= keep;
#pragma unroll
      for (int i = 0; i < NI; ++i) {
        const float w = __expf(l[i] - mb);
        z += w;
#pragma unroll
        for (int e = 0; e < 4; ++e) acc[e] += (w != 0.f) ? v[i][e] * w : 0.f;
      }
      m = mb;
    }
  }
#pragma unroll
  for (int o = 32; o >= LPR; o >>= 1) {
    const float m2 = __shfl_xor(m, o), z2 = __shfl_xor(z, o);
    const float mn = fmaxf(m, m2);
    const float k1 = (m > -INFINITY) ? __expf(m - mn) : 0.f, k2 = (m2 > -INFINITY) ? __expf(m2 - mn) : 0.f;
    z = z * k1 + z2 * k2;
#pragma unroll
    for (int e = 0; e < 4; ++e) acc[e] = acc[e] * k1 + __shfl_xor(acc[e], o) * k2;
    m = mn;
  }
  const bool any = z > 0.f;
  if (grp == 0) *reinterpret_cast<f32x4 *>(out + row * D + col) = any ? acc * (1.f / z) : f32x4{0.f, 0.f, 0.f, 0.f};
  if (lane == 0) lse[row] = any ? m + __logf(z) : -INFINITY;
  TL_STAMP(1);  // stores issued
  TL_STORE(blockIdx.x, 6, 2);
}

// NI = splits per lane group and block: the smallest of 1, 2, 4, 8 that covers S in one block
template <int D>
void launch_merge(const float *part_out, const float *part_lse, int S, int64_t n_rows, float *out, float *lse,
                  hipStream_t st) {
  constexpr int GROUPS = 64 / (D / 4);
  const dim3 grid((unsigned)((n_rows + 3) / 4)), block(256);
  const int per_group = (S + GROUPS - 1) / GROUPS;
  if (per_group <= 1) hipLaunchKernelGGL((merge_kernel<D, 1>), grid, block, 0, st, part_out, part_lse, S, n_rows, out, lse);
  else if (per_group <= 2) hipLaunchKernelGGL((merge_kernel<D, 2>), grid, block, 0, st, part_out, part_lse, S, n_rows, out, lse);
  else if (per_group <= 4) hipLaunchKernelGGL((merge_kernel<D, 4>), grid, block, 0, st, part_out, part_lse, S, n_rows, out, lse);
  else hipLaunchKernelGGL((merge_kernel<D, 8>), grid, block, 0, st, part_out, part_lse, S, n_rows, out, lse);
}

// ---------------------------------------------------------------------------------------
// host side: validation, plan, launch
// ---------------------------------------------------------------------------------------

struct Plan {
  int variant;  // index into the kernel table
  int BM, TK;
  int n_row_blocks, n_chunks, chunk_keys;
};

// workgroup shapes (values of tva_shape in tva.h, minus one)
enum { V_K2 = TVA_SHAPE_R32_W2 - 1, V_M2K2 = TVA_SHAPE_R64_W4 - 1, V_M2K2_3 = TVA_SHAPE_R64_W4_DEEP - 1,
       V_M4K2 = TVA_SHAPE_R128_W8 - 1, V_W8 = TVA_SHAPE_R256_W8 - 1, V_LAST = V_W8 };

// query rows of the whole batch: every tree node, or only the nodes cu_Q selects
inline int64_t query_rows(const tva_args *a) { return a->cu_Q ? a->sum_Q : a->sum_T; }

// Which sequence each workgroup slot takes, when the host knows the cache lengths (tva_args.L_host).  An unsplit
// launch of one workgroup per (sequence, KV head) with 8 KV heads and 33 .. 64 sequences, of a shape of which two
// share a CU, fits the chip at once; in dispatch order the heads go round the 8 XCDs and the sequences round an XCD's
// 32 CUs, so that slots j and j + 32 of the B share a CU for the whole launch, and a CU that got two long sequences
// ends it (measured on 64 lengths from U{512..2048}: 73.6 us as drawn, 68.0 with a long and a short one per CU,
// 60.3 with all lengths at their mean).  So: the CUs with one slot get the longest sequences, every other CU a long
// and a short one.  Where workgroups land is the dispatcher's business, not a guarantee: this is a heuristic about
// time, and slot_seq is a permutation whatever L_host holds, so no result depends on it.
void fill_slots(const tva_args *a, const Plan &pl, AttnParams *p) {
  p->pair_slots = 0;
  for (uint32_t &w : p->slot_seq) w = 0;
  const bool two_per_cu = pl.variant == V_K2 || pl.variant == V_M2K2;
  const int n = a->B;
  if (!a->L_host || !two_per_cu || pl.n_chunks != 1 || pl.n_row_blocks != 1 || a->Hkv != 8 || n <= 32 || n > 64) return;
  int order[64];  // sequences, longest first (equal lengths: lower index first)
  for (int i = 0; i < n; ++i) order[i] = i;
  std::stable_sort(order, order + n, [&](int x, int y) { return a->L_host[x] > a->L_host[y]; });
  const int shared = n - 32;  // CUs 0 .. shared-1 of an XCD hold two slots (j and j + 32), the others one
  for (int j = 0; j < n; ++j) {
    const int rank = j >= 32 ? n - 1 - (j - 32) : j < shared ? (64 - n) + j : j - shared;
    p->slot_seq[j >> 2] |= (uint32_t)order[rank] << (8 * (j & 3));
  }
  p->pair_slots = n;
}

bool make_plan(const tva_args *a, Plan *pl) {
  if (!a || a->B <= 0 || a->Hq <= 0 || a->Hkv <= 0 || a->Hq % a->Hkv) return false;
  if (a->sum_T < 0 || a->max_T < 0 || a->max_L < 0 || a->num_splits < 0) return false;
  if (a->plan_shape < TVA_SHAPE_AUTO || a->plan_shape > V_LAST + 1) return false;
  const int G = a->Hq / a->Hkv;
  const int rows = (a->cu_Q ? a->max_Q : a->max_T) * G;
  // Workgroup shape, from sweeps over the benchmark shapes and batch / length variations of them.
  // Up to 32 rows per KV head: 32-row workgroups of two waves that split the keys of 64-key tiles.
  // More rows: 64-row workgroups of 2 x 2 waves (two row groups x two key groups).  Both keep a
  // two-stage ring, small enough that two workgroups share a CU and hide each other's start-up
  // and drain.  From 128 rows on, larger workgroups that read each key fewer times take over
  // where the launch can feed them:
  //  - 128-row workgroups of 4 x 2 waves when 96 .. 256 of them exist (one per CU; with two KV
  //    splits at most, and those 16 tiles or longer);
  //  - 256-row workgroups of eight waves (32 rows each, two waves per SIMD) when there would be more
  //    than 256 of the former, or when there are fewer than 96 but the keys are many: half a million
  //    over the (sequence, KV head) pairs, or half of that with long caches, which splits then
  //    spread over the chip.
  const int pairs = a->B * a->Hkv;
  const int64_t keys = (int64_t)pairs * a->max_L;
  const int n128 = pairs * ((rows + 127) / 128);
  const int s128 = n128 * 3 >= 512 ? 1 : 256 / (n128 > 0 ? n128 : 1);
  int variant = V_M2K2;
  if (rows <= 32) variant = V_K2;
  // (the draft stage's attention of one or two sequences -- queries are the newest nodes, at most 48 rows per KV head:
  // two 32-row workgroups, the second three quarters empty, beat one of 64 rows by 0.4 .. 1.1 us of 12; from eight
  // sequences on the 64-row shape wins)
  else if (a->cu_Q && rows <= 48 && pairs <= 16) variant = V_K2;
  else if (rows >= 128) {
    if (n128 >= 96 && n128 <= 256 && (s128 == 1 || a->max_L / s128 >= 16 * 64)) variant = V_M4K2;
    else if (n128 > 256 || keys >= (512 << 10) || (keys >= (256 << 10) && a->max_L >= 4096)) variant = V_W8;
  }
  // tuning and test aid: the caller names the workgroup shape
  const bool forced = a->plan_shape != TVA_SHAPE_AUTO;
  if (forced) variant = a->plan_shape - 1;
  if (a->kv_fp8 && variant == V_M2K2_3) variant = V_M2K2;  // (8-bit K/V: no deep variant of the 2 x 2 shape)
  pl->variant = variant;
  pl->BM = variant == V_W8 ? 256 : variant == V_M4K2 ? 128 : variant == V_K2 ? 32 : 64;
  pl->TK = 64;
  pl->n_row_blocks = rows > 0 ? (rows + pl->BM - 1) / pl->BM : 1;
  int S = a->num_splits;
  const int max_by_len = a->max_L > 0 ? (a->max_L + pl->TK - 1) / pl->TK : 1;
  const int natural = a->B * a->Hkv * pl->n_row_blocks;
  const bool two_per_cu = variant == V_K2 || variant == V_M2K2;
  if (S == 0 && two_per_cu) {
    // The small shapes (two workgroups fit a CU): the number of splits that minimises a model of the
    // launch's duration, fitted to sweeps of the split count over B = 1 .. 8, caches of 256 .. 2048 keys and
    // trees of 1 .. 72 nodes on the benchmark head shape:
    //   (tiles of the longest split, the tree's own tiles counted with the last one) x time per tile
    //      x 1 while every workgroup has a CU to itself (256), x 1.5 while two share one (512),
    //   + with splits: a merge pass (second launch, 3.0 us) and the partial rows written and read back
    //     (0.30 us per MB).
    // Splits keep two tiles or more (one, in launches of at most 128 workgroups over six tiles or more) and
    // together stay within 512 workgroups.
    const int tiles = max_by_len, tree_tiles = (a->max_T + pl->TK - 1) / pl->TK;
    const double tile_us = 1.30 * a->D / 128.0;
    const double part_mb = 2.0 * query_rows(a) * a->Hq * (a->D + 1) * sizeof(float) * 1e-6;
    double best = 0.0;
    S = 1;
    for (int s = 1; s <= (tiles > 1 ? tiles : 1); ++s) {
      const int ckt = (tiles + s - 1) / s, nch = (tiles + ckt - 1) / ckt;
      if (nch != s) continue;  // the same split length as a smaller count
      const int64_t wgs = (int64_t)natural * nch;
      // splits of one tile only while half the CUs would stay empty otherwise, and not on four or five tiles
      // (measured at 256 keys: the unsplit pass is as fast as four one-tile splits and needs no merge)
      if (ckt < 2 && (wgs > 128 || tiles < 6)) break;
      // (no split once the unsplit launch already has a workgroup for every CU: measured at B = 16 and 32,
      // splitting then only adds the merge)
      if (nch > 1 && (wgs > 512 || natural >= 256)) break;
      const int last = tiles - (nch - 1) * ckt + tree_tiles;
      const int longest = nch > 1 && ckt > last ? ckt : last;
      const double share = wgs <= 256 ? 1.0 : 1.5 * (double)((wgs + 511) / 512);
      double cost = tile_us * longest * share;
      if (nch > 1) cost += 3.0 + 0.30 * part_mb * nch;
      if (s == 1 || cost < best - 1e-9) best = cost, S = nch;
    }
  } else if (S == 0) {
    // one workgroup per CU (256) if the batch allows, but no split shorter than two tiles:
    // every split costs a partial O of the size of the output, written and read back
    S = natural * 3 >= 512 ? 1 : (256 + natural - 1) / natural;  // two thirds of the CUs busy beats a merge pass
    if (S > 1 && natural * S > 256) --S;  // no second round for a few
    const int cap = a->max_L > 0 ? (a->max_L + 2 * pl->TK - 1) / (2 * pl->TK) : 1;
    if (S > cap) S = cap;
    if (S > max_by_len) S = max_by_len;
    // A split has to save more tile time than its merge pass costs (a second launch and the partial rows
    // written and read back: about six tiles' worth): short caches are split less, or not at all.
    while (S > 1 && max_by_len - (max_by_len + S - 1) / S < 6) --S;
  }
  if (S > max_by_len) S = max_by_len;
  if (S < 1) S = 1;
  int ck = a->max_L > 0 ? (a->max_L + S - 1) / S : pl->TK;
  ck = (ck + pl->TK - 1) / pl->TK * pl->TK;
  if (a->num_splits == 0 && S > 1 && a->sum_L > 0 && a->B > 1) {
    // Cache lengths known to differ (their sum is given): the plan above aims at natural * S
    // workgroups, but the splits a shorter sequence does not reach are empty.  Sequence b needs
    // ceil(L_b / c) <= L_b / c + 1 splits of c keys, so with c >= sum_L / (S * B - B) the non-empty
    // ones of the whole batch still number at most S * B per (KV head, row block): one round as
    // planned, of shorter splits.  Only where splits stay long (16 tiles), so that their length and
    // not the fixed cost per workgroup is what the time follows.
    const int64_t slots = (int64_t)S * a->B - a->B;
    int64_t c = (a->sum_L + slots - 1) / slots;
    c = (c + pl->TK - 1) / pl->TK * pl->TK;
    if (c >= 16 * pl->TK && c < ck) ck = (int)c;
  }
  if (a->num_splits == 0 && S > 1 && a->L_host && a->B > 1) {
    // The lengths themselves are known: the shortest split (whole tiles, 16 or more) with which the non-empty
    // splits of the batch still number S * B, counted instead of bounded.
    const int64_t slots = (int64_t)S * a->B;
    auto fits = [&](int c) {
      int64_t n = 0;
      for (int b = 0; b < a->B; ++b) n += a->L_host[b] > 0 ? ((int64_t)a->L_host[b] + c - 1) / c : 1;
      return n <= slots;
    };
    while (ck - pl->TK >= 16 * pl->TK && fits(ck - pl->TK)) ck -= pl->TK;
  }
  pl->chunk_keys = ck;
  pl->n_chunks = a->max_L > 0 ? (a->max_L + ck - 1) / ck : 1;
  // one 2 x 2 workgroup per CU at most and long splits: a third ring stage (two tiles in flight)
  // pays; with more workgroups the second one on the CU hides more than the deeper ring would
  if (pl->variant == V_M2K2 && !forced && !a->kv_fp8 && (int64_t)pairs * pl->n_row_blocks * pl->n_chunks <= 256 && ck >= 12 * pl->TK)
    pl->variant = V_M2K2_3;
  return true;
}

typedef void (*attn_fn)(const AttnParams);

// Launch status.  An error some earlier HIP call of the process left behind is cleared before a
// launch, so that the status reflects this launch only; a failure is left in place (peeked, not
// consumed) for the caller's hipGetLastError, and named on stderr when TVA_VERBOSE is set.
inline void clear_stale_hip_error() { (void)hipGetLastError(); }
inline hipError_t launch_status(const char *what) {
  const hipError_t e = hipPeekAtLastError();
  if (e != hipSuccess && getenv("TVA_VERBOSE")) fprintf(stderr, "libtva: %s: %s\n", what, hipGetErrorString(e));
  return e;
}

template <int D, int WM, int WK, int RB, bool PAGED, int NST, bool KV8 = false>
hipError_t launch_attn(const AttnParams &p, dim3 grid, hipStream_t st) {
  using C = AttnCfg<D, WM, WK, RB, PAGED, NST, KV8>;
  // raising the dynamic-LDS limit is idempotent and needed once per device (and per instantiation)
  static std::atomic<uint64_t> attr_done{0};
  auto kfn = attn_kernel<D, WM, WK, RB, PAGED, NST, KV8>;
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) return hipErrorInvalidDevice;
  const uint64_t bit = (dev >= 0 && dev < 64) ? 1ull << dev : 0;
  if (!(attr_done.load(std::memory_order_relaxed) & bit)) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kfn),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, C::SMEM);
    if (e != hipSuccess) return e;
    attr_done.fetch_or(bit, std::memory_order_relaxed);
  }
  clear_stale_hip_error();
  hipLaunchKernelGGL(kfn, grid, dim3(C::NT), C::SMEM, st, p);
  return launch_status("attention kernel launch");
}

template <int D, bool PAGED>
hipError_t dispatch_variant(int variant, const AttnParams &p, dim3 grid, hipStream_t st) {
  switch (variant) {
    case V_W8: return launch_attn<D, 8, 1, 1, PAGED, 4>(p, grid, st);
    case V_M4K2: return launch_attn<D, 4, 2, 1, PAGED, 4>(p, grid, st);
    case V_M2K2_3: return launch_attn<D, 2, 2, 1, PAGED, 3>(p, grid, st);
    case V_K2: return launch_attn<D, 1, 2, 1, PAGED, 2>(p, grid, st);
    default: return launch_attn<D, 2, 2, 1, PAGED, 2>(p, grid, st);  // V_M2K2
  }
}

// 8-bit K/V (three landing slots each)
template <bool PAGED>
hipError_t dispatch_variant_fp8(int variant, const AttnParams &p, dim3 grid, hipStream_t st) {
  switch (variant) {
    case V_W8: return launch_attn<128, 8, 1, 1, PAGED, 3, true>(p, grid, st);
    case V_M4K2: return launch_attn<128, 4, 2, 1, PAGED, 3, true>(p, grid, st);
    case V_K2: return launch_attn<128, 1, 2, 1, PAGED, 3, true>(p, grid, st);
    default: return launch_attn<128, 2, 2, 1, PAGED, 3, true>(p, grid, st);  // V_M2K2
  }
}

}  // namespace

// ---------------------------------------------------------------------------------------
// scratch memory of tva_tree_verify_attn_static (the entry point that allocates nothing)
// ---------------------------------------------------------------------------------------
// A device array that is part of the code object: every GPU the library runs on holds its own copy,
// at its own address, from the moment the module is loaded there until the process ends.  In host
// code the array's name is only a handle for hipGetSymbolAddress; the address it returns for the
// current device is what kernels, copies and fills are given.  Nothing in it has to start at zero:
// the attention kernel writes every partial row and every partial log-sum-exp (also the "empty"
// marks of splits a short sequence does not reach) that the merge of the same call reads.
static __device__ __align__(256) unsigned char scratch[TVA_STATIC_SCRATCH_BYTES];

namespace {
constexpr int kMaxDevices = 64;
std::atomic<void *> scratch_addr[kMaxDevices];  // zero-initialised: not looked up yet

// Address of `scratch` on the current device; looked up once per device, with that device current.
int static_scratch(void **out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return TVA_HIP_ERROR;
  void *ptr = scratch_addr[dev].load(std::memory_order_acquire);
  if (!ptr) {
    const hipError_t e = hipGetSymbolAddress((void **)&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !ptr) {
      if (getenv("TVA_VERBOSE")) fprintf(stderr, "libtva: hipGetSymbolAddress(scratch): %s\n", hipGetErrorString(e));
      return TVA_HIP_ERROR;
    }
    scratch_addr[dev].store(ptr, std::memory_order_release);  // (two threads racing store the same value)
  }
  *out = ptr;
  return TVA_OK;
}
}  // namespace

extern "C" {

int tva_version(void) { return 7; }

int tva_timeline_read(uint64_t *dst, int32_t n_workgroups) {
#ifdef TVA_TIMELINE
  if (!dst || n_workgroups < 0 || n_workgroups > TL_MAX_WG) return TVA_INVALID_ARG;
  const hipError_t e = hipMemcpyFromSymbol(dst, HIP_SYMBOL(timeline), (size_t)n_workgroups * TL_SLOTS * sizeof(uint64_t), 0,
                                           hipMemcpyDeviceToHost);
  return e == hipSuccess ? TVA_OK : TVA_HIP_ERROR;
#else
  (void)dst;
  (void)n_workgroups;
  return TVA_UNSUPPORTED;
#endif
}

size_t tva_sizeof_args(void) { return sizeof(tva_args); }

const char *tva_strerror(int code) {
  switch (code) {
    case TVA_OK: return "ok";
    case TVA_INVALID_ARG: return "invalid argument";
    case TVA_UNSUPPORTED: return "unsupported shape";
    case TVA_WORKSPACE_TOO_SMALL: return "workspace too small";
    case TVA_HIP_ERROR: return "HIP launch error";
    case TVA_BAD_TREE: return "malformed tree (parent index outside [-1, i-1])";
    default: return "unknown status";
  }
}

int tva_build_ancestor_mask(const int32_t *parent, const int32_t *cu_T, int32_t B, int32_t max_T,
                            int32_t mask_words, uint64_t *mask, int32_t *err_flag, void *stream) {
  if (B < 0 || max_T < 0 || mask_words < 1 || mask_words * 64 < max_T) return TVA_INVALID_ARG;
  if (B == 0) return TVA_OK;
  if (!parent || !cu_T || !mask) return TVA_INVALID_ARG;
  int threads = ((max_T + 63) / 64) * 64;
  threads = threads < 64 ? 64 : (threads > 256 ? 256 : threads);
  clear_stale_hip_error();
  hipLaunchKernelGGL(anc_mask_kernel, dim3(B), dim3(threads), 0, (hipStream_t)stream, parent, cu_T, B,
                     mask_words, mask, err_flag);
  return launch_status("ancestor mask kernel launch") == hipSuccess ? TVA_OK : TVA_HIP_ERROR;
}

static int check_args(const tva_args *a, bool shapes_only) {
  if (!a) return TVA_INVALID_ARG;
  if (a->B <= 0 || a->Hq <= 0 || a->Hkv <= 0 || a->Hq % a->Hkv) return TVA_INVALID_ARG;
  if (a->sum_T < 0 || a->max_T < 0 || a->max_L < 0 || a->num_splits < 0) return TVA_INVALID_ARG;
  if (a->D != 64 && a->D != 128) return TVA_UNSUPPORTED;
  if (a->max_T > TVA_MAX_TREE) return TVA_UNSUPPORTED;
  if (a->mask_words < 1 || a->mask_words > 2 || a->mask_words * 64 < a->max_T) return TVA_UNSUPPORTED;
  if (a->kv_fp8 != 0 && a->kv_fp8 != 1) return TVA_INVALID_ARG;
  if (a->kv_fp8 && a->D != 128) return TVA_UNSUPPORTED;
  if (a->cu_Q && (a->sum_Q < 0 || a->max_Q < 0 || a->max_Q > a->max_T || a->sum_Q > a->sum_T)) return TVA_INVALID_ARG;
  if (a->plan_shape < TVA_SHAPE_AUTO || a->plan_shape > TVA_SHAPE_R256_W8) return TVA_INVALID_ARG;
  if (a->sum_L < 0) return TVA_INVALID_ARG;
  if (shapes_only) return TVA_OK;
  if (!(a->scale > 0.f)) return TVA_INVALID_ARG;
  if (a->sum_T == 0) return TVA_OK;
  if (!a->cu_T || !a->L || !a->q || !a->out || !a->lse) return TVA_INVALID_ARG;
  if ((a->k_tree == nullptr) != (a->v_tree == nullptr)) return TVA_INVALID_ARG;
  if (!a->anc_mask && !a->parent) return TVA_INVALID_ARG;
  const bool dense = a->cu_L != nullptr, paged = a->page_table != nullptr;
  if (dense == paged) return TVA_INVALID_ARG;
  const bool tree_in_cache = a->k_tree == nullptr;
  if ((a->max_L > 0 || tree_in_cache) && (!a->k_cache || !a->v_cache)) return TVA_INVALID_ARG;
  if (paged && (a->page_size <= 0 || a->max_pages <= 0)) return TVA_INVALID_ARG;
  // (with tree rows in the cache the table must cover L[b] + T_b positions of every sequence; only the two
  // bounds are known here, and the longest cache need not belong to the largest tree)
  if (paged && (int64_t)a->max_pages * a->page_size < (tree_in_cache && a->max_T > a->max_L ? a->max_T : a->max_L))
    return TVA_INVALID_ARG;
  if ((a->stride_page | a->stride_tok | a->stride_head) % (a->kv_fp8 ? 16 : 8)) return TVA_INVALID_ARG;  // 16-byte pieces
  if (a->stride_page < 0 || a->stride_tok < 0 || a->stride_head < 0) return TVA_INVALID_ARG;
  if (a->stride_tok >= (1 << 24)) return TVA_UNSUPPORTED;  // lane offsets inside a tile are 32-bit
  if (a->kv_fp8 && (!(a->k_scale >= 0.f) || !(a->v_scale >= 0.f))) return TVA_INVALID_ARG;
  return TVA_OK;
}

int32_t tva_plan_splits(const tva_args *a) {
  if (check_args(a, true) != TVA_OK) return -1;
  Plan pl;
  if (!make_plan(a, &pl)) return -1;
  return pl.n_chunks;
}

int32_t tva_plan_chunk_keys(const tva_args *a) {
  if (check_args(a, true) != TVA_OK) return -1;
  Plan pl;
  if (!make_plan(a, &pl)) return -1;
  return pl.chunk_keys;
}

int32_t tva_plan_slot_sequences(const tva_args *a, int32_t *slot_seq) {
  if (check_args(a, true) != TVA_OK || !slot_seq) return -1;
  Plan pl;
  if (!make_plan(a, &pl)) return -1;
  AttnParams p;
  fill_slots(a, pl, &p);
  for (int j = 0; j < p.pair_slots; ++j) slot_seq[j] = (int32_t)((p.slot_seq[j >> 2] >> (8 * (j & 3))) & 0xFFu);
  return p.pair_slots;
}

int32_t tva_plan_workgroup_rows(const tva_args *a) {
  if (check_args(a, true) != TVA_OK) return -1;
  Plan pl;
  if (!make_plan(a, &pl)) return -1;
  return pl.BM;
}

size_t tva_workspace_bytes(const tva_args *a) {
  if (check_args(a, true) != TVA_OK) return (size_t)-1;
  Plan pl;
  if (!make_plan(a, &pl)) return (size_t)-1;
  if (pl.n_chunks <= 1) return 0;
  return (size_t)pl.n_chunks * query_rows(a) * a->Hq * (a->D + 1) * sizeof(float);
}

static int run_attention(const tva_args *a, void *workspace, size_t workspace_bytes, void *stream, bool merge);

int tva_tree_verify_attn(const tva_args *a, void *stream) {
  return a ? run_attention(a, a->workspace, a->workspace_bytes, stream, true) : TVA_INVALID_ARG;
}

int tva_tree_verify_attn_splits(const tva_args *a, void *stream) {
  return a ? run_attention(a, a->workspace, a->workspace_bytes, stream, false) : TVA_INVALID_ARG;
}

size_t tva_static_scratch_bytes(void) { return TVA_STATIC_SCRATCH_BYTES; }

int tva_tree_verify_attn_static(const tva_args *a, void *stream) {
  if (!a) return TVA_INVALID_ARG;
  // the size is settled from the shapes alone, before any pointer or the device is looked at
  int rc = check_args(a, true);
  if (rc != TVA_OK) return rc;
  const size_t need = tva_workspace_bytes(a);
  if (need == (size_t)-1) return TVA_INVALID_ARG;
  if (need > TVA_STATIC_SCRATCH_BYTES) return TVA_WORKSPACE_TOO_SMALL;
  rc = check_args(a, false);
  if (rc != TVA_OK) return rc;
  void *ptr = nullptr;
  if (need > 0) {  // (a single split touches no scratch memory: no lookup either)
    rc = static_scratch(&ptr);
    if (rc != TVA_OK) return rc;
  }
  return run_attention(a, ptr, need > 0 ? TVA_STATIC_SCRATCH_BYTES : 0, stream, true);
}

static int run_attention(const tva_args *a, void *workspace, size_t workspace_bytes, void *stream, bool merge) {
  int rc = check_args(a, false);
  if (rc != TVA_OK) return rc;
  if (a->sum_T == 0 || a->max_T == 0 || query_rows(a) == 0) return TVA_OK;
  Plan pl;
  if (!make_plan(a, &pl)) return TVA_INVALID_ARG;
  const size_t need = pl.n_chunks > 1 ? (size_t)pl.n_chunks * query_rows(a) * a->Hq * (a->D + 1) * sizeof(float) : 0;
  if (need > 0 && (!workspace || workspace_bytes < need)) return TVA_WORKSPACE_TOO_SMALL;

  AttnParams p;
  p.q = (const __bf16 *)a->q;
  p.k_tree = (const __bf16 *)a->k_tree;
  p.v_tree = (const __bf16 *)a->v_tree;
  p.k_cache = (const __bf16 *)a->k_cache;
  p.v_cache = (const __bf16 *)a->v_cache;
  p.cu_T = a->cu_T;
  p.L = a->L;
  p.cu_L = a->cu_L;
  p.page_table = a->page_table;
  p.mask = a->anc_mask;
  p.parent = a->parent;
  p.out = a->out;
  p.lse = a->lse;
  p.part_out = need > 0 ? (float *)workspace : nullptr;
  p.part_lse = p.part_out ? p.part_out + (size_t)pl.n_chunks * query_rows(a) * a->Hq * a->D : nullptr;
  p.B = a->B;
  p.Hq = a->Hq;
  p.Hkv = a->Hkv;
  p.G = a->Hq / a->Hkv;
  p.g_shift = -1;
  for (int sft = 0; sft < 31; ++sft)
    if ((1 << sft) == p.G) p.g_shift = sft;
  p.sum_Q = (int)query_rows(a);
  p.cu_Q = a->cu_Q;
  p.W = a->mask_words;
  p.chunk_keys = pl.chunk_keys;
  p.n_chunks = pl.n_chunks;
  p.n_row_blocks = pl.n_row_blocks;
  p.max_L = a->max_L;
  fill_slots(a, pl, &p);
  p.page_size = a->page_size > 0 ? a->page_size : 1;
  p.page_shift = -1;
  for (int sft = 0; sft < 31; ++sft)
    if ((1 << sft) == p.page_size) p.page_shift = sft;
  p.max_pages = a->max_pages;
  p.stride_head = a->stride_head ? a->stride_head : a->D;
  p.stride_tok = a->stride_tok ? a->stride_tok : (int64_t)a->Hkv * a->D;
  p.stride_page = a->stride_page ? a->stride_page : (int64_t)p.page_size * p.stride_tok;
  p.scale_log2 = a->scale * kLog2e * ((a->kv_fp8 && a->k_scale > 0.f) ? a->k_scale : 1.f);
  p.v_scale = (a->kv_fp8 && a->v_scale > 0.f) ? a->v_scale : 1.f;

  if ((int64_t)a->B * pl.n_chunks > 65535 || pl.n_row_blocks > 65535) return TVA_UNSUPPORTED;
  const dim3 grid(a->Hkv, pl.n_row_blocks, a->B * pl.n_chunks);
  const bool paged = a->page_table != nullptr;
  hipStream_t st = (hipStream_t)stream;
  hipError_t e;
  if (a->kv_fp8)
    e = paged ? dispatch_variant_fp8<true>(pl.variant, p, grid, st) : dispatch_variant_fp8<false>(pl.variant, p, grid, st);
  else if (a->D == 128)
    e = paged ? dispatch_variant<128, true>(pl.variant, p, grid, st) : dispatch_variant<128, false>(pl.variant, p, grid, st);
  else
    e = paged ? dispatch_variant<64, true>(pl.variant, p, grid, st) : dispatch_variant<64, false>(pl.variant, p, grid, st);
  if (e != hipSuccess) return TVA_HIP_ERROR;

  if (merge && pl.n_chunks > 1) {
    const int64_t n_rows = (int64_t)query_rows(a) * a->Hq;
    clear_stale_hip_error();
    if (a->D == 128) launch_merge<128>(p.part_out, p.part_lse, pl.n_chunks, n_rows, a->out, a->lse, st);
    else launch_merge<64>(p.part_out, p.part_lse, pl.n_chunks, n_rows, a->out, a->lse, st);
    if (launch_status("merge kernel launch") != hipSuccess) return TVA_HIP_ERROR;
  }
  return TVA_OK;
}

int tva_merge_splits(const float *part_out, const float *part_lse, int32_t S, int64_t n_rows, int32_t D,
                     float *out, float *lse, void *stream) {
  if (S < 1 || n_rows < 0) return TVA_INVALID_ARG;
  if (D != 64 && D != 128) return TVA_UNSUPPORTED;
  if (n_rows == 0) return TVA_OK;
  if (!part_out || !part_lse || !out || !lse) return TVA_INVALID_ARG;
  if ((n_rows + 3) / 4 > 0x7fffffff) return TVA_UNSUPPORTED;
  hipStream_t st = (hipStream_t)stream;
  clear_stale_hip_error();
  if (D == 128) launch_merge<128>(part_out, part_lse, S, n_rows, out, lse, st);
  else launch_merge<64>(part_out, part_lse, S, n_rows, out, lse, st);
  return launch_status("merge kernel launch") == hipSuccess ? TVA_OK : TVA_HIP_ERROR;
}

}  // extern "C"
