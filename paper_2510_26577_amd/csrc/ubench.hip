// libtva_ubench: microbenchmarks of the MI355X (gfx950) rates the attention kernels are priced against.
//
// Not part of the hot path and not linked into libtva.so: a separate small library with its own C
// ABI (include/tva_ubench.h), run by `bench.py --microbench`.  Each probe is a kernel whose inner loop
// is one kind of work; lane 0 of every wave brackets the loop with the shader-clock counter (s_memtime)
// and the constant 100 MHz counter (s_memrealtime), so a result is cycles per iteration and the clock
// the chip ran at, independent of launch overhead.  The host side reports the slowest wave.
//
//   MFMA     v_mfma_f32_32x32x16_bf16 issue rate, N independent accumulators
//   MFMA+V   one MFMA followed by K independent vector instructions and E v_exp_f32: how much vector
//            work fits under a matrix instruction (the ratio the attention loop is built around)
//   EXP      v_exp_f32 rate;  FMA  v_fma_f32 rate
//   LDS      ds_read_b128 and ds_read_b64_tr_b16 bandwidth per CU, conflict-free addresses
//   STREAM   read of a buffer larger than every cache: vector loads and LDS-writing loads
//   L2       every workgroup re-reads one small buffer: what the L2 -> CU path delivers to each kind of load
//   EMPTY    an empty kernel (launch cost is measured by the caller: back-to-back launches in a graph)
// and one alternative kernel for comparison: attention for very few query rows on the vector ALUs only.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "tva_ubench.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ uint64_t shader_clock() { return __builtin_readcyclecounter(); }
__device__ __forceinline__ uint64_t real_clock() { return __builtin_amdgcn_s_memrealtime(); }

// per-wave record: shader cycles, 100 MHz ticks
__device__ __forceinline__ void record(uint64_t *out, uint64_t c0, uint64_t r0) {
  const uint64_t c1 = shader_clock(), r1 = real_clock();
  if ((threadIdx.x & 63) == 0) {
    const size_t w = ((size_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    out[2 * w] = c1 - c0;
    out[2 * w + 1] = r1 - r0;
  }
}

// One MFMA, then K v_fma_f32 and E v_exp_f32 on registers of their own, NACC accumulators in turn;
// the order inside an iteration is pinned with scheduling-group hints.
template <int NACC, int K, int E>
__global__ void __launch_bounds__(512) mfma_valu_kernel(int iters, float seed, uint64_t *out, float *sink) {
  constexpr int NA = NACC > 0 ? NACC : 1;  // NACC = 0: no MFMA at all, vector work only
  f32x16 acc[NA];
  for (int a = 0; a < NA; ++a)
    for (int i = 0; i < 16; ++i) acc[a][i] = seed * (a + i);
  bf16x8 x, y;
  for (int i = 0; i < 8; ++i) x[i] = (__bf16)(seed + i), y[i] = (__bf16)(seed - i);
  float f[K > 0 ? K : 1], e[E > 0 ? E : 1];
  for (int i = 0; i < (K > 0 ? K : 1); ++i) f[i] = seed + i;
  for (int i = 0; i < (E > 0 ? E : 1); ++i) e[i] = seed * 0.5f + i;
  const uint64_t c0 = shader_clock(), r0 = real_clock();
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int a = 0; a < NA; ++a) {
      if (NACC > 0) acc[a] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(x, y, acc[a], 0, 0, 0);
#pragma unroll
      for (int i = 0; i < K; ++i) f[i] = fmaf(f[i], 1.0001f, seed);
#pragma unroll
      for (int i = 0; i < E; ++i) e[i] = __builtin_amdgcn_exp2f(e[i]);
      if (NACC > 0) __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
      if (K + E > 0) __builtin_amdgcn_sched_group_barrier(0x402, K + E, 0);
    }
  }
  record(out, c0, r0);
  float s = 0.f;
  for (int a = 0; a < NA; ++a)
    for (int i = 0; i < 16; ++i) s += acc[a][i];
  for (int i = 0; i < (K > 0 ? K : 1); ++i) s += f[i];
  for (int i = 0; i < (E > 0 ? E : 1); ++i) s += e[i];
  if (s == 12345.678f) sink[threadIdx.x] = s;  // keeps the work alive, never true in practice
}

// LDS reads: 8 reads of 16 bytes (ds_read_b128), or 16 transpose reads of 8 bytes (ds_read_b64_tr_b16), per
// iteration, every lane at its own 16 (8) bytes of a 1 KiB (512 B) line per wave: no bank conflicts
template <bool TR>
__global__ void __launch_bounds__(512) lds_kernel(int iters, uint64_t *out, float *sink) {
  extern __shared__ __align__(16) unsigned char smem[];
  for (int i = threadIdx.x; i < 64 * 1024 / 4; i += blockDim.x) reinterpret_cast<float *>(smem)[i] = (float)i;
  __syncthreads();
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const uint32_t base = (uint32_t)(uintptr_t)smem + wave * 8192 + lane * (TR ? 8 : 16);
  u32x4 acc = {0, 0, 0, 0};
  const uint64_t c0 = shader_clock(), r0 = real_clock();
  for (int it = 0; it < iters; ++it) {
    if (TR) {
      s16x4 v[16];
#pragma unroll
      for (int j = 0; j < 16; ++j) asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(v[j]) : "v"(base), "n"(j * 512));
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
      for (int j = 0; j < 16; ++j) acc[j & 3] ^= (uint32_t)v[j][0];
    } else {
      u32x4 v[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(v[j]) : "v"(base), "n"(j * 1024));
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
      for (int j = 0; j < 8; ++j) acc ^= v[j];
    }
  }
  record(out, c0, r0);
  if (acc[0] + acc[1] + acc[2] + acc[3] == 0x12345678u) sink[threadIdx.x] = 1.f;
}

// streaming read: every workgroup walks its share of the buffer with 16-byte loads per lane; either into
// registers (with the non-temporal hint), or directly into LDS (the way the attention kernel's tile loads work),
// without (TO_LDS = 1) or with (TO_LDS = 2) that hint
template <int TO_LDS>
__global__ void __launch_bounds__(256) stream_kernel(const u32x4 *__restrict__ src, size_t n16, float *sink) {
  extern __shared__ __align__(16) unsigned char smem[];
  u32x4 acc = {0, 0, 0, 0};
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int wave = threadIdx.x >> 6;
  if (TO_LDS) {
    // 8 wave-wide loads of 1 KiB in flight per wave, each into its own slot
    int slot = 0;
    for (; i + 7 * stride < n16; i += 8 * stride) {
#pragma unroll
      for (int u = 0; u < 8; ++u)
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(src + i + u * stride),
                                         (__attribute__((address_space(3))) void *)(smem + (wave * 8 + u) * 1024), 16, 0,
                                         TO_LDS == 2 ? 2 : 0);
      ++slot;
    }
    __builtin_amdgcn_s_waitcnt(0);
    acc[0] = slot;
  } else {
    for (; i + 7 * stride < n16; i += 8 * stride) {
      u32x4 v[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) v[u] = __builtin_nontemporal_load(src + i + u * stride);
#pragma unroll
      for (int u = 0; u < 8; ++u) acc ^= v[u];
    }
  }
  if (acc[0] + acc[1] + acc[2] + acc[3] == 0x12345678u) sink[threadIdx.x] = 1.f;
}

// every workgroup reads the same small buffer `reps` times (so that all but the first reads are served by
// the L2 of its XCD): what the L2 -> CU path delivers, into registers or straight into LDS
template <bool TO_LDS>
__global__ void __launch_bounds__(256) l2_stream_kernel(const u32x4 *__restrict__ src, int n16, int reps, float *sink) {
  extern __shared__ __align__(16) unsigned char smem[];
  u32x4 acc = {0, 0, 0, 0};
  const int wave = threadIdx.x >> 6;
  for (int rep = 0; rep < reps; ++rep) {
    // (each workgroup starts somewhere else, so that they do not all ask for the same line at once)
    int i = (threadIdx.x + blockIdx.x * 4096) % n16;
    for (int k = 0; k + 8 * 256 <= n16; k += 8 * 256) {
      if (TO_LDS) {
#pragma unroll
        for (int u = 0; u < 8; ++u) {
          const int j = (i + u * 256) % n16;
          __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(src + j),
                                           (__attribute__((address_space(3))) void *)(smem + (wave * 8 + u) * 1024), 16, 0, 0);
        }
      } else {
        u32x4 v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = src[(i + u * 256) % n16];
#pragma unroll
        for (int u = 0; u < 8; ++u) acc ^= v[u];
      }
      i = (i + 8 * 256) % n16;
    }
    if (TO_LDS) __builtin_amdgcn_s_waitcnt(0);
  }
  if (acc[0] + acc[1] + acc[2] + acc[3] == 0x12345678u) sink[threadIdx.x] = 1.f;
}

__global__ void empty_kernel() {}

// ---- attention for very few query rows on the vector ALUs (see tva_ubench_valu_attn in the header) ----
__device__ __forceinline__ float wave_max(float x) {
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) x = fmaxf(x, __shfl_xor(x, o));
  return x;
}
__device__ __forceinline__ float wave_sum(float x) {
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) x += __shfl_xor(x, o);
  return x;
}
__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xFFFF0000u); }

template <int D>
__global__ void __launch_bounds__(256) valu_attn_kernel(const tva_ubench_attn_args p) {
  constexpr int RG = 4;          // query rows per workgroup
  constexpr int DW = D / 2;      // 32-bit words (bf16 pairs) per row
  __shared__ float qs[RG][D];  // the rows' q, widened once
  __shared__ float xm[4][RG], xl[4][RG];
  __shared__ float xo[4][RG][D];
  const int kvh = blockIdx.x, rg = blockIdx.y, b = blockIdx.z;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int G = p.Hq / p.Hkv;
  const int t0 = p.cu_T[b], Tb = p.cu_T[b + 1] - t0, Lb = p.L[b], cuL = p.cu_L[b];
  int Tq = Tb, tq0 = t0;
  if (p.cu_Q) {
    const int nq = p.cu_Q[b + 1] - p.cu_Q[b];
    Tq = nq < Tb ? nq : Tb;
    tq0 = p.cu_Q[b];
  }
  const int node_off = Tb - Tq, R = Tq * G;
  if (rg * RG >= R) return;
  const uint32_t *q32 = (const uint32_t *)p.q;
  for (int i = threadIdx.x; i < RG * DW; i += 256) {
    const int r = i / DW, c = i % DW;
    const int row = rg * RG + r < R ? rg * RG + r : R - 1;
    const uint32_t w = q32[((size_t)(tq0 + row / G) * p.Hq + kvh * G + row % G) * DW + c];
    qs[r][2 * c] = bf16_lo(w);
    qs[r][2 * c + 1] = bf16_hi(w);
  }
  __syncthreads();
  uint64_t mk[RG][2];
#pragma unroll
  for (int r = 0; r < RG; ++r) {
    const int row = rg * RG + r < R ? rg * RG + r : R - 1;
    const uint64_t *mp = p.mask + (size_t)(t0 + node_off + row / G) * p.mask_words;
    mk[r][0] = mp[0];
    mk[r][1] = p.mask_words > 1 ? mp[1] : 0;
  }
  const float scale_log2 = p.scale * 1.4426950408889634f;
  float m[RG], l[RG], o[RG][2];
#pragma unroll
  for (int r = 0; r < RG; ++r) m[r] = -INFINITY, l[r] = 0.f, o[r][0] = o[r][1] = 0.f;
  const uint32_t *kc32 = (const uint32_t *)p.k_cache, *vc32 = (const uint32_t *)p.v_cache;
  const uint32_t *kt32 = (const uint32_t *)p.k_tree, *vt32 = (const uint32_t *)p.v_tree;
  const int n_keys = Lb + Tb, n_tiles = (n_keys + 63) / 64;
  for (int tile = wave; tile < n_tiles; tile += 4) {
    // scores: lane = key
    const int kidx = tile * 64 + lane;
    const bool valid = kidx < n_keys;
    const int kc = valid ? kidx : n_keys - 1;
    const uint32_t *kp = kc < Lb ? kc32 + ((size_t)(cuL + kc) * p.Hkv + kvh) * DW
                                 : kt32 + ((size_t)(t0 + kc - Lb) * p.Hkv + kvh) * DW;
    u32x4 kr[DW / 4];
#pragma unroll
    for (int c = 0; c < DW / 4; ++c) kr[c] = reinterpret_cast<const u32x4 *>(kp)[c];
    float s[RG];
#pragma unroll
    for (int r = 0; r < RG; ++r) s[r] = 0.f;
#pragma unroll
    for (int c = 0; c < DW / 4; ++c) {
      float kf[8];
#pragma unroll
      for (int e = 0; e < 4; ++e) kf[2 * e] = bf16_lo(kr[c][e]), kf[2 * e + 1] = bf16_hi(kr[c][e]);
#pragma unroll
      for (int r = 0; r < RG; ++r) {
        // (the same address in every lane: broadcast reads)
        const f32x4 qa = *reinterpret_cast<const f32x4 *>(&qs[r][8 * c]), qb = *reinterpret_cast<const f32x4 *>(&qs[r][8 * c + 4]);
#pragma unroll
        for (int e = 0; e < 4; ++e) s[r] = fmaf(kf[e], qa[e], s[r]);
#pragma unroll
        for (int e = 0; e < 4; ++e) s[r] = fmaf(kf[4 + e], qb[e], s[r]);
      }
    }
    float pr[RG];
#pragma unroll
    for (int r = 0; r < RG; ++r) {
      bool ok = valid;
      if (kidx >= Lb) {
        const int n = kidx - Lb;
        ok = ok && ((mk[r][(n >> 6) & 1] >> (n & 63)) & 1ull);
      }
      const float sv = ok ? s[r] * scale_log2 : -INFINITY;
      const float m_new = fmaxf(m[r], wave_max(sv));
      const float alpha = (m_new == -INFINITY) ? 1.f : exp2f(m[r] - m_new);
      pr[r] = (m_new == -INFINITY) ? 0.f : exp2f(sv - m_new);
      l[r] = l[r] * alpha + pr[r];
      o[r][0] *= alpha;
      o[r][1] *= alpha;
      m[r] = m_new;
    }
    // output: lane = pair of head dimensions; key j's probability comes from lane j
    // (keys past the end have probability zero and re-read the last key's row)
    const int k0 = tile * 64;
#pragma unroll 1
    for (int j0 = 0; j0 < 64; j0 += 16) {
      uint32_t vw[16];
#pragma unroll
      for (int j = 0; j < 16; ++j) {
        const int key = k0 + j0 + j < n_keys ? k0 + j0 + j : n_keys - 1;
        const uint32_t *vp = key < Lb ? vc32 + ((size_t)(cuL + key) * p.Hkv + kvh) * DW
                                      : vt32 + ((size_t)(t0 + key - Lb) * p.Hkv + kvh) * DW;
        vw[j] = lane < DW ? vp[lane] : 0u;
      }
#pragma unroll
      for (int j = 0; j < 16; ++j) {
        const float vx = bf16_lo(vw[j]), vy = bf16_hi(vw[j]);
#pragma unroll
        for (int r = 0; r < RG; ++r) {
          const float pj = __uint_as_float(__builtin_amdgcn_readlane(__float_as_uint(pr[r]), j0 + j));
          o[r][0] = fmaf(pj, vx, o[r][0]);
          o[r][1] = fmaf(pj, vy, o[r][1]);
        }
      }
    }
  }
  // combine the four waves
#pragma unroll
  for (int r = 0; r < RG; ++r) {
    const float ls = wave_sum(l[r]);
    if (lane == 0) xm[wave][r] = m[r], xl[wave][r] = ls;
    if (lane < DW) xo[wave][r][2 * lane] = o[r][0], xo[wave][r][2 * lane + 1] = o[r][1];
  }
  __syncthreads();
  for (int i = threadIdx.x; i < RG * D; i += 256) {
    const int r = i / D, d = i % D;
    const int row = rg * RG + r;
    if (row >= R) continue;
    float M = -INFINITY;
    for (int w = 0; w < 4; ++w) M = fmaxf(M, xm[w][r]);
    float L = 0.f, O = 0.f;
    for (int w = 0; w < 4; ++w) {
      const float a = (xm[w][r] == -INFINITY) ? 0.f : exp2f(xm[w][r] - M);
      L += xl[w][r] * a;
      O += xo[w][r][d] * a;
    }
    const size_t og = (size_t)(tq0 + row / G) * p.Hq + kvh * G + row % G;
    p.out[og * D + d] = L > 0.f ? O / L : 0.f;
    if (d == 0) p.lse[og] = L > 0.f ? (M + log2f(L)) * 0.6931471805599453f : -INFINITY;
  }
}

template <typename F>
int launch_checked(F &&f) {
  (void)hipGetLastError();
  f();
  return hipPeekAtLastError() == hipSuccess ? 0 : -1;
}

}  // namespace

extern "C" {

int tva_ubench_mfma_valu(int32_t nacc, int32_t k, int32_t e, int32_t waves_per_simd, int32_t workgroups,
                         int32_t iters, uint64_t *out, float *sink, void *stream) {
  if ((waves_per_simd != 1 && waves_per_simd != 2) || workgroups < 1 || iters < 1 || !out || !sink) return -1;
  const dim3 grid(workgroups), block(256 * waves_per_simd);
  hipStream_t st = (hipStream_t)stream;
#define CASE(N, K, E) \
  if (nacc == N && k == K && e == E) \
    return launch_checked([&] { hipLaunchKernelGGL((mfma_valu_kernel<N, K, E>), grid, block, 0, st, iters, 1.0f, out, sink); });
  CASE(1, 0, 0) CASE(4, 0, 0)
  CASE(4, 2, 0) CASE(4, 4, 0) CASE(4, 6, 0) CASE(4, 8, 0) CASE(4, 10, 0) CASE(4, 12, 0) CASE(4, 16, 0)
  CASE(4, 0, 1) CASE(4, 0, 2) CASE(4, 0, 4)
  CASE(4, 5, 2) CASE(4, 3, 2)
  CASE(0, 8, 0) CASE(0, 0, 8)
#undef CASE
  return -2;
}

int tva_ubench_lds(int32_t transpose_reads, int32_t waves_per_simd, int32_t workgroups, int32_t iters, uint64_t *out,
                   float *sink, void *stream) {
  if ((waves_per_simd != 1 && waves_per_simd != 2) || workgroups < 1 || iters < 1 || !out || !sink) return -1;
  const dim3 grid(workgroups), block(256 * waves_per_simd);
  hipStream_t st = (hipStream_t)stream;
  if (transpose_reads) return launch_checked([&] { hipLaunchKernelGGL((lds_kernel<true>), grid, block, 64 * 1024, st, iters, out, sink); });
  return launch_checked([&] { hipLaunchKernelGGL((lds_kernel<false>), grid, block, 64 * 1024, st, iters, out, sink); });
}

int tva_ubench_stream(int32_t to_lds, const void *src, size_t bytes, int32_t workgroups, float *sink, void *stream) {
  if (!src || bytes < 16 || workgroups < 1 || !sink) return -1;
  hipStream_t st = (hipStream_t)stream;
  const u32x4 *p = (const u32x4 *)src;
  const size_t n16 = bytes / 16;
  if (to_lds == 2) return launch_checked([&] { hipLaunchKernelGGL((stream_kernel<2>), dim3(workgroups), dim3(256), 32 * 1024, st, p, n16, sink); });
  if (to_lds) return launch_checked([&] { hipLaunchKernelGGL((stream_kernel<1>), dim3(workgroups), dim3(256), 32 * 1024, st, p, n16, sink); });
  return launch_checked([&] { hipLaunchKernelGGL((stream_kernel<0>), dim3(workgroups), dim3(256), 0, st, p, n16, sink); });
}

int tva_ubench_valu_attn(const tva_ubench_attn_args *a, void *stream) {
  if (!a || !a->q || !a->k_cache || !a->v_cache || !a->k_tree || !a->v_tree || !a->mask || !a->cu_T || !a->L || !a->cu_L ||
      !a->out || !a->lse)
    return -1;
  if (a->B < 1 || a->Hkv < 1 || a->Hq < a->Hkv || a->Hq % a->Hkv || (a->D != 64 && a->D != 128) || a->mask_words < 1 ||
      a->mask_words > 2 || a->max_rows < 1 || a->B > 65535)
    return -1;
  const dim3 grid(a->Hkv, (a->max_rows + 3) / 4, a->B), block(256);
  hipStream_t st = (hipStream_t)stream;
  if (a->D == 128) return launch_checked([&] { hipLaunchKernelGGL((valu_attn_kernel<128>), grid, block, 0, st, *a); });
  return launch_checked([&] { hipLaunchKernelGGL((valu_attn_kernel<64>), grid, block, 0, st, *a); });
}

int tva_ubench_reread(int32_t to_lds, const void *src, size_t bytes, int32_t reps, int32_t workgroups, float *sink, void *stream) {
  if (!src || bytes < 8 * 256 * 16 || bytes > (1u << 30) || reps < 1 || workgroups < 1 || !sink) return -1;
  hipStream_t st = (hipStream_t)stream;
  const u32x4 *p = (const u32x4 *)src;
  const int n16 = (int)(bytes / 16);
  if (to_lds) return launch_checked([&] { hipLaunchKernelGGL((l2_stream_kernel<true>), dim3(workgroups), dim3(256), 32 * 1024, st, p, n16, reps, sink); });
  return launch_checked([&] { hipLaunchKernelGGL((l2_stream_kernel<false>), dim3(workgroups), dim3(256), 0, st, p, n16, reps, sink); });
}

int tva_ubench_empty(void *stream) {
  return launch_checked([&] { hipLaunchKernelGGL(empty_kernel, dim3(1), dim3(64), 0, (hipStream_t)stream); });
}

}  // extern "C"
