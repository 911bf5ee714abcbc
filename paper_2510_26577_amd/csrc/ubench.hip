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
//   EMPTY    an empty kernel (launch cost is measured by the caller: back-to-back launches in a graph)
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
// registers, or directly into LDS (the way the attention kernel's tile loads work)
template <bool TO_LDS>
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
                                         (__attribute__((address_space(3))) void *)(smem + (wave * 8 + u) * 1024), 16, 0, 0);
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

__global__ void empty_kernel() {}

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
  if (to_lds) return launch_checked([&] { hipLaunchKernelGGL((stream_kernel<true>), dim3(workgroups), dim3(256), 32 * 1024, st, p, n16, sink); });
  return launch_checked([&] { hipLaunchKernelGGL((stream_kernel<false>), dim3(workgroups), dim3(256), 0, st, p, n16, sink); });
}

int tva_ubench_empty(void *stream) {
  return launch_checked([&] { hipLaunchKernelGGL(empty_kernel, dim3(1), dim3(64), 0, (hipStream_t)stream); });
}

}  // extern "C"
