// Measurement helpers: stream copy, back-to-back MFMA loop, LDS read loop (gfx950).
#include "bsp_bench.h"

#include <hip/hip_runtime.h>

#include "bsp.h"
#include "bsp_device.h"

namespace {

__global__ __launch_bounds__(256) void bench_copy(u32x4_t* __restrict__ dst,
                                                  const u32x4_t* __restrict__ src, int64_t n) {
  const int64_t stride = (int64_t)gridDim.x * 256 * 4;
  for (int64_t i = (int64_t)blockIdx.x * 256 * 4 + threadIdx.x; i < n; i += stride) {
    u32x4_t v[4];
#pragma unroll
    for (int k = 0; k < 4; ++k)
      if (i + k * 256 < n) v[k] = __builtin_nontemporal_load(src + i + k * 256);
#pragma unroll
    for (int k = 0; k < 4; ++k)
      if (i + k * 256 < n) __builtin_nontemporal_store(v[k], dst + i + k * 256);
  }
}

__global__ __launch_bounds__(256) void bench_mfma(float* sink, int iters, int64_t* clocks) {
  const int lane = threadIdx.x & 63;
  const int64_t c0 = clock64(), r0 = wall_clock64();
  u32x4_t a = {0x3f803f80u + lane, 0x3f803f80u, 0x3f803f80u, 0x3f803f80u};
  u32x4_t b = {0x3f003f00u, 0x3f003f00u + lane, 0x3f003f00u, 0x3f003f00u};
  f32x4_t acc[8];
#pragma unroll
  for (int k = 0; k < 8; ++k) acc[k] = f32x4_t{0.f, 0.f, 0.f, 0.f};
  for (int it = 0; it < iters; ++it) {
    // written out so that the compiler neither moves the accumulators about nor reorders
#pragma unroll
    for (int k = 0; k < 8; ++k)
      asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+v"(acc[k]) : "v"(a), "v"(b));
  }
  float s = 0.f;
#pragma unroll
  for (int k = 0; k < 8; ++k) s += acc[k].x + acc[k].y + acc[k].z + acc[k].w;
  if (lane == 0) sink[blockIdx.x * 4 + (threadIdx.x >> 6)] = s;
  if (clocks && blockIdx.x == 0 && threadIdx.x == 0) {
    clocks[0] = clock64() - c0;
    clocks[1] = wall_clock64() - r0;
  }
}

__global__ __launch_bounds__(256) void bench_lds(float* sink, int iters) {
  __shared__ __align__(16) unsigned char lds[32768];
  for (int i = threadIdx.x; i < 32768 / 4; i += 256) ((uint32_t*)lds)[i] = i;
  __syncthreads();
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const unsigned char* base = lds + wave * 8192 + lane * 16;
  u32x4_t s = {0, 0, 0, 0};
  for (int it = 0; it < iters; ++it) {
    u32x4_t v[8];
    const uint32_t addr = (uint32_t)(uintptr_t)base;
#pragma unroll
    for (int k = 0; k < 8; ++k)
      asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(v[k]) : "v"(addr), "n"(k * 1024));
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
    for (int k = 0; k < 8; ++k) s.x ^= v[k].x;
  }
  const uint32_t r = s.x + s.y + s.z + s.w;
  if (r == 0x12345678u || lane == 0) sink[blockIdx.x * 4 + wave] = (float)r;
}

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

}  // namespace

extern "C" {

int bsp_bench_copy(void* dst, const void* src, int64_t bytes, void* stream) {
  if (!dst || !src) return BSP_ERR_NULL;
  if (bytes < 0 || (bytes & 15)) return BSP_ERR_SHAPE;
  if (!aligned16(dst) || !aligned16(src)) return BSP_ERR_ALIGN;
  if (bytes == 0) return BSP_OK;
  const int64_t n = bytes / 16;
  int64_t blocks = (n + 1023) / 1024;
  if (blocks > 256 * 16) blocks = 256 * 16;
  hipLaunchKernelGGL(bench_copy, dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)stream,
                     (u32x4_t*)dst, (const u32x4_t*)src, n);
  return hipGetLastError() == hipSuccess ? BSP_OK : BSP_ERR_HIP;
}

int bsp_bench_mfma_bf16(float* sink, int32_t waves, int32_t iters, int64_t* clocks, void* stream) {
  if (!sink) return BSP_ERR_NULL;
  if (waves <= 0 || (waves & 3) || iters < 0) return BSP_ERR_SHAPE;
  hipLaunchKernelGGL(bench_mfma, dim3((unsigned)(waves / 4)), dim3(256), 0, (hipStream_t)stream,
                     sink, iters, clocks);
  return hipGetLastError() == hipSuccess ? BSP_OK : BSP_ERR_HIP;
}

int bsp_bench_lds_read(float* sink, int32_t waves, int32_t iters, void* stream) {
  if (!sink) return BSP_ERR_NULL;
  if (waves <= 0 || (waves & 3) || iters < 0) return BSP_ERR_SHAPE;
  hipLaunchKernelGGL(bench_lds, dim3((unsigned)(waves / 4)), dim3(256), 0, (hipStream_t)stream,
                     sink, iters);
  return hipGetLastError() == hipSuccess ? BSP_OK : BSP_ERR_HIP;
}

}  // extern "C"
