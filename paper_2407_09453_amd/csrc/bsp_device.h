// Device-side helpers shared by the bsp kernels (gfx950 only).
#ifndef BSP_DEVICE_H
#define BSP_DEVICE_H

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "bsp_plan.h"

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4_t;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2_t;

struct bf16_raw {
  uint16_t v;
};

// Everything a layer launch needs; passed by value.
struct ConvParams {
  const void* X;
  void* Y;
  const float* bias;
  const void* payload;
  const int32_t* plan;
  const int32_t* row_ptr;  // the compressed block rows themselves (for kernels that stream them)
  const int32_t* col_idx;
  int32_t B, L, J, I, O, H, K, M, N;
  int32_t sh, sw, ph, pw;
  int32_t P;  // B*M*N output pixels
  // fused epilogue: Y = act(round(conv + bias) + residual), then rounded to the element type
  const void* residual;  // same shape and element type as Y, or null
  int32_t relu;          // act = max(., 0) when nonzero, identity otherwise
};

// A kernel's argument block lies in a few 64-byte lines of memory, and the compiler reads each
// argument where the code first needs it, basic block by basic block: a first use of a new line
// is a miss of the scalar cache, and a kernel's opening takes several of them one after the
// other.  This asks for one word of every line of an argument block of type Args at once and
// waits for all of them (the words go nowhere), so that what follows hits.  The first statement
// of a kernel; nothing past the end of Args is read.
template <typename Args>
__device__ __forceinline__ void kernarg_touch() {
  constexpr int kLines = (int)((sizeof(Args) + 63) / 64);
  const auto* p = __builtin_amdgcn_kernarg_segment_ptr();
  uint32_t t0, t1, t2, t3, t4, t5;
  if constexpr (kLines >= 6)
    asm volatile(
        "s_load_dword %0, %6, 0x0\n\ts_load_dword %1, %6, 0x40\n\ts_load_dword %2, %6, 0x80\n\t"
        "s_load_dword %3, %6, 0xc0\n\ts_load_dword %4, %6, 0x100\n\ts_load_dword %5, %6, 0x140\n\t"
        "s_waitcnt lgkmcnt(0)"
        : "=&s"(t0), "=&s"(t1), "=&s"(t2), "=&s"(t3), "=&s"(t4), "=&s"(t5)
        : "s"(p)
        : "memory");
  else if constexpr (kLines == 5)
    asm volatile(
        "s_load_dword %0, %5, 0x0\n\ts_load_dword %1, %5, 0x40\n\ts_load_dword %2, %5, 0x80\n\t"
        "s_load_dword %3, %5, 0xc0\n\ts_load_dword %4, %5, 0x100\n\ts_waitcnt lgkmcnt(0)"
        : "=&s"(t0), "=&s"(t1), "=&s"(t2), "=&s"(t3), "=&s"(t4)
        : "s"(p)
        : "memory");
  else if constexpr (kLines == 4)
    asm volatile(
        "s_load_dword %0, %4, 0x0\n\ts_load_dword %1, %4, 0x40\n\ts_load_dword %2, %4, 0x80\n\t"
        "s_load_dword %3, %4, 0xc0\n\ts_waitcnt lgkmcnt(0)"
        : "=&s"(t0), "=&s"(t1), "=&s"(t2), "=&s"(t3)
        : "s"(p)
        : "memory");
  else if constexpr (kLines == 3)
    asm volatile(
        "s_load_dword %0, %3, 0x0\n\ts_load_dword %1, %3, 0x40\n\ts_load_dword %2, %3, 0x80\n\t"
        "s_waitcnt lgkmcnt(0)"
        : "=&s"(t0), "=&s"(t1), "=&s"(t2)
        : "s"(p)
        : "memory");
}

__device__ __forceinline__ uint16_t f32_to_bf16_rne(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7F800000u) == 0x7F800000u && (u & 0x007FFFFFu)) return (uint16_t)((u >> 16) | 0x0040u);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}
__device__ __forceinline__ float bf16_bits_to_f32(uint16_t h) {
  return __uint_as_float((uint32_t)h << 16);
}

// D(16x16, fp32) += A(16x32, bf16) * B(32x16, bf16).  Lane l supplies row l%16
// of A and column l%16 of B, eight consecutive k each (the same eight for both
// operands: group l/16), and holds D[4*(l/16) + r][l%16] for r = 0..3.
__device__ __forceinline__ f32x4_t mfma_bf16_16x16x32(u32x4_t a, u32x4_t b, f32x4_t c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a),
                                                 __builtin_bit_cast(bf16x8_t, b), c, 0, 0, 0);
}
// D(16x16) += A(16x4) * B(4x16) in fp32: lane l supplies A[l%16][l/16] and B[l/16][l%16].
__device__ __forceinline__ f32x4_t mfma_f32_16x16x4(float a, float b, f32x4_t c) {
  return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0);
}

struct PlanView {
  const int32_t* strip_ptr;
  const int32_t* chunk_xc;
  const int32_t* chunk_src;
};
__device__ __forceinline__ PlanView plan_view(const int32_t* plan) {
  PlanView v;
  v.strip_ptr = plan + plan[BSP_PLAN_OFF_STRIP_W];
  v.chunk_xc = plan + plan[BSP_PLAN_OFF_XC_W];
  v.chunk_src = plan + plan[BSP_PLAN_OFF_SRC_W];
  return v;
}

// Fused epilogue on four bf16 results packed in v (channels c..c+3 of one pixel): adds the
// residual's channels (r4 points at channel c; `n` of the four exist), applies the
// activation, rounds again.  Without a residual the second rounding changes nothing.
__device__ __forceinline__ u32x2_t post_bf16x4(u32x2_t v, const uint16_t* r4, int n, bool vec,
                                               int relu) {
  float f[4] = {bf16_bits_to_f32((uint16_t)(v.x & 0xFFFF)), bf16_bits_to_f32((uint16_t)(v.x >> 16)),
                bf16_bits_to_f32((uint16_t)(v.y & 0xFFFF)), bf16_bits_to_f32((uint16_t)(v.y >> 16))};
  if (r4) {
    if (vec) {
      const u32x2_t r = *(const u32x2_t*)r4;
      f[0] += bf16_bits_to_f32((uint16_t)(r.x & 0xFFFF));
      f[1] += bf16_bits_to_f32((uint16_t)(r.x >> 16));
      f[2] += bf16_bits_to_f32((uint16_t)(r.y & 0xFFFF));
      f[3] += bf16_bits_to_f32((uint16_t)(r.y >> 16));
    } else {
#pragma unroll
      for (int k = 0; k < 4; ++k)
        if (k < n) f[k] += bf16_bits_to_f32(r4[k]);
    }
  }
  if (relu) {
#pragma unroll
    for (int k = 0; k < 4; ++k) f[k] = fmaxf(f[k], 0.f);
  }
  u32x2_t o;
  o.x = (uint32_t)f32_to_bf16_rne(f[0]) | ((uint32_t)f32_to_bf16_rne(f[1]) << 16);
  o.y = (uint32_t)f32_to_bf16_rne(f[2]) | ((uint32_t)f32_to_bf16_rne(f[3]) << 16);
  return o;
}

#endif
