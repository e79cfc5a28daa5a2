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
  int32_t B, L, J, I, O, H, K, M, N;
  int32_t sh, sw, ph, pw;
  int32_t P;  // B*M*N output pixels
};

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

#endif
