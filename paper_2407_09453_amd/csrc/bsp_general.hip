// General-shape block-sparse implicit-GEMM kernel: any H x K window, stride,
// padding, ragged channel counts, all three block granularities, fp32 or bf16.
// Operands go straight from global memory (through L1/L2) into MFMA registers;
// the shape-specialised kernels stage activations through LDS instead.
//
// One wave owns one strip of 16 output channels and MT tiles of 16 output
// pixels.  The contraction index of a strip is the list of (chunk, tap) pairs,
// chunk running over the strip's kept 8-channel groups: only kept blocks are
// visited (paper Section I, advantage 3).  bf16: one MFMA 16x16x32 consumes
// four pairs, one per 16-lane group.  fp32: one pair feeds two MFMA 16x16x4,
// the 16-lane group g supplying channels 2g and 2g+1 of the chunk.
#include "bsp_device.h"
#include "bsp_launch.h"

namespace {

template <int BO, int BI>
struct Gran {
  // Which of the (strip, chunk) cell's sources a weight row uses, and the row
  // of that block, for output channel `jn` (0..15) of the strip.
  __device__ static __forceinline__ int sub(int jn) { return BI == 4 ? 0 : jn / BO; }
  __device__ static __forceinline__ int row(int jn) { return jn % BO; }
};

template <int BO, int BI, int MT>
__global__ __launch_bounds__(256) void conv_general_bf16(ConvParams p) {
  kernarg_touch<ConvParams>();
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int jn = lane & 15, g = lane >> 4;
  const int strip = blockIdx.y;
  const PlanView pv = plan_view(p.plan);
  const int c0 = pv.strip_ptr[strip];
  const int nchunks = pv.strip_ptr[strip + 1] - c0;
  const int HK = p.H * p.K;
  const int npairs = nchunks * HK;
  const int pix_base = (blockIdx.x * 4 + wave) * (MT * 16);
  if (pix_base >= p.P) return;

  const uint16_t* X = (const uint16_t*)p.X;
  const uint16_t* Wp = (const uint16_t*)p.payload;
  const bool vecX = (p.I % 8) == 0;

  int iy0[MT], ix0[MT];
  int64_t xb[MT];
  bool vp[MT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) {
    const int pid = pix_base + mt * 16 + jn;
    vp[mt] = pid < p.P;
    const int pc = vp[mt] ? pid : 0;
    const int n = pc / (p.M * p.N);
    const int rem = pc - n * (p.M * p.N);
    const int m = rem / p.N;
    const int q = rem - m * p.N;
    iy0[mt] = m * p.sh - p.ph;
    ix0[mt] = q * p.sw - p.pw;
    xb[mt] = (int64_t)n * p.L * p.J * p.I;
  }

  f32x4_t acc[MT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) acc[mt] = f32x4_t{0.f, 0.f, 0.f, 0.f};

  const int sub = Gran<BO, BI>::sub(jn), row = Gran<BO, BI>::row(jn);
  int chunk = g / HK, tap = g % HK;
  for (int q0 = 0; q0 < npairs; q0 += 4) {
    const bool valid = (q0 + g) < npairs;
    u32x4_t a = u32x4_t{0u, 0u, 0u, 0u};
    int xc = 0, th = 0, tw = 0;
    if (valid) {
      const int ce = c0 + chunk;
      xc = pv.chunk_xc[ce];
      th = tap / p.K;
      tw = tap - th * p.K;
      if constexpr (BI >= 8) {
        const int src = pv.chunk_src[ce * BSP_MAXSUB + sub];
        if (src >= 0) a = *(const u32x4_t*)(Wp + src + (row * HK + tap) * BI);
      } else {
        const int s0 = pv.chunk_src[ce * BSP_MAXSUB + 0];
        const int s1 = pv.chunk_src[ce * BSP_MAXSUB + 1];
        if (s0 >= 0) {
          const u32x2_t lo = *(const u32x2_t*)(Wp + s0 + (row * HK + tap) * BI);
          a.x = lo.x;
          a.y = lo.y;
        }
        if (s1 >= 0) {
          const u32x2_t hi = *(const u32x2_t*)(Wp + s1 + (row * HK + tap) * BI);
          a.z = hi.x;
          a.w = hi.y;
        }
      }
    }
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
      const int iy = iy0[mt] + th, ix = ix0[mt] + tw;
      u32x4_t b = u32x4_t{0u, 0u, 0u, 0u};
      if (valid && vp[mt] && (unsigned)iy < (unsigned)p.L && (unsigned)ix < (unsigned)p.J) {
        const uint16_t* xp = X + xb[mt] + ((int64_t)iy * p.J + ix) * p.I + xc * BSP_CHUNK;
        if (vecX) {
          b = *(const u32x4_t*)xp;
        } else {
          uint32_t e[8];
#pragma unroll
          for (int t = 0; t < 8; ++t) e[t] = (xc * BSP_CHUNK + t < p.I) ? xp[t] : 0u;
          b.x = e[0] | (e[1] << 16);
          b.y = e[2] | (e[3] << 16);
          b.z = e[4] | (e[5] << 16);
          b.w = e[6] | (e[7] << 16);
        }
      }
      acc[mt] = mfma_bf16_16x16x32(a, b, acc[mt]);
    }
    tap += 4;
    while (tap >= HK) {
      tap -= HK;
      ++chunk;
    }
  }

  // epilogue: + bias, one rounding, store.  Lane holds channels 4g..4g+3 of pixel jn.
  const int ch = strip * BSP_STRIP + 4 * g;
  float bv[4];
#pragma unroll
  for (int r = 0; r < 4; ++r) bv[r] = (p.bias && ch + r < p.O) ? p.bias[ch + r] : 0.f;
  uint16_t* Y = (uint16_t*)p.Y;
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) {
    const int pid = pix_base + mt * 16 + jn;
    if (!vp[mt]) continue;
    uint16_t h[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) h[r] = f32_to_bf16_rne(acc[mt][r] + bv[r]);
    uint16_t* yp = Y + (int64_t)pid * p.O + ch;
    const bool vec = (p.O % 4) == 0 && ch + 3 < p.O;
    if (p.residual || p.relu) {
      u32x2_t v;
      v.x = (uint32_t)h[0] | ((uint32_t)h[1] << 16);
      v.y = (uint32_t)h[2] | ((uint32_t)h[3] << 16);
      const uint16_t* rp = p.residual ? (const uint16_t*)p.residual + (int64_t)pid * p.O + ch : nullptr;
      v = post_bf16x4(v, rp, p.O - ch, vec, p.relu);
      h[0] = (uint16_t)(v.x & 0xFFFF);
      h[1] = (uint16_t)(v.x >> 16);
      h[2] = (uint16_t)(v.y & 0xFFFF);
      h[3] = (uint16_t)(v.y >> 16);
    }
    if (vec) {
      u32x2_t v;
      v.x = (uint32_t)h[0] | ((uint32_t)h[1] << 16);
      v.y = (uint32_t)h[2] | ((uint32_t)h[3] << 16);
      *(u32x2_t*)yp = v;
    } else {
#pragma unroll
      for (int r = 0; r < 4; ++r)
        if (ch + r < p.O) yp[r] = h[r];
    }
  }
}

template <int BO, int BI, int MT>
__global__ __launch_bounds__(256) void conv_general_f32(ConvParams p) {
  kernarg_touch<ConvParams>();
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int jn = lane & 15, g = lane >> 4;
  const int strip = blockIdx.y;
  const PlanView pv = plan_view(p.plan);
  const int c0 = pv.strip_ptr[strip];
  const int nchunks = pv.strip_ptr[strip + 1] - c0;
  const int HK = p.H * p.K;
  const int pix_base = (blockIdx.x * 4 + wave) * (MT * 16);
  if (pix_base >= p.P) return;

  const float* X = (const float*)p.X;
  const float* Wp = (const float*)p.payload;
  const bool vecX = (p.I % 2) == 0;

  int iy0[MT], ix0[MT];
  int64_t xb[MT];
  bool vp[MT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) {
    const int pid = pix_base + mt * 16 + jn;
    vp[mt] = pid < p.P;
    const int pc = vp[mt] ? pid : 0;
    const int n = pc / (p.M * p.N);
    const int rem = pc - n * (p.M * p.N);
    const int m = rem / p.N;
    const int q = rem - m * p.N;
    iy0[mt] = m * p.sh - p.ph;
    ix0[mt] = q * p.sw - p.pw;
    xb[mt] = (int64_t)n * p.L * p.J * p.I;
  }
  f32x4_t acc[MT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) acc[mt] = f32x4_t{0.f, 0.f, 0.f, 0.f};

  // this lane's two channels of every chunk: 2g and 2g+1
  const int cc = 2 * g;
  const int sub = BI == 4 ? (cc >> 2) : Gran<BO, BI>::sub(jn);
  const int row = Gran<BO, BI>::row(jn);
  const int wcol = BI == 4 ? (cc & 3) : cc;

  for (int chunk = 0; chunk < nchunks; ++chunk) {
    const int ce = c0 + chunk;
    const int xc = pv.chunk_xc[ce];
    const int src = pv.chunk_src[ce * BSP_MAXSUB + sub];
    for (int tap = 0; tap < HK; ++tap) {
      const int th = tap / p.K, tw = tap - th * p.K;
      float a0 = 0.f, a1 = 0.f;
      if (src >= 0) {
        const float2 w2 = *(const float2*)(Wp + src + (row * HK + tap) * BI + wcol);
        a0 = w2.x;
        a1 = w2.y;
      }
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) {
        const int iy = iy0[mt] + th, ix = ix0[mt] + tw;
        float b0 = 0.f, b1 = 0.f;
        if (vp[mt] && (unsigned)iy < (unsigned)p.L && (unsigned)ix < (unsigned)p.J) {
          const int chn = xc * BSP_CHUNK + cc;
          const float* xp = X + xb[mt] + ((int64_t)iy * p.J + ix) * p.I + chn;
          if (vecX) {
            if (chn < p.I) {
              const float2 x2 = *(const float2*)xp;
              b0 = x2.x;
              b1 = x2.y;
            }
          } else {
            if (chn < p.I) b0 = xp[0];
            if (chn + 1 < p.I) b1 = xp[1];
          }
        }
        acc[mt] = mfma_f32_16x16x4(a0, b0, acc[mt]);
        acc[mt] = mfma_f32_16x16x4(a1, b1, acc[mt]);
      }
    }
  }

  const int ch = strip * BSP_STRIP + 4 * g;
  float bv[4];
#pragma unroll
  for (int r = 0; r < 4; ++r) bv[r] = (p.bias && ch + r < p.O) ? p.bias[ch + r] : 0.f;
  float* Y = (float*)p.Y;
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) {
    const int pid = pix_base + mt * 16 + jn;
    if (!vp[mt]) continue;
    float* yp = Y + (int64_t)pid * p.O + ch;
    float y[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      y[r] = acc[mt][r] + bv[r];
      if (p.residual && ch + r < p.O) y[r] += ((const float*)p.residual)[(int64_t)pid * p.O + ch + r];
      if (p.relu) y[r] = fmaxf(y[r], 0.f);
    }
    if ((p.O % 4) == 0 && ch + 3 < p.O) {
      *(float4*)yp = make_float4(y[0], y[1], y[2], y[3]);
    } else {
#pragma unroll
      for (int r = 0; r < 4; ++r)
        if (ch + r < p.O) yp[r] = y[r];
    }
  }
}

template <int BO, int BI>
int launch_gran(const ConvParams& p, int dtype, hipStream_t st) {
  const int nstrips = (p.O + BSP_STRIP - 1) / BSP_STRIP;
  // four pixel tiles per wave once there is enough work to fill the chip with them
  const bool big = (int64_t)p.P * nstrips >= (int64_t)256 * 1024;
  const int mt = big ? 4 : 1;
  dim3 grid((unsigned)((p.P + 64 * mt - 1) / (64 * mt)), (unsigned)nstrips);
  dim3 block(256);
  if (dtype == BSP_BF16) {
    if (big)
      hipLaunchKernelGGL((conv_general_bf16<BO, BI, 4>), grid, block, 0, st, p);
    else
      hipLaunchKernelGGL((conv_general_bf16<BO, BI, 1>), grid, block, 0, st, p);
  } else {
    if (big)
      hipLaunchKernelGGL((conv_general_f32<BO, BI, 4>), grid, block, 0, st, p);
    else
      hipLaunchKernelGGL((conv_general_f32<BO, BI, 1>), grid, block, 0, st, p);
  }
  return hipGetLastError() == hipSuccess ? BSP_OK : BSP_ERR_HIP;
}

}  // namespace

int bsp_launch_general(const ConvParams& p, int dtype, int bo, int bi, hipStream_t st) {
  if (bo == 8 && bi == 8) return launch_gran<8, 8>(p, dtype, st);
  if (bo == 4 && bi == 16) return launch_gran<4, 16>(p, dtype, st);
  if (bo == 16 && bi == 4) return launch_gran<16, 4>(p, dtype, st);
  return BSP_ERR_UNSUPPORTED;
}
