// 8-bit integer layers (paper Section I: the sparse model is quantized "to 8-bit integer
// computations"; Section III: weights 8 bits, bias 32 bits; Section V: INT8 tensors with
// power-of-two scales).  General-shape block-sparse implicit GEMM on int8 codes with
// exact 32-bit accumulation: any H x K window, stride, padding, ragged channel counts,
// all three block granularities.
//
// Same decomposition as the general floating-point kernel: one wave owns one strip of 16
// output channels and MT tiles of 16 output pixels; the contraction index of a strip is
// the list of (chunk, tap) pairs over the strip's kept 8-channel groups, so only kept
// blocks are visited.  One MFMA i32 16x16x32 (int8 operands) consumes four pairs, one
// per 16-lane group, each lane supplying the eight codes of its pair.
#include "bsp_device.h"
#include "bsp_launch.h"

namespace {

typedef __attribute__((ext_vector_type(4))) int i32x4_t;

// D(16x16, i32) += A(16x32, i8) * B(32x16, i8).  Lane l supplies row l%16 of A and column
// l%16 of B, eight consecutive k each (group l/16), and holds D[4*(l/16) + r][l%16].
__device__ __forceinline__ i32x4_t mfma_i8_16x16x32(u32x2_t a, u32x2_t b, i32x4_t c) {
  return __builtin_amdgcn_mfma_i32_16x16x32_i8(__builtin_bit_cast(long, a),
                                               __builtin_bit_cast(long, b), c, 0, 0, 0);
}

struct I8Params {
  ConvParams p;       // X, payload: int8; bias: int32 (through the float pointer); Y: see below
  int32_t y_i8;       // 1: Y is int8 (shifted, rounded, saturated), 0: Y is the int32 sum
  int32_t shift;
};

template <int BO, int BI, int MT>
__global__ __launch_bounds__(256) void conv_general_i8(I8Params q) {
  kernarg_touch<I8Params>();
  const ConvParams& p = q.p;
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

  const uint8_t* X = (const uint8_t*)p.X;
  const uint8_t* Wp = (const uint8_t*)p.payload;
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
    const int qq = rem - m * p.N;
    iy0[mt] = m * p.sh - p.ph;
    ix0[mt] = qq * p.sw - p.pw;
    xb[mt] = (int64_t)n * p.L * p.J * p.I;
  }

  i32x4_t acc[MT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) acc[mt] = i32x4_t{0, 0, 0, 0};

  // which of the (strip, chunk) cell's blocks this lane's output channel lies in, and its row
  const int sub = BI == 4 ? 0 : jn / BO, row = jn % BO;
  int chunk = g / HK, tap = g % HK;
  for (int q0 = 0; q0 < npairs; q0 += 4) {
    const bool valid = (q0 + g) < npairs;
    u32x2_t a = u32x2_t{0u, 0u};
    int xc = 0, th = 0, tw = 0;
    if (valid) {
      const int ce = c0 + chunk;
      xc = pv.chunk_xc[ce];
      th = tap / p.K;
      tw = tap - th * p.K;
      if constexpr (BI >= 8) {
        const int src = pv.chunk_src[ce * BSP_MAXSUB + sub];
        if (src >= 0) a = *(const u32x2_t*)(Wp + src + (row * HK + tap) * BI);
      } else {  // two 4-wide blocks share the chunk
        const int s0 = pv.chunk_src[ce * BSP_MAXSUB + 0];
        const int s1 = pv.chunk_src[ce * BSP_MAXSUB + 1];
        if (s0 >= 0) a.x = *(const uint32_t*)(Wp + s0 + (row * HK + tap) * BI);
        if (s1 >= 0) a.y = *(const uint32_t*)(Wp + s1 + (row * HK + tap) * BI);
      }
    }
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
      const int iy = iy0[mt] + th, ix = ix0[mt] + tw;
      u32x2_t b = u32x2_t{0u, 0u};
      if (valid && vp[mt] && (unsigned)iy < (unsigned)p.L && (unsigned)ix < (unsigned)p.J) {
        const uint8_t* xp = X + xb[mt] + ((int64_t)iy * p.J + ix) * p.I + xc * BSP_CHUNK;
        if (vecX) {
          b = *(const u32x2_t*)xp;
        } else {
          uint32_t e[8];
#pragma unroll
          for (int t = 0; t < 8; ++t) e[t] = (xc * BSP_CHUNK + t < p.I) ? xp[t] : 0u;
          b.x = e[0] | (e[1] << 8) | (e[2] << 16) | (e[3] << 24);
          b.y = e[4] | (e[5] << 8) | (e[6] << 16) | (e[7] << 24);
        }
      }
      acc[mt] = mfma_i8_16x16x32(a, b, acc[mt]);
    }
    tap += 4;
    while (tap >= HK) {
      tap -= HK;
      ++chunk;
    }
  }

  // epilogue: + 32-bit bias, then either the sum itself or the power-of-two rescale.
  // Lane holds channels 4g..4g+3 of pixel jn.
  const int ch = strip * BSP_STRIP + 4 * g;
  const int32_t* bias = (const int32_t*)p.bias;
  int bv[4];
#pragma unroll
  for (int r = 0; r < 4; ++r) bv[r] = (bias && ch + r < p.O) ? bias[ch + r] : 0;
  const int half = q.shift > 0 ? (1 << (q.shift - 1)) : 0;
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) {
    const int pid = pix_base + mt * 16 + jn;
    if (!vp[mt]) continue;
    int v[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) v[r] = acc[mt][r] + bv[r];
    if (q.y_i8) {
      uint32_t packed = 0;
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        // 64-bit so that adding the rounding half cannot wrap
        const long long s = ((long long)v[r] + half) >> q.shift;
        const int c = s < -128 ? -128 : (s > 127 ? 127 : (int)s);
        packed |= (uint32_t)(c & 0xFF) << (8 * r);
      }
      uint8_t* yp = (uint8_t*)p.Y + (int64_t)pid * p.O + ch;
      if ((p.O % 4) == 0 && ch + 3 < p.O) {
        *(uint32_t*)yp = packed;
      } else {
#pragma unroll
        for (int r = 0; r < 4; ++r)
          if (ch + r < p.O) yp[r] = (uint8_t)(packed >> (8 * r));
      }
    } else {
      int32_t* yp = (int32_t*)p.Y + (int64_t)pid * p.O + ch;
      if ((p.O % 4) == 0 && ch + 3 < p.O) {
        *(i32x4_t*)yp = i32x4_t{v[0], v[1], v[2], v[3]};
      } else {
#pragma unroll
        for (int r = 0; r < 4; ++r)
          if (ch + r < p.O) yp[r] = v[r];
      }
    }
  }
}

template <int BO, int BI>
int launch_gran(const I8Params& q, hipStream_t st) {
  const ConvParams& p = q.p;
  const int nstrips = (p.O + BSP_STRIP - 1) / BSP_STRIP;
  // four pixel tiles per wave once there is enough work to fill the chip with them
  const bool big = (int64_t)p.P * nstrips >= (int64_t)256 * 1024;
  const int mt = big ? 4 : 1;
  dim3 grid((unsigned)((p.P + 64 * mt - 1) / (64 * mt)), (unsigned)nstrips);
  dim3 block(256);
  if (big)
    hipLaunchKernelGGL((conv_general_i8<BO, BI, 4>), grid, block, 0, st, q);
  else
    hipLaunchKernelGGL((conv_general_i8<BO, BI, 1>), grid, block, 0, st, q);
  return hipGetLastError() == hipSuccess ? BSP_OK : BSP_ERR_HIP;
}

}  // namespace

int bsp_launch_i8(const ConvParams& p, int y_i8, int shift, int bo, int bi, hipStream_t st) {
  I8Params q;
  q.p = p;
  q.y_i8 = y_i8;
  q.shift = shift;
  if (bo == 8 && bi == 8) return launch_gran<8, 8>(q, st);
  if (bo == 4 && bi == 16) return launch_gran<4, 16>(q, st);
  if (bo == 16 && bi == 4) return launch_gran<16, 4>(q, st);
  return BSP_ERR_UNSUPPORTED;
}
