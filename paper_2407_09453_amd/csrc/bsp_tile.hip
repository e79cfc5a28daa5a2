// LDS-tiled block-sparse implicit-GEMM convolution, bf16 in / fp32 accumulate.
//
// One workgroup (4 waves) owns a TH x TW tile of output pixels of one image and
// a group of strips (16 output channels each).  The input patch the tile needs
// (halo included, zero-filled where it leaves the image, so padding costs no
// branches in the hot loop) is staged once into LDS, one slab of input
// channels at a time, and reused by every strip of the group.  A wave takes a
// strip and walks its steps from the plan: per step one contiguous 1 KB weight
// fragment (already in MFMA operand order) and, per 16-pixel tile, one 16-byte
// LDS read per lane gathered by the step's (chunk, tap) descriptor, feeding
// v_mfma_f32_16x16x32_bf16.  Only kept blocks have steps (paper Section I,
// advantages 3-4); the epilogue adds the fp32 bias and rounds once to bf16.
#include "bsp_device.h"
#include "bsp_launch.h"

namespace {

struct TileCfg {
  int32_t TH, TW;            // output tile, pixels
  int32_t TPH, TPW;          // staged input patch, pixels
  int32_t lsh, lsw;          // LDS pixels per output pixel step
  int32_t gsh, gsw;          // input pixels per LDS pixel step
  int32_t tiles_y, tiles_x;  // tiles per image
  int32_t row_bytes;         // LDS bytes per staged pixel (slab*2 + pad)
  int32_t slab, nslabs;      // channels per slab, slabs
  int32_t spc;               // strips per workgroup (4 when nslabs > 1)
  int32_t nstrips;
};

template <int NT>
__global__ __launch_bounds__(256) void conv_tile_bf16(ConvParams p, TileCfg t) {
  extern __shared__ __align__(16) unsigned char lds[];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int jn = lane & 15, g = lane >> 4;

  const int tpi = t.tiles_y * t.tiles_x;
  const int tile = blockIdx.x;
  const int n = tile / tpi;
  const int trem = tile - n * tpi;
  const int tyi = trem / t.tiles_x;
  const int txi = trem - tyi * t.tiles_x;
  const int oy0 = tyi * t.TH, ox0 = txi * t.TW;
  const int iy_org = oy0 * p.sh - p.ph, ix_org = ox0 * p.sw - p.pw;

  const int32_t* plan = p.plan;
  const int32_t* slab_ptr = plan + plan[BSP_PLAN_OFF_SLAB_W];
  const int32_t* xdesc = plan + plan[BSP_PLAN_OFF_XDESC_W];
  const u32x4_t* wfrag = (const u32x4_t*)(plan + plan[BSP_PLAN_OFF_WFRAG_W]);

  int base[NT];
  bool pv[NT];
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) {
    const int pi = nt * 16 + jn;
    const int ty = pi / t.TW, tx = pi - ty * t.TW;
    pv[nt] = pi < t.TH * t.TW && oy0 + ty < p.M && ox0 + tx < p.N;
    base[nt] = pv[nt] ? ((ty * t.lsh) * t.TPW + tx * t.lsw) * t.row_bytes : 0;
  }

  const uint16_t* X = (const uint16_t*)p.X;
  const int PP = t.slab / BSP_CHUNK;  // 16-byte pieces per staged pixel
  const int npieces = t.TPH * t.TPW * PP;

  f32x4_t acc[NT];

  for (int sl = 0; sl < t.nslabs; ++sl) {
    if (sl) __syncthreads();
    // ---- stage the slab: global -> registers -> LDS, four pieces in flight per thread
    for (int i0 = tid; i0 < npieces; i0 += 256 * 4) {
      u32x4_t v[4];
      int dst[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int idx = i0 + u * 256;
        v[u] = u32x4_t{0u, 0u, 0u, 0u};
        dst[u] = -1;
        if (idx < npieces) {
          const int pix = idx / PP, part = idx - pix * PP;
          const int py = pix / t.TPW, px = pix - py * t.TPW;
          const int iy = iy_org + py * t.gsh, ix = ix_org + px * t.gsw;
          const int ch = sl * t.slab + part * BSP_CHUNK;
          dst[u] = pix * t.row_bytes + part * 16;
          if ((unsigned)iy < (unsigned)p.L && (unsigned)ix < (unsigned)p.J && ch < p.I)
            v[u] = *(const u32x4_t*)(X + (((int64_t)n * p.L + iy) * p.J + ix) * p.I + ch);
        }
      }
#pragma unroll
      for (int u = 0; u < 4; ++u)
        if (dst[u] >= 0) *(u32x4_t*)(lds + dst[u]) = v[u];
    }
    __syncthreads();

    // ---- contraction over this slab's steps, strip by strip
    for (int si = wave; si < t.spc; si += 4) {
      const int strip = blockIdx.y * t.spc + si;
      if (strip >= t.nstrips) break;
      if (sl == 0) {
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) acc[nt] = f32x4_t{0.f, 0.f, 0.f, 0.f};
      }
      int s = slab_ptr[strip * (t.nslabs + 1) + sl];
      const int s1 = slab_ptr[strip * (t.nslabs + 1) + sl + 1];
      if (s < s1) {
        u32x4_t a_next = wfrag[(int64_t)s * 64 + lane];
        int d_next = xdesc[s * 4 + g];
        for (; s < s1; ++s) {
          const u32x4_t a = a_next;
          const int d = d_next;
          if (s + 1 < s1) {
            a_next = wfrag[(int64_t)(s + 1) * 64 + lane];
            d_next = xdesc[(s + 1) * 4 + g];
          }
          const int xoff =
              (((d >> 16) & 0xFF) * t.TPW + ((d >> 24) & 0xFF)) * t.row_bytes + (d & 0xFFFF) * 16;
#pragma unroll
          for (int nt = 0; nt < NT; ++nt) {
            const u32x4_t b = *(const u32x4_t*)(lds + base[nt] + xoff);
            acc[nt] = mfma_bf16_16x16x32(a, b, acc[nt]);
          }
        }
      }
      if (sl == t.nslabs - 1) {
        // epilogue: lane holds channels 4g..4g+3 of pixel jn of every pixel tile
        const int ch = strip * BSP_STRIP + 4 * g;
        float bv[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) bv[r] = (p.bias && ch + r < p.O) ? p.bias[ch + r] : 0.f;
        uint16_t* Y = (uint16_t*)p.Y;
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
          if (!pv[nt]) continue;
          const int pi = nt * 16 + jn;
          const int ty = pi / t.TW, tx = pi - ty * t.TW;
          const int64_t pid = ((int64_t)n * p.M + oy0 + ty) * p.N + ox0 + tx;
          uint16_t h[4];
#pragma unroll
          for (int r = 0; r < 4; ++r) h[r] = f32_to_bf16_rne(acc[nt][r] + bv[r]);
          uint16_t* yp = Y + pid * p.O + ch;
          if ((p.O % 4) == 0 && ch + 3 < p.O) {
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
    }
  }
}

constexpr int kMaxLds = 64 * 1024;

// Pick the output tile: most useful pixels per MFMA pixel slot, then least halo.
bool choose_tile(const ConvParams& p, int slab, int* NT, TileCfg* t) {
  const bool pointwise = p.H == 1 && p.K == 1;
  const int row_bytes = slab * 2 + 16;
  static const int nts[] = {4, 7, 8};
  static const int tws[] = {4, 7, 8, 14, 16, 28, 32, 56, 64, 112, 128};
  double best = -1.0;
  for (int nt : nts)
    for (int tw : tws) {
      if (tw > nt * 16) continue;
      const int TW = tw < p.N ? tw : p.N;
      int TH = nt * 16 / TW;
      if (TH > p.M) TH = p.M;
      if (TH < 1) continue;
      const int lsh = pointwise ? 1 : p.sh, lsw = pointwise ? 1 : p.sw;
      const int TPH = (TH - 1) * lsh + (pointwise ? 1 : p.H);
      const int TPW = (TW - 1) * lsw + (pointwise ? 1 : p.K);
      const int64_t ldsb = (int64_t)TPH * TPW * row_bytes;
      if (ldsb > kMaxLds) continue;
      const int tiles_y = (p.M + TH - 1) / TH, tiles_x = (p.N + TW - 1) / TW;
      const double util = (double)p.M * p.N / ((double)tiles_y * tiles_x * nt * 16);
      const double halo = (double)TPH * TPW / ((double)TH * TW * lsh * lsw);
      const double score = util - 0.02 * halo + 0.001 * nt;
      if (score > best) {
        best = score;
        *NT = nt;
        t->TH = TH;
        t->TW = TW;
        t->TPH = TPH;
        t->TPW = TPW;
        t->lsh = lsh;
        t->lsw = lsw;
        t->gsh = pointwise ? p.sh : 1;
        t->gsw = pointwise ? p.sw : 1;
        t->tiles_y = tiles_y;
        t->tiles_x = tiles_x;
        t->row_bytes = row_bytes;
      }
    }
  return best >= 0.0;
}

}  // namespace

bool bsp_tile_supported(const ConvParams& p, int dtype) {
  return dtype == BSP_BF16 && (p.I % 8) == 0 && p.H <= 255 && p.K <= 255;
}

int bsp_launch_tile(const ConvParams& p_in, int dtype, hipStream_t st) {
  if (!bsp_tile_supported(p_in, dtype)) return BSP_ERR_UNSUPPORTED;
  ConvParams p = p_in;
  // a 1x1, stride-1, unpadded layer is a plain matrix product over all B*M*N
  // pixels: flatten them into one long row so tiles never straddle image edges
  if (p.H == 1 && p.K == 1 && p.sh == 1 && p.sw == 1 && p.ph == 0 && p.pw == 0) {
    p.J = p.N = p.P;
    p.L = p.M = 1;
    p.B = 1;
  }
  TileCfg t;
  int NT = 0;
  t.slab = bsp_slab_channels(p.I, p.H, p.K);
  t.nslabs = ((p.I + 7) / 8 + t.slab / 8 - 1) / (t.slab / 8);
  t.nstrips = (p.O + BSP_STRIP - 1) / BSP_STRIP;
  if (!choose_tile(p, t.slab, &NT, &t)) return BSP_ERR_UNSUPPORTED;
  const int64_t ntiles = (int64_t)p.B * t.tiles_y * t.tiles_x;
  int sw = 1;
  if (t.nslabs == 1) {
    for (int cand : {8, 4, 2}) {
      const int64_t groups = (t.nstrips + 4 * cand - 1) / (4 * cand);
      if (4 * cand <= t.nstrips + 3 && ntiles * groups >= 1024) {
        sw = cand;
        break;
      }
    }
  }
  t.spc = 4 * sw;
  const int64_t groups = (t.nstrips + t.spc - 1) / t.spc;
  if (ntiles > 0x7FFFFFFF || groups > 65535) return BSP_ERR_SHAPE;
  dim3 grid((unsigned)ntiles, (unsigned)groups), block(256);
  const size_t ldsb = (size_t)t.TPH * t.TPW * t.row_bytes;
  switch (NT) {
    case 4: hipLaunchKernelGGL(conv_tile_bf16<4>, grid, block, ldsb, st, p, t); break;
    case 7: hipLaunchKernelGGL(conv_tile_bf16<7>, grid, block, ldsb, st, p, t); break;
    case 8: hipLaunchKernelGGL(conv_tile_bf16<8>, grid, block, ldsb, st, p, t); break;
    default: return BSP_ERR_UNSUPPORTED;
  }
  return hipGetLastError() == hipSuccess ? BSP_OK : BSP_ERR_HIP;
}
