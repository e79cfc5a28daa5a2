// LDS-tiled block-sparse implicit-GEMM convolution, bf16 in / fp32 accumulate.
//
// Persistent workgroups (4 waves) walk a list of work items; an item is a
// TH x TW tile of output pixels of one image times a group of strips (16 output
// channels each).  The input patch a tile needs (halo included, zero-filled
// where it leaves the image, so padding costs no branches in the hot loop) is
// staged into LDS one slab of input channels at a time and reused by every
// strip of the group; the global loads for the NEXT slab or tile are issued
// before the current one is computed and land in registers meanwhile.  A wave
// takes a strip and walks its steps from the plan: per step one contiguous
// 1 KB weight fragment (already in MFMA operand order, prefetched several
// steps ahead) and, per 16-pixel tile, one 16-byte LDS read per lane gathered
// by the step's (chunk, tap) descriptor, feeding v_mfma_f32_16x16x32_bf16.
// Only kept blocks have steps (paper Section I, advantages 3-4); the epilogue
// adds the fp32 bias and rounds once to bf16.
#include "bsp_device.h"
#include "bsp_launch.h"

#include <array>
#include <map>
#include <mutex>

namespace {

struct TileCfg {
  int32_t TH, TW;            // output tile, pixels
  int32_t TPH, TPW;          // staged input patch, pixels
  int32_t lsh, lsw;          // LDS pixels per output pixel step
  int32_t gsh, gsw;          // input pixels per LDS pixel step
  int32_t tiles_y, tiles_x;  // tiles per image
  int32_t row_bytes;         // LDS bytes per staged pixel (slab*2 + pad)
  int32_t pitch;             // LDS bytes per staged patch row (TPW*row_bytes + pad)
  int32_t tile2x8;           // 1: a 16-pixel tile is 2 rows x 8 columns, 0: 16 consecutive pixels
  int32_t slab, nslabs;      // channels per slab, slabs
  int32_t spc;               // strips per work item (4 when nslabs > 1)
  int32_t nstrips;
  int32_t ntiles;            // B * tiles_y * tiles_x
  int32_t nitems;            // ntiles * strip groups
};

constexpr int kStagePieces = 8;  // 16-byte pieces a thread keeps in flight while staging
constexpr int kWDepth = 4;       // weight fragments prefetched ahead

typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
typedef __attribute__((ext_vector_type(2))) float f32x2_t;
// two fp32 -> packed bf16 pair, round to nearest even (v_cvt_pk_bf16_f32)
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  const f32x2_t v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}

// One step: a = weight fragment, d = its descriptor.  Every pixel tile of the
// wave reads its 16 bytes of activations at the step's gathered offset.
template <int NT>
__device__ __forceinline__ void mma_step(f32x4_t (&acc)[NT], const u32x4_t a, const int d,
                                         const unsigned char* lds, const int (&base)[NT],
                                         const int pitch, const int row_bytes) {
  const int xoff = ((d >> 16) & 0xFF) * pitch + ((d >> 24) & 0xFF) * row_bytes + (d & 0xFFFF) * 16;
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) {
    const u32x4_t b = *(const u32x4_t*)(lds + base[nt] + xoff);
    acc[nt] = mfma_bf16_16x16x32(a, b, acc[nt]);
  }
}

// All steps [s0, s1) of one (strip, slab); fragments are fetched kWDepth steps ahead.
template <int NT>
__device__ __forceinline__ void run_steps(f32x4_t (&acc)[NT], const u32x4_t* __restrict__ wf,
                                          const int32_t* __restrict__ xd, const int s0,
                                          const int s1, const int lane, const int g,
                                          const unsigned char* lds, const int (&base)[NT],
                                          const int pitch, const int row_bytes) {
  if (s0 >= s1) return;
  const int last = s1 - 1;
  u32x4_t w[kWDepth];
  int d[kWDepth];
#pragma unroll
  for (int u = 0; u < kWDepth; ++u) {
    const int i = min(s0 + u, last);
    w[u] = wf[(int64_t)i * 64 + lane];
    d[u] = xd[i * 4 + g];
  }
  int s = s0;
  for (; s + kWDepth <= s1; s += kWDepth) {
#pragma unroll
    for (int u = 0; u < kWDepth; ++u) {
      const u32x4_t a = w[u];
      const int dd = d[u];
      const int i = min(s + u + kWDepth, last);
      w[u] = wf[(int64_t)i * 64 + lane];
      d[u] = xd[i * 4 + g];
      mma_step<NT>(acc, a, dd, lds, base, pitch, row_bytes);
    }
  }
  const int rem = s1 - s;
#pragma unroll
  for (int u = 0; u < kWDepth - 1; ++u)
    if (u < rem) mma_step<NT>(acc, w[u], d[u], lds, base, pitch, row_bytes);
}

template <int NT>
__global__ __launch_bounds__(256) void conv_tile_bf16(ConvParams p, TileCfg t) {
  extern __shared__ __align__(16) unsigned char lds[];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int jn = lane & 15, g = lane >> 4;

  const int32_t* plan = p.plan;
  const int32_t* slab_ptr = plan + plan[BSP_PLAN_OFF_SLAB_W];
  const int32_t* xdesc = plan + plan[BSP_PLAN_OFF_XDESC_W];
  const u32x4_t* wfrag = (const u32x4_t*)(plan + plan[BSP_PLAN_OFF_WFRAG_W]);
  const uint16_t* X = (const uint16_t*)p.X;

  // ---- per-thread staging map: piece u of this thread -> LDS offset, patch pixel, channel
  const int PP = t.slab / BSP_CHUNK;  // 16-byte pieces per staged pixel
  const int npieces = t.TPH * t.TPW * PP;
  int sdst[kStagePieces], sinfo[kStagePieces];
#pragma unroll
  for (int u = 0; u < kStagePieces; ++u) {
    const int idx = tid + u * 256;
    const int pix = idx / PP, part = idx - pix * PP;
    const int py = pix / t.TPW, px = pix - py * t.TPW;
    sdst[u] = idx < npieces ? py * t.pitch + px * t.row_bytes + part * 16 : -1;
    sinfo[u] = (py * t.gsh) | ((px * t.gsw) << 10) | (part << 20);
  }
  // ---- per-lane output pixel map
  int pyx[NT], base[NT];
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) {
    const int pi = nt * 16 + jn;
    int ty, tx;
    if (t.tile2x8) {  // pixel tiles are 2 rows x 8 columns
      const int tpr = t.TW >> 3;
      const int tr = nt / tpr, tc = nt - tr * tpr;
      ty = tr * 2 + (jn >> 3);
      tx = tc * 8 + (jn & 7);
    } else {
      ty = pi / t.TW;
      tx = pi - ty * t.TW;
    }
    const bool in_tile = ty < t.TH && tx < t.TW;
    pyx[nt] = in_tile ? (ty | (tx << 16)) : -1;
    base[nt] = in_tile ? (ty * t.lsh) * t.pitch + (tx * t.lsw) * t.row_bytes : 0;
  }

  // work units: (item, slab) pairs in order; unit -> where its patch comes from
  const int tpi = t.tiles_y * t.tiles_x;
  auto decode = [&](int item, int* n, int* oy0, int* ox0, int* sg) {
    const int tile = item % t.ntiles;
    *sg = item / t.ntiles;
    *n = tile / tpi;
    const int trem = tile - *n * tpi;
    const int tyi = trem / t.tiles_x;
    *oy0 = tyi * t.TH;
    *ox0 = (trem - tyi * t.tiles_x) * t.TW;
  };
  u32x4_t sv[kStagePieces];
  auto issue_loads = [&](int item, int sl) {
    int n, oy0, ox0, sg;
    decode(item, &n, &oy0, &ox0, &sg);
    const int iy_org = oy0 * p.sh - p.ph, ix_org = ox0 * p.sw - p.pw;
    const int64_t img = (int64_t)n * p.L;
#pragma unroll
    for (int u = 0; u < kStagePieces; ++u) {
      sv[u] = u32x4_t{0u, 0u, 0u, 0u};
      const int iy = iy_org + (sinfo[u] & 0x3FF), ix = ix_org + ((sinfo[u] >> 10) & 0x3FF);
      const int ch = sl * t.slab + (sinfo[u] >> 20) * BSP_CHUNK;
      if (sdst[u] >= 0 && (unsigned)iy < (unsigned)p.L && (unsigned)ix < (unsigned)p.J && ch < p.I)
        sv[u] = *(const u32x4_t*)(X + ((img + iy) * p.J + ix) * p.I + ch);
    }
  };

  f32x4_t acc[NT];
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) acc[nt] = f32x4_t{0.f, 0.f, 0.f, 0.f};
  int item = blockIdx.x;
  if (item >= t.nitems) return;
  issue_loads(item, 0);
  int sl = 0;
  while (true) {
    // registers -> LDS (the previous unit's readers are past the barrier below)
#pragma unroll
    for (int u = 0; u < kStagePieces; ++u)
      if (sdst[u] >= 0) *(u32x4_t*)(lds + sdst[u]) = sv[u];
    __syncthreads();
    // next unit's loads fly while this one is computed
    int nitem = item, nsl = sl + 1;
    if (nsl == t.nslabs) {
      nsl = 0;
      nitem = item + gridDim.x;
    }
    const bool more = nitem < t.nitems;
    if (more) issue_loads(nitem, nsl);

    int n, oy0, ox0, sg;
    decode(item, &n, &oy0, &ox0, &sg);
    for (int si = wave; si < t.spc; si += 4) {
      const int strip = sg * t.spc + si;
      if (strip >= t.nstrips) break;
      const int s0 = slab_ptr[strip * (t.nslabs + 1) + sl];
      const int s1 = slab_ptr[strip * (t.nslabs + 1) + sl + 1];
      run_steps<NT>(acc, wfrag, xdesc, s0, s1, lane, g, lds, base, t.pitch, t.row_bytes);
      if (sl == t.nslabs - 1) {
        // epilogue: lane holds channels 4g..4g+3 of pixel jn of every pixel tile
        const int ch = strip * BSP_STRIP + 4 * g;
        float bv[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) bv[r] = (p.bias && ch + r < p.O) ? p.bias[ch + r] : 0.f;
        uint16_t* Y = (uint16_t*)p.Y;
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
          const int oy = oy0 + (pyx[nt] & 0xFFFF), ox = ox0 + (pyx[nt] >> 16);
          u32x2_t v;
          v.x = pack_bf16x2(acc[nt][0] + bv[0], acc[nt][1] + bv[1]);
          v.y = pack_bf16x2(acc[nt][2] + bv[2], acc[nt][3] + bv[3]);
          acc[nt] = f32x4_t{0.f, 0.f, 0.f, 0.f};
          if (pyx[nt] < 0 || oy >= p.M || ox >= p.N) continue;
          const int64_t pid = ((int64_t)n * p.M + oy) * p.N + ox;
          uint16_t* yp = Y + pid * p.O + ch;
          if ((p.O % 4) == 0 && ch + 3 < p.O) {
            *(u32x2_t*)yp = v;
          } else {
            if (ch + 0 < p.O) yp[0] = (uint16_t)(v.x & 0xFFFF);
            if (ch + 1 < p.O) yp[1] = (uint16_t)(v.x >> 16);
            if (ch + 2 < p.O) yp[2] = (uint16_t)(v.y & 0xFFFF);
            if (ch + 3 < p.O) yp[3] = (uint16_t)(v.y >> 16);
          }
        }
      }
    }
    if (!more) break;
    item = nitem;
    sl = nsl;
    __syncthreads();  // everyone is done reading LDS before it is overwritten
  }
}

// LDS passes one (chunk, tap) read of all pixel tiles costs beyond the conflict-free
// minimum: per 16-pixel tile, the worst number of lanes that fall on the same
// 16-byte slot of a 256-byte bank cycle (and, for each half of the tile, of a
// 128-byte cycle), minus one.  0 = conflict free.
int conflict_excess(const TileCfg& t, int NT) {
  int excess = 0;
  for (int nt = 0; nt < NT; ++nt) {
    int cnt16[16] = {0}, lo8[8] = {0}, hi8[8] = {0}, worst = 1;
    for (int jn = 0; jn < 16; ++jn) {
      int ty, tx;
      if (t.tile2x8) {
        const int tpr = t.TW >> 3;
        ty = (nt / tpr) * 2 + (jn >> 3);
        tx = (nt % tpr) * 8 + (jn & 7);
      } else {
        ty = (nt * 16 + jn) / t.TW;
        tx = (nt * 16 + jn) % t.TW;
      }
      if (ty >= t.TH || tx >= t.TW) continue;
      const int slot = ((ty * t.lsh) * t.pitch + (tx * t.lsw) * t.row_bytes) / 16;
      const int a = ++cnt16[slot & 15];
      const int b = jn < 8 ? ++lo8[slot & 7] : ++hi8[slot & 7];
      if (a > worst) worst = a;
      if (b > worst) worst = b;
    }
    excess += worst - 1;
  }
  return excess;
}

constexpr int kMaxLds = 64 * 1024;

// Pick the output tile: most useful pixels per MFMA pixel slot, least halo, no
// LDS bank conflicts; then the LDS paddings that achieve the latter.
bool choose_tile(const ConvParams& p, int slab, int* NT, TileCfg* out) {
  const bool pointwise = p.H == 1 && p.K == 1;
  static const int nts[] = {4, 7, 8};
  static const int tws[] = {4, 7, 8, 14, 16, 24, 28, 32, 56, 64, 112, 128};
  double best = -1.0;
  for (int nt : nts)
    for (int tw : tws)
      for (int mode = 0; mode < 2; ++mode) {
        TileCfg t = *out;
        t.tile2x8 = mode;
        if (tw > nt * 16) continue;
        t.TW = tw < p.N ? tw : p.N;
        if (mode == 1) {
          if ((t.TW % 8) != 0 || p.M < 2 || nt < t.TW / 8) continue;
          t.TH = 2 * (nt / (t.TW / 8));
        } else {
          t.TH = nt * 16 / t.TW;
        }
        if (t.TH > p.M) t.TH = p.M;
        if (t.TH < 1) continue;
        t.lsh = pointwise ? 1 : p.sh;
        t.lsw = pointwise ? 1 : p.sw;
        t.gsh = pointwise ? p.sh : 1;
        t.gsw = pointwise ? p.sw : 1;
        t.TPH = (t.TH - 1) * t.lsh + (pointwise ? 1 : p.H);
        t.TPW = (t.TW - 1) * t.lsw + (pointwise ? 1 : p.K);
        if (t.TPH * t.gsh >= 1024 || t.TPW * t.gsw >= 1024) continue;
        if ((int64_t)t.TPH * t.TPW * (slab / BSP_CHUNK) > 256 * kStagePieces) continue;
        t.tiles_y = (p.M + t.TH - 1) / t.TH;
        t.tiles_x = (p.N + t.TW - 1) / t.TW;
        // paddings: fewest conflicts first, then least LDS
        int best_ex = 1 << 30;
        int64_t best_lds = 0;
        int brp = 0, bpp = 0;
        for (int rp = 0; rp <= 112; rp += 16)
          for (int pp = 0; pp <= 240; pp += 16) {
            t.row_bytes = slab * 2 + rp;
            t.pitch = t.TPW * t.row_bytes + pp;
            const int64_t ldsb = (int64_t)t.TPH * t.pitch;
            if (ldsb > kMaxLds) continue;
            const int ex = conflict_excess(t, nt);
            if (ex < best_ex || (ex == best_ex && ldsb < best_lds)) {
              best_ex = ex;
              best_lds = ldsb;
              brp = rp;
              bpp = pp;
            }
          }
        if (best_ex == (1 << 30)) continue;
        t.row_bytes = slab * 2 + brp;
        t.pitch = t.TPW * t.row_bytes + bpp;
        const double util = (double)p.M * p.N / ((double)t.tiles_y * t.tiles_x * nt * 16);
        const double halo = (double)t.TPH * t.TPW / ((double)t.TH * t.TW * t.lsh * t.lsw);
        const double score = util - 0.02 * halo - 0.05 * best_ex / nt + 0.001 * nt;
        if (score > best) {
          best = score;
          *NT = nt;
          *out = t;
        }
      }
  return best >= 0.0;
}

int device_cus() {
  static int cus = 0;
  if (cus == 0) {
    int dev = 0, v = 0;
    if (hipGetDevice(&dev) == hipSuccess &&
        hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && v > 0)
      cus = v;
    else
      cus = 256;
  }
  return cus;
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
  {
    // the search is a pure function of the shape: remember its answers
    static std::mutex mu;
    static std::map<std::array<int32_t, 10>, std::pair<int, TileCfg>> memo;
    const std::array<int32_t, 10> key = {p.M, p.N, p.I, p.O, p.H, p.K, p.sh, p.sw, p.ph, p.pw};
    std::lock_guard<std::mutex> lock(mu);
    auto it = memo.find(key);
    if (it == memo.end()) {
      t.slab = bsp_slab_channels(p.I, p.H, p.K);
      t.nslabs = ((p.I + 7) / 8 + t.slab / 8 - 1) / (t.slab / 8);
      t.nstrips = (p.O + BSP_STRIP - 1) / BSP_STRIP;
      if (!choose_tile(p, t.slab, &NT, &t)) NT = 0;
      if (memo.size() > 4096) memo.clear();
      it = memo.emplace(key, std::make_pair(NT, t)).first;
    }
    NT = it->second.first;
    t = it->second.second;
    if (NT == 0) return BSP_ERR_UNSUPPORTED;
  }
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
  const int64_t nitems = ntiles * groups;
  if (nitems > 0x7FFFFFFF) return BSP_ERR_SHAPE;
  t.ntiles = (int32_t)ntiles;
  t.nitems = (int32_t)nitems;
  // persistent grid: at most two workgroups per CU, every workgroup the same item count
  const int64_t max_wg = 2 * (int64_t)device_cus();
  const int64_t per = (nitems + max_wg - 1) / max_wg;
  const int64_t nwg = (nitems + per - 1) / per;
  dim3 grid((unsigned)nwg), block(256);
  const size_t ldsb = (size_t)t.TPH * t.pitch;
  switch (NT) {
    case 4: hipLaunchKernelGGL(conv_tile_bf16<4>, grid, block, ldsb, st, p, t); break;
    case 7: hipLaunchKernelGGL(conv_tile_bf16<7>, grid, block, ldsb, st, p, t); break;
    case 8: hipLaunchKernelGGL(conv_tile_bf16<8>, grid, block, ldsb, st, p, t); break;
    default: return BSP_ERR_UNSUPPORTED;
  }
  return hipGetLastError() == hipSuccess ? BSP_OK : BSP_ERR_HIP;
}
