// Weights-resident variant of the LDS-tiled bf16 kernel, for layers whose whole
// weight set for a group of four strips fits in LDS next to one input patch
// (single slab of input channels, short strips: 3x3 layers with 64 input
// channels, 1x1 layers with up to 256).
//
// Such layers have so few steps per strip that fetching weight fragments from
// L2 while computing never reaches a steady state; the memory latency of every
// fragment is exposed.  Here a persistent workgroup copies its four strips'
// fragments into LDS once (each wave its own strip, all loads in flight
// together), turns the step descriptors into ready LDS offsets, and then walks
// many pixel tiles: the hot loop reads only LDS (weights, offsets, activations,
// each one step ahead) and issues MFMAs, while the global loads for the next
// tile's patch are already in flight in registers.
#include "bsp_launch.h"
#include "bsp_tile.h"

#include <array>
#include <map>
#include <mutex>

namespace {

struct WresCfg {
  int32_t xbuf_bytes;     // LDS bytes of the input patch
  int32_t obuf_off;       // LDS offset of the output staging tile: [NT*16 pixels][64 ch + pad]
  int32_t region_bytes;   // LDS bytes per wave: maxsteps fragments + maxsteps offset quads
  int32_t maxsteps;       // most steps any strip has
  int32_t groups;         // strip groups (of four)
  int32_t wg_per_group;   // workgroups sharing one strip group
  int32_t off_slab, off_xdesc, off_wfrag;  // plan sections, in words (read on the host)
  FastDiv d_groups;
};

constexpr int kWBatch = 12;   // per wave; the waves sharing a strip split its fragments
constexpr int kPH = 2;        // waves per strip, each taking a share of the tile's pixel tiles  // weight fragments a lane keeps in flight while copying

template <int NT>
__device__ __forceinline__ void load_b_at(u32x4_t (&b)[NT], const int xoff,
                                          const unsigned char* lds, const int (&base)[NT]) {
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) b[nt] = *(const u32x4_t*)(lds + base[nt] + xoff);
}

template <int NT, int PH>
__global__ __launch_bounds__(256 * PH, 1) void conv_wres_bf16(ConvParams p, TileCfg t, WresCfg c) {
  constexpr int kThreads = 256 * PH;
  extern __shared__ __align__(16) unsigned char lds[];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave_all = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wave = wave_all & 3;   // which strip of the group
  const int half = wave_all >> 2;  // which share of the tile's pixel tiles
  const int jn = lane & 15, g = lane >> 4;

  const uint32_t bid = blockIdx.x;
  const int cidx = (int)fdiv(bid, c.d_groups);
  const int sg = (int)bid - cidx * c.groups;
  int tile = cidx;
  if (tile >= t.ntiles) return;

  const uint16_t* X = (const uint16_t*)p.X;
  const int tpi = t.tiles_y * t.tiles_x;

  // ---- per-thread staging map (same for every tile): piece u -> LDS offset, patch pixel, channel
  const int PP = t.slab / BSP_CHUNK;
  const int npieces = t.TPH * t.TPW * PP;
  int sdst[kStageBatch], sinfo[kStageBatch], soff[kStageBatch];
#pragma unroll
  for (int u = 0; u < kStageBatch; ++u) {
    const int idx = tid + u * kThreads;
    const uint32_t pix = fdiv((uint32_t)idx, t.d_pp);
    const int part = idx - (int)pix * PP;
    const int py = (int)fdiv(pix, t.d_tpw);
    const int px = (int)pix - py * t.TPW;
    const bool live = idx < npieces && part * BSP_CHUNK < p.I;
    sdst[u] = idx < npieces ? py * t.pitch + px * t.row_bytes + part * 16 : -1;
    sinfo[u] = live ? ((py * t.gsh) | ((px * t.gsw) << 16)) : -1;
    soff[u] = ((py * t.gsh) * p.J + px * t.gsw) * p.I + part * BSP_CHUNK;  // elements from the patch origin
  }
  u32x4_t sv[kStageBatch];
  // X + origin of the patch may point before the image (padding); only in-image pieces are read
  auto issue_patch = [&](int tl) {
    const int n = (int)fdiv((uint32_t)tl, t.d_tpi);
    const int trem = tl - n * tpi;
    const int tyi = (int)fdiv((uint32_t)trem, t.d_tiles_x);
    const int iy_org = tyi * t.TH * p.sh - p.ph;
    const int ix_org = (trem - tyi * t.tiles_x) * t.TW * p.sw - p.pw;
    const uint16_t* org = X + (((int64_t)n * p.L + iy_org) * p.J + ix_org) * p.I;
    const bool interior = iy_org >= 0 && ix_org >= 0 && iy_org + (t.TPH - 1) * t.gsh < p.L &&
                          ix_org + (t.TPW - 1) * t.gsw < p.J;
    if (interior) {
#pragma unroll
      for (int u = 0; u < kStageBatch; ++u) {
        sv[u] = u32x4_t{0u, 0u, 0u, 0u};
        if (sinfo[u] >= 0) sv[u] = *(const u32x4_t*)(org + soff[u]);
      }
    } else {
#pragma unroll
      for (int u = 0; u < kStageBatch; ++u) {
        sv[u] = u32x4_t{0u, 0u, 0u, 0u};
        const int iy = iy_org + (sinfo[u] & 0xFFFF), ix = ix_org + (sinfo[u] >> 16);
        if (sinfo[u] >= 0 && (unsigned)iy < (unsigned)p.L && (unsigned)ix < (unsigned)p.J)
          sv[u] = *(const u32x4_t*)(org + soff[u]);
      }
    }
  };
  auto store_patch = [&]() {
#pragma unroll
    for (int u = 0; u < kStageBatch; ++u)
      if (sdst[u] >= 0) *(u32x4_t*)(lds + sdst[u]) = sv[u];
  };

  issue_patch(tile);

  // ---- this wave's strip: fragments and ready-made LDS offsets into the wave's region
  const int32_t* plan = p.plan;
  const int32_t* slab_ptr = plan + c.off_slab;
  const int32_t* xdesc = plan + c.off_xdesc;
  const u32x4_t* wfrag = (const u32x4_t*)(plan + c.off_wfrag);
  const int strip = sg * 4 + wave;
  const bool valid = strip < t.nstrips;
  u32x4_t* wl = (u32x4_t*)(lds + c.xbuf_bytes + wave * c.region_bytes);
  int* xo = (int*)(lds + c.xbuf_bytes + wave * c.region_bytes + c.maxsteps * 1024);
  int nst = 0;
  float bv[4] = {0.f, 0.f, 0.f, 0.f};
  if (valid) {
    const int s0 = slab_ptr[strip * 2], s1 = slab_ptr[strip * 2 + 1];
    nst = min(s1 - s0, c.maxsteps);
    // request everything first (fragments, descriptors, bias), consume afterwards, so the
    // memory latencies overlap each other and the patch loads already in flight
    const int ch = strip * BSP_STRIP + 4 * g;
    int dsc[2] = {0, 0};  // descriptors of (step, group) pairs lane and lane + 64
#pragma unroll
    for (int k = 0; k < 2; ++k)
      if (half == 0 && lane + 64 * k < nst * 4) dsc[k] = xdesc[s0 * 4 + lane + 64 * k];
#pragma unroll
    for (int r = 0; r < 4; ++r) bv[r] = (p.bias && ch + r < p.O) ? p.bias[ch + r] : 0.f;
    // the PH waves that share this strip copy alternate fragments
    for (int b0 = half; b0 < nst; b0 += kWBatch * PH) {
      u32x4_t wv[kWBatch];
#pragma unroll
      for (int u = 0; u < kWBatch; ++u)
        if (b0 + u * PH < nst) wv[u] = wfrag[(int64_t)(s0 + b0 + u * PH) * 64 + lane];
#pragma unroll
      for (int u = 0; u < kWBatch; ++u)
        if (b0 + u * PH < nst) wl[(b0 + u * PH) * 64 + lane] = wv[u];
    }
#pragma unroll
    for (int k = 0; k < 2; ++k)
      if (half == 0 && lane + 64 * k < nst * 4) {
        const int d = dsc[k];
        xo[lane + 64 * k] =
            ((d >> 16) & 0xFF) * t.pitch + ((d >> 24) & 0xFF) * t.row_bytes + (d & 0xFFFF) * 16;
      }
    for (int i = lane + 128; half == 0 && i < nst * 4; i += 64) {  // strips longer than 32 steps
      const int d = xdesc[s0 * 4 + i];
      xo[i] = ((d >> 16) & 0xFF) * t.pitch + ((d >> 24) & 0xFF) * t.row_bytes + (d & 0xFFFF) * 16;
    }
  }

  // ---- per-lane output pixel map: LDS base, position in the tile, offset in Y from the tile origin
  int base[NT];
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) {
    const int gt = half * NT + nt;  // pixel tile within the workgroup's tile
    int ty, tx;
    if (t.tile2x8) {
      const int tr = (int)fdiv((uint32_t)gt, t.d_tpr), tc = gt - tr * (t.TW >> 3);
      ty = tr * 2 + (jn >> 3);
      tx = tc * 8 + (jn & 7);
    } else {
      const int pi = gt * 16 + jn;
      ty = (int)fdiv((uint32_t)pi, t.d_tw);
      tx = pi - ty * t.TW;
    }
    const bool in_tile = ty < t.TH && tx < t.TW;
    base[nt] = in_tile ? (ty * t.lsh) * t.pitch + (tx * t.lsw) * t.row_bytes : 0;
  }

#ifdef BSP_EXP_STAGGER
  if (blockIdx.x >= 256) __builtin_amdgcn_s_sleep(BSP_EXP_STAGGER);
#endif
  // ---- cooperative store map: the tile's results leave LDS as whole 16-byte pieces, eight
  // consecutive lanes covering the 64 output channels (128 bytes) of one pixel
  constexpr int kOutRow = 4 * BSP_STRIP * 2 + 16;        // bytes per pixel in the staging tile
  constexpr int kOutPieces = (NT * PH * 16 * 8 + kThreads - 1) / kThreads;  // pieces per thread
  int csrc[kOutPieces], cpyx[kOutPieces], coff[kOutPieces];
#pragma unroll
  for (int k = 0; k < kOutPieces; ++k) {
    const int q = tid + k * kThreads;
    const int pi = q >> 3, part = q & 7;
    const int nt = pi >> 4, j = pi & 15;
    int ty, tx;
    if (t.tile2x8) {
      const int tr = (int)fdiv((uint32_t)nt, t.d_tpr), tc = nt - tr * (t.TW >> 3);
      ty = tr * 2 + (j >> 3);
      tx = tc * 8 + (j & 7);
    } else {
      ty = (int)fdiv((uint32_t)pi, t.d_tw);
      tx = pi - ty * t.TW;
    }
    const bool live = nt < NT * PH && ty < t.TH && tx < t.TW && sg * 64 + part * 8 < p.O;
    csrc[k] = c.obuf_off + pi * kOutRow + part * 16;
    cpyx[k] = live ? (ty | (tx << 16)) : -1;
    coff[k] = (ty * p.N + tx) * p.O + sg * 64 + part * 8;
  }
  // where this lane's four channels of pixel jn of pixel tile nt go in the staging tile
  const int orow = c.obuf_off + (half * NT * 16 + jn) * kOutRow + wave * (BSP_STRIP * 2) + g * 8;

  store_patch();
  __syncthreads();

  uint16_t* Y = (uint16_t*)p.Y;
  int prev = -1;  // tile whose results sit in the staging tile
  auto flush = [&](int tl) {
    const int n = (int)fdiv((uint32_t)tl, t.d_tpi);
    const int trem = tl - n * tpi;
    const int tyi = (int)fdiv((uint32_t)trem, t.d_tiles_x);
    const int oy0 = tyi * t.TH, ox0 = (trem - tyi * t.tiles_x) * t.TW;
    uint16_t* yorg = Y + (((int64_t)n * p.M + oy0) * p.N + ox0) * p.O;
    const bool whole = oy0 + t.TH <= p.M && ox0 + t.TW <= p.N;
#pragma unroll
    for (int k = 0; k < kOutPieces; ++k) {
      if (cpyx[k] < 0) continue;
      if (!whole && (oy0 + (cpyx[k] & 0xFFFF) >= p.M || ox0 + (cpyx[k] >> 16) >= p.N)) continue;
      *(u32x4_t*)(yorg + coff[k]) = *(const u32x4_t*)(lds + csrc[k]);
    }
  };
  while (true) {
    const int next = tile + c.wg_per_group;
    const bool more = next < t.ntiles;
    if (more) issue_patch(next);  // lands in registers while this tile is computed

    if (valid) {
      f32x4_t acc[NT];
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) acc[nt] = f32x4_t{0.f, 0.f, 0.f, 0.f};
      if (nst > 0) {
        // everything one step ahead: fragment a, activations b; offsets two steps ahead
        u32x4_t a[2], b[2][NT];
        const int lastq = nst - 1;
        int x1 = xo[min(1, lastq) * 4 + g];
        a[0] = wl[lane];
        load_b_at<NT>(b[0], xo[g], lds, base);
        for (int s = 0; s < nst; s += 2) {
          const int x2 = xo[min(s + 2, lastq) * 4 + g];
          a[1] = wl[min(s + 1, lastq) * 64 + lane];
          load_b_at<NT>(b[1], x1, lds, base);
          do_mma<NT>(acc, a[0], b[0]);
          if (s + 1 < nst) {
            x1 = xo[min(s + 3, lastq) * 4 + g];
            a[0] = wl[min(s + 2, lastq) * 64 + lane];
            load_b_at<NT>(b[0], x2, lds, base);
            do_mma<NT>(acc, a[1], b[1]);
          }
        }
      }
      // epilogue: lane holds channels 4g..4g+3 of pixel jn of every pixel tile
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) {
        u32x2_t v;
        v.x = pack_bf16x2(acc[nt][0] + bv[0], acc[nt][1] + bv[1]);
        v.y = pack_bf16x2(acc[nt][2] + bv[2], acc[nt][3] + bv[3]);
        *(u32x2_t*)(lds + orow + nt * 16 * kOutRow) = v;
      }
    }
    prev = tile;
    __syncthreads();  // results staged; everyone is done reading the patch
    flush(prev);
    if (!more) break;
    store_patch();
    __syncthreads();
    tile = next;
  }
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

constexpr int64_t kLdsPerCu = 160 * 1024;

template <int NT, int PH>
int launch(const ConvParams& p, const TileCfg& t, const WresCfg& c, dim3 grid, size_t ldsb,
           hipStream_t st) {
  static bool raised = false;  // dynamic LDS above 64 KB has to be allowed once per kernel
  if (!raised) {
    if (hipFuncSetAttribute((const void*)conv_wres_bf16<NT, PH>,
                            hipFuncAttributeMaxDynamicSharedMemorySize,
                            (int)kLdsPerCu) != hipSuccess)
      return BSP_ERR_HIP;
    raised = true;
  }
  hipLaunchKernelGGL((conv_wres_bf16<NT, PH>), grid, dim3(256 * PH), ldsb, st, p, t, c);
  return hipGetLastError() == hipSuccess ? BSP_OK : BSP_ERR_HIP;
}

}  // namespace

int bsp_launch_wres(const ConvParams& p_in, int dtype, const void* plan_host, hipStream_t st) {
  if (!plan_host || dtype != BSP_BF16 || (p_in.I % 8) != 0 || (p_in.O % 8) != 0)
    return BSP_ERR_UNSUPPORTED;
  const int32_t* hdr = (const int32_t*)plan_host;
  if (hdr[BSP_PLAN_MAGIC_W] != BSP_PLAN_MAGIC || hdr[BSP_PLAN_VERSION_W] != BSP_PLAN_VERSION ||
      hdr[BSP_PLAN_O_W] != p_in.O || hdr[BSP_PLAN_I_W] != p_in.I || hdr[BSP_PLAN_H_W] != p_in.H ||
      hdr[BSP_PLAN_K_W] != p_in.K || hdr[BSP_PLAN_DTYPE_W] != BSP_BF16)
    return BSP_ERR_UNSUPPORTED;
  if (hdr[BSP_PLAN_NSLABS_W] != 1 || hdr[BSP_PLAN_MAXSTEPS_W] < 1) return BSP_ERR_UNSUPPORTED;
  ConvParams p = p_in;
  if (p.H == 1 && p.K == 1 && p.sh == 1 && p.sw == 1 && p.ph == 0 && p.pw == 0) {
    p.J = p.N = p.P;
    p.L = p.M = 1;
    p.B = 1;
  }
  WresCfg c;
  c.maxsteps = hdr[BSP_PLAN_MAXSTEPS_W];
  c.region_bytes = c.maxsteps * (1024 + 16);
  const int64_t wbytes = 4ll * c.region_bytes;
  if (wbytes > kLdsPerCu - 32 * 1024) return BSP_ERR_UNSUPPORTED;

  TileCfg t;
  int NT = 0;
  {
    static std::mutex mu;
    static std::map<std::array<int32_t, 11>, std::pair<int, TileCfg>> memo;
    const std::array<int32_t, 11> key = {p.M, p.N, p.I, p.O, p.H, p.K, p.sh, p.sw, p.ph, p.pw,
                                         c.maxsteps};
    std::lock_guard<std::mutex> lock(mu);
    auto it = memo.find(key);
    if (it == memo.end()) {
      t.slab = bsp_slab_channels(p.I, p.H, p.K);
      t.nslabs = 1;
      t.nstrips = (p.O + BSP_STRIP - 1) / BSP_STRIP;
      // two workgroups per CU if the patch leaves room for that, else one
      // eight waves (two per strip) and one workgroup per CU; the LDS left after the
      // weights holds the patch and the results staging tile
      if (!bsp_choose_tile(p, t.slab, kLdsPerCu - wbytes, 512 * kStageBatch, kPH,
                           4 * BSP_STRIP * 2 + 16, &NT, &t))
        NT = 0;
      if (memo.size() > 4096) memo.clear();
      it = memo.emplace(key, std::make_pair(NT, t)).first;
    }
    NT = it->second.first;
    t = it->second.second;
    if (NT == 0) return BSP_ERR_UNSUPPORTED;
  }
  if (t.TPH * t.gsh >= 1024 || t.TPW * t.gsw >= 1024) return BSP_ERR_UNSUPPORTED;
  const int64_t ntiles = (int64_t)p.B * t.tiles_y * t.tiles_x;
  c.xbuf_bytes = (t.TPH * t.pitch + 15) & ~15;
  c.obuf_off = c.xbuf_bytes + (int32_t)wbytes;
  const size_t ldsb = (size_t)c.obuf_off + (size_t)NT * kPH * 16 * (4 * BSP_STRIP * 2 + 16);
  if ((int64_t)ldsb > kLdsPerCu) return BSP_ERR_UNSUPPORTED;
  c.groups = (t.nstrips + 3) / 4;
  // persistent grid: as many workgroups as fit at once, every one the same tile count
  const int64_t per_cu = 1;
  int64_t slots = per_cu * device_cus() / c.groups;
  if (slots < 1) slots = 1;
  c.wg_per_group = (int32_t)(ntiles < slots ? ntiles : slots);
  const int64_t nwg = (int64_t)c.wg_per_group * c.groups;
  const int64_t npieces = (int64_t)t.TPH * t.TPW * (t.slab / BSP_CHUNK);
  if (nwg >= (1 << 24) || ntiles >= (1 << 24) || npieces > 512 * kStageBatch ||
      (npieces + 2048) * t.TPW >= (1ll << 32))
    return BSP_ERR_UNSUPPORTED;
  t.spc = 4;
  t.ntiles = (int32_t)ntiles;
  t.d_pp = make_fastdiv(t.slab / BSP_CHUNK);
  t.d_tpw = make_fastdiv(t.TPW);
  t.d_tw = make_fastdiv(t.TW);
  t.d_tpr = make_fastdiv(t.TW >= 8 ? t.TW >> 3 : 1);
  t.d_ntiles = make_fastdiv((uint32_t)ntiles);
  t.d_tpi = make_fastdiv(t.tiles_y * t.tiles_x);
  t.d_tiles_x = make_fastdiv(t.tiles_x);
  c.d_groups = make_fastdiv(c.groups);
  c.off_slab = hdr[BSP_PLAN_OFF_SLAB_W];
  c.off_xdesc = hdr[BSP_PLAN_OFF_XDESC_W];
  c.off_wfrag = hdr[BSP_PLAN_OFF_WFRAG_W];
  dim3 grid((unsigned)nwg);
  switch (NT) {
    case 4: return launch<4, kPH>(p, t, c, grid, ldsb, st);
    case 7: return launch<7, kPH>(p, t, c, grid, ldsb, st);
    case 8: return launch<8, kPH>(p, t, c, grid, ldsb, st);
    default: return BSP_ERR_UNSUPPORTED;
  }
}
