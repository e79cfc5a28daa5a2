// LDS-resident variant of the tiled bf16 kernel: weights AND activations of the
// current slab of input channels live in LDS, the hot loop touches nothing else.
//
// A persistent workgroup of eight waves owns a group of four strips (wave w:
// strip w & 3, pixel-tile share w >> 2) and walks units = (pixel tile of an
// image, slab of input channels).  For each unit the input patch of the slab
// and the four strips' weight fragments of the slab are copied into LDS, the
// step descriptors are turned into ready LDS offsets, and the waves run the
// slab's steps reading only LDS (weights, offsets and activations each one
// step ahead of the MFMAs).  While a unit is computed, the global loads of the
// NEXT unit are already in flight into registers, so their latency is hidden
// and, since the loop issues no other vector memory operation, nothing queues
// up behind them.  When all of a layer's input channels fit one slab the
// weights are copied once and stay for every tile the workgroup visits.  After
// the last slab of a tile the results (+ bias, rounded once to bf16) go through
// an LDS staging tile and leave as whole 16-byte pieces, eight lanes per pixel.
//
// Only kept blocks have steps (paper Section I, advantages 3-4): work and
// weight traffic shrink with the mask, the patch traffic does not.
#include "bsp_launch.h"
#include "bsp_tile.h"

#include <array>
#include <map>
#include <mutex>

namespace {

constexpr int kPH = 2;             // waves per strip, each taking a share of the tile's pixel tiles
constexpr int kThreads = 256 * kPH;
constexpr int kXBatch = 8;         // 16-byte patch pieces a thread keeps in flight
constexpr int kWBatch = 10;        // weight fragments a lane keeps in flight (its share of a slab)
constexpr int kMaxSlabs = 32;
constexpr int kOutRow = 4 * BSP_STRIP * 2 + 16;  // bytes per pixel in the results staging tile

struct LdsCfg {
  int32_t wbuf_off;       // LDS offset of the weight regions (after the patch)
  int32_t region_bytes;   // per strip: maxsteps fragments + maxsteps offset quads
  int32_t obuf_off;       // LDS offset of the results staging tile
  int32_t sp_off;         // LDS offset of the step-range table [4][nslabs + 1]
  int32_t maxsteps;       // most steps any (strip, slab) has
  int32_t groups;         // strip groups (of four)
  int32_t wg_per_group;   // workgroups sharing one strip group
  int32_t off_slab, off_xdesc, off_wfrag;  // plan sections, in words (read on the host)
  FastDiv d_groups;
};

template <int NT>
__device__ __forceinline__ void load_b_at(u32x4_t (&b)[NT], const int xoff,
                                          const unsigned char* lds, const int (&base)[NT]) {
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) b[nt] = *(const u32x4_t*)(lds + base[nt] + xoff);
}

template <int NT>
__global__ __launch_bounds__(kThreads, 1) void conv_lds_bf16(ConvParams p, TileCfg t, LdsCfg c) {
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
  const int32_t* plan = p.plan;
  const int32_t* slab_ptr = plan + c.off_slab;
  const int32_t* xdesc = plan + c.off_xdesc;
  const u32x4_t* wfrag = (const u32x4_t*)(plan + c.off_wfrag);
  const int tpi = t.tiles_y * t.tiles_x;
  const int strip = sg * 4 + wave;
  const bool valid = strip < t.nstrips;
  const int nsl1 = t.nslabs + 1;

  // ---- step ranges of the group's four strips, all slabs: LDS table sp[4][nslabs+1]
  int* sp = (int*)(lds + c.sp_off);
  if (tid < 4 * nsl1) {
    const int w = tid / nsl1, k = tid - w * nsl1;
    const int st = sg * 4 + w;
    sp[tid] = st < t.nstrips ? slab_ptr[st * nsl1 + k] : 0;
  }

  // ---- per-thread patch map (same for every unit): piece u -> LDS offset, patch pixel, offset in X
  const int PP = t.slab / BSP_CHUNK;
  const int npieces = t.TPH * t.TPW * PP;
  int sdst[kXBatch], sinfo[kXBatch], soff[kXBatch];
#pragma unroll
  for (int u = 0; u < kXBatch; ++u) {
    const int idx = tid + u * kThreads;
    const uint32_t pix = fdiv((uint32_t)idx, t.d_pp);
    const int part = idx - (int)pix * PP;
    const int py = (int)fdiv(pix, t.d_tpw);
    const int px = (int)pix - py * t.TPW;
    sdst[u] = idx < npieces ? py * t.pitch + px * t.row_bytes + part * 16 : -1;
    sinfo[u] = idx < npieces ? ((py * t.gsh) | ((px * t.gsw) << 16) | (part << 26)) : -1;
    soff[u] = ((py * t.gsh) * p.J + px * t.gsw) * p.I + part * BSP_CHUNK;  // elements from the patch origin
  }

  // ---- registers the next unit's data lands in
  u32x4_t xv[kXBatch], wv[kWBatch];
  int dsc[2] = {0, 0};
  int w_nst = 0;  // steps of the (strip, slab) in flight
  u32x4_t* wl = (u32x4_t*)(lds + c.wbuf_off + wave * c.region_bytes);
  int* xo = (int*)(lds + c.wbuf_off + wave * c.region_bytes + c.maxsteps * 1024);

  // X + origin of the patch may point before the image (padding); only in-image pieces are read
  auto issue_patch = [&](int tl, int sl) {
    const int n = (int)fdiv((uint32_t)tl, t.d_tpi);
    const int trem = tl - n * tpi;
    const int tyi = (int)fdiv((uint32_t)trem, t.d_tiles_x);
    const int iy_org = tyi * t.TH * p.sh - p.ph;
    const int ix_org = (trem - tyi * t.tiles_x) * t.TW * p.sw - p.pw;
    const int ch0 = sl * t.slab;
    const uint16_t* org = X + (((int64_t)n * p.L + iy_org) * p.J + ix_org) * p.I + ch0;
    const bool interior = iy_org >= 0 && ix_org >= 0 && iy_org + (t.TPH - 1) * t.gsh < p.L &&
                          ix_org + (t.TPW - 1) * t.gsw < p.J && ch0 + t.slab <= p.I;
    if (interior) {
#pragma unroll
      for (int u = 0; u < kXBatch; ++u) {
        xv[u] = u32x4_t{0u, 0u, 0u, 0u};
        if (sinfo[u] >= 0) xv[u] = *(const u32x4_t*)(org + soff[u]);
      }
    } else {
#pragma unroll
      for (int u = 0; u < kXBatch; ++u) {
        xv[u] = u32x4_t{0u, 0u, 0u, 0u};
        const int iy = iy_org + (sinfo[u] & 0x3FF), ix = ix_org + ((sinfo[u] >> 16) & 0x3FF);
        const int ch = ch0 + (sinfo[u] >> 26) * BSP_CHUNK;
        if (sinfo[u] >= 0 && (unsigned)iy < (unsigned)p.L && (unsigned)ix < (unsigned)p.J && ch < p.I)
          xv[u] = *(const u32x4_t*)(org + soff[u]);
      }
    }
  };
  // this wave's share of its strip's fragments of a slab (alternate steps) and, on the
  // first of the two waves, the step descriptors; s0 / steps come from the LDS table
  auto issue_weights = [&](int s0, int nst) {
    w_nst = nst;
#pragma unroll
    for (int u = 0; u < kWBatch; ++u)
      if (half + u * kPH < nst) wv[u] = wfrag[(int64_t)(s0 + half + u * kPH) * 64 + lane];
#pragma unroll
    for (int k = 0; k < 2; ++k)
      if (half == 0 && lane + 64 * k < nst * 4) dsc[k] = xdesc[s0 * 4 + lane + 64 * k];
  };
  auto commit_patch = [&]() {
#pragma unroll
    for (int u = 0; u < kXBatch; ++u)
      if (sdst[u] >= 0) *(u32x4_t*)(lds + sdst[u]) = xv[u];
  };
  auto commit_weights = [&]() {
#pragma unroll
    for (int u = 0; u < kWBatch; ++u)
      if (half + u * kPH < w_nst) wl[(half + u * kPH) * 64 + lane] = wv[u];
#pragma unroll
    for (int k = 0; k < 2; ++k)
      if (half == 0 && lane + 64 * k < w_nst * 4) {
        const int d = dsc[k];
        xo[lane + 64 * k] =
            ((d >> 16) & 0xFF) * t.pitch + ((d >> 24) & 0xFF) * t.row_bytes + (d & 0xFFFF) * 16;
      }
  };

  // ---- first unit: patch first (needs nothing from the plan), then weights
  issue_patch(tile, 0);
  __syncthreads();  // step-range table visible
  const bool reload_w = t.nslabs > 1;
  if (valid) issue_weights(sp[wave * nsl1], sp[wave * nsl1 + 1] - sp[wave * nsl1]);
  float bv[4] = {0.f, 0.f, 0.f, 0.f};
  const int ch = strip * BSP_STRIP + 4 * g;
  if (valid) {
#pragma unroll
    for (int r = 0; r < 4; ++r) bv[r] = (p.bias && ch + r < p.O) ? p.bias[ch + r] : 0.f;
  }

  // ---- per-lane pixel map: LDS base of each of this wave's pixel tiles
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
  // ---- cooperative store map: results leave LDS as whole 16-byte pieces, eight
  // consecutive lanes covering the 64 output channels (128 bytes) of one pixel
  constexpr int kOutPieces = (NT * kPH * 16 * 8 + kThreads - 1) / kThreads;
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
    const bool live = nt < NT * kPH && ty < t.TH && tx < t.TW && sg * 64 + part * 8 < p.O;
    csrc[k] = c.obuf_off + pi * kOutRow + part * 16;
    cpyx[k] = live ? (ty | (tx << 16)) : -1;
    coff[k] = (ty * p.N + tx) * p.O + sg * 64 + part * 8;
  }
  // where this lane's four channels of pixel jn of pixel tile nt go in the staging tile
  const int orow = c.obuf_off + (half * NT * 16 + jn) * kOutRow + wave * (BSP_STRIP * 2) + g * 8;

  uint16_t* Y = (uint16_t*)p.Y;
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

  f32x4_t acc[NT];
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) acc[nt] = f32x4_t{0.f, 0.f, 0.f, 0.f};

  int sl = 0;
  bool w_pending = true;  // weights for the unit about to start are in registers, not yet in LDS
  while (true) {
    // ---- registers -> LDS for this unit
    commit_patch();
    if (w_pending && valid) commit_weights();
    const int nst = valid ? sp[wave * nsl1 + sl + 1] - sp[wave * nsl1 + sl] : 0;
    __syncthreads();

    // ---- next unit's loads fly while this one is computed
    int ntile = tile, nsl = sl + 1;
    if (nsl == t.nslabs) {
      nsl = 0;
      ntile = tile + c.wg_per_group;
    }
    const bool more = ntile < t.ntiles;
    // The two waves that share a SIMD go through "fetch the next unit" and "compute this
    // one" in opposite order, so one's address traffic overlaps the other's MFMAs.
    auto fetch_next = [&]() {
      if (!more) return;
      issue_patch(ntile, nsl);
      if (reload_w && valid)
        issue_weights(sp[wave * nsl1 + nsl], sp[wave * nsl1 + nsl + 1] - sp[wave * nsl1 + nsl]);
    };
    if (half == 0) fetch_next();
    w_pending = reload_w;

    // ---- this slab's steps, everything from LDS and one step ahead (offsets two)
    if (nst > 0) {
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
    if (half != 0) fetch_next();
    const bool last_slab = sl == t.nslabs - 1;
    if (last_slab && valid) {
      // lane holds channels 4g..4g+3 of pixel jn of every pixel tile
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) {
        u32x2_t v;
        v.x = pack_bf16x2(acc[nt][0] + bv[0], acc[nt][1] + bv[1]);
        v.y = pack_bf16x2(acc[nt][2] + bv[2], acc[nt][3] + bv[3]);
        acc[nt] = f32x4_t{0.f, 0.f, 0.f, 0.f};
        *(u32x2_t*)(lds + orow + nt * 16 * kOutRow) = v;
      }
    }
    __syncthreads();  // patch and weights may be overwritten; results are staged
    if (last_slab) flush(tile);
    if (!more) break;
    tile = ntile;
    sl = nsl;
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

template <int NT>
int launch(const ConvParams& p, const TileCfg& t, const LdsCfg& c, dim3 grid, size_t ldsb,
           hipStream_t st) {
  static bool raised = false;  // dynamic LDS above 64 KB has to be allowed once per kernel
  if (!raised) {
    if (hipFuncSetAttribute((const void*)conv_lds_bf16<NT>,
                            hipFuncAttributeMaxDynamicSharedMemorySize,
                            (int)kLdsPerCu) != hipSuccess)
      return BSP_ERR_HIP;
    raised = true;
  }
  hipLaunchKernelGGL(conv_lds_bf16<NT>, grid, dim3(kThreads), ldsb, st, p, t, c);
  return hipGetLastError() == hipSuccess ? BSP_OK : BSP_ERR_HIP;
}

}  // namespace

int bsp_launch_lds(const ConvParams& p_in, int dtype, const void* plan_host, hipStream_t st) {
  if (!plan_host || dtype != BSP_BF16 || (p_in.I % 8) != 0 || (p_in.O % 8) != 0)
    return BSP_ERR_UNSUPPORTED;
  const int32_t* hdr = (const int32_t*)plan_host;
  if (hdr[BSP_PLAN_MAGIC_W] != BSP_PLAN_MAGIC || hdr[BSP_PLAN_VERSION_W] != BSP_PLAN_VERSION ||
      hdr[BSP_PLAN_O_W] != p_in.O || hdr[BSP_PLAN_I_W] != p_in.I || hdr[BSP_PLAN_H_W] != p_in.H ||
      hdr[BSP_PLAN_K_W] != p_in.K || hdr[BSP_PLAN_DTYPE_W] != BSP_BF16)
    return BSP_ERR_UNSUPPORTED;
  ConvParams p = p_in;
  if (p.H == 1 && p.K == 1 && p.sh == 1 && p.sw == 1 && p.ph == 0 && p.pw == 0) {
    p.J = p.N = p.P;
    p.L = p.M = 1;
    p.B = 1;
  }
  LdsCfg c;
  c.maxsteps = hdr[BSP_PLAN_MAXSLABSTEPS_W];
  const int nslabs = hdr[BSP_PLAN_NSLABS_W];
  // a lane copies every other step of a slab and two descriptors: bounds of this kernel
  if (c.maxsteps < 1 || c.maxsteps > kWBatch * kPH || c.maxsteps > 32 || nslabs > kMaxSlabs)
    return BSP_ERR_UNSUPPORTED;
  c.region_bytes = c.maxsteps * (1024 + 16);
  const int64_t wbytes = 4ll * c.region_bytes;
  const int64_t spbytes = 4 * (kMaxSlabs + 1) * 4;

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
      t.nslabs = ((p.I + 7) / 8 + t.slab / 8 - 1) / (t.slab / 8);
      t.nstrips = (p.O + BSP_STRIP - 1) / BSP_STRIP;
      // the LDS left after the weights holds the patch and the results staging tile
      if (!bsp_choose_tile(p, t.slab, kLdsPerCu - wbytes - spbytes, kThreads * kXBatch, kPH, kOutRow,
                           &NT, &t))
        NT = 0;
      if (memo.size() > 4096) memo.clear();
      it = memo.emplace(key, std::make_pair(NT, t)).first;
    }
    NT = it->second.first;
    t = it->second.second;
    if (NT == 0) return BSP_ERR_UNSUPPORTED;
  }
  if (t.nslabs != nslabs || t.slab != hdr[BSP_PLAN_SLAB_W]) return BSP_ERR_UNSUPPORTED;
  if (t.TPH * t.gsh >= 1024 || t.TPW * t.gsw >= 1024 || t.slab / BSP_CHUNK > 32)
    return BSP_ERR_UNSUPPORTED;
  const int64_t ntiles = (int64_t)p.B * t.tiles_y * t.tiles_x;
  c.wbuf_off = (t.TPH * t.pitch + 15) & ~15;
  c.obuf_off = c.wbuf_off + (int32_t)wbytes;
  c.sp_off = c.obuf_off + NT * kPH * 16 * kOutRow;
  const size_t ldsb = (size_t)c.sp_off + (size_t)spbytes;
  if ((int64_t)ldsb > kLdsPerCu) return BSP_ERR_UNSUPPORTED;
  c.groups = (t.nstrips + 3) / 4;
  // persistent grid: one workgroup per CU, shared out among the strip groups
  int64_t slots = device_cus() / c.groups;
  if (slots < 1) slots = 1;
  c.wg_per_group = (int32_t)(ntiles < slots ? ntiles : slots);
  const int64_t nwg = (int64_t)c.wg_per_group * c.groups;
  const int64_t npieces = (int64_t)t.TPH * t.TPW * (t.slab / BSP_CHUNK);
  if (nwg >= (1 << 24) || ntiles >= (1 << 24) || npieces > kThreads * kXBatch ||
      (npieces + 8 * kThreads) * t.TPW >= (1ll << 32) || (int64_t)p.L * p.J * p.I >= (1ll << 31))
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
    case 4: return launch<4>(p, t, c, grid, ldsb, st);
    case 7: return launch<7>(p, t, c, grid, ldsb, st);
    case 8: return launch<8>(p, t, c, grid, ldsb, st);
    default: return BSP_ERR_UNSUPPORTED;
  }
}
