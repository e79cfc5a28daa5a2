// LDS-tiled block-sparse implicit-GEMM convolution, bf16 in / fp32 accumulate.
//
// One workgroup (4 waves) owns a TH x TW tile of output pixels of one image and
// a group of strips (16 output channels each).  The input patch the tile needs
// (halo included, zero-filled where it leaves the image, so padding costs no
// branches in the hot loop) is staged into LDS, one slab of input channels at
// a time, and reused by every strip of the group.  A wave takes a strip and
// walks its steps from the plan: per step one contiguous 1 KB weight fragment
// (already in MFMA operand order, fetched four steps ahead) and, per 16-pixel
// tile, one 16-byte LDS read per lane gathered by the step's (chunk, tap)
// descriptor (issued one step ahead), feeding v_mfma_f32_16x16x32_bf16.  Only
// kept blocks have steps (paper Section I, advantages 3-4); the epilogue adds
// the fp32 bias and rounds once to bf16.
//
// Latency is what bounds small layers, so everything that does not depend on
// the activations (step ranges, first weight fragments, bias) is requested
// while the patch is still in flight, and a strip's successor is requested
// before the strip's own results are stored (vector memory operations retire
// in issue order, so a load issued behind a store would wait for it).
#include "bsp_launch.h"
#include "bsp_tile.h"

#include <algorithm>

#include <array>
#include <map>
#include <mutex>

#ifndef BSP_TILE_OCC
#define BSP_TILE_OCC 2
#endif

namespace {

// Ring of the next kWDepth (weight fragment, descriptor) pairs of a strip.
struct Ring {
  u32x4_t w[kWDepth];
  int d[kWDepth];
};
__device__ __forceinline__ void ring_fill(Ring& r, const u32x4_t* __restrict__ wf,
                                          const int32_t* __restrict__ xd, const int s0,
                                          const int s1, const int lane, const int g) {
  if (s0 >= s1) return;
#pragma unroll
  for (int u = 0; u < kWDepth; ++u) {
    const int i = min(s0 + u, s1 - 1);
    r.w[u] = wf[(int64_t)i * 64 + lane];
    r.d[u] = xd[i * 4 + g];
  }
}

// All steps [s0, s1) of one (strip, slab); r holds steps s0 .. s0+kWDepth-1 on
// entry.  The LDS reads of step s+1 are issued before the MFMAs of step s (two
// register sets), and the slot a step frees is refilled with the fragment
// kWDepth steps further on.
template <int NT>
__device__ __forceinline__ void run_steps(f32x4_t (&acc)[NT], Ring& r,
                                          const u32x4_t* __restrict__ wf,
                                          const int32_t* __restrict__ xd, const int s0,
                                          const int s1, const int lane, const int g,
                                          const unsigned char* lds, const int (&base)[NT],
                                          const int pitch, const int row_bytes) {
  static_assert(kWDepth % 2 == 0, "two activation register sets alternate");
  if (s0 >= s1) return;
  const int last = s1 - 1;
  u32x4_t b[2][NT];
  load_b<NT>(b[0], r.d[0], lds, base, pitch, row_bytes);
  int s = s0;
  for (; s + kWDepth <= s1; s += kWDepth) {
#pragma unroll
    for (int u = 0; u < kWDepth; ++u) {
      const u32x4_t a = r.w[u];
      load_b<NT>(b[(u + 1) & 1], r.d[(u + 1) % kWDepth], lds, base, pitch, row_bytes);
      const int i = min(s + u + kWDepth, last);
      r.w[u] = wf[(int64_t)i * 64 + lane];
      r.d[u] = xd[i * 4 + g];
      do_mma<NT>(acc, a, b[u & 1]);
    }
  }
  const int rem = s1 - s;  // fewer than kWDepth steps left; b[0] holds step s
#pragma unroll
  for (int u = 0; u < kWDepth - 1; ++u) {
    if (u < rem) {
      if (u + 1 < rem) load_b<NT>(b[(u + 1) & 1], r.d[u + 1], lds, base, pitch, row_bytes);
      do_mma<NT>(acc, r.w[u], b[u & 1]);
    }
  }
}

template <int NT>
__global__ __launch_bounds__(256, BSP_TILE_OCC) void conv_tile_bf16(ConvParams p, TileCfg t) {
  struct AllArgs {  // the argument block as the two arguments lie in it
    ConvParams p;
    TileCfg t;
  };
  kernarg_touch<AllArgs>();
  extern __shared__ __align__(16) unsigned char lds[];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int jn = lane & 15, g = lane >> 4;

  // workgroup -> (strip group, image, tile)
  const uint32_t bid = blockIdx.x;
  const int sg = (int)fdiv(bid, t.d_ntiles);
  const uint32_t tile = bid - (uint32_t)sg * t.ntiles;
  const int n = (int)fdiv(tile, t.d_tpi);
  const uint32_t trem = tile - (uint32_t)n * (t.tiles_y * t.tiles_x);
  const int tyi = (int)fdiv(trem, t.d_tiles_x);
  const int oy0 = tyi * t.TH, ox0 = (int)(trem - tyi * t.tiles_x) * t.TW;
  const int iy_org = oy0 * p.sh - p.ph, ix_org = ox0 * p.sw - p.pw;

  const int32_t* plan = p.plan;
  const int32_t* slab_ptr = plan + plan[BSP_PLAN_OFF_SLAB_W];
  const int32_t* xdesc = plan + plan[BSP_PLAN_OFF_XDESC_W];
  const u32x4_t* wfrag = (const u32x4_t*)(plan + plan[BSP_PLAN_OFF_WFRAG_W]);
  const uint16_t* X = (const uint16_t*)p.X;
  const int64_t img = (int64_t)n * p.L;

  Ring ring;
  int s0 = 0, s1 = 0;
  float bias_next[4] = {0.f, 0.f, 0.f, 0.f};
  // everything about (strip, slab) that can be requested before activations are there
  auto request = [&](int strip, int sl) {
    s0 = slab_ptr[strip * (t.nslabs + 1) + sl];
    s1 = slab_ptr[strip * (t.nslabs + 1) + sl + 1];
    ring_fill(ring, wfrag, xdesc, s0, s1, lane, g);
    if (sl == 0) {
      const int ch = strip * BSP_STRIP + 4 * g;
#pragma unroll
      for (int r = 0; r < 4; ++r) bias_next[r] = (p.bias && ch + r < p.O) ? p.bias[ch + r] : 0.f;
    }
  };

  // stage one slab: global -> registers -> LDS in batches; `early` runs once the
  // first batch of loads is in flight
  const int PP = t.slab / BSP_CHUNK;  // 16-byte pieces per staged pixel
  const int npieces = t.TPH * t.TPW * PP;
  auto stage = [&](int sl, auto&& early) {
    for (int b0 = 0; b0 < npieces; b0 += 256 * kStageBatch) {
      u32x4_t sv[kStageBatch];
      int sdst[kStageBatch];
#pragma unroll
      for (int u = 0; u < kStageBatch; ++u) {
        const int idx = b0 + tid + u * 256;
        const uint32_t pix = fdiv((uint32_t)idx, t.d_pp);
        const int part = idx - (int)pix * PP;
        const int py = (int)fdiv(pix, t.d_tpw);
        const int px = (int)pix - py * t.TPW;
        sdst[u] = idx < npieces ? py * t.pitch + px * t.row_bytes + part * 16 : -1;
        const int iy = iy_org + py * t.gsh, ix = ix_org + px * t.gsw;
        const int ch = sl * t.slab + part * BSP_CHUNK;
        sv[u] = u32x4_t{0u, 0u, 0u, 0u};
        if (sdst[u] >= 0 && (unsigned)iy < (unsigned)p.L && (unsigned)ix < (unsigned)p.J && ch < p.I)
          sv[u] = *(const u32x4_t*)(X + ((img + iy) * p.J + ix) * p.I + ch);
      }
      if (b0 == 0) early();
#pragma unroll
      for (int u = 0; u < kStageBatch; ++u)
        if (sdst[u] >= 0) *(u32x4_t*)(lds + sdst[u]) = sv[u];
    }
  };

  int strip = sg * t.spc + wave;
  const int strip_end = min((sg + 1) * t.spc, t.nstrips);
  bool valid = strip < strip_end;

  stage(0, [&] {
    if (valid) request(strip, 0);
  });

  // per-lane output pixel map
  int pyx[NT], base[NT];
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) {
    int ty, tx;
    if (t.tile2x8) {  // pixel tiles are 2 rows x 8 columns
      const int tr = (int)fdiv((uint32_t)nt, t.d_tpr), tc = nt - tr * (t.TW >> 3);
      ty = tr * 2 + (jn >> 3);
      tx = tc * 8 + (jn & 7);
    } else {
      const int pi = nt * 16 + jn;
      ty = (int)fdiv((uint32_t)pi, t.d_tw);
      tx = pi - ty * t.TW;
    }
    const bool in_tile = ty < t.TH && tx < t.TW;
    pyx[nt] = in_tile ? (ty | (tx << 16)) : -1;
    base[nt] = in_tile ? (ty * t.lsh) * t.pitch + (tx * t.lsw) * t.row_bytes : 0;
  }
  f32x4_t acc[NT];
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) acc[nt] = f32x4_t{0.f, 0.f, 0.f, 0.f};
  __syncthreads();

  int sl = 0;
  while (true) {
    if (valid)
      run_steps<NT>(acc, ring, wfrag, xdesc, s0, s1, lane, g, lds, base, t.pitch, t.row_bytes);
    if (sl + 1 < t.nslabs) {  // same strip, next slab of input channels (spc == 4 here)
      ++sl;
      __syncthreads();  // everyone is done reading LDS before it is overwritten
      stage(sl, [&] {
        if (valid) request(strip, sl);
      });
      __syncthreads();
      continue;
    }
    // strip finished: request its successor first, then store
    float bv[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) bv[r] = bias_next[r];
    const int nstrip = strip + 4;
    const bool nvalid = valid && nstrip < strip_end;
    if (nvalid) request(nstrip, 0);
    if (valid) {
      // lane holds channels 4g..4g+3 of pixel jn of every pixel tile
      const int ch = strip * BSP_STRIP + 4 * g;
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
        if (p.residual || p.relu)
          v = post_bf16x4(v, p.residual ? (const uint16_t*)p.residual + pid * p.O + ch : nullptr,
                          p.O - ch, (p.O % 4) == 0 && ch + 3 < p.O, p.relu);
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
    if (!nvalid) break;
    strip = nstrip;
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

// Pick the output tile: most useful pixels per MFMA pixel slot, least halo, no
// LDS bank conflicts; then the LDS paddings that achieve the latter.
}  // namespace

bool bsp_choose_tile(const ConvParams& p, int slab, int64_t max_lds, int max_pieces, int nt_scale,
                     int out_row_bytes, int min_nt, int slots, int* NT, TileCfg* out) {
  const bool pointwise = p.H == 1 && p.K == 1;
  static const int nts[] = {2, 4, 7, 8};
  static const int tws[] = {4, 7, 8, 14, 16, 24, 28, 32, 56, 64, 112, 128, 224, 256};
  double best = -1.0;
  for (int nt1 : nts)
    for (int tw : tws)
      for (int mode = 0; mode < 2; ++mode) {
        if (nt1 < min_nt) continue;
        const int nt = nt1 * nt_scale;
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
        t.tiles_y = (p.M + t.TH - 1) / t.TH;
        t.tiles_x = (p.N + t.TW - 1) / t.TW;
        if (max_pieces > 0 && (int64_t)t.TPH * t.TPW * (slab / BSP_CHUNK) > max_pieces) continue;
        // paddings: fewest conflicts first, then least LDS
        int best_ex = 1 << 30;
        int64_t best_lds = 0;
        int brp = 0, bpp = 0;
        for (int rp = 0; rp <= 112; rp += 16)
          for (int pp = 0; pp <= 240; pp += 16) {
            t.row_bytes = slab * 2 + rp;
            t.pitch = t.TPW * t.row_bytes + pp;
            const int64_t ldsb = (int64_t)t.TPH * t.pitch + (int64_t)nt * 16 * out_row_bytes;
            if (ldsb > max_lds) continue;
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
        double util = (double)p.M * p.N / ((double)t.tiles_y * t.tiles_x * nt * 16);
        if (slots > 0) {
          // persistent grid of `slots` workgroups per strip group: what counts is how many
          // rounds of units the busiest workgroup runs and what a unit costs, a fixed part
          // (barriers, writing the next unit into LDS; `fixed` 16-pixel tiles' worth of
          // compute) plus its pixel tiles.  Small layers then get smaller tiles on more CUs.
          const double steps = std::max(1.0, 0.75 * (slab / BSP_CHUNK) * (pointwise ? 1 : p.H * p.K) / 4.0);
          const double fixed = 64.0 / steps;
          const int64_t ntiles = (int64_t)p.B * t.tiles_y * t.tiles_x;
          const int64_t rounds = (ntiles + slots - 1) / slots;
          // (blended with the plain slot utilisation: the total work still costs bandwidth)
          util = 0.7 * ((double)p.B * p.M * p.N / 16.0 / slots) / ((double)rounds * (fixed + nt)) + 0.3 * util;
        }
        const double halo = (double)t.TPH * t.TPW / ((double)t.TH * t.TW * t.lsh * t.lsw);
        const double score = util - 0.02 * halo - 0.05 * best_ex / nt + 0.001 * nt;
        if (score > best) {
          best = score;
          *NT = nt1;
          *out = t;
        }
      }
  return best >= 0.0;
}

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
      if (!bsp_choose_tile(p, t.slab, 64 * 1024, 0, 1, 0, 4, 0, &NT, &t)) NT = 0;
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
  const int64_t nwg = ntiles * groups;
  // the multiply-high divisions are exact only while dividend * divisor < 2^32
  const int64_t npieces = (int64_t)t.TPH * t.TPW * (t.slab / BSP_CHUNK);
  if (nwg >= (1 << 30) || nwg * ntiles >= (1ll << 32) ||
      (npieces + 2048) * (t.slab / BSP_CHUNK) >= (1ll << 32) ||
      (npieces + 2048) * t.TPW >= (1ll << 32))
    return BSP_ERR_UNSUPPORTED;
  t.ntiles = (int32_t)ntiles;
  t.d_pp = make_fastdiv(t.slab / BSP_CHUNK);
  t.d_tpw = make_fastdiv(t.TPW);
  t.d_tw = make_fastdiv(t.TW);
  t.d_tpr = make_fastdiv(t.TW >= 8 ? t.TW >> 3 : 1);
  t.d_ntiles = make_fastdiv((uint32_t)ntiles);
  t.d_tpi = make_fastdiv(t.tiles_y * t.tiles_x);
  t.d_tiles_x = make_fastdiv(t.tiles_x);
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
