// LDS-resident tiled kernel: weights AND activations of the current slab of input channels
// live in LDS, the hot loop touches nothing else.  bf16 layers (fp32 accumulation), first
// layers with at most four input channels, and int8 layers (exact int32 sums).
//
// A persistent workgroup of twelve waves owns a group of four strips (64 output channels)
// and walks units = (pixel tile of an image, slab of input channels).  Eight waves compute
// (wave w: strip w & 3, pixel-tile share w >> 2), four move data.  For each unit the input
// patch of the slab and the four strips' weight fragments of the slab are copied into LDS,
// the step descriptors are turned into ready LDS offsets, and the compute waves run the
// slab's steps reading only LDS (weights, offsets and activations each one step ahead of
// the MFMAs).  While a unit is computed, the global loads of the NEXT unit are already in
// flight into registers (the patch in the mover waves, the weight fragments in spare
// registers of the compute waves), so their latency is hidden.  When all of a layer's input
// channels fit one slab the weights are copied once and stay for every tile the workgroup
// visits.  After the last slab of a tile the results (+ bias, rounded once) go through an
// LDS staging tile and leave as whole 16-byte pieces; a residual add and a ReLU can be
// applied on the way out.
//
// Only kept blocks have steps (paper Section I, advantages 3-4): work and weight traffic
// shrink with the mask, the patch traffic does not.
#include "bsp_launch.h"
#include "bsp_tile.h"

#include <array>
#include <cstdlib>
#include <type_traits>
#include <map>
#include <mutex>

namespace {

typedef __attribute__((ext_vector_type(4))) int i32x4_t;

constexpr int kPH = 2;              // compute waves per strip, each taking a share of the pixel tiles
constexpr int kComputeThreads = 256 * kPH;
constexpr int kLoaderWaves = 4;     // one per strip of the group
constexpr int kLoaderThreads = 64 * kLoaderWaves;
constexpr int kThreads = kComputeThreads + kLoaderThreads;
constexpr int kXBatch = 11;         // 16-byte patch pieces a loader thread keeps in flight
constexpr int kXBatchFlat = 14;     // the same for flattened pointwise layers (no address maps to keep)
constexpr int kWHalf = 10;         // weight fragments a loader lane keeps in flight (one slab of a strip)
constexpr int kMaxSlabs = 32;
constexpr int kOutRow = 4 * BSP_STRIP * 2 + 16;  // bytes per pixel in the results staging tile
constexpr int kOutRowI8 = 4 * BSP_STRIP + 16;     // the same for int8 results

struct LdsCfg {
  int32_t wbuf_off;       // LDS offset of the weight regions (after the patch)
  int32_t region_bytes;   // per strip: maxsteps fragments + maxsteps offset quads
  int32_t obuf_off;       // LDS offset of the results staging tile
  int32_t sp_off;         // LDS offset of the step-range table [4][nslabs + 1]
  int32_t maxsteps;       // most steps any (strip, slab) has
  int32_t lgpp;           // >= 0: a flattened pointwise layer (movers without maps)
  int32_t wload;          // steps of a slab each of a strip's waves stages: ceil(maxsteps / kPH)
  int32_t nsteps;         // steps in the whole plan
  int32_t mover_first;    // raise the data movers' wave priority
  int32_t shift;          // int8 results: rounding right shift of the 32-bit sums
  int32_t part_bytes;     // LDS bytes between a pixel's consecutive 16-byte chunks: 16 when a
                          // pixel's chunks lie side by side, the plane size when every chunk
                          // index has a plane of its own (then t.row_bytes is 16)
  int32_t groups;         // strip groups (of four)
  int32_t wg_per_group;   // workgroups sharing one strip group
  int32_t off_slab, off_xdesc, off_wfrag;  // plan sections, in words (read on the host)
  // advancing a thread's patch piece by the number of loader threads: uniform steps of
  // (channel part, patch column), of the LDS offset, of the element offset from the patch
  // origin and of the image row / column, then what a carry out of the channel parts
  // (cp_*) and out of the patch columns (cx_*) adds
  int32_t s_part, s_px, s_l, s_g, s_iy, s_ix;
  int32_t cp_l, cp_g;
  int32_t cx_l, cx_g, cx_ix;
  FastDiv d_groups;
};

template <int NT>
__device__ __forceinline__ void load_b_at(u32x4_t (&b)[NT], const int xoff,
                                          const unsigned char* lds, const int (&base)[NT]) {
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) b[nt] = *(const u32x4_t*)(lds + base[nt] + xoff);
}

// position (row, column) inside the workgroup's tile of pixel j of pixel tile gt
__device__ __forceinline__ void tile_pos(const TileCfg& t, int gt, int j, int* ty, int* tx) {
  if (t.tile2x8) {
    const int tr = (int)fdiv((uint32_t)gt, t.d_tpr), tc = gt - tr * (t.TW >> 3);
    *ty = tr * 2 + (j >> 3);
    *tx = tc * 8 + (j & 7);
  } else {
    const int pi = gt * 16 + j;
    *ty = (int)fdiv((uint32_t)pi, t.d_tw);
    *tx = pi - *ty * t.TW;
  }
}

// Twelve waves, two roles.  Waves 0-7 compute: wave w owns strip w & 3 of the group and
// share w >> 2 of the tile's pixel tiles; during a unit (one slab of one tile) it touches
// nothing but LDS and the matrix cores, apart from having its share of the strip's next
// weight fragments in flight into spare registers.  Waves 8-11 move data: while a unit is
// computed they have the next unit's patch in flight into their registers, after the
// barrier they write it into LDS, and they carry finished results from the LDS staging
// tile to global memory.  Two barriers per unit, taken by all twelve waves.  Single-slab
// layers (weights stay in LDS):
//   E  compute is done with the patch (the movers may overwrite it) and the staging tile
//      has been drained (results may go in)
//   A  the next patch is in LDS and the results are staged
// otherwise:
//   B  compute is done with the patch and the weights; results, if any, are staged
//   A  the next unit's patch and weights are in LDS
// KIND: what a 16-byte chunk of a pixel holds.
enum { kBf16 = 0, kBf16Narrow = 1, kInt8 = 2 };

template <int NT, int KIND, bool RELOAD, bool FLAT>
__global__ __launch_bounds__(kThreads, 1) void conv_lds(ConvParams p, TileCfg t, LdsCfg c) {
  struct AllArgs {  // the argument block as the three arguments lie in it
    ConvParams p;
    TileCfg t;
    LdsCfg c;
  };
  kernarg_touch<AllArgs>();
  constexpr bool NARROW = KIND == kBf16Narrow;
  // int8 codes: a chunk is sixteen channels, the MFMA is i32 16x16x64, sums are exact 32-bit
  // integers, the results are int8 after a rounding shift (c.shift).  The data movers see
  // pairs of codes as one 2-byte element (p.I counts such pairs), so the patch path is the
  // same; the staging tile holds 64 bytes per pixel and leaves as 16-byte pieces of 16 channels.
  constexpr bool I8 = KIND == kInt8;
  constexpr int OUT_ROW = I8 ? kOutRowI8 : kOutRow;
  extern __shared__ __align__(16) unsigned char lds[];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave_all = __builtin_amdgcn_readfirstlane(tid >> 6);
  const bool loader = wave_all >= 4 * kPH;

  const uint32_t bid = blockIdx.x;
  const int cidx = (int)fdiv(bid, c.d_groups);
  const int sg = (int)bid - cidx * c.groups;
  int tile = cidx;
  if (tile >= t.ntiles) return;

  const int tpi = t.tiles_y * t.tiles_x;
  const int nsl1 = t.nslabs + 1;
  // RELOAD: the layer has several slabs, so the weights of the next one are staged while
  // this one is computed (registers for that; the step loop then prefetches less deeply)
  constexpr bool reload_w = RELOAD;
  const int32_t* plan = p.plan;

  // which tile / slab follows (tile, sl), and whether there is one
  auto advance = [&](int tl, int sl, int* ntl, int* nsl) {
    *ntl = tl;
    *nsl = sl + 1;
    if (*nsl == t.nslabs) {
      *nsl = 0;
      *ntl = tl + c.wg_per_group;
    }
    return *ntl < t.ntiles;
  };

  if (loader) {
    // =================================================================== data movers
    // few instructions, but where units are short everything waits on them: then they
    // issue ahead of the compute waves
    if (c.mover_first) __builtin_amdgcn_s_setprio(3);
    const int ltid = tid - kComputeThreads;
    const uint16_t* X = (const uint16_t*)p.X;
    // The patch is cut into 16-byte pieces (pixel-major, 8 channels each); this thread
    // moves pieces ltid, ltid + 256, ...  For each of them it keeps, from the first unit
    // on: the element offset from the patch origin (-1: no such piece), the LDS offset,
    // and (channel part) << 20 | (image rows from the origin) << 10 | (image columns).
    // Piece -> (channel part, patch column, patch row) is found by division for the first
    // piece and advanced by the uniform step with two carries for the others.
    const int PP = t.slab / BSP_CHUNK;
    const int npieces = t.TPH * t.TPW * PP;
    // FLAT: a pointwise layer whose pixels were flattened into one row; piece -> (pixel, part)
    // is then one division by a constant, no maps are kept and the registers go to a longer
    // batch (larger tiles)
    constexpr int XB = FLAT ? kXBatchFlat : kXBatch;
    int xg[FLAT ? 1 : kXBatch], xl[FLAT ? 1 : kXBatch], xq[FLAT ? 1 : kXBatch];
    // the results staging tile: piece q = ltid + 256 k is channels 8 (q & 7).. of pixel q >> 3
    // (filled in once the first unit's loads are on their way)
    constexpr int PPP = I8 ? 4 : 8;          // 16-byte pieces per staged pixel
    constexpr int PXK = kLoaderThreads / PPP;  // pixels per round of the 256 threads
    constexpr int NF = (NT * kPH * 16 + PXK - 1) / PXK;
    const int fpart = ltid % PPP, fpix = ltid / PPP;
    int fpos[NF], foff[NF];

    u32x4_t xv[XB];
    // X + origin of the patch may point before the image (padding); only in-image pieces are read
    struct Origin {
      const uint16_t* org;
      int iy, ix, ch0;
    };
    auto origin = [&](int tl, int sl) {
      const int n = (int)fdiv((uint32_t)tl, t.d_tpi);
      const int trem = tl - n * tpi;
      const int tyi = (int)fdiv((uint32_t)trem, t.d_tiles_x);
      Origin o;
      o.iy = tyi * t.TH * p.sh - p.ph;
      o.ix = (trem - tyi * t.tiles_x) * t.TW * p.sw - p.pw;
      o.ch0 = sl * t.slab;
      o.org = X + (((int64_t)n * p.L + o.iy) * p.J + o.ix) * p.I + o.ch0;
      return o;
    };
    auto load_piece = [&](int u, const Origin& o) {
      xv[u] = u32x4_t{0u, 0u, 0u, 0u};
      if constexpr (FLAT) {
        const int i = ltid + u * kLoaderThreads;
        const int pix = (int)fdiv((uint32_t)i, t.d_pp), part = i - pix * PP;
        if (i < npieces && o.ix + pix < p.J && o.ch0 + part * BSP_CHUNK < p.I)
          xv[u] = *(const u32x4_t*)(o.org + (int64_t)pix * p.I + part * BSP_CHUNK);
        return;
      }
      const int q = xq[u];
      if (xg[u] >= 0 && (unsigned)(o.iy + ((q >> 10) & 1023)) < (unsigned)p.L &&
          (unsigned)(o.ix + (q & 1023)) < (unsigned)p.J && o.ch0 + (q >> 20) * BSP_CHUNK < p.I) {
        if constexpr (!NARROW) {
          xv[u] = *(const u32x4_t*)(o.org + xg[u]);
        } else {  // the pixel's p.I <= 4 channels, one by one (no branch between the loads);
                  // the rest of the chunk stays zero
          const uint16_t* e = o.org + xg[u];
          const uint32_t h0 = e[0], h1 = e[min(1, p.I - 1)], h2 = e[min(2, p.I - 1)],
                         h3 = e[min(3, p.I - 1)];
          xv[u] = u32x4_t{h0 | (p.I > 1 ? h1 << 16 : 0u), (p.I > 2 ? h2 : 0u) | (p.I > 3 ? h3 << 16 : 0u),
                          0u, 0u};
        }
      }
    };
    // first unit: build the maps piece by piece, each piece's load leaving right away
    auto first_patch = [&](int tl) {
      const Origin o = origin(tl, 0);
      if constexpr (FLAT) {
#pragma unroll
        for (int u = 0; u < XB; ++u) load_piece(u, o);
        return;
      }
      const int pix = (int)fdiv((uint32_t)ltid, t.d_pp);
      int part = ltid - pix * PP;
      const int py0 = (int)fdiv((uint32_t)pix, t.d_tpw);
      int px = pix - py0 * t.TPW;
      int l = py0 * t.pitch + px * t.row_bytes + part * c.part_bytes;
      uint32_t g = (uint32_t)((py0 * t.gsh * p.J + px * t.gsw) * p.I + part * BSP_CHUNK);
      int iy = py0 * t.gsh, ix = px * t.gsw;
#pragma unroll
      for (int u = 0; u < kXBatch; ++u) {
        const bool exists = ltid + u * kLoaderThreads < npieces;
        xg[u] = exists ? (int)g : -1;
        xl[u] = l;
        xq[u] = part << 20 | iy << 10 | ix;
        load_piece(u, o);
        part += c.s_part; px += c.s_px; l += c.s_l; g += (uint32_t)c.s_g; iy += c.s_iy; ix += c.s_ix;
        if (part >= PP) { part -= PP; px += 1; l += c.cp_l; g += (uint32_t)c.cp_g; ix += t.gsw; }
        if (px >= t.TPW) { px -= t.TPW; l += c.cx_l; g += (uint32_t)c.cx_g; iy += t.gsh; ix -= c.cx_ix; }
      }
    };
    auto issue_patch = [&](int tl, int sl) {
      const Origin o = origin(tl, sl);
#pragma unroll
      for (int u = 0; u < XB; ++u) load_piece(u, o);
    };
    auto commit_patch = [&]() {
      if constexpr (FLAT) {
#pragma unroll
        for (int u = 0; u < XB; ++u) {
          const int i = ltid + u * kLoaderThreads;
          const int pix = (int)fdiv((uint32_t)i, t.d_pp);
          if (i < npieces) *(u32x4_t*)(lds + pix * t.row_bytes + (i - pix * PP) * c.part_bytes) = xv[u];
        }
        return;
      }
#pragma unroll
      for (int u = 0; u < kXBatch; ++u)
        if (xg[u] >= 0) *(u32x4_t*)(lds + xl[u]) = xv[u];
    };
    // results of tile tl: LDS staging tile -> Y as whole 16-byte pieces, eight consecutive
    // lanes covering the 64 output channels (128 bytes) of one pixel
    auto flush = [&](int tl) {
      const int n = (int)fdiv((uint32_t)tl, t.d_tpi);
      const int trem = tl - n * tpi;
      const int tyi = (int)fdiv((uint32_t)trem, t.d_tiles_x);
      const int oy0 = tyi * t.TH, ox0 = (trem - tyi * t.tiles_x) * t.TW;
      // element offsets; an element of Y is 2 bytes (bf16) or 1 byte (int8)
      constexpr int YES = I8 ? 1 : 2;
      unsigned char* yorg = (unsigned char*)p.Y + ((((int64_t)n * p.M + oy0) * p.N + ox0) * p.O + sg * 64) * YES;
      const unsigned char* rorg = (const unsigned char*)p.residual + (yorg - (unsigned char*)p.Y);
      const int my = p.M - oy0, mx = p.N - ox0;  // rows / columns of the tile inside the image
      // a few pieces at a time: all reads first, then the stores, so that neither waits on
      // the other.  Plain: four staged pieces.  Fused: two staged pieces and their two
      // residual pieces (the same registers in all).
      auto batch = [&](auto bs_tag, auto fused_tag) {
        constexpr int BS = decltype(bs_tag)::value;
        constexpr bool FUSED = decltype(fused_tag)::value;
#pragma unroll
        for (int k0 = 0; k0 < NF; k0 += BS) {
          u32x4_t ov[BS], rv[FUSED ? BS : 1];
          bool ok[BS];
#pragma unroll
          for (int k = k0; k < k0 + BS && k < NF; ++k) {
            const int f = fpos[k];
            ok[k - k0] = f >= 0 && (f >> 16) < my && (f & 0xFFFF) < mx;
            if constexpr (FUSED) {
              rv[k - k0] = u32x4_t{0u, 0u, 0u, 0u};
              if (p.residual && ok[k - k0]) rv[k - k0] = *(const u32x4_t*)(rorg + foff[k] * YES);
            }
          }
#pragma unroll
          for (int k = k0; k < k0 + BS && k < NF; ++k)
            ov[k - k0] = *(const u32x4_t*)(lds + c.obuf_off + (fpix + PXK * k) * OUT_ROW + fpart * 16);
#pragma unroll
          for (int k = k0; k < k0 + BS && k < NF; ++k) {
            if (!ok[k - k0]) continue;
            u32x4_t o = ov[k - k0];
            if constexpr (FUSED) {  // eight channels: + residual, activation, second rounding
              const u32x4_t r = rv[k - k0];
              const uint32_t in[4] = {o.x, o.y, o.z, o.w}, rr[4] = {r.x, r.y, r.z, r.w};
              uint32_t out[4];
#pragma unroll
              for (int q = 0; q < 4; ++q) {
                float lo = bf16_bits_to_f32((uint16_t)(in[q] & 0xFFFF)) +
                           bf16_bits_to_f32((uint16_t)(rr[q] & 0xFFFF));
                float hi = bf16_bits_to_f32((uint16_t)(in[q] >> 16)) +
                           bf16_bits_to_f32((uint16_t)(rr[q] >> 16));
                if (p.relu) {
                  lo = fmaxf(lo, 0.f);
                  hi = fmaxf(hi, 0.f);
                }
                out[q] = pack_bf16x2(lo, hi);
              }
              o = u32x4_t{out[0], out[1], out[2], out[3]};
            }
            // streaming store: results are not read again here, and lines left dirty in L2
            // would all be written back in one burst when the kernel ends
            __builtin_nontemporal_store(o, (u32x4_t*)(yorg + foff[k] * YES));
          }
        }
      };
      if (!I8 && (p.residual || p.relu))
        batch(std::integral_constant<int, 2>{}, std::true_type{});
      else
        batch(std::integral_constant<int, (NT >= 8 ? 4 : NF)>{}, std::false_type{});
    };

    int sl = 0;
    first_patch(tile);
#pragma unroll
    for (int k = 0; k < NF; ++k) {
      const int pi = fpix + PXK * k;
      int ty, tx;
      tile_pos(t, pi >> 4, pi & 15, &ty, &tx);
      fpos[k] = (pi < NT * kPH * 16 && ty < t.TH && tx < t.TW && sg * 64 + fpart * (64 / PPP) < p.O)
                    ? (ty << 16 | tx)
                    : -1;
      foff[k] = (ty * p.N + tx) * p.O + fpart * (64 / PPP);  // in elements of Y
    }
    commit_patch();
    __syncthreads();  // A: first unit is in LDS
    int flush_tile = -1;
    while (true) {
      int ntile, nsl;
      const bool more = advance(tile, sl, &ntile, &nsl);
      if (more) issue_patch(ntile, nsl);  // lands in registers during the compute phase
      // the previous tile's results, while the compute waves work on (tile, sl).  After the
      // loads: a store's data registers may not be touched until the store has completed,
      // so anything issued behind the stores would first wait for them.
      if (flush_tile >= 0) flush(flush_tile);
      flush_tile = sl == t.nslabs - 1 ? tile : -1;
      // E (single-slab layers): the compute waves are done with the patch and go on to stage
      // their results, so the next patch can go in at once and B is not needed;
      // B (otherwise): the compute waves are done with the patch and the weights
      __syncthreads();
      if (more) commit_patch();
      __syncthreads();  // A: next unit is in LDS (single-slab: and the results are staged)
      if (!more) break;
      tile = ntile;
      sl = nsl;
    }
    flush(tile);
    return;
  }

  // ===================================================================== compute waves
  const int wave = wave_all & 3;   // which strip of the group
  const int half = wave_all >> 2;  // which share of the tile's pixel tiles
  const int jn = lane & 15, g = lane >> 4;
  const int strip = sg * 4 + wave;
  const bool valid = strip < t.nstrips;
  const int32_t* slab_ptr = plan + c.off_slab + (valid ? strip : 0) * nsl1;
  const int32_t* xdesc = plan + c.off_xdesc;
  const u32x4_t* wfrag = (const u32x4_t*)(plan + c.off_wfrag);
  u32x4_t* wl = (u32x4_t*)(lds + c.wbuf_off + wave * c.region_bytes);
  int* xo = (int*)(lds + c.wbuf_off + wave * c.region_bytes + c.maxsteps * 1024);

  // The strip's weight fragments of a slab go global -> registers -> LDS, this wave moving
  // steps [half * kWHalf, half * kWHalf + kWHalf) of them, and with them the LDS offsets
  // the steps' activation fragments are read at.
  u32x4_t wv[kWHalf];  // live across the step loop only when RELOAD
  int dsc = 0, w_n = 0;
  // All kWHalf loads are always issued, in one straight line so that they are in flight
  // together; those past the wave's share repeat its last fragment and are dropped.
  auto issue_weights = [&](int s0, int s1) {
    w_n = max(0, min(s1 - s0 - half * c.wload, c.wload));
    const int f = s0 + half * c.wload;
    const int last = min(max(f + w_n, s0 + 1), c.nsteps) - 1;  // a fragment that exists
    // (no more loads than any strip of the layer can need: c.wload, the same for every wave
    // and unit, so the loads still leave in one straight line)
#pragma unroll
    for (int u = 0; u < kWHalf; ++u) {
      u32x4_t v = u32x4_t{0u, 0u, 0u, 0u};
      if (u < c.wload) v = wfrag[(int64_t)min(f + u, last) * 64 + lane];
      wv[u] = v;
    }
    if (lane < w_n * 4) dsc = xdesc[f * 4 + lane];
  };
  auto commit_weights = [&]() {
#pragma unroll
    for (int u = 0; u < kWHalf; ++u)
      if (u < w_n) wl[(half * c.wload + u) * 64 + lane] = wv[u];
    if (lane < w_n * 4)
      xo[half * c.wload * 4 + lane] = ((dsc >> 16) & 0xFF) * t.pitch +
                                     ((dsc >> 24) & 0xFF) * t.row_bytes + (dsc & 0xFFFF) * c.part_bytes;
  };

  // the strip's step ranges go to LDS once: later slabs then cost an LDS read, not a trip
  // to global memory in front of the step loop
  int* sp = (int*)(lds + c.sp_off) + wave * nsl1;
  if (RELOAD && half == 0)
    for (int k = lane; k < nsl1; k += 64) sp[k] = valid ? slab_ptr[k] : 0;
  int s_lo = valid ? slab_ptr[0] : 0, s_hi = valid ? slab_ptr[1] : 0;  // steps of the current slab
  issue_weights(s_lo, s_hi);

  using acc_t = typename std::conditional<I8, i32x4_t, f32x4_t>::type;
  using bias_t = typename std::conditional<I8, int32_t, float>::type;
  bias_t bv[4] = {0, 0, 0, 0};
  const int ch = strip * BSP_STRIP + 4 * g;
  if (valid) {
#pragma unroll
    for (int r = 0; r < 4; ++r)
      bv[r] = (p.bias && ch + r < p.O) ? ((const bias_t*)p.bias)[ch + r] : (bias_t)0;
  }
  int base[NT];  // LDS base of this lane's pixel in each of the wave's pixel tiles
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) {
    int ty, tx;
    tile_pos(t, half * NT + nt, jn, &ty, &tx);
    base[nt] = (ty < t.TH && tx < t.TW) ? (ty * t.lsh) * t.pitch + (tx * t.lsw) * t.row_bytes : 0;
  }
  // where this lane's four channels of pixel jn of pixel tile nt go in the staging tile
  const int orow = c.obuf_off + (half * NT * 16 + jn) * OUT_ROW +
                   (I8 ? wave * BSP_STRIP + g * 4 : wave * (BSP_STRIP * 2) + g * 8);

  acc_t acc[NT];
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) acc[nt] = acc_t{0, 0, 0, 0};
  auto mma = [&](const u32x4_t& a, const u32x4_t (&b)[NT]) {
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
      if constexpr (I8)
        acc[nt] = __builtin_amdgcn_mfma_i32_16x16x64_i8(__builtin_bit_cast(i32x4_t, a),
                                                        __builtin_bit_cast(i32x4_t, b[nt]), acc[nt], 0, 0, 0);
      else
        acc[nt] = mfma_bf16_16x16x32(a, b[nt], acc[nt]);
    }
  };

  int sl = 0;
  commit_weights();
  __syncthreads();  // A
  while (true) {
    int ntile, nsl;
    const bool more = advance(tile, sl, &ntile, &nsl);
    const int nst = s_hi - s_lo;
    if (reload_w && more) {  // next slab's fragments: in flight while this one is computed
      s_lo = sp[nsl];
      s_hi = sp[nsl + 1];
      issue_weights(s_lo, s_hi);
    }
    // this slab's steps, everything from LDS and D - 1 steps ahead of the MFMAs (offsets one
    // more): the fragments of step s + D - 1 are requested before the MFMAs of step s go out.
    // Two steps ahead where the registers allow it: one step does not cover the LDS latency.
    if (nst > 0) {
      constexpr int D = (NT >= 8 || (RELOAD && NT > 4)) ? 2 : 3;
      u32x4_t a[D], b[D][NT];
      int x[D];
      const int lastq = nst - 1;
#pragma unroll
      for (int u = 0; u < D; ++u) x[u] = xo[min(u, lastq) * 4 + g];
#pragma unroll
      for (int u = 0; u < D - 1; ++u) {
        a[u] = wl[min(u, lastq) * 64 + lane];
        load_b_at<NT>(b[u], x[u], lds, base);
      }
      for (int s = 0; s < nst; s += D) {
#pragma unroll
        for (int u = 0; u < D; ++u) {
          if (s + u < nst) {
            const int nx = (u + D - 1) % D;  // buffer of step s + u + D - 1
            const int xn = xo[min(s + u + D, lastq) * 4 + g];
            a[nx] = wl[min(s + u + D - 1, lastq) * 64 + lane];
            load_b_at<NT>(b[nx], x[nx], lds, base);
            x[u] = xn;  // the offset of step s + u + D takes the place of step s + u's
            mma(a[u], b[u]);
          }
        }
      }
    }
    if (!reload_w) __syncthreads();  // E (the staging tile has been drained by now)
    if (sl == t.nslabs - 1 && valid) {
      // + bias, one rounding; lane holds channels 4g..4g+3 of pixel jn of every pixel tile
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) {
        if constexpr (I8) {
          // exact sum + 32-bit bias, rounding right shift (ties upward), saturation to int8
          uint32_t packed = 0;
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            const long long sft = ((long long)acc[nt][r] + bv[r] + (c.shift > 0 ? 1ll << (c.shift - 1) : 0)) >> c.shift;
            const int q = sft < -128 ? -128 : (sft > 127 ? 127 : (int)sft);
            packed |= (uint32_t)(q & 0xFF) << (8 * r);
          }
          *(uint32_t*)(lds + orow + nt * 16 * OUT_ROW) = packed;
        } else {
          u32x2_t v;
          v.x = pack_bf16x2(acc[nt][0] + bv[0], acc[nt][1] + bv[1]);
          v.y = pack_bf16x2(acc[nt][2] + bv[2], acc[nt][3] + bv[3]);
          *(u32x2_t*)(lds + orow + nt * 16 * OUT_ROW) = v;
        }
        acc[nt] = acc_t{0, 0, 0, 0};
      }
    }
    if (reload_w) {
      __syncthreads();  // B
      if (more) commit_weights();
    }
    __syncthreads();  // A
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

template <int NT, int KIND, bool RELOAD, bool FLAT>
int launch_one(const ConvParams& p, const TileCfg& t, const LdsCfg& c, dim3 grid, size_t ldsb,
               hipStream_t st) {
  static bool raised = false;  // dynamic LDS above 64 KB has to be allowed once per kernel
  if (!raised) {
    if (hipFuncSetAttribute((const void*)conv_lds<NT, KIND, RELOAD, FLAT>,
                            hipFuncAttributeMaxDynamicSharedMemorySize,
                            (int)kLdsPerCu) != hipSuccess)
      return BSP_ERR_HIP;
    raised = true;
  }
  hipLaunchKernelGGL((conv_lds<NT, KIND, RELOAD, FLAT>), grid, dim3(kThreads), ldsb, st, p, t, c);
  return hipGetLastError() == hipSuccess ? BSP_OK : BSP_ERR_HIP;
}

template <int NT, int KIND>
int launch(const ConvParams& p, const TileCfg& t, const LdsCfg& c, dim3 grid, size_t ldsb,
           hipStream_t st) {
  if constexpr (KIND == kBf16Narrow) {  // first layers have one slab
    return launch_one<NT, KIND, false, false>(p, t, c, grid, ldsb, st);
  } else {
    if constexpr (NT <= 4) {  // flattened pointwise layers take the small tile counts
      if (c.lgpp >= 0)
        return t.nslabs > 1 ? launch_one<NT, KIND, true, true>(p, t, c, grid, ldsb, st)
                            : launch_one<NT, KIND, false, true>(p, t, c, grid, ldsb, st);
    }
    return t.nslabs > 1 ? launch_one<NT, KIND, true, false>(p, t, c, grid, ldsb, st)
                        : launch_one<NT, KIND, false, false>(p, t, c, grid, ldsb, st);
  }
}

}  // namespace

namespace {

// dtype BSP_BF16: bf16 layers.  dtype BSP_I8: int8 codes in, int8 results after `shift`.
int launch_lds(const ConvParams& p_in, int dtype, const void* plan_host, int shift, hipStream_t st) {
  const bool i8 = dtype == BSP_I8;
  // input channels: whole 16-byte chunks (8 bf16 or 16 int8), or, for bf16, at most 4 in all
  // (a first layer's RGB planes), which the data movers then gather element by element into
  // one zero-padded chunk.  int8 results leave as pieces of 16 channels.
  if (!plan_host || (dtype != BSP_BF16 && !i8)) return BSP_ERR_UNSUPPORTED;
  if (i8 ? ((p_in.I % 16) != 0 || (p_in.O % 16) != 0)
         : (((p_in.I % 8) != 0 && p_in.I > 4) || (p_in.O % 8) != 0))
    return BSP_ERR_UNSUPPORTED;
  const int32_t* hdr = (const int32_t*)plan_host;
  if (hdr[BSP_PLAN_MAGIC_W] != BSP_PLAN_MAGIC || hdr[BSP_PLAN_VERSION_W] != BSP_PLAN_VERSION ||
      hdr[BSP_PLAN_O_W] != p_in.O || hdr[BSP_PLAN_I_W] != p_in.I || hdr[BSP_PLAN_H_W] != p_in.H ||
      hdr[BSP_PLAN_K_W] != p_in.K || hdr[BSP_PLAN_DTYPE_W] != dtype)
    return BSP_ERR_UNSUPPORTED;
  ConvParams p = p_in;
  bool flattened = false;
  const int plan_slab = i8 ? hdr[BSP_PLAN_SLAB_W] / 2 : hdr[BSP_PLAN_SLAB_W];
  if (i8) p.I /= 2;  // from here on an input element is a pair of codes (2 bytes, like a bf16)
  const int out_row = i8 ? kOutRowI8 : kOutRow;
  if (p.H == 1 && p.K == 1 && p.sh == 1 && p.sw == 1 && p.ph == 0 && p.pw == 0) {
    p.J = p.N = p.P;
    p.L = p.M = 1;
    p.B = 1;
    flattened = true;
  }
  LdsCfg c;
  c.maxsteps = hdr[BSP_PLAN_MAXSLABSTEPS_W];
  const int nslabs = hdr[BSP_PLAN_NSLABS_W];
  // a compute wave stages half the steps of a slab of its strip, one descriptor per lane
  if (c.maxsteps < 1 || c.maxsteps > kWHalf * kPH || c.maxsteps > 32 || nslabs > kMaxSlabs)
    return BSP_ERR_UNSUPPORTED;
  c.wload = (c.maxsteps + kPH - 1) / kPH;  // each of a strip's waves stages this many steps
  c.region_bytes = c.maxsteps * (1024 + 16);
  const int64_t wbytes = 4ll * c.region_bytes;

  // flattened pointwise layers: the movers keep no maps and move longer batches, so the tiles
  // can be larger
  const int lgpp = flattened ? 0 : -1;
  const int max_pieces = kLoaderThreads * (lgpp >= 0 ? kXBatchFlat : kXBatch);
  TileCfg t;
  int NT = 0;
  {
    static std::mutex mu;
    static std::map<std::array<int32_t, 13>, std::pair<int, TileCfg>> memo;
    const std::array<int32_t, 13> key = {p.B, p.M, p.N, p.I, p.O, p.H, p.K, p.sh, p.sw, p.ph, p.pw,
                                         c.maxsteps, dtype};
    std::lock_guard<std::mutex> lock(mu);
    auto it = memo.find(key);
    if (it == memo.end()) {
      t.slab = bsp_slab_channels(p.I, p.H, p.K);
      t.nslabs = ((p.I + 7) / 8 + t.slab / 8 - 1) / (t.slab / 8);
      t.nstrips = (p.O + BSP_STRIP - 1) / BSP_STRIP;
      // the LDS left after the weights holds the patch and the results staging tile
      const int groups = (t.nstrips + 3) / 4;
      const int64_t room = kLdsPerCu - wbytes - 4 * (kMaxSlabs + 1) * 4;
      const int slots = std::max(1, device_cus() / groups);
      if (!bsp_choose_tile(p, t.slab, room, max_pieces, kPH, out_row, 2, slots, &NT, &t)) NT = 0;
      // the long batches exist for the small tile counts only
      if (NT > 4 && (int64_t)t.TPH * t.TPW * (t.slab / BSP_CHUNK) > kLoaderThreads * kXBatch &&
          !bsp_choose_tile(p, t.slab, room, kLoaderThreads * kXBatch, kPH, out_row, 2, slots, &NT, &t))
        NT = 0;
      if (memo.size() > 4096) memo.clear();
      it = memo.emplace(key, std::make_pair(NT, t)).first;
    }
    NT = it->second.first;
    t = it->second.second;
    if (NT == 0) return BSP_ERR_UNSUPPORTED;
  }
  if (t.nslabs != nslabs || t.slab != plan_slab) return BSP_ERR_UNSUPPORTED;
  if (t.TPH * t.gsh >= 1024 || t.TPW * t.gsw >= 1024 || t.slab / BSP_CHUNK > 32)
    return BSP_ERR_UNSUPPORTED;
  const int64_t ntiles = (int64_t)p.B * t.tiles_y * t.tiles_x;
  const int movers = kLoaderThreads;  // threads that move the patch
  c.part_bytes = 16;
  int64_t patch_bytes = (int64_t)t.TPH * t.pitch;
  c.wbuf_off = (int32_t)((patch_bytes + 15) & ~15);
  c.obuf_off = c.wbuf_off + (int32_t)wbytes;
  c.sp_off = c.obuf_off + NT * kPH * 16 * out_row;
  const size_t ldsb = (size_t)c.sp_off + 4 * (kMaxSlabs + 1) * 4;
  if ((int64_t)ldsb > kLdsPerCu) return BSP_ERR_UNSUPPORTED;
  c.groups = (t.nstrips + 3) / 4;
  // persistent grid: one workgroup per CU, shared out among the strip groups
  int64_t slots = device_cus() / c.groups;
  if (slots < 1) slots = 1;
  c.wg_per_group = (int32_t)(ntiles < slots ? ntiles : slots);
  const int64_t nwg = (int64_t)c.wg_per_group * c.groups;
  const int64_t npieces = (int64_t)t.TPH * t.TPW * (t.slab / BSP_CHUNK);
  // the multiply-high divisions of a tile number (by tiles per image, then by tiles per row;
  // of a workgroup number by the strip groups) are exact while dividend * divisor < 2^32
  if (ntiles * std::max<int64_t>((int64_t)t.tiles_y * t.tiles_x, t.tiles_x) >= (1ll << 32) ||
      nwg * c.groups >= (1ll << 32))
    return BSP_ERR_UNSUPPORTED;
  if (nwg >= (1 << 24) || ntiles >= (1 << 24) ||
      npieces > max_pieces ||
      (npieces + kXBatchFlat * kLoaderThreads) * t.TPW >= (1ll << 32) || (int64_t)p.L * p.J * p.I >= (1ll << 31))
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
  {
    const int PP = t.slab / BSP_CHUNK;
    const int spix = movers / PP;  // pixels per step, then its rows and columns
    c.s_part = movers % PP;
    const int s_py = spix / t.TPW;
    c.s_px = spix % t.TPW;
    c.s_l = s_py * t.pitch + c.s_px * t.row_bytes + c.s_part * c.part_bytes;
    c.s_g = (s_py * t.gsh * p.J + c.s_px * t.gsw) * p.I + c.s_part * BSP_CHUNK;
    c.s_iy = s_py * t.gsh;
    c.s_ix = c.s_px * t.gsw;
    c.cp_l = t.row_bytes - PP * c.part_bytes;
    c.cp_g = t.gsw * p.I - PP * BSP_CHUNK;
    c.cx_l = t.pitch - t.TPW * t.row_bytes;
    c.cx_g = (t.gsh * p.J - t.TPW * t.gsw) * p.I;
    c.cx_ix = t.TPW * t.gsw;
  }
  // long compute phases (windows over several slabs) hide the movers anyway, and their
  // instructions then only take issue slots from the matrix cores
  c.mover_first = !(p.H * p.K > 1 && nslabs > 1);
  c.shift = shift;
  c.lgpp = (lgpp >= 0 && NT <= 4) ? lgpp : -1;
  c.nsteps = hdr[BSP_PLAN_NSTEPS_W];
  c.off_slab = hdr[BSP_PLAN_OFF_SLAB_W];
  c.off_xdesc = hdr[BSP_PLAN_OFF_XDESC_W];
  c.off_wfrag = hdr[BSP_PLAN_OFF_WFRAG_W];
  dim3 grid((unsigned)nwg);
  if (i8) {
    switch (NT) {
      case 2: return launch<2, kInt8>(p, t, c, grid, ldsb, st);
      case 4: return launch<4, kInt8>(p, t, c, grid, ldsb, st);
      case 7: return launch<7, kInt8>(p, t, c, grid, ldsb, st);
      case 8: return launch<8, kInt8>(p, t, c, grid, ldsb, st);
      default: return BSP_ERR_UNSUPPORTED;
    }
  }
  if ((p.I % 8) != 0) {  // first layers are large: the two large tile shapes are enough
    if (NT == 7) return launch<7, kBf16Narrow>(p, t, c, grid, ldsb, st);
    if (NT == 8) return launch<8, kBf16Narrow>(p, t, c, grid, ldsb, st);
    return BSP_ERR_UNSUPPORTED;
  }
  switch (NT) {
    case 2: return launch<2, kBf16>(p, t, c, grid, ldsb, st);
    case 4: return launch<4, kBf16>(p, t, c, grid, ldsb, st);
    case 7: return launch<7, kBf16>(p, t, c, grid, ldsb, st);
    case 8: return launch<8, kBf16>(p, t, c, grid, ldsb, st);
    default: return BSP_ERR_UNSUPPORTED;
  }
}

}  // namespace

int bsp_launch_lds(const ConvParams& p, int dtype, const void* plan_host, hipStream_t st) {
  if (dtype != BSP_BF16) return BSP_ERR_UNSUPPORTED;
  return launch_lds(p, dtype, plan_host, 0, st);
}

int bsp_launch_lds_i8(const ConvParams& p, const void* plan_host, int shift, hipStream_t st) {
  if (p.residual || p.relu) return BSP_ERR_UNSUPPORTED;
  return launch_lds(p, BSP_I8, plan_host, shift, st);
}
