// Three consecutive layers on one output tile with both intermediates kept in LDS (paper
// Section VI, depth-wise tiling): 1x1 (I -> C), 3x3 with padding 1 (C -> C), 1x1 (C -> O), a
// ReLU after each, an optional residual added before the last one.  bf16, fp32 accumulation;
// every intermediate is rounded to bf16 where the per-layer path would store it.
//
// A workgroup of 16 waves owns BR output rows of one image, all J columns.
//   A. 1x1 over the band's input rows (one halo row above and below).  The rows are one
//      contiguous range of pixels: they are streamed through two LDS buffers in chunks of
//      16*CT pixels (waves 12..15 only move data, global_load_lds; waves 0..11 compute).
//      Results go to T1, an LDS image of (BR + 2) x (J + 2) pixels x C channels whose border
//      (padding and rows outside the image) stays zero.
//   B. 3x3 from T1: a work item is a strip of 16 output channels and 16 output columns, all BR
//      rows; an activation fragment read once serves the three window rows (as in the
//      row-band kernel).  Results go to T2 (BR x J pixels x C channels), which reuses the
//      chunk buffers.
//   C. 1x1 from T2, 64 pixels x 16 strips at a time; the results of a round are gathered in
//      LDS as whole output lines (reusing T1), then written with the residual and the ReLU.
// Weights come from the three layers' row-band plan sections (bsp_plan.h); only kept blocks
// are multiplied.  LDS pixels are swizzled as in bsp_pw.hip (slot = piece ^ f(pixel)).
#include "bsp_launch.h"
#include "bsp_tile.h"

#include <algorithm>
#include <cstdlib>

namespace {

struct LayerPlan {
  const int32_t* rstrip;
  const int32_t* rslab;
  const unsigned char* rdesc;
  const unsigned char* rfrag;
  const float* bias;
  int32_t nstrips, nslabs, sc;  // sc: 16-byte pieces per slab
  int64_t wbytes;               // weight fragments of the whole layer
};

struct ChainArgs {
  const unsigned char* X;
  unsigned char* Y;
  const unsigned char* residual;
  LayerPlan l1, l2, l3;
  int32_t B, L, J, I, C, O;
  int32_t nbands;
  int32_t Jp;                        // T1 row pitch in pixels (J + 2)
  int32_t CT;                        // lane tiles per chunk of phase A
  int32_t pitchX, xs_shift, xs_mask; // staged input pixel: bytes, swizzle
  int32_t pitchC, cs_shift, cs_mask; // T1 / T2 pixel
  int32_t xbuf, nbuf;                // bytes of one chunk buffer; how many there are (2 or 4)
  int32_t odbl;                      // two output images in phase C (one barrier per round) or one (two)
  int32_t adv_pix, adv_rem;          // 4096 / pitchX and 4096 % pitchX: from one request of a mover to its next
  int32_t t1_off;                    // LDS offset of T1 (and of the output image of phase C)
  int32_t opitch;                    // bytes per pixel of the output image
  int32_t relu;
  FastDiv d_J, d_pitchX, d_ct;
#ifdef BSP_ROWS_TUNE
  long long* trace;
#endif
};

#ifdef BSP_ROWS_TUNE
#define CH_MARK(k)                                                                                   \
  do {                                                                                               \
    if (a.trace && lane == 0) a.trace[((size_t)blockIdx.x * 16 + wave) * 8 + (k)] = wall_clock64(); \
  } while (0)
#else
#define CH_MARK(k)
#endif

typedef __attribute__((address_space(1))) const void* gptr_t;
typedef __attribute__((address_space(3))) void* lptr_t;

constexpr int kComputeA = 12;  // compute waves of phase A; the other four move data

template <int BR>
__global__ __launch_bounds__(1024) void conv_chain(ChainArgs a) {
  kernarg_touch<ChainArgs>();
  extern __shared__ __align__(16) unsigned char lds[];
  const int tid = threadIdx.x, lane = tid & 63, g = lane >> 4, c = lane & 15;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int n = (int)blockIdx.x / a.nbands, band = (int)blockIdx.x - n * a.nbands;
  const int y0 = band * BR;
  const int ra = max(y0 - 1, 0), rb = min(y0 + BR + 1, a.L);
  const int npx = (rb - ra) * a.J;          // input pixels of the band, contiguous in X
  const int roff = ra - (y0 - 1);           // T1 row of the first of them
  const uint32_t gp0 = (uint32_t)(n * a.L + ra) * (uint32_t)a.J;
  const int CH = a.CT * 16;
  const int nch = (npx + CH - 1) / CH;
  unsigned char* T1 = lds + a.t1_off;
  unsigned char* T2 = lds;
  const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)lds;

  CH_MARK(0);
  // ---- T1's border must read as zero: clear all of it (phase A overwrites the inside)
  {
    const int n16 = ((BR + 2) * a.Jp * a.pitchC) >> 4;
    for (int i = tid; i < n16; i += (int)blockDim.x) ((u32x4_t*)T1)[i] = u32x4_t{0, 0, 0, 0};
  }

  CH_MARK(1);
  // ================= phase A
  if (wave >= kComputeA) {
    // ---- data movers: chunk k goes to buffer k % nbuf; its KiB requests are dealt out to the
    // four movers (request rq to mover rq % 4), so that asking for a chunk is short.  Barrier k
    // tells the compute waves that chunk k has landed and everybody that chunk k - 1 has been
    // consumed: its buffer then takes chunk k + nbuf - 1, nbuf - 1 chunks being in flight while
    // one is worked on.  A wave's copies complete in order, so "chunk k has landed" is "at
    // most as many of my requests are outstanding as I made for the chunks after it"; for
    // the last chunks (one of which may have requests that are skipped) that is zero.
    const int mw = wave - kComputeA;
    const int nreq = (CH * a.pitchX) >> 10;
    const int nbm = a.nbuf - 1;  // (two or four buffers)
    const int per = (nreq - mw + 3) >> 2;  // my requests per chunk
    auto request = [&](int k) {
      const uint32_t buf = lds0 + (uint32_t)(k & nbm) * (uint32_t)a.xbuf;
      const uint32_t o0 = (uint32_t)mw * 1024u + (uint32_t)lane * 16u;
      uint32_t lp = fdiv(o0, a.d_pitchX);
      uint32_t rem = o0 - lp * (uint32_t)a.pitchX;
      for (int rq = mw; rq < nreq; rq += 4) {
        const uint32_t piece = (rem >> 4) ^ ((lp >> a.xs_shift) & (uint32_t)a.xs_mask);
        const uint32_t q = (uint32_t)k * (uint32_t)CH + lp;
        if (q < (uint32_t)npx && piece * 8u < (uint32_t)a.I)
          __builtin_amdgcn_global_load_lds((gptr_t)(a.X + ((gp0 + q) * (uint32_t)a.I + piece * 8u) * 2u),
                                           (lptr_t)(uintptr_t)(buf + (uint32_t)rq * 1024u), 16, 0, 0);
        rem += (uint32_t)a.adv_rem;
        lp += (uint32_t)a.adv_pix;
        if (rem >= (uint32_t)a.pitchX) {
          rem -= (uint32_t)a.pitchX;
          ++lp;
        }
      }
    };
    // wait until at most n of this wave's copies are outstanding (n a multiple of `per`)
    auto wait_le = [&](int n) {
      switch (n) {
#define BSP_CASE(v) \
  case v: __builtin_amdgcn_s_waitcnt(0x0F70 | ((v) & 15) | (((v) >> 4) << 14)); break;
        BSP_CASE(1) BSP_CASE(2) BSP_CASE(3) BSP_CASE(4) BSP_CASE(6) BSP_CASE(8) BSP_CASE(9) BSP_CASE(12)
        BSP_CASE(16) BSP_CASE(18) BSP_CASE(24) BSP_CASE(32) BSP_CASE(36) BSP_CASE(48)
#undef BSP_CASE
        default: __builtin_amdgcn_s_waitcnt(0); break;
      }
    };
    for (int k = 0; k < nbm && k < nch; ++k) request(k);  // the first chunks
    for (int k = 0; k < nch; ++k) {
      const int after = min(nbm - 1, nch - 1 - k);  // chunks asked for after chunk k so far
      if (k + nbm >= nch) __builtin_amdgcn_s_waitcnt(0);
      else wait_le(after * per);
      __builtin_amdgcn_s_barrier();  // barrier k (the bare instruction: a fence would wait for every copy in flight)
      if (k + nbm < nch) request(k + nbm);
    }
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();  // T1 is complete
  } else {
    // ---- compute waves: work item = (strip, lane tile of the chunk); wave w takes items w,
    // w + 12, ...  What the first item needs from the plan is fetched once, before the chunks.
    const int nitems = a.l1.nstrips * a.CT;
    struct Item {
      int lo, hi, chan, t;
      f32x4_t bv;
    };
    auto setup = [&](int item) {
      Item it;
      const int strip = (int)fdiv((uint32_t)item, a.d_ct);
      it.t = item - strip * a.CT;
      it.lo = a.l1.rslab[strip * 2];
      it.hi = a.l1.rslab[strip * 2 + 1];
      it.chan = a.l1.rstrip[strip * 4 + g];
      it.bv = f32x4_t{0.f, 0.f, 0.f, 0.f};
      if (a.l1.bias && it.chan >= 0)
        it.bv = f32x4_t{a.l1.bias[it.chan], a.l1.bias[it.chan + 1], a.l1.bias[it.chan + 2], a.l1.bias[it.chan + 3]};
      return it;
    };
    const bool mine = wave < nitems;
    Item first = setup(mine ? wave : 0);
    // A wave with a single item whose strip has at most eight steps keeps that strip's
    // weights in registers for all chunks.
    const bool resident = nitems <= kComputeA && first.hi - first.lo <= 8;
    u32x4_t wres[8];
    int dres[8];
#pragma unroll
    for (int d = 0; d < 8; ++d) {
      wres[d] = u32x4_t{0, 0, 0, 0};
      dres[d] = 0;
      if (resident && mine && first.lo + d < first.hi) {
        dres[d] = *(const int*)(a.l1.rdesc + ((uint32_t)(first.lo + d) * 16u + (uint32_t)g * 4u));
        wres[d] = *(const u32x4_t*)(a.l1.rfrag + ((uint32_t)(first.lo + d) * 1024u + (uint32_t)lane * 16u));
      }
    }
    for (int k = 0; k < nch; ++k) {
      // (streamed weights) the first item's first step, asked for before the wait for the chunk
      int d0 = 0;
      u32x4_t w0 = {0, 0, 0, 0};
      if (!resident && mine && first.lo < first.hi) {
        d0 = *(const int*)(a.l1.rdesc + ((uint32_t)first.lo * 16u + (uint32_t)g * 4u));
        w0 = *(const u32x4_t*)(a.l1.rfrag + ((uint32_t)first.lo * 1024u + (uint32_t)lane * 16u));
      }
      __syncthreads();  // barrier k (the clearing of T1 above is also behind it)
      const unsigned char* xb = lds + (k & (a.nbuf - 1)) * a.xbuf;
      for (int item = wave; item < nitems; item += kComputeA) {
        Item it = first;
        if (item != wave) {
          it = setup(item);
          if (it.lo < it.hi) {
            d0 = *(const int*)(a.l1.rdesc + ((uint32_t)it.lo * 16u + (uint32_t)g * 4u));
            w0 = *(const u32x4_t*)(a.l1.rfrag + ((uint32_t)it.lo * 1024u + (uint32_t)lane * 16u));
          }
        }
        const int lp = it.t * 16 + c;
        const uint32_t swz = ((uint32_t)lp >> a.xs_shift) & (uint32_t)a.xs_mask;
        const uint32_t base = (uint32_t)lp * (uint32_t)a.pitchX;
        f32x4_t acc = {0.f, 0.f, 0.f, 0.f};
        if (resident) {
          const int ns = it.hi - it.lo;
          u32x4_t f[8];
#pragma unroll
          for (int d = 0; d < 8; ++d)
            if (d < ns) f[d] = *(const u32x4_t*)(xb + base + ((((uint32_t)dres[d] & 0xFFu) ^ swz) << 4));
#pragma unroll
          for (int d = 0; d < 8; ++d)
            if (d < ns) acc = mfma_bf16_16x16x32(wres[d], f[d], acc);
        } else {
          for (int cs = it.lo; cs < it.hi; ++cs) {  // one step ahead
            const int nx = min(cs + 1, it.hi - 1);
            const int d1 = *(const int*)(a.l1.rdesc + ((uint32_t)nx * 16u + (uint32_t)g * 4u));
            const u32x4_t w1 = *(const u32x4_t*)(a.l1.rfrag + ((uint32_t)nx * 1024u + (uint32_t)lane * 16u));
            const u32x4_t f = *(const u32x4_t*)(xb + base + ((((uint32_t)d0 & 0xFFu) ^ swz) << 4));
            acc = mfma_bf16_16x16x32(w0, f, acc);
            d0 = d1;
            w0 = w1;
          }
        }
        // bias, ReLU, one rounding, into T1 (zero border untouched)
        const int q = k * CH + lp;
        if (q < npx && it.chan >= 0) {
          f32x4_t v = acc + it.bv;
          if (a.relu) v = f32x4_t{fmaxf(v.x, 0.f), fmaxf(v.y, 0.f), fmaxf(v.z, 0.f), fmaxf(v.w, 0.f)};
          const int row = (int)fdiv((uint32_t)q, a.d_J), col = q - row * a.J;
          const uint32_t tp = (uint32_t)((roff + row) * a.Jp + col + 1);
          const uint32_t piece = (uint32_t)it.chan >> 3;
          const uint32_t ad = tp * (uint32_t)a.pitchC + ((piece ^ ((tp >> a.cs_shift) & (uint32_t)a.cs_mask)) << 4) +
                              (((uint32_t)it.chan & 4u) << 1);
          *(u32x2_t*)(T1 + ad) = u32x2_t{pack_bf16x2(v.x, v.y), pack_bf16x2(v.z, v.w)};
        }
      }
    }
    __syncthreads();  // T1 is complete
  }

  CH_MARK(2);
  // ================= phase B: 3x3 from T1 into T2 (which reuses the chunk buffers)
  {
    const int ctb = (a.J + 15) >> 4;  // column tiles
    const int nitems = a.l2.nstrips * ctb;
    for (int item = wave; item < nitems; item += 16) {
      const int strip = item / ctb, x0 = (item - strip * ctb) * 16;
      const int chan = a.l2.rstrip[strip * 4 + g];
      const int x = min(x0 + c, a.J - 1);  // lanes past the row's end repeat its last column (never stored)
      f32x4_t acc[BR];
#pragma unroll
      for (int r = 0; r < BR; ++r) acc[r] = f32x4_t{0.f, 0.f, 0.f, 0.f};
      // lane i holds the first step of slab i; a strip's steps are numbered consecutively
      const int vr = a.l2.rslab[strip * (a.l2.nslabs + 1) + min(lane, a.l2.nslabs)];
      const int s_first = __builtin_amdgcn_readlane(vr, 0), s_end = __builtin_amdgcn_readlane(vr, a.l2.nslabs);
      int sl = 0, s_next = __builtin_amdgcn_readlane(vr, 1);
      auto wload = [&](int cs, int& d, u32x4_t (&w)[3]) {
        d = *(const int*)(a.l2.rdesc + ((uint32_t)cs * 16u + (uint32_t)g * 4u));
#pragma unroll
        for (int dy = 0; dy < 3; ++dy)
          w[dy] = *(const u32x4_t*)(a.l2.rfrag + (((uint32_t)cs * 3u + dy) * 1024u + (uint32_t)lane * 16u));
      };
      int d0 = 0, d1 = 0;
      u32x4_t w0[3] = {}, w1[3] = {};
      if (s_first < s_end) wload(s_first, d0, w0);
      for (int cs = s_first; cs < s_end; ++cs) {  // one step ahead
        wload(min(cs + 1, s_end - 1), d1, w1);
        while (cs >= s_next) {
          ++sl;
          s_next = __builtin_amdgcn_readlane(vr, min(sl + 1, a.l2.nslabs));
        }
        const uint32_t desc = (uint32_t)d0;
        const uint32_t unit = (uint32_t)(sl * a.l2.sc) + (desc & 0xFFu), dx = (desc >> 8) & 0xFFu;
        u32x4_t f[BR + 2];
#pragma unroll
        for (int fr = 0; fr < BR + 2; ++fr) {
          const uint32_t tp = (uint32_t)(fr * a.Jp + x) + dx;
          f[fr] = *(const u32x4_t*)(T1 + tp * (uint32_t)a.pitchC +
                                    ((unit ^ ((tp >> a.cs_shift) & (uint32_t)a.cs_mask)) << 4));
        }
#pragma unroll
        for (int dy = 0; dy < 3; ++dy)
#pragma unroll
          for (int r = 0; r < BR; ++r) acc[r] = mfma_bf16_16x16x32(w0[dy], f[r + dy], acc[r]);
        d0 = d1;
#pragma unroll
        for (int dy = 0; dy < 3; ++dy) w0[dy] = w1[dy];
      }
      if (x0 + c < a.J && chan >= 0) {
        f32x4_t bv = {0.f, 0.f, 0.f, 0.f};
        if (a.l2.bias) bv = f32x4_t{a.l2.bias[chan], a.l2.bias[chan + 1], a.l2.bias[chan + 2], a.l2.bias[chan + 3]};
        const uint32_t piece = (uint32_t)chan >> 3;
#pragma unroll
        for (int r = 0; r < BR; ++r) {
          f32x4_t v = acc[r] + bv;
          if (a.relu) v = f32x4_t{fmaxf(v.x, 0.f), fmaxf(v.y, 0.f), fmaxf(v.z, 0.f), fmaxf(v.w, 0.f)};
          const uint32_t tp = (uint32_t)(r * a.J + x0 + c);
          const uint32_t ad = tp * (uint32_t)a.pitchC + ((piece ^ ((tp >> a.cs_shift) & (uint32_t)a.cs_mask)) << 4) +
                              (((uint32_t)chan & 4u) << 1);
          *(u32x2_t*)(T2 + ad) = u32x2_t{pack_bf16x2(v.x, v.y), pack_bf16x2(v.z, v.w)};
        }
      }
    }
  }
  CH_MARK(3);
  __syncthreads();  // T2 is complete, T1 is free
  CH_MARK(4);

  // ================= phase C: 1x1 from T2, a round of 64 pixels x 16 strips at a time
  {
    const int rows_out = min(BR, a.L - y0);
    const int npx2 = rows_out * a.J;
    const int nrounds = (npx2 + 63) >> 6;
    const int npass = (a.l3.nstrips + 15) >> 4;
    unsigned char* ot = T1;
    const uint32_t yp0 = (uint32_t)(n * a.L + y0) * (uint32_t)a.J;  // the band's first output pixel
    for (int pass = 0; pass < npass; ++pass) {
      const int strip = pass * 16 + wave;
      const bool active = strip < a.l3.nstrips;
      const int sq = active ? strip : 0;
      const int lo = a.l3.rslab[sq * 2], hi = active ? a.l3.rslab[sq * 2 + 1] : lo;
      const int chan = active ? a.l3.rstrip[sq * 4 + g] : -1;
      f32x4_t bv = {0.f, 0.f, 0.f, 0.f};
      if (a.l3.bias && chan >= 0) bv = f32x4_t{a.l3.bias[chan], a.l3.bias[chan + 1], a.l3.bias[chan + 2], a.l3.bias[chan + 3]};
      const int range0 = pass * 256;  // the pass's first output channel (strips are in window order)
      int df0 = 0, df1 = 0;
      u32x4_t wf0 = {0, 0, 0, 0}, wf1 = {0, 0, 0, 0};
      if (lo < hi) {
        df0 = *(const int*)(a.l3.rdesc + ((uint32_t)lo * 16u + (uint32_t)g * 4u));
        wf0 = *(const u32x4_t*)(a.l3.rfrag + ((uint32_t)lo * 1024u + (uint32_t)lane * 16u));
        const int s1 = min(lo + 1, hi - 1);
        df1 = *(const int*)(a.l3.rdesc + ((uint32_t)s1 * 16u + (uint32_t)g * 4u));
        wf1 = *(const u32x4_t*)(a.l3.rfrag + ((uint32_t)s1 * 1024u + (uint32_t)lane * 16u));
      }
      const int cpp = min(32, (a.O - range0) >> 3);  // 16-byte pieces per pixel in this pass
      for (int round = 0; round < nrounds; ++round) {
        // what this thread will write at the end of the round, and the residual that goes
        // with it: asked for now, used after the round's arithmetic
        bool ovalid[2];
        uint32_t ooff[2];
        u32x4_t res[2];
#pragma unroll
        for (int it = 0; it < 2; ++it) {
          const int i = tid + it * 1024, pixel = i >> 5, kk = i & 31;
          const int p2 = round * 64 + pixel;
          ovalid[it] = kk < cpp && p2 < npx2;
          ooff[it] = ((yp0 + (uint32_t)p2) * (uint32_t)a.O + (uint32_t)(range0 + kk * 8)) * 2u;
          res[it] = u32x4_t{0, 0, 0, 0};
          if (ovalid[it] && a.residual) res[it] = *(const u32x4_t*)(a.residual + ooff[it]);
        }
        f32x4_t acc[4];
        uint32_t base[4], swz[4];
#pragma unroll
        for (int t = 0; t < 4; ++t) {
          acc[t] = f32x4_t{0.f, 0.f, 0.f, 0.f};
          const uint32_t tp = (uint32_t)min(round * 64 + t * 16 + c, npx2 - 1);
          base[t] = tp * (uint32_t)a.pitchC;
          swz[t] = (tp >> a.cs_shift) & (uint32_t)a.cs_mask;
        }
        // the strip's first two steps stay in registers for all rounds; later ones are
        // streamed one step ahead
        int d0 = df0, d1 = df1;
        u32x4_t w0 = wf0, w1 = wf1;
        for (int cs = lo; cs < hi; ++cs) {
          int d2 = d1;
          u32x4_t w2 = w1;
          if (cs + 2 < hi) {
            d2 = *(const int*)(a.l3.rdesc + ((uint32_t)(cs + 2) * 16u + (uint32_t)g * 4u));
            w2 = *(const u32x4_t*)(a.l3.rfrag + ((uint32_t)(cs + 2) * 1024u + (uint32_t)lane * 16u));
          }
          const uint32_t unit = (uint32_t)d0 & 0xFFu;
#pragma unroll
          for (int t = 0; t < 4; ++t) {
            const u32x4_t f = *(const u32x4_t*)(T2 + base[t] + ((unit ^ swz[t]) << 4));
            acc[t] = mfma_bf16_16x16x32(w0, f, acc[t]);
          }
          d0 = d1;
          w0 = w1;
          d1 = d2;
          w1 = w2;
        }
        // the round's results as whole output lines in LDS (two images used in turn, so one
        // barrier per round is enough)
        unsigned char* oi = ot + (a.odbl ? (round & 1) * (64 * a.opitch) : 0);
        if (chan >= 0) {
#pragma unroll
          for (int t = 0; t < 4; ++t) {
            const f32x4_t v = acc[t] + bv;
            *(u32x2_t*)(oi + (t * 16 + c) * a.opitch + (chan - range0) * 2) =
                u32x2_t{pack_bf16x2(v.x, v.y), pack_bf16x2(v.z, v.w)};
          }
        }
        __syncthreads();
#pragma unroll
        for (int it = 0; it < 2; ++it) {
          if (!ovalid[it]) continue;
          const int i = tid + it * 1024, pixel = i >> 5, kk = i & 31;
          const u32x4_t v = *(const u32x4_t*)(oi + pixel * a.opitch + kk * 16);
          u32x2_t l2 = {v.x, v.y}, h2 = {v.z, v.w};
          if (a.residual || a.relu) {
            l2 = post_bf16x4_reg(l2, u32x2_t{res[it].x, res[it].y}, a.residual != nullptr, a.relu);
            h2 = post_bf16x4_reg(h2, u32x2_t{res[it].z, res[it].w}, a.residual != nullptr, a.relu);
          }
          __builtin_nontemporal_store(u32x4_t{l2.x, l2.y, h2.x, h2.y}, (u32x4_t*)(a.Y + ooff[it]));
        }
        if (!a.odbl) __syncthreads();
      }
      __syncthreads();  // before the next pass reuses the images
    }
  }
  CH_MARK(5);
}

constexpr int kLdsLimit = 160 * 1024;

template <int BR>
int launch_chain(const ChainArgs& a, dim3 grid, size_t ldsb, hipStream_t st) {
  static bool raised = false;  // dynamic LDS above 64 KB has to be allowed once per kernel
  if (!raised) {
    if (hipFuncSetAttribute((const void*)conv_chain<BR>, hipFuncAttributeMaxDynamicSharedMemorySize, kLdsLimit) !=
        hipSuccess)
      return BSP_ERR_HIP;
    raised = true;
  }
  hipLaunchKernelGGL((conv_chain<BR>), grid, dim3(1024), ldsb, st, a);
  return hipGetLastError() == hipSuccess ? BSP_OK : BSP_ERR_HIP;
}

// The row-band section of one layer's plan, checked against the layer.
bool layer_plan(const bsp_weights* w, const float* bias, int H, LayerPlan* out) {
  if (!w || !w->plan_host || !w->plan || w->dtype != BSP_BF16 || w->H != H || w->K != H) return false;
  const int32_t* hdr = (const int32_t*)w->plan_host;
  if (hdr[BSP_PLAN_MAGIC_W] != BSP_PLAN_MAGIC || hdr[BSP_PLAN_VERSION_W] != BSP_PLAN_VERSION ||
      hdr[BSP_PLAN_O_W] != w->O || hdr[BSP_PLAN_I_W] != w->I || hdr[BSP_PLAN_H_W] != w->H ||
      hdr[BSP_PLAN_OFF_ROWS_W] == 0)
    return false;
  const int32_t* rs = hdr + hdr[BSP_PLAN_OFF_ROWS_W];
  if (rs[BSP_ROWS_CW_W] != 8) return false;  // 8-channel contraction units (8x8 and 4x16 blocks)
  if (H == 1 && (rs[BSP_ROWS_NSLABS_W] != 1 || rs[BSP_ROWS_WINDOW_W] != 4)) return false;
  const int32_t* sec = (const int32_t*)w->plan + hdr[BSP_PLAN_OFF_ROWS_W];
  out->rstrip = sec + rs[BSP_ROWS_OFF_STRIP_W];
  out->rslab = sec + rs[BSP_ROWS_OFF_SLAB_W];
  out->rdesc = (const unsigned char*)(sec + rs[BSP_ROWS_OFF_DESC_W]);
  out->rfrag = (const unsigned char*)(sec + rs[BSP_ROWS_OFF_FRAG_W]);
  out->bias = bias;
  out->nstrips = rs[BSP_ROWS_NSTRIPS_W];
  out->nslabs = rs[BSP_ROWS_NSLABS_W];
  out->sc = rs[BSP_ROWS_SLAB_W] / 8;
  out->wbytes = (int64_t)rs[BSP_ROWS_NCS_W] * H * 1024;
  return true;
}

void pixel_pitch(int channels, int* pitch, int* shift, int* mask) {
  const int raw = channels * 2;
  *pitch = raw <= 128 ? 128 : (raw + 255) & ~255;
  if (*pitch % 256 == 0) {
    *shift = 0;
    *mask = 15;
  } else {
    *shift = 1;
    *mask = 7;
  }
}

}  // namespace

int bsp_launch_chain(const bsp_weights* w1, const bsp_weights* w2, const bsp_weights* w3, const void* X,
                     const float* bias1, const float* bias2, const float* bias3, const void* residual, void* Y,
                     int B, int L, int J, int relu, hipStream_t st) {
  ChainArgs a{};
#ifdef BSP_ROWS_TUNE
  if (const char* e = std::getenv("BSP_PW_TRACE_PTR")) a.trace = (long long*)std::strtoull(e, nullptr, 16);
#endif
  if (!layer_plan(w1, bias1, 1, &a.l1) || !layer_plan(w2, bias2, 3, &a.l2) || !layer_plan(w3, bias3, 1, &a.l3))
    return BSP_ERR_UNSUPPORTED;
  if (w1->O != w2->I || w2->O != w2->I || w3->I != w2->O) return BSP_ERR_SHAPE;
  a.X = (const unsigned char*)X;
  a.Y = (unsigned char*)Y;
  a.residual = (const unsigned char*)residual;
  a.B = B;
  a.L = L;
  a.J = J;
  a.I = w1->I;
  a.C = w2->I;
  a.O = w3->O;
  a.relu = relu;
  if (B < 1 || L < 1 || J < 1) return BSP_ERR_SHAPE;
  if ((int64_t)B * L * J * a.I * 2 >= (1ll << 31) || (int64_t)B * L * J * a.O * 2 >= (1ll << 31))
    return BSP_ERR_UNSUPPORTED;
  pixel_pitch(a.I, &a.pitchX, &a.xs_shift, &a.xs_mask);
  pixel_pitch(a.C, &a.pitchC, &a.cs_shift, &a.cs_mask);
  a.Jp = J + 2;
  a.opitch = 512 + 16;
  // rows per band: enough workgroups for the chip, as few halo rows as that allows
  int BR = 7;
  for (int cand : {7, 4, 2}) {
    BR = cand;
    if ((int64_t)B * ((L + cand - 1) / cand) >= 200) break;
  }
  for (;;) {
    const int64_t t1 = (int64_t)(BR + 2) * a.Jp * a.pitchC;
    const int64_t t2 = (int64_t)BR * J * a.pitchC;
    // most data in flight first: four chunk buffers and two output images, then less
    int ct = 0, nbuf = 0, odbl = 0;
    for (int nb : {4, 2}) {
      for (int od : {1, 0}) {
        const int64_t region1 = std::max<int64_t>(t1, (od ? 2 : 1) * 64 * a.opitch);
        for (int cand : {3, 2, 1}) {
          const int64_t region0 = (std::max<int64_t>((int64_t)nb * cand * 16 * a.pitchX, t2) + 255) & ~255ll;
          if (region0 + region1 <= kLdsLimit) {
            ct = cand;
            break;
          }
        }
        if (ct) {
          nbuf = nb;
          odbl = od;
          break;
        }
      }
      if (ct) break;
    }
    if (ct) {
      a.CT = ct;
      a.nbuf = nbuf;
      a.odbl = odbl;
      a.xbuf = ct * 16 * a.pitchX;
      a.t1_off = (int32_t)((std::max<int64_t>((int64_t)nbuf * a.xbuf, t2) + 255) & ~255ll);
      a.adv_pix = 4096 / a.pitchX;  // a mover's requests of one chunk are 4 KiB apart
      a.adv_rem = 4096 % a.pitchX;
      const int64_t ldsb = a.t1_off + std::max<int64_t>(t1, (odbl ? 2 : 1) * 64 * a.opitch);
      if (ldsb <= kLdsLimit) {
        a.nbands = (L + BR - 1) / BR;
        a.d_J = make_fastdiv((uint32_t)J);
        a.d_pitchX = make_fastdiv((uint32_t)a.pitchX);
        a.d_ct = make_fastdiv((uint32_t)a.CT);
        // multiply-high divisions are exact while dividend * divisor < 2^32
        if ((int64_t)(BR + 2) * J * J >= (1ll << 32) || (int64_t)a.xbuf * a.pitchX >= (1ll << 32) ||
            (int64_t)a.l1.nstrips * a.CT * a.CT >= (1ll << 32) || (int64_t)B * a.nbands >= (1ll << 31))
          return BSP_ERR_UNSUPPORTED;
        // Every band streams all three layers' weights: worth it only while that stays below
        // what the intermediates would have cost in memory traffic (their round trips are about
        // what X and Y cost).  Deep, small-image bottlenecks are faster layer by layer; a
        // caller's kernel mask (BSP_KERNEL_CHAIN in any of the three) overrides the rule.
        const bool forced = ((w1->kernels | w2->kernels | w3->kernels) & BSP_KERNEL_CHAIN) != 0;
        const int64_t wtraffic = (a.l1.wbytes + a.l2.wbytes + a.l3.wbytes) * B * a.nbands;
        if (!forced && wtraffic > (int64_t)B * L * J * (a.I + a.O) * 2) return BSP_ERR_UNSUPPORTED;
        dim3 grid((unsigned)(B * a.nbands));
        switch (BR) {
          case 7: return launch_chain<7>(a, grid, (size_t)ldsb, st);
          case 4: return launch_chain<4>(a, grid, (size_t)ldsb, st);
          case 2: return launch_chain<2>(a, grid, (size_t)ldsb, st);
        }
      }
    }
    if (BR == 7)
      BR = 4;
    else if (BR == 4)
      BR = 2;
    else
      return BSP_ERR_UNSUPPORTED;  // the intermediates do not fit LDS
  }
}
