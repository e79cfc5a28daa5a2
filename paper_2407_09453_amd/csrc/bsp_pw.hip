// Pointwise (1x1) bf16 layers as a block-sparse matrix product, fp32 accumulation:
// Y[pixel][o] = bias[o] + sum over the kept blocks of row o of W[o][i] * X[pixel][i]
// (paper Eq. (5) with H = K = 1; only kept blocks are multiplied, Section I advantages 3-4).
//
// Work split.  A workgroup owns MT = 16 * PT * PG consecutive output pixels and NS strips of
// 16 output channels.  All input channels of its pixels are copied once from global memory
// straight into LDS (global_load_lds, one contiguous KiB per request); nothing is staged
// twice and there is no loop over channel slabs.  A staged pixel is `pitch` bytes; its
// 16-byte pieces are permuted by the pixel's position (slot = piece ^ f(pixel)) so that the
// sixteen pixels of a lane tile fall into sixteen different bank groups.  Wave (strip s,
// pixel group q) walks the strip's column steps: per step one weight fragment (streamed from
// the plan through a ring of D registers, requested D steps ahead), PT activation fragments
// from LDS at the channels the step's descriptor names, PT MFMAs.  Results leave straight
// from the accumulators; two lane tiles exchange halves across lane rows first so that every
// lane stores the 16 contiguous bytes of one 8-channel block row.
//
// Staged pixels past the layer's last pixel are never written to LDS and never stored: each
// MFMA column depends on its own pixel only.
#include "bsp_launch.h"
#include "bsp_tile.h"

#include <algorithm>
#include <cstdio>
#include <cstdlib>

namespace {

struct PwArgs {
  const unsigned char* X;
  unsigned char* Y;
  const float* bias;
  const unsigned char* residual;
  const int32_t* rstrip;
  const int32_t* rslab;
  const unsigned char* rdesc;
  const unsigned char* rfrag;
  int32_t relu, nstrips;
  int32_t P, I, O;
  int32_t S, L, J, N, MN;          // S > 1: output pixel (img, y, x) reads input pixel (img, y*S, x*S)
  int32_t pitch, swz_shift, swz_mask;
  int32_t MT, lpg, NS, nreq;       // pixels per tile, log2 of the pixel groups, strips, KiB requests per tile
  int32_t mtiles, nsplit, per_xcd;
  int32_t pair;                    // results leave as 16-byte pieces (lane tiles paired)
  int32_t win_out, out_off, opitch;  // results gathered in LDS as whole output lines: where, bytes per pixel there
  int32_t adv_pix, adv_rem;        // (waves * 1024) / pitch and % pitch: a wave's step from request to request
  FastDiv d_mn, d_n, d_pitch, d_nsplit, d_cpp;
#ifdef BSP_ROWS_TUNE
  long long* trace;
#endif
};

#ifdef BSP_ROWS_TUNE
#define PW_MARK(k)                                                                                   \
  do {                                                                                               \
    if (a.trace && lane == 0) a.trace[((size_t)blockIdx.x * 16 + wave) * 8 + (k)] = wall_clock64(); \
  } while (0)
#else
#define PW_MARK(k)
#endif

typedef __attribute__((address_space(1))) const void* gptr_t;
typedef __attribute__((address_space(3))) void* lptr_t;

template <int PT, bool CW4, int D, int MAXT>
__global__ __launch_bounds__(MAXT) void conv_pw(PwArgs a) {
  kernarg_touch<PwArgs>();
  extern __shared__ __align__(16) unsigned char lds[];
  const int tid = threadIdx.x, lane = tid & 63, g = lane >> 4, c = lane & 15;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int nwaves = (int)(blockDim.x >> 6);
  // consecutive workgroups of one XCD share a pixel tile (its second reader hits that L2)
  const int xcd = blockIdx.x & 7, slot_wg = blockIdx.x >> 3;
  if (slot_wg >= a.per_xcd) return;
  const int q = xcd * a.per_xcd + slot_wg;
  const int mt = (int)fdiv((uint32_t)q, a.d_nsplit);
  if (mt >= a.mtiles) return;
  const int ns = q - mt * a.nsplit;
  const int pix0 = mt * a.MT;
  PW_MARK(0);

  // ---- this wave's strip and pixel group.  Its step range and output channels are wave-uniform:
  // scalar loads, asked for here and waited for once the tile's copies are on their way (a
  // vector load would have to queue behind those copies, and a wait here would delay them)
  const int sidx = wave >> a.lpg, pg = wave & ((1 << a.lpg) - 1);
  const int strip = ns * a.NS + sidx;
  const bool active = sidx < a.NS && strip < a.nstrips;
  const int sq = active ? strip : 0;
  u32x2_t lohi;
  u32x4_t ch4;
  {
    const int32_t* ps = a.rslab + sq * 2;
    const int32_t* pc = a.rstrip + sq * 4;
    asm volatile("s_load_dwordx2 %0, %2, 0x0\n\ts_load_dwordx4 %1, %3, 0x0"
                 : "=&s"(lohi), "=&s"(ch4)
                 : "s"(ps), "s"(pc)
                 : "memory");
  }

  // ---- stage the tile: request rq fills LDS bytes [rq * 1024, rq * 1024 + 1024)
  const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)lds;
  {
    // lane state: the staged pixel its 16 bytes belong to and their offset in it; from one
    // request of this wave to the next both advance by constants
    const uint32_t o0 = (uint32_t)wave * 1024u + (uint32_t)lane * 16u;
    uint32_t lp = fdiv(o0, a.d_pitch);
    uint32_t rem = o0 - lp * (uint32_t)a.pitch;
    for (int rq = wave; rq < a.nreq; rq += nwaves) {
      const uint32_t piece = (rem >> 4) ^ ((lp >> a.swz_shift) & (uint32_t)a.swz_mask);
      const uint32_t p = (uint32_t)pix0 + lp;
      uint32_t ip = p;
      if (a.S > 1) {
        const uint32_t img = fdiv(p, a.d_mn), r2 = p - img * (uint32_t)a.MN;
        const uint32_t oy = fdiv(r2, a.d_n), ox = r2 - oy * (uint32_t)a.N;
        ip = (img * (uint32_t)a.L + oy * (uint32_t)a.S) * (uint32_t)a.J + ox * (uint32_t)a.S;
      }
      if (p < (uint32_t)a.P && piece * 8u < (uint32_t)a.I)
        __builtin_amdgcn_global_load_lds((gptr_t)(a.X + (ip * (uint32_t)a.I + piece * 8u) * 2u),
                                         (lptr_t)(uintptr_t)(lds0 + (uint32_t)rq * 1024u), 16, 0, 0);
      rem += (uint32_t)a.adv_rem;
      lp += (uint32_t)a.adv_pix;
      if (rem >= (uint32_t)a.pitch) {
        rem -= (uint32_t)a.pitch;
        ++lp;
      }
    }
  }
  PW_MARK(1);
  // ---- the step range and channels asked for above have to be there now (the registers pass
  // through the wait, so that no use of them is moved above it)
  asm volatile("s_waitcnt lgkmcnt(0)" : "+s"(lohi), "+s"(ch4) : : "memory");
  PW_MARK(2);
  const int lo = (int)lohi.x, hi = active ? (int)lohi.y : lo;
  const int nsteps = hi - lo;
  // first output channel of this lane's four rows
  const int chan = !active ? -1 : g == 0 ? (int)ch4.x : g == 1 ? (int)ch4.y : g == 2 ? (int)ch4.z : (int)ch4.w;

  const uint32_t frag_lane = (uint32_t)lane * 16u, desc_lane = (uint32_t)g * 4u;
  u32x4_t wr[D];  // weight fragments of the next D steps, oldest in slot 0
  int dr[D];      // their item descriptors
  int fnext = lo;
  // Slot d takes the next step; past the strip's end it asks for the last step again (a valid
  // address, never used).  Every pass of the ring loop thus issues the same loads whatever
  // the step count, so the wait before a slot's use can be for exactly that slot.
  auto fetch = [&](int d) {
    const int cs = min(fnext, hi - 1);
    ++fnext;
    dr[d] = *(const int*)(a.rdesc + ((uint32_t)cs * 16u + desc_lane));
    wr[d] = *(const u32x4_t*)(a.rfrag + ((uint32_t)cs * 1024u + frag_lane));
  };
  // the first D steps, and no more than the strip has
#pragma unroll
  for (int d = 0; d < D; ++d) {
    dr[d] = 0;
    wr[d] = u32x4_t{0, 0, 0, 0};
    if (d < nsteps) fetch(d);
  }
  f32x4_t bv = {0.f, 0.f, 0.f, 0.f};
  if (a.bias && chan >= 0) bv = f32x4_t{a.bias[chan], a.bias[chan + 1], a.bias[chan + 2], a.bias[chan + 3]};

  f32x4_t acc[PT];
#pragma unroll
  for (int t = 0; t < PT; ++t) acc[t] = f32x4_t{0.f, 0.f, 0.f, 0.f};

  PW_MARK(3);
  __builtin_amdgcn_s_waitcnt(0);  // this wave's requests have landed
  PW_MARK(4);
  __syncthreads();                // everybody's have
  PW_MARK(5);
  if (!active && !a.win_out) return;  // (with win_out every wave helps to store the tile)

  const int lp0 = pg * (PT * 16) + c;  // this lane's pixel of the wave's first lane tile
  const uint32_t swz = ((uint32_t)lp0 >> a.swz_shift) & (uint32_t)a.swz_mask;  // the same in every lane tile
  const uint32_t base = (uint32_t)lp0 * (uint32_t)a.pitch;
  const uint32_t tstep = 16u * (uint32_t)a.pitch;

  // the activation fragments of the step in slot d
  auto read = [&](int d, u32x4_t (&f)[PT]) {
    uint32_t desc = (uint32_t)dr[d];
    // the descriptor is decoded here, at its use: decoded where it is loaded, every
    // pass of the loop would wait for all the ring's loads at once
    asm volatile("" : "+v"(desc));
    if (CW4) {
      const uint32_t u0 = desc & 0xFFu, u1 = (desc >> 16) & 0xFFu;
      const uint32_t a0 = base + (((u0 >> 1) ^ swz) << 4) + ((u0 & 1u) << 3);
      const uint32_t a1 = base + (((u1 >> 1) ^ swz) << 4) + ((u1 & 1u) << 3);
#pragma unroll
      for (int t = 0; t < PT; ++t) {
        const u32x2_t p0 = *(const u32x2_t*)(lds + a0 + t * tstep);
        const u32x2_t p1 = *(const u32x2_t*)(lds + a1 + t * tstep);
        f[t] = u32x4_t{p0.x, p0.y, p1.x, p1.y};
      }
    } else {
      const uint32_t ad = base + (((desc & 0xFFu) ^ swz) << 4);
#pragma unroll
      for (int t = 0; t < PT; ++t) f[t] = *(const u32x4_t*)(lds + ad + t * tstep);
    }
  };
  auto mfmas = [&](int d, const u32x4_t (&f)[PT]) {
#pragma unroll
    for (int t = 0; t < PT; ++t) acc[t] = mfma_bf16_16x16x32(wr[d], f[t], acc[t]);
  };

  // A step's fragments are read from LDS while the step before it is in the matrix cores.
  u32x4_t fa[PT], fb[PT];
  int cs0 = lo;
  if (nsteps > 0) read(0, fa);
  // whole passes over the ring while more than D steps remain: every slot is used and then
  // refilled in place, after the MFMAs that read it
  for (; cs0 + D < hi; cs0 += D) {
#pragma unroll
    for (int d = 0; d < D; d += 2) {
      read(d + 1, fb);
      mfmas(d, fa);
      __builtin_amdgcn_sched_barrier(0);
      fetch(d);
      __builtin_amdgcn_sched_barrier(0);
      read((d + 2) % D, fa);
      mfmas(d + 1, fb);
      __builtin_amdgcn_sched_barrier(0);
      fetch(d + 1);
      __builtin_amdgcn_sched_barrier(0);
    }
  }
  // the last steps (at most D): nothing is asked for any more
#pragma unroll
  for (int d = 0; d < D; d += 2) {
    if (cs0 + d + 1 < hi) read(d + 1, fb);
    if (cs0 + d < hi) mfmas(d, fa);
    if (d + 2 < D && cs0 + d + 2 < hi) read(d + 2, fa);
    if (cs0 + d + 1 < hi) mfmas(d + 1, fb);
  }

  // ---- results: bias, one rounding, then the optional residual add and ReLU
#pragma unroll
  for (int t = 0; t < PT; ++t) acc[t] += bv;
#ifdef BSP_ROWS_TUNE
  asm volatile("" ::"v"(acc[0]));
#endif
  PW_MARK(6);
  const int ptile0 = pix0 + pg * (PT * 16);
  // lane rows 0/1 (and 2/3) hold the two halves of one 8-channel block row: after an exchange
  // an even row has all eight channels of lane tile t, an odd row those of lane tile t + 1
  const int ch8 = __builtin_amdgcn_ds_bpermute(((lane & 32) + c) << 2, chan);  // the even row's channel
  const int odd = g & 1;
  auto paired = [&](int t) {
    const uint32_t x0 = pack_bf16x2(acc[t].x, acc[t].y), y0 = pack_bf16x2(acc[t].z, acc[t].w);
    const uint32_t x1 = pack_bf16x2(acc[t + 1].x, acc[t + 1].y), y1 = pack_bf16x2(acc[t + 1].z, acc[t + 1].w);
    const auto sx = __builtin_amdgcn_permlane16_swap(x0, x1, false, false);
    const auto sy = __builtin_amdgcn_permlane16_swap(y0, y1, false, false);
    return u32x4_t{sx[0], sy[0], sx[1], sy[1]};
  };
  if (a.win_out) {
    // The workgroup's strips cover a contiguous range of output channels: every wave puts its
    // pieces where they belong in an LDS image of the tile's output lines, then all threads
    // copy that image out, 16 contiguous bytes per lane.
    unsigned char* ot = lds + a.out_off;
    const int range0 = ns * a.NS * 16;
    const int lpix = pg * (PT * 16) + c;
    if (PT >= 2 && a.pair) {
#pragma unroll
      for (int t = 0; t + 1 < PT; t += 2) {
        const u32x4_t v = paired(t);
        if (ch8 >= 0) *(u32x4_t*)(ot + (lpix + (t + odd) * 16) * a.opitch + (ch8 - range0) * 2) = v;
      }
    } else {
#pragma unroll
      for (int t = 0; t < PT; ++t) {
        const u32x2_t v = {pack_bf16x2(acc[t].x, acc[t].y), pack_bf16x2(acc[t].z, acc[t].w)};
        if (chan >= 0) *(u32x2_t*)(ot + (lpix + t * 16) * a.opitch + (chan - range0) * 2) = v;
      }
    }
    // what this thread copies out afterwards, and the residual that goes with it: asked for
    // now, used after the barrier
    const int cpp = a.NS * 2;  // 16-byte pieces per pixel
    const int total = a.MT * cpp;
    constexpr int NIT = PT >= 2 ? PT / 2 : 1;  // pieces per thread: 16 * PT * NS * 2 over 64 * NS * PG threads
    uint32_t ooff[NIT], lsrc[NIT];
    bool ovalid[NIT];
    u32x4_t res[NIT];
#pragma unroll
    for (int it = 0; it < NIT; ++it) {
      const int i = tid + it * (int)blockDim.x;
      const int pixel = (int)fdiv((uint32_t)min(i, total - 1), a.d_cpp), k = min(i, total - 1) - pixel * cpp;
      const int ch = range0 + k * 8, gp = pix0 + pixel;
      ovalid[it] = i < total && gp < a.P && ch < a.O;
      ooff[it] = ((uint32_t)gp * (uint32_t)a.O + (uint32_t)ch) * 2u;
      lsrc[it] = (uint32_t)(pixel * a.opitch + k * 16);
      res[it] = u32x4_t{0, 0, 0, 0};
      if (ovalid[it] && a.residual) res[it] = *(const u32x4_t*)(a.residual + ooff[it]);
    }
    __syncthreads();
#pragma unroll
    for (int it = 0; it < NIT; ++it) {
      if (!ovalid[it]) continue;
      const u32x4_t v = *(const u32x4_t*)(ot + lsrc[it]);
      u32x2_t l2 = {v.x, v.y}, h2 = {v.z, v.w};
      if (a.residual || a.relu) {
        l2 = post_bf16x4_reg(l2, u32x2_t{res[it].x, res[it].y}, a.residual != nullptr, a.relu);
        h2 = post_bf16x4_reg(h2, u32x2_t{res[it].z, res[it].w}, a.residual != nullptr, a.relu);
      }
      // (whole output lines leave as streaming stores: no burst of dirty L2 lines is left for the
      // end of the kernel; pieces scattered over a line, below, are better merged in L2)
      __builtin_nontemporal_store(u32x4_t{l2.x, l2.y, h2.x, h2.y}, (u32x4_t*)(a.Y + ooff[it]));
    }
    // (a workgroup with several pixel groups has more pieces per thread than NIT covers)
    for (int i = tid + NIT * (int)blockDim.x; i < total; i += (int)blockDim.x) {
      const int pixel = (int)fdiv((uint32_t)i, a.d_cpp), k = i - pixel * cpp;
      const int ch = range0 + k * 8, gp = pix0 + pixel;
      if (gp >= a.P || ch >= a.O) continue;
      const u32x4_t v = *(const u32x4_t*)(ot + pixel * a.opitch + k * 16);
      const uint32_t off = ((uint32_t)gp * (uint32_t)a.O + (uint32_t)ch) * 2u;
      u32x2_t l2 = {v.x, v.y}, h2 = {v.z, v.w};
      if (a.residual || a.relu) {
        u32x4_t r = {0, 0, 0, 0};
        if (a.residual) r = *(const u32x4_t*)(a.residual + off);
        l2 = post_bf16x4_reg(l2, u32x2_t{r.x, r.y}, a.residual != nullptr, a.relu);
        h2 = post_bf16x4_reg(h2, u32x2_t{r.z, r.w}, a.residual != nullptr, a.relu);
      }
      __builtin_nontemporal_store(u32x4_t{l2.x, l2.y, h2.x, h2.y}, (u32x4_t*)(a.Y + off));
    }
  } else if (PT >= 2 && a.pair) {
#pragma unroll
    for (int t = 0; t + 1 < PT; t += 2) {
      u32x4_t v = paired(t);
      const int pixel = ptile0 + (t + odd) * 16 + c;
      if (pixel >= a.P || ch8 < 0) continue;
      const uint32_t off = ((uint32_t)pixel * (uint32_t)a.O + (uint32_t)ch8) * 2u;
      if (a.residual || a.relu) {
        const uint16_t* rp = a.residual ? (const uint16_t*)(a.residual + off) : nullptr;
        const u32x2_t l2 = post_bf16x4(u32x2_t{v.x, v.y}, rp, 4, true, a.relu);
        const u32x2_t h2 = post_bf16x4(u32x2_t{v.z, v.w}, rp ? rp + 4 : nullptr, 4, true, a.relu);
        v = u32x4_t{l2.x, l2.y, h2.x, h2.y};
      }
      *(u32x4_t*)(a.Y + off) = v;
    }
  } else {
#pragma unroll
    for (int t = 0; t < PT; ++t) {
      const int pixel = ptile0 + t * 16 + c;
      if (pixel >= a.P || chan < 0) continue;
      u32x2_t v = {pack_bf16x2(acc[t].x, acc[t].y), pack_bf16x2(acc[t].z, acc[t].w)};
      const uint32_t off = ((uint32_t)pixel * (uint32_t)a.O + (uint32_t)chan) * 2u;
      if (a.residual || a.relu)
        v = post_bf16x4(v, a.residual ? (const uint16_t*)(a.residual + off) : nullptr, 4, true, a.relu);
      *(u32x2_t*)(a.Y + off) = v;
    }
  }
#ifdef BSP_ROWS_TUNE
  __builtin_amdgcn_s_waitcnt(0);
#endif
  PW_MARK(7);
}

constexpr int kLdsLimit = 160 * 1024;

template <int PT, bool CW4, int D, int MAXT>
int launch_inst(const PwArgs& a, dim3 grid, int threads, size_t ldsb, hipStream_t st) {
  static bool raised = false;  // dynamic LDS above 64 KB has to be allowed once per kernel
  if (!raised) {
    if (hipFuncSetAttribute((const void*)conv_pw<PT, CW4, D, MAXT>, hipFuncAttributeMaxDynamicSharedMemorySize,
                            kLdsLimit) != hipSuccess)
      return BSP_ERR_HIP;
    raised = true;
  }
  hipLaunchKernelGGL((conv_pw<PT, CW4, D, MAXT>), grid, dim3(threads), ldsb, st, a);
  return hipGetLastError() == hipSuccess ? BSP_OK : BSP_ERR_HIP;
}

// Ring depth D: strips of at most 2 (4) steps take instances with as many registers for
// weights, which leaves room for more waves per SIMD; deep asks for 16 (workgroups of at most
// 512 threads, which may then use 256 registers per lane); otherwise 8.
template <bool CW4, int D, int MAXT>
int launch_d(const PwArgs& a, int PT, dim3 grid, int threads, size_t ldsb, hipStream_t st) {
  if (threads > MAXT) return BSP_ERR_UNSUPPORTED;
  switch (PT) {
    case 1: return launch_inst<1, CW4, D, MAXT>(a, grid, threads, ldsb, st);
    case 2: return launch_inst<2, CW4, D, MAXT>(a, grid, threads, ldsb, st);
    case 4: return launch_inst<4, CW4, D, MAXT>(a, grid, threads, ldsb, st);
    case 8: return launch_inst<8, CW4, D, (D >= 8 ? 512 : MAXT)>(a, grid, threads, ldsb, st);  // 8 lane tiles and a ring of 8 need more than 128 registers
  }
  return BSP_ERR_UNSUPPORTED;
}

template <bool CW4>
int launch_pt(const PwArgs& a, int PT, int depth, dim3 grid, int threads, size_t ldsb, hipStream_t st) {
  if (PT == 8 && depth >= 8 && threads > 512) return BSP_ERR_UNSUPPORTED;
  switch (depth) {
    case 2: return launch_d<CW4, 2, 1024>(a, PT, grid, threads, ldsb, st);
    case 4: return launch_d<CW4, 4, 1024>(a, PT, grid, threads, ldsb, st);
    case 8: return launch_d<CW4, 8, 1024>(a, PT, grid, threads, ldsb, st);
    case 16: return launch_d<CW4, 16, 512>(a, PT, grid, threads, ldsb, st);
  }
  return BSP_ERR_UNSUPPORTED;
}

struct PwChoice {
  int PT, PG, NS;
  int wout;      // results leave through an LDS image of whole output lines
  int deep = 0;  // ring depth override (0: from the plan's longest strip)
};

inline int cdiv(int64_t a, int64_t b) { return (int)((a + b - 1) / b); }

// Tile choice, from per-shape timings of ResNet50-, VGG16- and InceptionV3-shaped pointwise
// layers (several configurations each): one pixel group; four lane tiles per wave unless the
// tile's channels then exceed 128 KiB of LDS; few strips per workgroup while pixels are
// plentiful or the tile is thin (many small workgroups hide each other's latencies), many when they are not
// (every strip group re-reads the tile from L2, which is what bounds deep layers); whole-line
// output for layers that widen (their output is the bulk of the traffic).
PwChoice pw_choose(int P, int I, int O, int nstrips, int pitch, bool windowed) {
  PwChoice c{4, 1, 1, 0};
  while (c.PT > 1 && 16 * c.PT * pitch > 128 * 1024) c.PT /= 2;
  int ns = (P >= 50000 || (I <= 128 && P >= 20000)) ? 4 : (I >= 512 ? 16 : 8);
  ns = std::min(ns, nstrips);
  if (ns >= 4) ns &= ~3;
  c.NS = std::max(ns, 1);
  // enough workgroups for the chip: fewer strips each first, then smaller pixel tiles
  while ((int64_t)cdiv(P, 16 * c.PT) * cdiv(nstrips, c.NS) < 160) {
    if (c.NS >= 8)
      c.NS = (c.NS / 2) & ~3;
    else if (c.PT > 1)
      c.PT /= 2;
    else
      break;
  }
  // few pixel tiles and few strips (a narrow layer on a small image): measured, tiles of 32
  // pixels, two workgroups or so per CU, beat tiles of 64 by about half a microsecond
  if (c.PT == 4 && cdiv(P, 64) < 96 && nstrips <= 16) {
    c.PT = 2;
    c.NS = nstrips <= 8 ? nstrips : 4;
  }
  const int64_t xb = (int64_t)16 * c.PT * pitch, ob = (int64_t)16 * c.PT * (c.NS * 32 + 16);
  c.wout = windowed && (c.NS % 4 == 0 || c.NS >= nstrips) && O >= I && xb + ob <= kLdsLimit;
  return c;
}

}  // namespace

int bsp_launch_pw(const ConvParams& p, int dtype, const void* plan_host, hipStream_t st) {
  if (dtype != BSP_BF16 || !plan_host) return BSP_ERR_UNSUPPORTED;
  const int32_t* hdr = (const int32_t*)plan_host;
  if (hdr[BSP_PLAN_MAGIC_W] != BSP_PLAN_MAGIC || hdr[BSP_PLAN_VERSION_W] != BSP_PLAN_VERSION ||
      hdr[BSP_PLAN_O_W] != p.O || hdr[BSP_PLAN_I_W] != p.I || hdr[BSP_PLAN_H_W] != p.H ||
      hdr[BSP_PLAN_K_W] != p.K || hdr[BSP_PLAN_DTYPE_W] != dtype || hdr[BSP_PLAN_OFF_ROWS_W] == 0)
    return BSP_ERR_UNSUPPORTED;
  const int32_t* rs = hdr + hdr[BSP_PLAN_OFF_ROWS_W];
  if (p.H != 1 || p.K != 1 || p.ph != 0 || p.pw != 0 || p.sh != p.sw || p.sh < 1) return BSP_ERR_UNSUPPORTED;
  if (rs[BSP_ROWS_NSLABS_W] != 1 || p.P <= 64) return BSP_ERR_UNSUPPORTED;  // (FC layers: streaming kernels)
  if ((int64_t)p.B * p.L * p.J * p.I * 2 >= (1ll << 31) || (int64_t)p.P * p.O * 2 >= (1ll << 31))
    return BSP_ERR_UNSUPPORTED;
  const int nstrips = rs[BSP_ROWS_NSTRIPS_W];
  const int raw = p.I * 2;
  const int pitch = raw <= 128 ? 128 : (raw + 255) & ~255;
#ifdef BSP_ROWS_TUNE
  long long* a_trace = nullptr;
#endif
  const int maxsteps = rs[BSP_ROWS_MAXSTRIPSTEPS_W];
  const int depth0 = maxsteps <= 2 ? 2 : maxsteps <= 4 ? 4 : 8;
  PwChoice ch = pw_choose(p.P, p.I, p.O, nstrips, pitch, rs[BSP_ROWS_WINDOW_W] == 4);
#ifdef BSP_ROWS_TUNE  // experiments only: never defined in the product build
  if (const char* e = std::getenv("BSP_PWK_TUNE")) {
    int q[5] = {0, 0, 0, 0, 0};
    if (sscanf(e, "%d,%d,%d,%d,%d", q, q + 1, q + 2, q + 3, q + 4) >= 4) {
      ch = PwChoice{q[0], q[1], q[2], q[3]};
      ch.deep = q[4];
    }
  }
  if (const char* e = std::getenv("BSP_PW_TRACE_PTR")) a_trace = (long long*)std::strtoull(e, nullptr, 16);
  if (std::getenv("BSP_ROWS_VERBOSE"))
    fprintf(stderr, "pw: P=%d I=%d O=%d S=%d strips=%d steps=%d | PT=%d PG=%d NS=%d wout=%d\n", p.P, p.I, p.O,
            p.sh, nstrips, rs[BSP_ROWS_NCS_W], ch.PT, ch.PG, ch.NS, ch.wout);
#endif
  if (ch.PT < 1 || ch.PG < 1 || ch.NS < 1) return BSP_ERR_UNSUPPORTED;
  PwArgs a{};
  const int32_t* sec = p.plan + hdr[BSP_PLAN_OFF_ROWS_W];
#ifdef BSP_ROWS_TUNE
  a.trace = a_trace;
#endif
  a.X = (const unsigned char*)p.X;
  a.Y = (unsigned char*)p.Y;
  a.bias = p.bias;
  a.residual = (const unsigned char*)p.residual;
  a.relu = p.relu;
  a.rstrip = sec + rs[BSP_ROWS_OFF_STRIP_W];
  a.rslab = sec + rs[BSP_ROWS_OFF_SLAB_W];
  a.rdesc = (const unsigned char*)(sec + rs[BSP_ROWS_OFF_DESC_W]);
  a.rfrag = (const unsigned char*)(sec + rs[BSP_ROWS_OFF_FRAG_W]);
  a.nstrips = nstrips;
  a.P = p.P;
  a.I = p.I;
  a.O = p.O;
  a.S = p.sh;
  a.L = p.L;
  a.J = p.J;
  a.N = p.N;
  a.MN = p.M * p.N;
  a.pitch = pitch;
  if (pitch % 256 == 0) {
    a.swz_shift = 0;
    a.swz_mask = 15;
  } else {
    a.swz_shift = 1;
    a.swz_mask = 7;
  }
  a.MT = 16 * ch.PT * ch.PG;
  a.lpg = 0;
  while ((1 << a.lpg) < ch.PG) ++a.lpg;
  if ((1 << a.lpg) != ch.PG) return BSP_ERR_UNSUPPORTED;
  a.NS = ch.NS;
  const int64_t xbytes = (int64_t)a.MT * pitch;
  // whole-line output through LDS: the plan keeps windows of four strips together and the
  // workgroup takes whole windows (or every strip there is)
  a.win_out = ch.wout && rs[BSP_ROWS_WINDOW_W] == 4 && (ch.NS % 4 == 0 || ch.NS >= nstrips);
  a.out_off = (int32_t)xbytes;
  a.opitch = ch.NS * 32 + 16;
  const int64_t ldsb = xbytes + (a.win_out ? (int64_t)a.MT * a.opitch : 0);
  if (ldsb > kLdsLimit || ch.PG * ch.NS > 16 || ch.PG * ch.NS < 1) return BSP_ERR_UNSUPPORTED;
  a.nreq = (int32_t)(xbytes / 1024);
  a.d_cpp = make_fastdiv((uint32_t)(ch.NS * 2));
  a.mtiles = cdiv(p.P, a.MT);
  a.nsplit = cdiv(nstrips, ch.NS);
  const int64_t wgs = (int64_t)a.mtiles * a.nsplit;
  a.per_xcd = cdiv(wgs, 8);
  a.pair = hdr[BSP_PLAN_BO_W] != 4 && ch.PT >= 2;
  // multiply-high divisions are exact while dividend * divisor < 2^32
  const int64_t pmax = (int64_t)a.mtiles * a.MT;  // pixel numbers the staging loop divides
  if (pmax * std::max(a.MN, a.N) >= (1ll << 32) || (int64_t)a.per_xcd * 8 * a.nsplit >= (1ll << 32) ||
      xbytes * pitch >= (1ll << 32) || (int64_t)a.per_xcd * 8 >= (1ll << 31))
    return BSP_ERR_UNSUPPORTED;
  a.d_mn = make_fastdiv((uint32_t)a.MN);
  a.d_n = make_fastdiv((uint32_t)a.N);
  a.d_pitch = make_fastdiv((uint32_t)pitch);
  a.d_nsplit = make_fastdiv((uint32_t)a.nsplit);
  const int threads = 64 * ch.PG * ch.NS;
  a.adv_pix = (threads * 16) / pitch;
  a.adv_rem = (threads * 16) % pitch;
  dim3 grid((unsigned)(a.per_xcd * 8));
  const int depth = ch.deep ? ch.deep : depth0;
  return rs[BSP_ROWS_CW_W] == 4 ? launch_pt<true>(a, ch.PT, depth, grid, threads, (size_t)ldsb, st)
                                 : launch_pt<false>(a, ch.PT, depth, grid, threads, (size_t)ldsb, st);
}
