// 3x3 layers (stride 1, padding 1 or 0, bf16) whose input channels fit one slab of the row-band plan
// section (at most 128): one workgroup per band of BR output rows x chunk of CW columns (as
// many sixteen-column tiles as make a workgroup of four waves with the layer's strips, or the
// whole row where that is narrower), all output channels.
//
// The band's input rows (one halo row above and below, one halo column left and right of the
// chunk) are runs of whole pixels of image rows, so they are copied global -> LDS with no
// gather at all: an LDS image of (BR + 2) rows of Jp = CW + 2 pixels with the bank permutation
// slot = piece ^ f(patch column), the same in every row; the halo columns that lie outside the
// image and the rows outside the image are cleared (they are never copied into: no ordering
// between clearing and copying is needed).  Wave (strip s, column tile t)
// owns 16 output columns x BR rows of strip s: per column step it reads the BR + 2 patch rows
// of the step's (unit, dx) item once and issues 3 * BR MFMAs (output row r, window row dy
// uses patch row r + dy), weights streamed from the plan through a register ring as in the
// row-band kernel.  The results of all strips are gathered in LDS as whole output lines (the
// band's output is one contiguous range of Y) and leave 16 bytes per lane with the optional
// residual and ReLU.  With 56-pixel rows and 64 channels the launcher makes chunks of sixteen
// columns: four waves per workgroup and, at batch 32, four workgroups per CU.
#include "bsp_launch.h"
#include "bsp_tile.h"

#include <algorithm>
#include <cstdlib>

namespace {

struct BandArgs {
  const unsigned char* X;
  unsigned char* Y;
  const float* bias;
  const unsigned char* residual;
  const int32_t* rstrip;
  const int32_t* rslab;
  const unsigned char* rdesc;
  const unsigned char* rfrag;
  int32_t relu, nstrips;
  int32_t B, L, J, I, O;
  int32_t M, N, pad;  // output rows and columns; padding 1 (M = L, N = J) or 0 (M = L - 2, N = J - 2)
  int32_t nbands, ctiles;
  int32_t cw, nchunks;  // columns per chunk (a multiple of 16 when there are several chunks), chunks per row
  int32_t Jp, pitch, swz_shift, swz_mask;
  int32_t ppr;      // pixels per KiB request
  int32_t rpr;      // requests per image row
  int32_t opitch;   // bytes per pixel of the output image
  int32_t llpp;     // log2 of the 16-byte slots per staged pixel
  FastDiv d_rpr, d_ctiles, d_cpp, d_nbands, d_nchunks, d_rowp;
#ifdef BSP_ROWS_TUNE
  long long* trace;
#endif
};

#ifdef BSP_ROWS_TUNE
#define BAND_MARK(k)                                                                                 \
  do {                                                                                               \
    if (a.trace && lane == 0) a.trace[((size_t)blockIdx.x * 16 + wave) * 8 + (k)] = wall_clock64(); \
  } while (0)
#else
#define BAND_MARK(k)
#endif

typedef __attribute__((address_space(1))) const void* gptr_t;
typedef __attribute__((address_space(3))) void* lptr_t;

template <int BR, int D>
__global__ __launch_bounds__(1024) void conv_band3(BandArgs a) {
  extern __shared__ __align__(16) unsigned char lds[];
  kernarg_touch<BandArgs>();
  const int tid = threadIdx.x, lane = tid & 63, g = lane >> 4, c = lane & 15;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int nwaves = (int)(blockDim.x >> 6);
  // consecutive workgroups go to different XCDs: all bands of an image are given to one XCD, so
  // that the halo rows two neighbouring bands share are fetched from HBM once
  const int xcd = blockIdx.x & 7, slot_wg = blockIdx.x >> 3;
  const int grp8 = (int)fdiv((uint32_t)slot_wg, a.d_nbands), bc = slot_wg - grp8 * a.nbands;  // nbands counts (band, chunk) pairs
  const int n = xcd + 8 * grp8;
  if (n >= a.B) return;
  const int band = (int)fdiv((uint32_t)bc, a.d_nchunks), chunk = bc - band * a.nchunks;
  const int y0 = band * BR, x0 = chunk * a.cw;
  const int Jc = min(a.cw, a.N - x0);  // this chunk's output columns: patch column pc holds image column x0 - pad + pc
  const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)lds;
  const int rowbytes = a.Jp * a.pitch;

  BAND_MARK(0);
  // this wave's strip and column tile; its step range and channels are asked for here (scalar
  // loads) and waited for after the copies have been issued
  const int strip = (int)fdiv((uint32_t)wave, a.d_ctiles), ct = wave - strip * a.ctiles;
  const bool active = strip < a.nstrips;
  const int sq = active ? strip : 0;
  u32x2_t lohi;
  u32x4_t ch4;
  {
    const int32_t* ps = a.rslab + sq * 2;
    const int32_t* pc = a.rstrip + sq * 4;
    asm volatile("s_load_dwordx2 %0, %2, 0x0\n\ts_load_dwordx4 %1, %3, 0x0" : "=&s"(lohi), "=&s"(ch4) : "s"(ps), "s"(pc) : "memory");
  }
  // ---- copies: a request is 1 KiB = a group of ppr pixels of one patch row.  A wave keeps to
  // one group of columns (everything that depends on the column is computed once) and walks
  // down the rows, which costs a few scalar instructions per request; where there are more
  // waves than groups the waves of a group share its rows.
  {
    const int lpp = a.pitch >> 4;                 // 16-byte slots per pixel (a power of two)
    const int sp = lane >> a.llpp, slot = lane & (lpp - 1);
    const int pc0 = (a.pad && x0 == 0) ? 1 : 0;  // (with padding the first chunk's left halo column lies outside the image)
    const int nwg = min(nwaves, a.rpr);           // waves side by side over the groups
    int nwr = 1;                                  // waves of a group over its rows
    while ((nwr + 1) * nwg <= nwaves) ++nwr;
    int wg = wave, wr = 0;
    while (wg >= nwg) {
      wg -= nwg;
      ++wr;
    }
    if (wr < nwr) {
      for (int grp = wg; grp < a.rpr; grp += nwg) {
        const int pc = pc0 + grp * a.ppr + sp, col = x0 - a.pad + pc;
        const uint32_t piece = (uint32_t)slot ^ (((uint32_t)pc >> a.swz_shift) & (uint32_t)a.swz_mask);
        const bool lane_ok = pc < Jc + 2 && (unsigned)col < (unsigned)a.J && piece * 8u < (uint32_t)a.I;
        const uint32_t goff = ((uint32_t)col * (uint32_t)a.I + piece * 8u) * 2u;
        const uint32_t ldst = lds0 + (uint32_t)(pc0 + grp * a.ppr) * (uint32_t)a.pitch;
        const uint32_t grow = (uint32_t)a.J * (uint32_t)a.I * 2u;  // bytes of an image row
        if (!lane_ok) continue;  // (the lanes are masked once per group; a row outside the image is a scalar branch)
        // (the byte offset stays a 32-bit number that wraps: the row above the first image is at
        // "minus one row", and only the sum with the later steps is a real offset)
        uint32_t src = (uint32_t)(n * a.L + y0 - a.pad + wr) * grow + goff;
        const uint32_t sstep = (uint32_t)nwr * grow, dstep = (uint32_t)(nwr * rowbytes);
        uint32_t dst = ldst + (uint32_t)(wr * rowbytes);
        for (int row = y0 - a.pad + wr; row < y0 - a.pad + BR + 2; row += nwr, src += sstep, dst += dstep)
          if ((unsigned)row < (unsigned)a.L)
            __builtin_amdgcn_global_load_lds((gptr_t)(a.X + src), (lptr_t)(uintptr_t)dst, 16, 0, 0);
      }
    }
  }
  BAND_MARK(1);
  // ---- what is never copied into must read as zero: the halo columns where they lie outside
  // the image (patch column 0 of the first chunk, Jc + 1 of the last), whole rows outside it
  {
    const int lpp = a.pitch >> 4;  // slots per pixel (a power of two)
    const bool left = a.pad && x0 == 0, right = a.pad && x0 + Jc == a.N;
    for (int i = tid; i < (BR + 2) * 2 * lpp; i += (int)blockDim.x) {
      const int bp = i >> a.llpp, fr = bp >> 1, side = bp & 1;
      if (side == 0 ? !left : !right) continue;
      const int pc = side == 0 ? 0 : Jc + 1;
      ((u32x4_t*)lds)[((fr * a.Jp + pc) << a.llpp) + (i & (lpp - 1))] = u32x4_t{0, 0, 0, 0};
    }
#pragma unroll
    for (int fr = 0; fr < BR + 2; ++fr) {
      if ((unsigned)(y0 - a.pad + fr) < (unsigned)a.L) continue;
      for (int i = tid; i < (Jc + 2) * lpp; i += (int)blockDim.x)
        ((u32x4_t*)lds)[((fr * a.Jp) << a.llpp) + i] = u32x4_t{0, 0, 0, 0};
    }
  }

  BAND_MARK(2);
  // ---- the step range and channels asked for at the top have to be there now (the registers
  // pass through the wait, so that no use of them is moved above it)
  asm volatile("s_waitcnt lgkmcnt(0)" : "+s"(lohi), "+s"(ch4) : : "memory");
  const int lo = (int)lohi.x, hi = active ? (int)lohi.y : lo;
  const int chan = !active ? -1 : g == 0 ? (int)ch4.x : g == 1 ? (int)ch4.y : g == 2 ? (int)ch4.z : (int)ch4.w;

  const uint32_t frag_lane = (uint32_t)lane * 16u, desc_lane = (uint32_t)g * 4u;
  u32x4_t wr[D][3];
  int dr[D];
  int fnext = lo;
  auto fetch = [&](int d) {
    const int cs = min(fnext, hi - 1);  // past the end: the last step again, never used
    ++fnext;
    dr[d] = *(const int*)(a.rdesc + ((uint32_t)cs * 16u + desc_lane));
#pragma unroll
    for (int dy = 0; dy < 3; ++dy)
      wr[d][dy] = *(const u32x4_t*)(a.rfrag + (((uint32_t)cs * 3u + dy) * 1024u + frag_lane));
  };
  if (hi > lo) {
#pragma unroll
    for (int d = 0; d < D; ++d) fetch(d);
  }
  f32x4_t bv = {0.f, 0.f, 0.f, 0.f};
  if (a.bias && chan >= 0) bv = f32x4_t{a.bias[chan], a.bias[chan + 1], a.bias[chan + 2], a.bias[chan + 3]};

  f32x4_t acc[BR];
#pragma unroll
  for (int r = 0; r < BR; ++r) acc[r] = f32x4_t{0.f, 0.f, 0.f, 0.f};

  BAND_MARK(3);
  __builtin_amdgcn_s_waitcnt(0);
  __syncthreads();  // the patch is in LDS
  BAND_MARK(4);

  const int x = min(ct * 16 + c, Jc - 1);  // (column of the chunk) lanes past its end repeat its last column (never stored)
  auto step = [&](int d) {
    uint32_t desc = (uint32_t)dr[d];
    asm volatile("" : "+v"(desc));  // decoded at its use, so that the wait is for this slot only
    const uint32_t unit = desc & 0xFFu, tp = (uint32_t)x + ((desc >> 8) & 0xFFu);  // image column x + dx
    const uint32_t ad = tp * (uint32_t)a.pitch + ((unit ^ ((tp >> a.swz_shift) & (uint32_t)a.swz_mask)) << 4);
    u32x4_t f[BR + 2];
#pragma unroll
    for (int fr = 0; fr < BR + 2; ++fr) f[fr] = *(const u32x4_t*)(lds + ad + fr * rowbytes);
#pragma unroll
    for (int dy = 0; dy < 3; ++dy)
#pragma unroll
      for (int r = 0; r < BR; ++r) acc[r] = mfma_bf16_16x16x32(wr[d][dy], f[r + dy], acc[r]);
  };
  if (active) {
    int cs0 = lo;
    for (; cs0 + D < hi; cs0 += D) {
#pragma unroll
      for (int d = 0; d < D; ++d) {
        step(d);
        __builtin_amdgcn_sched_barrier(0);
        fetch(d);  // refilled in place, after the MFMAs that read it
        __builtin_amdgcn_sched_barrier(0);
      }
    }
#pragma unroll
    for (int d = 0; d < D; ++d)
      if (cs0 + d < hi) step(d);
  }
  BAND_MARK(5);
  __syncthreads();  // everybody is done with the patch: its LDS becomes the output image

  // ---- results as whole output lines in LDS, then out
  if (chan >= 0 && ct * 16 + c < Jc) {
#pragma unroll
    for (int r = 0; r < BR; ++r) {
      const f32x4_t v = acc[r] + bv;
      *(u32x2_t*)(lds + (r * a.cw + ct * 16 + c) * a.opitch + chan * 2) =
          u32x2_t{pack_bf16x2(v.x, v.y), pack_bf16x2(v.z, v.w)};
    }
  }
  const int rows_out = min(BR, a.M - y0);
  const int cpp = a.O >> 3;  // 16-byte pieces per pixel
  const int rowp = a.cw * cpp;  // pieces per row of the output image
  const int total = rows_out * rowp;
  // piece i of the image: row r, column xl of the chunk, piece k of the pixel; a row of the chunk
  // is one contiguous run of Y
  const uint32_t y_off0 = (uint32_t)((n * a.M + y0) * a.N + x0) * (uint32_t)a.O * 2u;
  const uint32_t y_row = (uint32_t)a.N * (uint32_t)a.O * 2u;
  auto locate = [&](int i, uint32_t& src, uint32_t& dst) {
    const int pixel = (int)fdiv((uint32_t)i, a.d_cpp), k = i - pixel * cpp;
    src = (uint32_t)(pixel * a.opitch + k * 16);
    if (a.nchunks == 1) {  // whole rows: the band's output is one contiguous range
      dst = y_off0 + (uint32_t)i * 16u;
      return i < total;
    }
    const int r = (int)fdiv((uint32_t)i, a.d_rowp), rem = i - r * rowp;
    dst = y_off0 + (uint32_t)r * y_row + (uint32_t)rem * 16u;
    return i < total && pixel - r * a.cw < Jc;
  };
  constexpr int NIT = 4;
  uint32_t lsrc[NIT], ydst[NIT];
  bool ok[NIT];
  u32x4_t res[NIT];
#pragma unroll
  for (int it = 0; it < NIT; ++it) {
    ok[it] = locate(min(tid + it * (int)blockDim.x, max(total - 1, 0)), lsrc[it], ydst[it]) &&
             tid + it * (int)blockDim.x < total;
    res[it] = u32x4_t{0, 0, 0, 0};
    if (ok[it] && a.residual) res[it] = *(const u32x4_t*)(a.residual + ydst[it]);
  }
  __syncthreads();
  BAND_MARK(6);
  auto out_piece = [&](uint32_t src, uint32_t dst, u32x4_t r) {
    const u32x4_t v = *(const u32x4_t*)(lds + src);
    u32x2_t l2 = {v.x, v.y}, h2 = {v.z, v.w};
    if (a.residual || a.relu) {
      l2 = post_bf16x4_reg(l2, u32x2_t{r.x, r.y}, a.residual != nullptr, a.relu);
      h2 = post_bf16x4_reg(h2, u32x2_t{r.z, r.w}, a.residual != nullptr, a.relu);
    }
    // (streaming store: no burst of dirty L2 lines is left for the end of the kernel)
    __builtin_nontemporal_store(u32x4_t{l2.x, l2.y, h2.x, h2.y}, (u32x4_t*)(a.Y + dst));
  };
#pragma unroll
  for (int it = 0; it < NIT; ++it)
    if (ok[it]) out_piece(lsrc[it], ydst[it], res[it]);
  for (int i = tid + NIT * (int)blockDim.x; i < total; i += (int)blockDim.x) {
    uint32_t src, dst;
    if (!locate(i, src, dst)) continue;
    u32x4_t r = {0, 0, 0, 0};
    if (a.residual) r = *(const u32x4_t*)(a.residual + dst);
    out_piece(src, dst, r);
  }
#ifdef BSP_ROWS_TUNE
  __builtin_amdgcn_s_waitcnt(0);
#endif
  BAND_MARK(7);
}

constexpr int kLdsLimit = 160 * 1024;

template <int BR>
int launch_band(const BandArgs& a, dim3 grid, int threads, size_t ldsb, hipStream_t st) {
  static bool raised = false;  // dynamic LDS above 64 KB has to be allowed once per kernel
  if (!raised) {
    if (hipFuncSetAttribute((const void*)conv_band3<BR, 2>, hipFuncAttributeMaxDynamicSharedMemorySize, kLdsLimit) !=
        hipSuccess)
      return BSP_ERR_HIP;
    raised = true;
  }
  hipLaunchKernelGGL((conv_band3<BR, 2>), grid, dim3(threads), ldsb, st, a);
  return hipGetLastError() == hipSuccess ? BSP_OK : BSP_ERR_HIP;
}

}  // namespace

int bsp_launch_band(const ConvParams& p, int dtype, const void* plan_host, hipStream_t st) {
  if (dtype != BSP_BF16 || !plan_host) return BSP_ERR_UNSUPPORTED;
  const int32_t* hdr = (const int32_t*)plan_host;
  if (hdr[BSP_PLAN_MAGIC_W] != BSP_PLAN_MAGIC || hdr[BSP_PLAN_VERSION_W] != BSP_PLAN_VERSION ||
      hdr[BSP_PLAN_O_W] != p.O || hdr[BSP_PLAN_I_W] != p.I || hdr[BSP_PLAN_H_W] != p.H ||
      hdr[BSP_PLAN_K_W] != p.K || hdr[BSP_PLAN_DTYPE_W] != dtype || hdr[BSP_PLAN_OFF_ROWS_W] == 0)
    return BSP_ERR_UNSUPPORTED;
  const int32_t* rs = hdr + hdr[BSP_PLAN_OFF_ROWS_W];
  if (p.H != 3 || p.K != 3 || p.sh != 1 || p.sw != 1 || p.ph != p.pw || p.ph < 0 || p.ph > 1) return BSP_ERR_UNSUPPORTED;
  if (rs[BSP_ROWS_NSLABS_W] != 1 || rs[BSP_ROWS_CW_W] != 8 || p.I > 128) return BSP_ERR_UNSUPPORTED;
  if ((int64_t)p.B * p.L * p.J * p.I * 2 >= (1ll << 31) || (int64_t)p.P * p.O * 2 >= (1ll << 31))
    return BSP_ERR_UNSUPPORTED;
  const int nstrips = rs[BSP_ROWS_NSTRIPS_W];
  BandArgs a{};
#ifdef BSP_ROWS_TUNE
  if (const char* e = std::getenv("BSP_PW_TRACE_PTR")) a.trace = (long long*)std::strtoull(e, nullptr, 16);
#endif
  const int raw = p.I * 2;
  a.pitch = raw <= 128 ? 128 : 256;
  if (a.pitch % 256 == 0) {
    a.swz_shift = 0;
    a.swz_mask = 15;
  } else {
    a.swz_shift = 1;
    a.swz_mask = 7;
  }
  a.ppr = 1024 / a.pitch;
  a.opitch = p.O * 2 + 16;
  // Column tiles per workgroup: one wave per (strip, column tile), sixteen waves at most.  One
  // column tile (chunks of sixteen columns) wherever that still makes a workgroup of four waves:
  // measured on every 3x3 shape of the three networks, many small workgroups (several per CU,
  // each in another phase) beat one large one per CU by 5 to 35 %, although the chunks' halo
  // columns are copied twice.
  const int ct_all = (p.N + 15) / 16;
  if (nstrips < 1 || nstrips > 16) return BSP_ERR_UNSUPPORTED;
  int ct = std::min(ct_all, std::max(1, 4 / nstrips));
#ifdef BSP_ROWS_TUNE
  if (const char* e = std::getenv("BSP_BAND_CT")) ct = std::max(1, std::min(ct, std::atoi(e)));
#endif
  int BR = 7;
  int64_t ldsb = 0;
  for (; ct >= 1; --ct) {
    a.cw = ct == ct_all ? p.N : 16 * ct;
    a.nchunks = (p.N + a.cw - 1) / a.cw;
    // rows per band: seven unless that leaves CUs without a workgroup, or unless a workgroup
    // has nine to twelve waves: three per SIMD, of which the seven-row instance (94 registers,
    // five waves per SIMD) lets a CU hold one workgroup and the four-row instance (70 registers,
    // seven waves) two (InceptionV3's 80 -> 192 layer at 73x73: 33 -> 29 us)
    BR = (int64_t)p.B * ((p.M + 6) / 7) * a.nchunks >= 200 ? 7 : 4;
    if ((nstrips * ct + 3) / 4 == 3) BR = 4;
#ifdef BSP_ROWS_TUNE
    if (const char* e = std::getenv("BSP_BAND_BR")) BR = std::atoi(e) == 4 ? 4 : 7;
#endif
    a.Jp = a.cw + 2;
    const int64_t patch = (int64_t)(BR + 2) * a.Jp * a.pitch;
    const int64_t outimg = (int64_t)BR * a.cw * a.opitch;
    ldsb = std::max(patch, outimg);
    if (ldsb <= kLdsLimit) break;
  }
  if (ct < 1) return BSP_ERR_UNSUPPORTED;
  // (rows in several chunks with fewer than four strips or thin pixels: measured slower than the
  // LDS-resident kernel, which takes them)
  if (a.nchunks > 1 && (nstrips < 4 || p.I < 64)) return BSP_ERR_UNSUPPORTED;
  a.ctiles = ct;
  // requests per patch row: a chunk's columns and its halo columns inside the image
  a.rpr = ((a.nchunks == 1 && p.ph == 1 ? p.J : a.cw + 2) + a.ppr - 1) / a.ppr;
  a.nbands = ((p.M + BR - 1) / BR) * a.nchunks;  // (band, chunk) pairs of an image
  const int32_t* sec = p.plan + hdr[BSP_PLAN_OFF_ROWS_W];
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
  a.B = p.B;
  a.L = p.L;
  a.J = p.J;
  a.M = p.M;
  a.N = p.N;
  a.pad = p.ph;
  a.I = p.I;
  a.O = p.O;
  a.d_rpr = make_fastdiv((uint32_t)a.rpr);
  a.d_ctiles = make_fastdiv((uint32_t)a.ctiles);
  a.d_cpp = make_fastdiv((uint32_t)(p.O >> 3));
  a.d_nbands = make_fastdiv((uint32_t)a.nbands);
  a.d_nchunks = make_fastdiv((uint32_t)a.nchunks);
  a.d_rowp = make_fastdiv((uint32_t)(a.cw * (p.O >> 3)));
  a.llpp = a.pitch == 128 ? 3 : 4;
  // multiply-high divisions are exact while dividend * divisor < 2^32
  const int64_t nwg = (int64_t)((p.B + 7) / 8) * a.nbands * 8;  // eight images at a time, one per XCD
  if (nwg * a.nbands >= (1ll << 32) || nwg >= (1ll << 31) || (int64_t)(BR + 2) * a.rpr * a.rpr >= (1ll << 32) ||
      (int64_t)(BR * a.cw * (p.O >> 3) + 8192) * a.cw * (p.O >> 3) >= (1ll << 32))
    return BSP_ERR_UNSUPPORTED;
  const int threads = 64 * nstrips * a.ctiles;
  dim3 grid((unsigned)nwg);
  return BR == 7 ? launch_band<7>(a, grid, threads, (size_t)ldsb, st) : launch_band<4>(a, grid, threads, (size_t)ldsb, st);
}
