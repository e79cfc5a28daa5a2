// Row-band kernel: block-sparse implicit-GEMM convolution for bf16 layers (fp32 accumulation)
// in which one activation fragment, once in registers, serves every window row.
//
// Work split.  A workgroup owns a pixel tile (NI images x NB bands of BR output rows x TW
// output columns) and a group of strips of 16 output channels.  The tile's pixels are seen as
// columns: a column is BR vertically consecutive output pixels, sixteen columns make a
// lane tile (the N side of a 16x16 MFMA tile).
//
// Staging.  Per slab of input channels the tile's input patch (halo included) is copied
// from global memory straight into LDS (global_load_lds: 64 lanes x 16 bytes per request land
// as one contiguous KiB); staged pixels outside the image are cleared once and never
// requested.  A staged pixel occupies a power-of-two number of 16-byte slots, its pieces
// permuted by the pixel's position (slot = piece ^ f(pixel)) so that the sixteen pixels a
// lane group reads fall into sixteen different bank groups.
//
// conv_rows: a wave owns one strip, NT lane tiles and, when the
// contraction is split (KS > 1), every KS-th column step.  Per step it reads, for each lane
// tile, the NF = (BR-1)*S + H patch rows of the step's items once, takes the step's H weight
// fragments (one per window row, streamed from the plan through a ring of registers), and
// issues H*BR MFMAs per lane tile: output row r, window row dy uses patch row r*S + dy.  So
// an activation fragment read from LDS feeds up to H MFMAs and a weight fragment BR*NT.  The
// last wave of the workgroup only moves data: it requests the next slab while the others
// compute.
//
// Pointwise (1x1) layers are not served here (bsp_pw.hip).
//
// Only kept blocks have items (paper Section I, advantages 3-4); a strip groups block rows
// with similar kept columns (bsp_plan.h).
#include "bsp_launch.h"
#include "bsp_tile.h"

#include <algorithm>
#include <cstdio>
#include <cstdlib>

namespace {

struct RowsArgs {
  const unsigned char* X;
  unsigned char* Y;
  const float* bias;
  const unsigned char* residual;
  const int32_t* rstrip;
  const int32_t* rslab;
  const int32_t* rdesc;
  const u32x4_t* rfrag;
  int32_t relu;
  int32_t nstrips, nslabs, ncs;
  int32_t sc;                      // 16-byte pieces of a pixel per plan slab (slab / 8)
  int32_t G, nstaged, scs;         // plan slabs staged together, staged slabs, pieces with data (G * sc)
  int32_t NM;                      // data-mover waves (the last NM of the workgroup)
  int32_t lscp;                    // log2 of the pieces a staged pixel occupies (power of two >= sc)
  int32_t swz_shift, swz_mask;     // piece p of pixel q sits in slot p ^ ((q >> shift) & mask)
  int32_t B, L, J, I, O, M, N;
  int32_t ph, pw, stride;          // stride = S * gs
  int32_t gs;                      // input pixels per staged pixel (1)
  int32_t TW, NB, NI, PR, PC, PCp; // PC staged columns that are read, PCp the row pitch (multiple of 16)
  int32_t tiles_x, tiles_y, ntiles;
  int32_t ncols;                   // NI * NB * TW
  int32_t SG, PTW, KS, nsg;        // strips, lane-tile groups and contraction shares per workgroup; strip groups
  int32_t per_xcd;                 // workgroups per XCD slot range
  int32_t bufbytes;                // one patch buffer
  int32_t orow;                    // bytes per pixel in the results staging tile
  int32_t red_bytes;               // LDS bytes of the split-contraction partials
  int32_t tbl_off;                 // LDS offset of the tables
  int32_t piece8;                  // results leave as 8-byte pieces (4x16 blocks)
  int32_t direct;                  // results leave straight from the accumulators, 8 bytes per lane
  int32_t ylimit;                  // output pixels that exist
  int32_t lsg, lptw;               // log2 of SG and PTW
  FastDiv d_pcp, d_pr, d_np, d_br, d_nsg, d_tpi, d_tx, d_perimg, d_tw;
#ifdef BSP_ROWS_TUNE
  long long* trace;
  int nodma;  // experiments: 1 = the data movers request nothing (timing only, results wrong)
#endif
};

#ifdef BSP_ROWS_TUNE
#define ROWS_MARK(k)                                                                                       \
  do {                                                                                                     \
    if (a.trace && (threadIdx.x & 63) == 0) a.trace[((size_t)blockIdx.x * 16 + (threadIdx.x >> 6)) * 8 + (k)] = wall_clock64(); \
  } while (0)
#else
#define ROWS_MARK(k)
#endif

struct TilePos {
  int img0, y0, x0, sgi;
};

template <int H, int S, int BR>
constexpr bool row_needed(int fr) {
  for (int r = 0; r < BR; ++r)
    for (int dy = 0; dy < H; ++dy)
      if (r * S + dy == fr) return true;
  return false;
}

// workgroup -> (tile, strip group): consecutive workgroups of one XCD share a tile
__device__ __forceinline__ bool rows_tile(const RowsArgs& a, int BR, TilePos* t) {
  const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
  if (slot >= a.per_xcd) return false;
  const int q = xcd * a.per_xcd + slot;
  const int tile = (int)fdiv((uint32_t)q, a.d_nsg);
  if (tile >= a.ntiles) return false;
  t->sgi = q - tile * a.nsg;
  const int tpi = a.tiles_x * a.tiles_y;
  const int ig = (int)fdiv((uint32_t)tile, a.d_tpi), trem = tile - ig * tpi;
  const int ty = (int)fdiv((uint32_t)trem, a.d_tx), tx = trem - ty * a.tiles_x;
  t->img0 = ig * a.NI;
  t->y0 = ty * a.NB * BR;
  t->x0 = tx * a.TW;
  return true;
}

// Per column of the tile: first output pixel (or -1), rows that exist, first staged pixel.
__device__ __forceinline__ void rows_tables(const RowsArgs& a, const TilePos& t, int BR, int S, int nslots,
                                            int32_t* colbase, int32_t* colrows, int32_t* colpix) {
  const int tid = threadIdx.x;
  if (tid < nslots) {
    int cb = -1, rows = 0, lp = 0;
    if (tid < a.ncols) {
      const int per_img = a.NB * a.TW;
      const int img = (int)fdiv((uint32_t)tid, a.d_perimg), rem = tid - img * per_img;
      const int band = (int)fdiv((uint32_t)rem, a.d_tw), x = rem - band * a.TW;
      lp = (img * a.PR + band * BR * S) * a.PCp + x * S;
      const int gi = t.img0 + img, gy = t.y0 + band * BR, gx = t.x0 + x;
      if (gi < a.B && gx < a.N && gy < a.M) {
        cb = (gi * a.M + gy) * a.N + gx;
        rows = min(BR, a.M - gy);
      }
    }
    colbase[tid] = cb;
    colrows[tid] = rows;
    colpix[tid] = lp;
  }
}

// Sixteen zero bytes: what the copies read for the staged pixels that lie outside the image.
__device__ __align__(16) const unsigned char rows_zero16[16] = {0};

// Request staged slab sl (G plan slabs) of the tile's patch with the nw waves numbered w = 0 .. nw - 1:
// side by side over the staged rows and, where there are fewer rows than waves, over the
// requests of a row as well.  Nothing waits here; the copies complete in the background (vmcnt of
// the requesting wave).  A staged pixel outside the image (padding) is copied from the zero
// bytes above, so the patch needs no clearing: clearing by LDS stores cost the small layers,
// whose patches are mostly padding, more than the copies themselves.
__device__ __forceinline__ void rows_stage(const RowsArgs& a, const TilePos& t, unsigned char* lds, int sl,
                                           int w, int nw) {
  const int lane = threadIdx.x & 63;
  const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)lds;
  const uint32_t buf = lds0 + (sl & 1) * a.bufbytes;
  const int lppi = 6 - a.lscp;          // log2 of the pixels one request covers
  const int sub_pix = lane >> a.lscp;   // this lane's pixel within the request
  const int sidx = lane & ((1 << a.lscp) - 1);  // and its slot within the pixel
  const int iy0 = t.y0 * a.stride - a.ph, ix0 = t.x0 * a.stride - a.pw;
  const int groups = a.PCp >> lppi;     // requests per staged row
  const int nrows = a.NI * a.PR;
  // wave w = (wr over the rows, wg over a row's requests)
  const int nwr = min(nw, nrows);
  int wr = w, wg = 0, nwg = 1;
  while (wr >= nwr) {
    wr -= nwr;
    ++wg;
  }
  while ((nwg + 1) * nwr <= nw) ++nwg;
  if (wg >= nwg) return;
  // lane j: the j-th staged row of this wave, where it starts in X; kRowPad: a row above or
  // below the image; kRowNone: an image past the end of the batch (nothing is stored from it)
  constexpr uint32_t kRowNone = 0xFFFFFFFFu, kRowPad = 0xFFFFFFFEu;
  uint32_t rowsrc = kRowNone;
  const int myrow = wr + lane * nwr;
  if (myrow < nrows) {
    const int img = (int)fdiv((uint32_t)myrow, a.d_pr), pr = myrow - img * a.PR;
    const int gi = t.img0 + img, gy = iy0 + pr * a.gs;
    if (gi < a.B) rowsrc = (unsigned)gy < (unsigned)a.L ? (uint32_t)((gi * a.L + gy) * a.J) * (uint32_t)a.I * 2u : kRowPad;
  }
  const unsigned char* zero = rows_zero16;
  const bool fill = sl == 0;  // the padding of both buffers is written with the first slab (all waves share that); later slabs leave it alone
  for (int gq = wg; gq < groups; gq += nwg) {
    const int pc = (gq << lppi) + sub_pix;               // staged column of this lane
    const int cq = sidx ^ ((pc >> a.swz_shift) & a.swz_mask);
    const int gx = ix0 + pc * a.gs;
    const int ch = (sl * a.scs + cq) * 8;
    const bool wanted = cq < a.scs && ch < a.I && pc < a.PC;  // a slot some column step reads
    const bool col_real = wanted && (unsigned)gx < (unsigned)a.J;
    const uint32_t col_off = ((uint32_t)gx * (uint32_t)a.I + (uint32_t)ch) * 2u;
    const bool some_pad = __ballot(wanted && !col_real) != 0;
    uint32_t dst = buf + ((uint32_t)(wr * a.PCp + (gq << lppi)) << (a.lscp + 4));
    const uint32_t dst_step = (uint32_t)(nwr * a.PCp) << (a.lscp + 4);
    if (!fill) {
      // Later slabs (the data movers' work, and what bounds the layers with several slabs): the
      // real pixels only, four rows per pass with no branch taken inside a pass.  A lane past
      // the wave's last row holds kRowNone, which is no real row either.
      for (int j = 0, row = wr; row < nrows; j += 4, row += 4 * nwr, dst += 4 * dst_step) {
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          const uint32_t src = __builtin_amdgcn_readlane(rowsrc, j + u);  // (rows per wave <= 64: j + u <= 63)
#ifdef BSP_ROWS_TUNE
          if (a.nodma & 1) continue;
#endif
          if (src < kRowPad && col_real)
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(a.X + src + col_off),
                                             (__attribute__((address_space(3))) void*)(uintptr_t)(dst + u * dst_step), 16, 0, 0);
        }
      }
      continue;
    }
    for (int j = 0, row = wr; row < nrows; ++j, row += nwr, dst += dst_step) {
      const uint32_t src = __builtin_amdgcn_readlane(rowsrc, j);
      if (src == kRowNone) continue;
      const bool row_real = src != kRowPad;
      // the real pixels from X (one scalar base per row, one offset per lane), the padding from the zero bytes
      if (row_real && col_real)
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(a.X + src + col_off),
                                         (__attribute__((address_space(3))) void*)(uintptr_t)dst, 16, 0, 0);
      if (fill && (some_pad || !row_real)) {
        if (wanted && !(row_real && col_real)) {
          __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)zero,
                                           (__attribute__((address_space(3))) void*)(uintptr_t)dst, 16, 0, 0);
          if (a.nstaged > 1)
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)zero,
                                             (__attribute__((address_space(3))) void*)(uintptr_t)(dst + a.bufbytes), 16, 0, 0);
        }
      }
    }
  }
}

// Where a lane finds its 16 bytes of a column step's patch row 0 (the other rows lie rowbytes
// apart); with 4-channel units the 16 bytes are two pieces of 8.
struct RowsAd {
  uint32_t a0, a1;
};
template <bool CW4>
__device__ __forceinline__ RowsAd rows_addr(const RowsArgs& a, uint32_t desc, int pixb, uint32_t uoff) {
  RowsAd r;
  if (CW4) {
    uint32_t ad[2];
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const uint32_t it = (desc >> (16 * h)) & 0xFFFFu;
      const uint32_t unit = (it & 0xFFu) + 2u * uoff, pj = (uint32_t)pixb + (it >> 8);
      ad[h] = (((pj << a.lscp) + ((unit >> 1) ^ ((pj >> a.swz_shift) & a.swz_mask))) << 4) + ((unit & 1u) << 3);
    }
    r.a0 = ad[0];
    r.a1 = ad[1];
  } else {
    const uint32_t unit = (desc & 0xFFu) + uoff, pj = (uint32_t)pixb + ((desc >> 8) & 0xFFu);
    r.a0 = ((pj << a.lscp) + (unit ^ ((pj >> a.swz_shift) & a.swz_mask))) << 4;
    r.a1 = 0;
  }
  return r;
}
template <bool CW4>
__device__ __forceinline__ u32x4_t rows_frag(const unsigned char* buf, const RowsAd& ad, int rowoff) {
  if (CW4) {
    const u32x2_t p0 = *(const u32x2_t*)(buf + ad.a0 + rowoff);
    const u32x2_t p1 = *(const u32x2_t*)(buf + ad.a1 + rowoff);
    return u32x4_t{p0.x, p0.y, p1.x, p1.y};
  }
  return *(const u32x4_t*)(buf + ad.a0 + rowoff);
}

// The patch rows one column step needs, for one lane tile: f[fr] for the needed fr.
template <int H, int S, int BR, bool CW4>
__device__ __forceinline__ void rows_read(const RowsArgs& a, const unsigned char* buf, uint32_t desc, int pixb,
                                          int rowbytes, uint32_t uoff, u32x4_t (&f)[(BR - 1) * S + H]) {
  constexpr int NF = (BR - 1) * S + H;
  const RowsAd ad = rows_addr<CW4>(a, desc, pixb, uoff);
#pragma unroll
  for (int fr = 0; fr < NF; ++fr) {
    if (!row_needed<H, S, BR>(fr)) continue;
    f[fr] = rows_frag<CW4>(buf, ad, fr * rowbytes);
  }
}

// One lane tile's results straight from the accumulators: 8 bytes (four channels of one
// pixel) per lane; bias, one rounding, optional residual add and ReLU.
template <int BR>
__device__ __forceinline__ void rows_store_direct(const RowsArgs& a, const f32x4_t (&acc)[BR], int ch, int cb,
                                                  int rows, bool add_bias) {
  if (ch < 0 || cb < 0) return;
  f32x4_t bv = {0.f, 0.f, 0.f, 0.f};
  if (add_bias && a.bias) bv = f32x4_t{a.bias[ch], a.bias[ch + 1], a.bias[ch + 2], a.bias[ch + 3]};
#pragma unroll
  for (int r = 0; r < BR; ++r) {
    if (r >= rows || cb + r * a.N >= a.ylimit) continue;
    const f32x4_t v = acc[r] + bv;
    u32x2_t o;
    o.x = pack_bf16x2(v.x, v.y);
    o.y = pack_bf16x2(v.z, v.w);
    const uint32_t off = ((uint32_t)(cb + r * a.N) * (uint32_t)a.O + (uint32_t)ch) * 2u;
    if (a.residual || a.relu)
      o = post_bf16x4(o, a.residual ? (const uint16_t*)(a.residual + off) : nullptr, 4, true, a.relu);
    *(u32x2_t*)(a.Y + off) = o;
  }
}

template <int H, int S, int BR, int NT, bool CW4, int D>
__global__ __launch_bounds__(640) __attribute__((amdgpu_waves_per_eu(H == 3 && NT == 1 && (S == 1 || BR == 4) ? 4 : 3))) void conv_rows(RowsArgs a) {
  // (not in the one-row-window instances: there it costs scalar registers the kernel does not
  // have, and the spills cost more than the misses)
  if constexpr (H != 1) kernarg_touch<RowsArgs>();
  // The opening (tile position, tables, the first slab's requests) reads some fifty words of the
  // arguments, and the compiler would read each where a basic block first needs it, waiting for
  // the scalar cache every time (35 waits in a row before the first MFMA).  Naming them as inputs
  // of empty statements here makes it read them together (23 waits, 70 instructions fewer).
  if constexpr (H != 1) {
    asm volatile("" : :
                 "s"(a.per_xcd), "s"(a.nsg), "s"(a.ntiles), "s"(a.tiles_x), "s"(a.tiles_y), "s"(a.NI),
                 "s"(a.NB), "s"(a.TW), "s"(a.tbl_off), "s"(a.PTW), "s"(a.ncols), "s"(a.PR), "s"(a.PCp),
                 "s"(a.B), "s"(a.N), "s"(a.M), "s"(a.SG), "s"(a.NM), "s"(a.lsg), "s"(a.lptw));
    asm volatile("" : :
                 "s"(a.nstrips), "s"(a.ncs), "s"(a.lscp), "s"(a.nslabs), "s"(a.KS), "s"(a.bufbytes),
                 "s"(a.stride), "s"(a.ph), "s"(a.pw), "s"(a.PC), "s"(a.gs), "s"(a.L), "s"(a.J), "s"(a.I),
                 "s"(a.swz_shift), "s"(a.swz_mask), "s"(a.scs), "s"(a.nstaged));
    asm volatile("" : :
                 "s"(a.d_nsg.d), "s"(a.d_nsg.mul), "s"(a.d_tpi.d), "s"(a.d_tpi.mul), "s"(a.d_tx.d),
                 "s"(a.d_tx.mul), "s"(a.d_perimg.d), "s"(a.d_perimg.mul), "s"(a.d_tw.d), "s"(a.d_tw.mul),
                 "s"(a.d_pr.d), "s"(a.d_pr.mul));
  }
  constexpr int NF = (BR - 1) * S + H;
  extern __shared__ __align__(16) unsigned char lds[];
  const int tid = threadIdx.x;
  const int nthreads = blockDim.x - 64 * a.NM;  // compute threads; the last NM waves move data
  const int wave = tid >> 6, lane = tid & 63, g = lane >> 4, c = lane & 15;
  TilePos tp;
  if (!rows_tile(a, BR, &tp)) return;

  int32_t* colbase = (int32_t*)(lds + a.tbl_off);
  const int nslots = a.PTW * NT * 16;
  int32_t* colrows = colbase + nslots;
  int32_t* colpix = colrows + nslots;
  int32_t* chans = colpix + nslots;
  ROWS_MARK(0);
  rows_tables(a, tp, BR, S, nslots, colbase, colrows, colpix);
  // the output channels of the workgroup's strips: asked for now, put into LDS only when the
  // results are (a wait for this load any earlier would also wait for the patch's copies)
  int chan_v = -1;
  if (tid < a.SG * 4) {
    const int st = tp.sgi * a.SG + (tid >> 2);
    if (st < a.nstrips) chan_v = a.rstrip[st * 4 + (tid & 3)];
  }

  const int wave_u = __builtin_amdgcn_readfirstlane(wave);
  const bool mover = wave_u * 64 >= nthreads;
  // SG and PTW are powers of two
  const int sl_local = wave_u & (a.SG - 1), sub = wave_u >> a.lsg;
  const int pt = sub & (a.PTW - 1), ks = mover ? -1 : sub >> a.lptw;
  const int strip = tp.sgi * a.SG + sl_local;
  const bool active = !mover && strip < a.nstrips && a.ncs > 0;

  f32x4_t acc[NT][BR];
#pragma unroll
  for (int j = 0; j < NT; ++j)
#pragma unroll
    for (int r = 0; r < BR; ++r) acc[j][r] = f32x4_t{0.f, 0.f, 0.f, 0.f};

  const int rowbytes = a.PCp << (a.lscp + 4);

  // ---- compute waves: the strip's column steps come from the plan through a ring of registers,
  // D steps ahead (weight fragments and item descriptors).  A strip's steps are numbered
  // consecutively through all its slabs; with the contraction split KS ways (a power of two)
  // this wave takes the steps whose number is ks modulo KS, so its sequence is one arithmetic
  // progression from start to finish and the ring never has to be turned at a slab's end.
  // The first D steps are asked for before the patch is: their latency passes while the
  // requests for the patch are being issued.
  // entry i: the first step of slab i.  The table is read with scalar loads (the plan is never
  // written by a kernel): the address is made a scalar explicitly
  typedef const __attribute__((address_space(4))) int32_t* cptr_t;
  const uint64_t rsl_v = (uint64_t)(uintptr_t)(a.rslab + (active ? strip : 0) * (a.nslabs + 1));
  // (the builtin returns a signed int: widened through uint32_t, or the low half's top bit would spill over the high half)
  const uint32_t rsl_lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)rsl_v);
  const uint32_t rsl_hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(rsl_v >> 32));
  const cptr_t rsl = (cptr_t)(uintptr_t)((uint64_t)rsl_lo | ((uint64_t)rsl_hi << 32));
  const int ksm = a.KS - 1;
  int s_first = 0, s_end = 0, fnext = 0;
  const uint32_t frag_lane = (uint32_t)lane * 16u, desc_lane = (uint32_t)g * 4u;
  const unsigned char* fragb = (const unsigned char*)a.rfrag;
  const unsigned char* descb = (const unsigned char*)a.rdesc;
  u32x4_t wr[D][H];  // weight fragments of the next D steps of the sequence
  int dr[D];         // their item descriptors
  // Slot d takes the next step of the sequence; past the end it asks for the last step
  // again (never used): every pass through the unrolled loop below issues the same loads,
  // which lets the compiler wait for exactly the slot it needs.
  auto fetch = [&](int d) {
    const int cs = max(0, min(fnext, s_end - 1));
    fnext += a.KS;
    dr[d] = *(const int*)(descb + ((uint32_t)cs * 16u + desc_lane));
    const uint32_t off = (uint32_t)cs * (uint32_t)(H * 1024) + frag_lane;
#pragma unroll
    for (int dy = 0; dy < H; ++dy) wr[d][dy] = *(const u32x4_t*)(fragb + off + dy * 1024);
  };
  if (!mover) {
    // the strip's first and last step as scalar loads (the plan is never written by a kernel)
    s_first = rsl[0];
    s_end = rsl[a.nslabs];
    fnext = s_first + ((ks - s_first) & ksm);
    if (active) {
#pragma unroll
      for (int d = 0; d < D; ++d) {
        fetch(d);
        __builtin_amdgcn_sched_barrier(0);
      }
    }
  }
  ROWS_MARK(1);
  rows_stage(a, tp, lds, 0, wave_u, (int)(blockDim.x >> 6));  // the first slab: all waves together
  ROWS_MARK(2);

  if (mover) {
    // ---- the data movers request the next staged slab while the compute waves work on the
    // current one; the barrier at the end of a slab tells them it has landed and tells the
    // movers that the other buffer is free.
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();                  // the first slab is in LDS
    for (int ss = 1; ss < a.nstaged; ++ss) {
      rows_stage(a, tp, lds, ss, wave_u - (nthreads >> 6), a.NM);
      __builtin_amdgcn_s_waitcnt(0);  // everything requested so far is in LDS
      __syncthreads();                // slab ss - 1 is done everywhere
    }
    __syncthreads();                  // the last slab is done
  } else {
    ROWS_MARK(3);
    if (tid < a.SG * 4) chans[tid] = chan_v;  // (wave 0 is a compute wave)
    __builtin_amdgcn_s_waitcnt(0);  // this wave's share of the first patch has landed
    __syncthreads();                // the first slab's patch and the tables are in LDS
    ROWS_MARK(4);
    int pixb[NT];
#pragma unroll
    for (int j = 0; j < NT; ++j) pixb[j] = colpix[(pt * NT + j) * 16 + c];
    u32x4_t f[NT][NF];  // the patch rows of the step at hand

    // A step's MFMAs run patch row by patch row (row k feeds output rows k - dy), and as soon as
    // the ones that read row k have been issued the next step's row k is asked for into the same
    // registers: the matrix cores work through a step while the next one's fragments arrive.
    // A step reads nothing but the next step's fragments, so where the next step lies in the
    // next staged slab the wave passes that slab's barrier before the step, not after it.
    constexpr bool ROLL = H > 1;  // (a one-row window's fragments feed one MFMA each: read per step)
    int cs = s_first + ((ks - s_first) & ksm);  // this wave's next step
    int sl = 0, ss = 0;                          // a plan slab; the staged slab the workgroup is at
    int hi = rsl[1];                             // where plan slab sl ends
    const unsigned char* buf = lds;
    uint32_t uoff = 0;  // where plan slab sl's pieces start in a staged pixel
    // (uniform) make sl the slab of step at < s_end; on the way into a later staged slab, the
    // barriers that say the slabs before it are done everywhere and it has landed
    auto enter = [&](int at) {
      while (at >= hi) {
        ++sl;
        hi = rsl[sl + 1];
      }
      while ((ss + 1) * a.G <= sl) {
        __syncthreads();
        ++ss;
      }
      buf = lds + (ss & 1) * a.bufbytes;
      uoff = (uint32_t)((sl - ss * a.G) * a.sc);
    };
    auto step = [&](int d) {
      if (!ROLL) {
        enter(cs);
#pragma unroll
        for (int j = 0; j < NT; ++j) rows_read<H, S, BR, CW4>(a, buf, (uint32_t)dr[d], pixb[j], rowbytes, uoff, f[j]);
#pragma unroll
        for (int dy = 0; dy < H; ++dy)
#pragma unroll
          for (int j = 0; j < NT; ++j)
#pragma unroll
            for (int r = 0; r < BR; ++r)
              acc[j][r] = mfma_bf16_16x16x32(wr[d][dy], f[j][r * S + dy], acc[j][r]);
        cs += a.KS;
      } else {
        // (the last step of all asks for its own fragments again: nobody reads them)
        const int nxt = cs + a.KS;
        const bool pre = nxt < s_end;
        if (pre) enter(nxt);
        const uint32_t dn = (uint32_t)(pre ? dr[(d + 1) % D] : dr[d]);
        RowsAd nad[NT];
#pragma unroll
        for (int j = 0; j < NT; ++j) nad[j] = rows_addr<CW4>(a, dn, pixb[j], uoff);
#pragma unroll
        for (int k = 0; k < NF; ++k) {
#pragma unroll
          for (int dy = 0; dy < H; ++dy) {
            if (k - dy < 0 || (k - dy) % S != 0 || (k - dy) / S >= BR) continue;
#pragma unroll
            for (int j = 0; j < NT; ++j)
              acc[j][(k - dy) / S] = mfma_bf16_16x16x32(wr[d][dy], f[j][k], acc[j][(k - dy) / S]);
          }
#ifdef BSP_ROWS_TUNE
          if (a.nodma & 2) continue;  // experiments: the fragments are not read again (timing only)
#endif
          if (row_needed<H, S, BR>(k)) {
#pragma unroll
            for (int j = 0; j < NT; ++j) f[j][k] = rows_frag<CW4>(buf, nad[j], k * rowbytes);
          }
        }
        cs = nxt;
      }
    };
    if (ROLL && active && cs < s_end) {
      enter(cs);
#pragma unroll
      for (int j = 0; j < NT; ++j) rows_read<H, S, BR, CW4>(a, buf, (uint32_t)dr[0], pixb[j], rowbytes, uoff, f[j]);
    }
    if (active) {
      // passes that refill the ring while more than D steps remain (a slot is refilled only
      // after the MFMAs that read it, in place: requested earlier, the new fragments would
      // need registers of their own), then the steps the ring already holds
      while (cs + D * a.KS < s_end) {
#pragma unroll
        for (int d = 0; d < D; ++d) {
          step(d);
          __builtin_amdgcn_sched_barrier(0);
          fetch(d);
          __builtin_amdgcn_sched_barrier(0);
        }
      }
#pragma unroll
      for (int d = 0; d < D; ++d) {
        if (cs >= s_end) break;
        step(d);
      }
    }
    // the barriers of the staged slabs this wave had no step in: each slab's end is one
    while (ss < a.nstaged) {
      __syncthreads();
      ++ss;
    }
  }

  ROWS_MARK(5);
  // ---- results: optional sum over the contraction shares, then out
  unsigned char* red = lds;
  unsigned char* ostage = lds + a.red_bytes;
  if (a.KS > 1) {
    if (ks > 0) {
      const int w = ((ks - 1) * a.PTW + pt) * a.SG + sl_local;
      f32x4_t* dst = (f32x4_t*)red + (size_t)w * NT * BR * 64;
#pragma unroll
      for (int j = 0; j < NT; ++j)
#pragma unroll
        for (int r = 0; r < BR; ++r) dst[(j * BR + r) * 64 + lane] = acc[j][r];
    }
    __syncthreads();
    if (ks == 0) {
      for (int k = 1; k < a.KS; ++k) {
        const int w = ((k - 1) * a.PTW + pt) * a.SG + sl_local;
        const f32x4_t* src = (const f32x4_t*)red + (size_t)w * NT * BR * 64;
#pragma unroll
        for (int j = 0; j < NT; ++j)
#pragma unroll
          for (int r = 0; r < BR; ++r) acc[j][r] += src[(j * BR + r) * 64 + lane];
      }
    }
  }
  if (a.direct) {
    if (!mover && ks == 0 && strip < a.nstrips) {
      const int ch = chans[sl_local * 4 + g];
#pragma unroll
      for (int j = 0; j < NT; ++j) {
        const int col = (pt * NT + j) * 16 + c;
        rows_store_direct<BR>(a, acc[j], ch, colbase[col], colrows[col], true);
      }
    }
    return;
  }
  // through an LDS staging tile, leaving as whole 16-byte (4x16 blocks: 8-byte) pieces
  if (!mover && ks == 0 && strip < a.nstrips) {
    const int ch = chans[sl_local * 4 + g];
    if (ch >= 0) {
      f32x4_t bv = {0.f, 0.f, 0.f, 0.f};
      if (a.bias) bv = f32x4_t{a.bias[ch], a.bias[ch + 1], a.bias[ch + 2], a.bias[ch + 3]};
#pragma unroll
      for (int j = 0; j < NT; ++j)
#pragma unroll
        for (int r = 0; r < BR; ++r) {
          const f32x4_t v = acc[j][r] + bv;
          u32x2_t o;
          o.x = pack_bf16x2(v.x, v.y);
          o.y = pack_bf16x2(v.z, v.w);
          const int pix = ((pt * NT + j) * 16 + c) * BR + r;
          *(u32x2_t*)(ostage + pix * a.orow + (sl_local * 4 + g) * 8) = o;
        }
    }
  }
  __syncthreads();
  ROWS_MARK(6);
  const int nopix = nslots * BR;
  if (!a.piece8) {
    const int np = a.SG * 2;
    for (int idx = tid; idx < nopix * np; idx += blockDim.x) {
      const int pix = (int)fdiv((uint32_t)idx, a.d_np), pc = idx - pix * np;
      const int col = (int)fdiv((uint32_t)pix, a.d_br), r = pix - col * BR;
      const int cb = colbase[col], ch = chans[pc * 2];
      if (cb < 0 || r >= colrows[col] || ch < 0 || cb + r * a.N >= a.ylimit) continue;
      u32x4_t v = *(const u32x4_t*)(ostage + pix * a.orow + pc * 16);
      const uint32_t off = ((uint32_t)(cb + r * a.N) * (uint32_t)a.O + (uint32_t)ch) * 2u;
      if (a.residual || a.relu) {
        const uint16_t* rp = a.residual ? (const uint16_t*)(a.residual + off) : nullptr;
        const u32x2_t lo2 = post_bf16x4(u32x2_t{v.x, v.y}, rp, 4, true, a.relu);
        const u32x2_t hi2 = post_bf16x4(u32x2_t{v.z, v.w}, rp ? rp + 4 : nullptr, 4, true, a.relu);
        v = u32x4_t{lo2.x, lo2.y, hi2.x, hi2.y};
      }
      *(u32x4_t*)(a.Y + off) = v;
    }
  } else {
    const int np = a.SG * 4;
    for (int idx = tid; idx < nopix * np; idx += blockDim.x) {
      const int pix = (int)fdiv((uint32_t)idx, a.d_np), pc = idx - pix * np;
      const int col = (int)fdiv((uint32_t)pix, a.d_br), r = pix - col * BR;
      const int cb = colbase[col], ch = chans[pc];
      if (cb < 0 || r >= colrows[col] || ch < 0 || cb + r * a.N >= a.ylimit) continue;
      u32x2_t v = *(const u32x2_t*)(ostage + pix * a.orow + pc * 8);
      const uint32_t off = ((uint32_t)(cb + r * a.N) * (uint32_t)a.O + (uint32_t)ch) * 2u;
      if (a.residual || a.relu) {
        const uint16_t* rp = a.residual ? (const uint16_t*)(a.residual + off) : nullptr;
        v = post_bf16x4(v, rp, 4, true, a.relu);
      }
      *(u32x2_t*)(a.Y + off) = v;
    }
  }
#ifdef BSP_ROWS_TUNE
  __builtin_amdgcn_s_waitcnt(0);
#endif
  ROWS_MARK(7);
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

constexpr int kLdsLimit = 160 * 1024;

template <int H, int S, int BR, int NT, bool CW4, int D>
int launch_inst(const RowsArgs& a, dim3 grid, int threads, size_t ldsb, hipStream_t st) {
  static size_t raised = 65536;  // dynamic LDS above 64 KB has to be allowed per kernel
  if (ldsb > raised) {
    if (hipFuncSetAttribute((const void*)conv_rows<H, S, BR, NT, CW4, D>,
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)ldsb) != hipSuccess)
      return BSP_ERR_HIP;
    raised = ldsb;
  }
  hipLaunchKernelGGL((conv_rows<H, S, BR, NT, CW4, D>), grid, dim3(threads), ldsb, st, a);
  return hipGetLastError() == hipSuccess ? BSP_OK : BSP_ERR_HIP;
}

template <int H, int S, bool CW4>
int launch_hs(const RowsArgs& a, int BR, int NT, dim3 grid, int threads, size_t ldsb, hipStream_t st) {
  constexpr int D = H == 1 ? 8 : (H == 3 ? 3 : 2);
  if (BR == 7 && NT == 1) return launch_inst<H, S, 7, 1, CW4, D>(a, grid, threads, ldsb, st);
  if (BR == 4 && NT == 1) return launch_inst<H, S, 4, 1, CW4, D>(a, grid, threads, ldsb, st);
  if constexpr (H <= 3) {  // (two column tiles of a seven-row window do not fit the register file)
    if (BR == 4 && NT == 2) return launch_inst<H, S, 4, 2, CW4, D>(a, grid, threads, ldsb, st);
  }
  return BSP_ERR_UNSUPPORTED;
}

struct Choice {
  int BR, NT, TW, NB, NI, SG, PTW, KS;
  double cost;
  int G = 1;   // plan slabs staged together
  int NM = 1;  // data-mover waves
};

struct Geometry {
  int PR, PC, PCp, lscp, tiles_x, tiles_y, slots, orow;
  int64_t ntiles, bufbytes, red, body, ldsb;
};

inline int ceil_log2(int v) {
  int l = 0;
  while ((1 << l) < v) ++l;
  return l;
}

// Everything that follows from a choice; false when it does not fit.
bool rows_geometry(const ConvParams& p, int slab, int S, const Choice& c, Geometry* g) {
  g->slots = c.PTW * c.NT * 16;
  if (c.NI * c.NB * c.TW > g->slots || c.SG * c.PTW * c.KS > 8) return false;
  g->PR = (c.NB * c.BR - 1) * S + p.H;
  if (c.NI * g->PR > 64) return false;  // a wave keeps one staged row per lane
  g->PC = (c.TW - 1) * S + p.K;
  g->PCp = (g->PC + 15) & ~15;
  g->lscp = ceil_log2(c.G * slab / 8);
  if (g->lscp < 2 || g->lscp > 6) return false;  // a request covers between one and sixteen pixels of a row
  g->bufbytes = ((int64_t)c.NI * g->PR * g->PCp) << (g->lscp + 4);
  g->orow = c.SG * 32 + 16;
  g->red = c.KS > 1 ? (int64_t)(c.KS - 1) * c.PTW * c.SG * c.NT * c.BR * 1024 : 0;
  const int nslabs = (p.I + slab - 1) / slab;
  const int nstaged = (nslabs + c.G - 1) / c.G;
  const int64_t patch = nstaged > 1 ? 2 * g->bufbytes : g->bufbytes;
  g->body = std::max<int64_t>(patch, g->red + (int64_t)g->slots * c.BR * g->orow);
  g->body = (g->body + 15) & ~15ll;
  g->ldsb = g->body + (int64_t)g->slots * 12 + c.SG * 16;
  if (g->ldsb > kLdsLimit) return false;
  g->tiles_x = (p.N + c.TW - 1) / c.TW;
  g->tiles_y = ((p.M + c.BR - 1) / c.BR + c.NB - 1) / c.NB;
  g->ntiles = (int64_t)((p.B + c.NI - 1) / c.NI) * g->tiles_y * g->tiles_x;
  return true;
}

}  // namespace

// Tile and role choice.  Cost model (clock cycles, rough): matrix-core time of the busiest
// SIMD against the time the CU needs to pull in patches and weights, plus fixed costs.
static bool rows_choose(const ConvParams& p, const int32_t* rs, int S, Choice* best) {
  const int nstrips = rs[BSP_ROWS_NSTRIPS_W], nslabs = rs[BSP_ROWS_NSLABS_W];
  const int slab = rs[BSP_ROWS_SLAB_W];
  const double steps_per_strip = (double)rs[BSP_ROWS_NCS_W] / std::max(1, nstrips);
  const int cus = device_cus();
  best->cost = 1e300;
  for (int BR : {7, 4}) {
    for (int NT : {1, 2}) {
      if (BR == 7 && NT == 2) continue;
      // (two column tiles of 4-channel units at stride 2 do not fit the register file)
      if (NT == 2 && S == 2 && p.H > 1 && rs[BSP_ROWS_CW_W] == 4) continue;
      if (NT == 2 && p.H > 3) continue;
      for (int SG : {1, 2, 4, 8}) {
        if (SG > nstrips && SG != 1) continue;
        for (int KS : {1, 2, 4}) {
          for (int PTW : {1, 2, 4, 8}) {
            const int waves = SG * PTW * KS;
            if (waves > 8) continue;
            const int slots = PTW * NT * 16;  // columns a workgroup can hold
            for (int G : {1, 2, 4}) {
              if (G > 1 && G / 2 >= nslabs) continue;
              for (int mode = 0; mode < 4; ++mode) {
                Choice c{BR, NT, 0, 1, 1, SG, PTW, KS, 0.0};
                c.G = G;
                if (mode == 0) {           // whole image rows, several bands
                  c.TW = p.N;
                  if (c.TW > slots) continue;
                  c.NB = std::min(slots / c.TW, (p.M + BR - 1) / BR);
                } else if (mode == 3) {    // whole image rows, one band (a smaller patch per workgroup, more workgroups)
                  c.TW = p.N;
                  if (c.TW > slots || std::min(slots / c.TW, (p.M + BR - 1) / BR) < 2) continue;
                } else if (mode == 1) {    // several images, every band of each
                  c.TW = p.N;
                  c.NB = (p.M + BR - 1) / BR;
                  if (c.TW * c.NB > slots) continue;
                  c.NI = std::min(slots / (c.TW * c.NB), p.B);
                  if (c.NI < 2) continue;
                } else {                   // part of a row
                  if (p.N <= slots) continue;
                  const int parts = (p.N + slots - 1) / slots;
                  c.TW = (p.N + parts - 1) / parts;
                }
                Geometry g;
                if (!rows_geometry(p, slab, S, c, &g)) continue;
                const int nstaged = (nslabs + G - 1) / G;
                c.NM = nstaged > 1 ? (waves >= 8 ? 2 : 1) : 0;
                const int nsg = (nstrips + SG - 1) / SG;
                const int64_t nwg = g.ntiles * nsg;
                // rough times in ns.  A wave alone on its SIMD issues about one instruction per
                // eight cycles, so a column step costs its MFMAs plus its other instructions;
                // a second wave on the SIMD hides most of that
                const double step_mfma = p.H * BR * NT * 8.0, step_other = (20.0 + 10.0 * NT * ((BR - 1) * S + p.H)) * 4.0;
                // workgroups a CU holds at once: LDS, and the registers (between 77 and 168 per
                // lane: three to six waves per SIMD, as the kernel's instances are compiled), a
                // workgroup's waves being dealt round over the four SIMDs from the first one on
                // (two workgroups of ten waves need six waves on a SIMD, not five)
                const int occ = p.H == 1 ? (NT == 2 ? 4 : BR == 4 ? 6 : 5) : (p.H == 3 && NT == 1 && (S == 1 || BR == 4) ? 4 : 3);
                const int wg_per_cu = (int)std::max<int64_t>(
                    1, std::min<int64_t>(kLdsLimit / g.ldsb, occ / ((waves + c.NM + 3) / 4)));
                const double conc = std::min<double>(wg_per_cu, std::max(1.0, (double)nwg / cus));
                const double per_simd = std::max(1.0, waves * conc / 4.0);
                const double t_step = per_simd >= 2.0 ? std::max(step_mfma * per_simd, (step_mfma + step_other) * per_simd / 2.0)
                                                      : step_mfma + step_other;
                const double t_compute = steps_per_strip / KS * t_step;
                const double t_stage0 = 700.0 + (double)g.bufbytes / (60.0 / conc);
                const double t_mover = nstaged > 1 ? (double)(nstaged - 1) * g.bufbytes / 16.0 / 64.0 * 110.0 / std::max(1, c.NM) : 0.0;
                const double t_epi = 500.0 + 100.0 * NT * BR / 7.0 + (KS > 1 ? 400.0 : 0.0);
                const double t_wg = t_stage0 + std::max(t_compute, t_mover) + 250.0 * nstaged + t_epi;
                const double rounds = std::ceil((double)nwg / ((double)cus * wg_per_cu));
                c.cost = rounds * t_wg;
#ifdef BSP_ROWS_TUNE
                if (std::getenv("BSP_ROWS_COSTS"))
                  fprintf(stderr, "cand %d,%d,%d,%d,%d,%d,%d,%d,%d,%d nwg=%lld wgcu=%d conc=%.2f stage0=%.0f comp=%.0f mover=%.0f epi=%.0f nst=%d rounds=%.0f cost=%.0f\n",
                          c.BR, c.NT, c.TW, c.NB, c.NI, c.SG, c.PTW, c.KS, c.G, c.NM, (long long)nwg, wg_per_cu, conc, t_stage0,
                          t_compute, t_mover, t_epi, nstaged, rounds, c.cost);
#endif
                if (c.cost < best->cost) *best = c;
              }
            }
          }
        }
      }
    }
  }
  return best->cost < 1e299;
}

// What the kernel takes from the layer, the plan and the chosen tile.
static int rows_fill_common(const ConvParams& p, const ConvParams& v, const int32_t* hdr, const int32_t* rs, int gs,
                            const Choice& ch, const Geometry& geo, RowsArgs* out) {
  RowsArgs& a = *out;
  const int32_t* sec = p.plan + hdr[BSP_PLAN_OFF_ROWS_W];
  a.X = (const unsigned char*)p.X;
  a.Y = (unsigned char*)p.Y;
  a.bias = p.bias;
  a.residual = (const unsigned char*)p.residual;
  a.relu = p.relu;
  a.rstrip = sec + rs[BSP_ROWS_OFF_STRIP_W];
  a.rslab = sec + rs[BSP_ROWS_OFF_SLAB_W];
  a.rdesc = sec + rs[BSP_ROWS_OFF_DESC_W];
  a.rfrag = (const u32x4_t*)(sec + rs[BSP_ROWS_OFF_FRAG_W]);
  a.nstrips = rs[BSP_ROWS_NSTRIPS_W];
  a.nslabs = rs[BSP_ROWS_NSLABS_W];
  a.ncs = rs[BSP_ROWS_NCS_W];  // 0: an all-zero mask, no step exists anywhere
  a.sc = rs[BSP_ROWS_SLAB_W] / 8;
  a.G = ch.G;
  a.nstaged = (a.nslabs + ch.G - 1) / ch.G;
  a.scs = ch.G * a.sc;
  a.NM = ch.NM;
  a.lscp = geo.lscp;
  {
    const int bits = std::min(geo.lscp, 4);  // swizzle: 16 consecutive pixels, 16 distinct bank groups
    a.swz_shift = 4 - bits;
    a.swz_mask = (1 << bits) - 1;
  }
  a.B = v.B;
  a.L = v.L;
  a.J = v.J;
  a.I = p.I;
  a.O = p.O;
  a.M = v.M;
  a.N = v.N;
  a.ph = p.ph;
  a.pw = p.pw;
  a.stride = p.sh;
  a.gs = gs;
  a.TW = ch.TW;
  a.NB = ch.NB;
  a.NI = ch.NI;
  a.PR = geo.PR;
  a.PC = geo.PC;
  a.PCp = geo.PCp;
  a.tiles_x = geo.tiles_x;
  a.tiles_y = geo.tiles_y;
  a.ntiles = (int32_t)geo.ntiles;
  a.ncols = ch.NI * ch.NB * ch.TW;
  a.SG = ch.SG;
  a.PTW = ch.PTW;
  a.KS = ch.KS;
  a.nsg = (a.nstrips + ch.SG - 1) / ch.SG;
  a.per_xcd = ((a.ntiles + 7) / 8) * a.nsg;
  a.bufbytes = (int32_t)geo.bufbytes;
  a.orow = geo.orow;
  a.red_bytes = (int32_t)geo.red;
  a.piece8 = hdr[BSP_PLAN_BO_W] == 4;
  a.direct = 1;
  a.tbl_off = (int32_t)geo.body;
  a.ylimit = p.P;
  const int64_t nstage = geo.bufbytes / 16;
  if (geo.ntiles >= (1 << 24) || nstage >= (1 << 24) || (int64_t)a.per_xcd * 8 >= (1ll << 31))
    return BSP_ERR_UNSUPPORTED;
  a.lsg = ceil_log2(ch.SG);
  a.lptw = ceil_log2(ch.PTW);
  a.d_nsg = make_fastdiv(a.nsg);
  a.d_tpi = make_fastdiv(a.tiles_x * a.tiles_y);
  a.d_tx = make_fastdiv(a.tiles_x);
  a.d_perimg = make_fastdiv(ch.NB * ch.TW);
  a.d_tw = make_fastdiv(ch.TW);
  a.d_pcp = make_fastdiv(a.PCp);
  a.d_pr = make_fastdiv(a.PR);
  a.d_np = make_fastdiv(a.piece8 ? ch.SG * 4 : ch.SG * 2);
  a.d_br = make_fastdiv(ch.BR);
  // the multiply-high divisions are exact while dividend * divisor < 2^32; staged pixels are
  // counted up to the next multiple of the workgroup size
  if ((nstage + 1024) * std::max(a.PCp, a.PR) >= (1ll << 32) ||
      (int64_t)a.per_xcd * 8 * std::max(a.nsg, a.tiles_x * a.tiles_y) >= (1ll << 32))
    return BSP_ERR_UNSUPPORTED;
  return BSP_OK;
}

int bsp_launch_rows(const ConvParams& p, int dtype, const void* plan_host, hipStream_t st) {
  if (dtype != BSP_BF16 || !plan_host) return BSP_ERR_UNSUPPORTED;
  const int32_t* hdr = (const int32_t*)plan_host;
  if (hdr[BSP_PLAN_MAGIC_W] != BSP_PLAN_MAGIC || hdr[BSP_PLAN_VERSION_W] != BSP_PLAN_VERSION ||
      hdr[BSP_PLAN_O_W] != p.O || hdr[BSP_PLAN_I_W] != p.I || hdr[BSP_PLAN_H_W] != p.H ||
      hdr[BSP_PLAN_K_W] != p.K || hdr[BSP_PLAN_DTYPE_W] != dtype || hdr[BSP_PLAN_OFF_ROWS_W] == 0)
    return BSP_ERR_UNSUPPORTED;
  const int32_t* rs = hdr + hdr[BSP_PLAN_OFF_ROWS_W];
  if (p.sh != p.sw || (p.sh != 1 && p.sh != 2)) return BSP_ERR_UNSUPPORTED;
  if (p.H != 1 && p.H != 3 && !(p.H == 7 && p.sh == 1)) return BSP_ERR_UNSUPPORTED;  // (window heights the kernel is compiled for)
  if ((int64_t)p.B * p.L * p.J * p.I * 2 >= (1ll << 31) || (int64_t)p.P * p.O * 2 >= (1ll << 31))
    return BSP_ERR_UNSUPPORTED;
  if (p.H == 1 && p.K == 1) return BSP_ERR_UNSUPPORTED;  // pointwise layers: bsp_pw.hip
  if (p.H == 1 && p.sh != 1) return BSP_ERR_UNSUPPORTED;  // (one-row windows are compiled for stride 1 only)
  const int cw = rs[BSP_ROWS_CW_W];
  const int slab = rs[BSP_ROWS_SLAB_W];
  const int S = p.sh;   // staged pixels per output pixel step
  const int gs = 1;     // input pixels per staged pixel
  const ConvParams& v = p;
  Choice ch;
  if (!rows_choose(v, rs, S, &ch)) return BSP_ERR_UNSUPPORTED;
#ifdef BSP_ROWS_TUNE  // experiments only: never defined in the product build
  if (const char* e = std::getenv("BSP_ROWS_TUNE")) {
    int q[10] = {0, 0, 0, 0, 0, 0, 0, 0, 1, 1};
    if (sscanf(e, "%d,%d,%d,%d,%d,%d,%d,%d,%d,%d", q, q + 1, q + 2, q + 3, q + 4, q + 5, q + 6, q + 7, q + 8, q + 9) >= 8) {
      ch = Choice{q[0], q[1], q[2] > 0 ? q[2] : v.N, q[3], q[4], q[5], q[6], q[7], 0.0};
      ch.G = q[8];
      ch.NM = (rs[BSP_ROWS_NSLABS_W] + ch.G - 1) / ch.G > 1 ? std::max(1, q[9]) : 0;
    }
  }
  if (std::getenv("BSP_ROWS_VERBOSE"))
    fprintf(stderr, "rows: M=%d N=%d B=%d I=%d O=%d H=%d s=%d | BR=%d NT=%d TW=%d NB=%d NI=%d SG=%d PTW=%d KS=%d G=%d NM=%d cost=%.0f\n",
            v.M, v.N, v.B, p.I, p.O, p.H, p.sh, ch.BR, ch.NT, ch.TW, ch.NB, ch.NI, ch.SG, ch.PTW, ch.KS, ch.G, ch.NM, ch.cost);
#endif
  Geometry geo;
  if (!rows_geometry(v, slab, S, ch, &geo)) return BSP_ERR_UNSUPPORTED;

  RowsArgs a{};
  if (int rc = rows_fill_common(p, v, hdr, rs, gs, ch, geo, &a)) return rc;
  // Small outputs of one-row windows (at most 2 MB: InceptionV3's 1x7 and 1x3 layers) leave
  // straight from the accumulators, 8 bytes per lane: no staging tile, no barrier (measured
  // 0.3-0.5 us faster on each of them; the other window heights and larger outputs are as
  // fast or faster as 16-byte pieces).
  a.direct = p.H == 1 && (int64_t)p.P * p.O * 2 <= (2ll << 20);
#ifdef BSP_ROWS_TUNE
  if (const char* e = std::getenv("BSP_PW_TRACE_PTR")) a.trace = (long long*)std::strtoull(e, nullptr, 16);
  if (const char* e = std::getenv("BSP_ROWS_NODMA")) a.nodma = std::atoi(e);
#endif
#ifdef BSP_ROWS_TUNE
  if (std::getenv("BSP_ROWS_DIRECT")) a.direct = 1;
#endif
  if ((int64_t)geo.slots * ch.BR * ch.SG * 4 * std::max(ch.SG * 4, ch.BR) >= (1ll << 32)) return BSP_ERR_UNSUPPORTED;
  const int threads = 64 * (ch.SG * ch.PTW * ch.KS + ch.NM);  // compute waves + the data movers
  dim3 grid((unsigned)(a.per_xcd * 8));
  const size_t ldsb = (size_t)geo.ldsb;
  if (cw == 4) {
    if (p.H == 1) return launch_hs<1, 1, true>(a, ch.BR, ch.NT, grid, threads, ldsb, st);
    if (p.H == 7) return launch_hs<7, 1, true>(a, ch.BR, ch.NT, grid, threads, ldsb, st);
    return S == 1 ? launch_hs<3, 1, true>(a, ch.BR, ch.NT, grid, threads, ldsb, st)
                  : launch_hs<3, 2, true>(a, ch.BR, ch.NT, grid, threads, ldsb, st);
  }
  if (p.H == 1) return launch_hs<1, 1, false>(a, ch.BR, ch.NT, grid, threads, ldsb, st);
  if (p.H == 7) return launch_hs<7, 1, false>(a, ch.BR, ch.NT, grid, threads, ldsb, st);
  return S == 1 ? launch_hs<3, 1, false>(a, ch.BR, ch.NT, grid, threads, ldsb, st)
                : launch_hs<3, 2, false>(a, ch.BR, ch.NT, grid, threads, ldsb, st);
}
