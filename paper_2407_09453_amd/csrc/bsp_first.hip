// Layers with at most four input channels (a network's first layer; bf16, windows up to 7x7,
// any stride and padding, 32 or 64 output channels): one workgroup per band of BR output rows
// of an image, all columns, all output channels.
//
// A pixel of such a layer is a few bytes, so the window itself is the contraction: index
// k = (dy * K + dx) * I + i, 32 per MFMA step (one step for a 3x3 window over three channels,
// five for 7x7).  The band's input rows are staged in LDS as they lie in memory, between zero
// halo columns; a lane gathers its eight values of a step two bytes at a time (the offsets
// depend on the step and the lane group only: a small table in registers).  The weights of
// the whole layer stay in registers, in the plan's operand order, which interleaves the
// output channels over the strips so that a lane ends up with 4 * NS consecutive channels
// of its pixel: a lane tile leaves as whole lines, 16 bytes per lane and store.
#include "bsp_launch.h"
#include "bsp_plan.h"
#include "bsp_tile.h"

#include <algorithm>
#include <cstdlib>

namespace {

struct FirstArgs {
  const unsigned char* X;
  unsigned char* Y;
  const float* bias;
  const unsigned char* residual;
  const unsigned char* frag;
  int32_t relu;
  int32_t B, L, J, C, O, M, N, H, K, S, ph, pw;
  int32_t BR, PR, nbands, tiles_x;
  int32_t lead;    // bytes before a staged row's first (halo) pixel: makes image column 0 dword aligned
  int32_t lpitch;  // bytes per staged row (a multiple of four)
  int32_t Kt;      // H * K * C
  int32_t rowel;   // J * C: elements of an image row
  int32_t units;   // copy units per image row
  int32_t ub;      // bytes per copy unit: 16, 4 or 2, the largest that divides a row's bytes
  int32_t halo;    // 16-bit elements of a staged row outside the image
  FastDiv d_nbands, d_tx, d_units, d_kc, d_halo;
};

template <int NS, int STEPS>
__global__ __launch_bounds__(256) void conv_first(FirstArgs a) {
  kernarg_touch<FirstArgs>();
  extern __shared__ __align__(16) unsigned char lds[];
  const int tid = threadIdx.x, lane = tid & 63, g = lane >> 4, c = lane & 15;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  // consecutive workgroups go to different XCDs: all bands of an image are given to one XCD, so
  // that the halo rows two neighbouring bands share are fetched from HBM once
  const int xcd = blockIdx.x & 7, slot_wg = blockIdx.x >> 3;
  const int grp8 = (int)fdiv((uint32_t)slot_wg, a.d_nbands), band = slot_wg - grp8 * a.nbands;
  const int n = xcd + 8 * grp8;
  if (n >= a.B) return;
  const int y0 = band * a.BR, iy0 = y0 * a.S - a.ph;
  const int data0 = a.lead + a.pw * a.C * 2;  // where image column 0 lies in a staged row

  // ---- the band's input rows, as they lie in memory: 16 bytes per lane and load where a row's
  // bytes are a multiple of 16, else dwords (an even number of elements) or 16-bit elements.
  // Four loads are in flight per lane before the first is written to LDS, and every lane
  // loads, from a row that exists (a load under a condition would be waited for on the spot,
  // one memory latency per load).
  {
    const int total = a.PR * a.units;
    const uint32_t img = (uint32_t)(n * a.L) * (uint32_t)a.rowel * 2u;
    constexpr int NB = 4;  // (eight was measured 0.8 us slower on 299-pixel rows and no faster elsewhere)
    if (a.ub == 16) {
      for (int i0 = tid; i0 < total; i0 += NB * 256) {
        u32x4_t v[NB];
        int dst[NB];
#pragma unroll
        for (int u = 0; u < NB; ++u) {
          const int idx = i0 + u * 256, ic = min(idx, total - 1);
          const int r = (int)fdiv((uint32_t)ic, a.d_units), d = ic - r * a.units;
          const int gy = iy0 + r;
          dst[u] = idx < total && (unsigned)gy < (unsigned)a.L ? r * a.lpitch + data0 + d * 16 : -1;
          v[u] = *(const u32x4_t*)(a.X + img + (uint32_t)min(max(gy, 0), a.L - 1) * (uint32_t)a.rowel * 2u + d * 16);
        }
#pragma unroll
        for (int u = 0; u < NB; ++u) {
          if (dst[u] < 0) continue;
#pragma unroll
          for (int k = 0; k < 4; ++k) *(uint32_t*)(lds + dst[u] + 4 * k) = v[u][k];  // (image column 0 is dword aligned in LDS, no more)
        }
      }
    } else {
      for (int i0 = tid; i0 < total; i0 += NB * 256) {
        uint32_t v[NB];
        int dst[NB];
#pragma unroll
        for (int u = 0; u < NB; ++u) {
          const int idx = i0 + u * 256, ic = min(idx, total - 1);
          const int r = (int)fdiv((uint32_t)ic, a.d_units), d = ic - r * a.units;
          const int gy = iy0 + r;
          dst[u] = idx < total && (unsigned)gy < (unsigned)a.L ? r * a.lpitch + data0 + d * a.ub : -1;
          const unsigned char* src = a.X + img + (uint32_t)min(max(gy, 0), a.L - 1) * (uint32_t)a.rowel * 2u;
          v[u] = a.ub == 4 ? *(const uint32_t*)(src + d * 4) : (uint32_t) * (const uint16_t*)(src + d * 2);
        }
#pragma unroll
        for (int u = 0; u < NB; ++u) {
          if (dst[u] < 0) continue;
          if (a.ub == 4)
            *(uint32_t*)(lds + dst[u]) = v[u];
          else
            *(uint16_t*)(lds + dst[u]) = (uint16_t)v[u];
        }
      }
    }
  }
  // ---- what is never copied into must read as zero: the halo columns (and the alignment
  // bytes around them) of every row, whole rows outside the image
  {
    const int hl = data0 >> 1;  // elements before image column 0
    for (int idx = tid; idx < a.PR * a.halo; idx += 256) {
      const int r = (int)fdiv((uint32_t)idx, a.d_halo), e = idx - r * a.halo;
      const int off = e < hl ? e * 2 : data0 + a.rowel * 2 + (e - hl) * 2;
      *(uint16_t*)(lds + r * a.lpitch + off) = 0;
    }
    for (int r = 0; r < a.PR; ++r) {
      if ((unsigned)(iy0 + r) < (unsigned)a.L) continue;
      for (int i = tid; i < (a.lpitch >> 2); i += 256) *(uint32_t*)(lds + r * a.lpitch + i * 4) = 0;
    }
  }

  // ---- the layer's weights, the bias of this lane's channels, the gather offsets
  u32x4_t wf[STEPS][NS];
#pragma unroll
  for (int t = 0; t < STEPS; ++t)
#pragma unroll
    for (int s = 0; s < NS; ++s) wf[t][s] = *(const u32x4_t*)(a.frag + (uint32_t)(((t * NS + s) * 64 + lane) * 16));
  const int cb = g * 4 * NS;  // this lane's first output channel
  // off[t][q]: the byte offsets of contraction indices 32 t + 8 g + 2 q (low half) and + 1 (high
  // half) from the window's first element; indices past the window read that first element
  // again (their weights are zero)
  uint32_t off[STEPS][4];
  {
    const int kc = a.K * a.C;
#pragma unroll
    for (int t = 0; t < STEPS; ++t)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        uint32_t pair = 0;
#pragma unroll
        for (int h = 0; h < 2; ++h) {
          const int k = 32 * t + 8 * g + 2 * q + h;
          const int dy = (int)fdiv((uint32_t)k, a.d_kc), rr = k - dy * kc;
          const uint32_t o = k < a.Kt ? (uint32_t)(dy * a.lpitch + rr * 2) : 0u;
          pair |= o << (16 * h);
        }
        off[t][q] = pair;
      }
  }
  __syncthreads();  // the rows are in LDS

  const int rows_out = min(a.BR, a.M - y0);
  const int ntiles = rows_out * a.tiles_x;
  for (int tile = wave; tile < ntiles; tile += 4) {
    const int r = (int)fdiv((uint32_t)tile, a.d_tx), tx = tile - r * a.tiles_x;
    const int xq = tx * 16 + c, x = min(xq, a.N - 1);  // lanes past the row's end repeat its last pixel (never stored)
    const unsigned char* win = lds + (r * a.S) * a.lpitch + a.lead + (x * a.S) * a.C * 2;
    // the accumulators start from the bias of the lane's channels (read again for every lane
    // tile, from cache: cheaper than 4 * NS registers held through the loop)
    f32x4_t acc[NS];
#pragma unroll
    for (int s = 0; s < NS; ++s) {
      acc[s] = f32x4_t{0.f, 0.f, 0.f, 0.f};
      if (a.bias) acc[s] = f32x4_t{a.bias[cb + 4 * s], a.bias[cb + 4 * s + 1], a.bias[cb + 4 * s + 2], a.bias[cb + 4 * s + 3]};
    }
#pragma unroll
    for (int t = 0; t < STEPS; ++t) {
      u32x4_t bf;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const uint32_t lo = *(const uint16_t*)(win + (off[t][q] & 0xFFFFu));
        const uint32_t hi = *(const uint16_t*)(win + (off[t][q] >> 16));
        bf[q] = lo | (hi << 16);
      }
#pragma unroll
      for (int s = 0; s < NS; ++s) acc[s] = mfma_bf16_16x16x32(wf[t][s], bf, acc[s]);
    }
    // the lane's 4 * NS channels as 16-byte pieces (bias added, rounded once)
    u32x4_t piece[NS / 2];
#pragma unroll
    for (int h = 0; h < NS / 2; ++h)
      piece[h] = u32x4_t{pack_bf16x2(acc[2 * h].x, acc[2 * h].y), pack_bf16x2(acc[2 * h].z, acc[2 * h].w),
                         pack_bf16x2(acc[2 * h + 1].x, acc[2 * h + 1].y), pack_bf16x2(acc[2 * h + 1].z, acc[2 * h + 1].w)};
    const uint32_t mine = ((uint32_t)((n * a.M + y0 + r) * a.N + xq) * (uint32_t)a.O + (uint32_t)cb) * 2u;
    auto out = [&](u32x4_t v, uint32_t dst) {
      u32x2_t l2 = {v.x, v.y}, h2 = {v.z, v.w};
      if (a.residual || a.relu) {
        u32x4_t rs = {0, 0, 0, 0};
        if (a.residual) rs = *(const u32x4_t*)(a.residual + dst);
        l2 = post_bf16x4_reg(l2, u32x2_t{rs.x, rs.y}, a.residual != nullptr, a.relu);
        h2 = post_bf16x4_reg(h2, u32x2_t{rs.z, rs.w}, a.residual != nullptr, a.relu);
      }
      // (streaming store of whole lines: no burst of dirty L2 lines is left for the end of the kernel)
      __builtin_nontemporal_store(u32x4_t{l2.x, l2.y, h2.x, h2.y}, (u32x4_t*)(a.Y + dst));
    };
    if (NS == 2) {
      // 64 bytes per pixel, four lanes of 16: a lane tile is one contiguous kilobyte
      if (xq < a.N) out(piece[0], mine);
    } else {
      // 128 bytes per pixel, four lanes of 32.  Neighbouring pixels (lanes c, c ^ 1) trade a
      // piece, so that the first store writes the even pixels whole (eight lanes of 16 bytes: a
      // line) and the second the odd ones; each lane storing its own two pieces would write
      // every line twice by halves, which the streaming store is several times slower at.
      const bool odd = c & 1;
      const u32x4_t send = odd ? piece[0] : piece[NS / 2 - 1];
      u32x4_t recv;
#pragma unroll
      for (int k = 0; k < 4; ++k)
        recv[k] = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)send[k], 0xB1, 0xF, 0xF, true);  // quad_perm [1, 0, 3, 2]
      const uint32_t line = (uint32_t)a.O * 2u;
      // even pixel: its first piece from the even lane, its second from the odd lane
      const uint32_t dst_e = (odd ? mine - line : mine) + (odd ? 16u : 0u);
      const uint32_t dst_o = (odd ? mine : mine + line) + (odd ? 16u : 0u);
      const int xe = xq & ~1;
      if (xe < a.N) out(odd ? recv : piece[0], dst_e);
      if (xe + 1 < a.N) out(odd ? piece[1] : recv, dst_o);
    }
  }
}

template <int NS, int STEPS>
int launch_first(const FirstArgs& a, dim3 grid, size_t ldsb, hipStream_t st) {
  hipLaunchKernelGGL((conv_first<NS, STEPS>), grid, dim3(256), ldsb, st, a);
  return hipGetLastError() == hipSuccess ? BSP_OK : BSP_ERR_HIP;
}

}  // namespace

int bsp_launch_first(const ConvParams& p, int dtype, const void* plan_host, hipStream_t st) {
  if (dtype != BSP_BF16 || !plan_host) return BSP_ERR_UNSUPPORTED;
  const int32_t* hdr = (const int32_t*)plan_host;
  if (hdr[BSP_PLAN_MAGIC_W] != BSP_PLAN_MAGIC || hdr[BSP_PLAN_VERSION_W] != BSP_PLAN_VERSION ||
      hdr[BSP_PLAN_O_W] != p.O || hdr[BSP_PLAN_I_W] != p.I || hdr[BSP_PLAN_H_W] != p.H ||
      hdr[BSP_PLAN_K_W] != p.K || hdr[BSP_PLAN_DTYPE_W] != dtype || hdr[BSP_PLAN_OFF_FIRST_W] == 0)
    return BSP_ERR_UNSUPPORTED;
  const int32_t* fs = hdr + hdr[BSP_PLAN_OFF_FIRST_W];
  const int NS = fs[BSP_FIRST_NS_W], steps = fs[BSP_FIRST_STEPS_W];
  if ((NS != 2 && NS != 4) || (steps != 1 && steps != 5)) return BSP_ERR_UNSUPPORTED;  // (the instances compiled)
  if (p.I > 4 || p.sh != p.sw || p.sh < 1 || p.sh > 4 || p.ph < 0 || p.pw < 0 || p.ph > 7 || p.pw > 7)
    return BSP_ERR_UNSUPPORTED;
  if ((int64_t)p.B * p.L * p.J * p.I * 2 >= (1ll << 31) || (int64_t)p.P * p.O * 2 >= (1ll << 31))
    return BSP_ERR_UNSUPPORTED;
  FirstArgs a{};
  a.X = (const unsigned char*)p.X;
  a.Y = (unsigned char*)p.Y;
  a.bias = p.bias;
  a.residual = (const unsigned char*)p.residual;
  a.frag = (const unsigned char*)(p.plan + hdr[BSP_PLAN_OFF_FIRST_W] + fs[BSP_FIRST_OFF_FRAG_W]);
  a.relu = p.relu;
  a.B = p.B;
  a.L = p.L;
  a.J = p.J;
  a.C = p.I;
  a.O = p.O;
  a.M = p.M;
  a.N = p.N;
  a.H = p.H;
  a.K = p.K;
  a.S = p.sh;
  a.ph = p.ph;
  a.pw = p.pw;
  // rows per band (measured on the three networks' first layers: larger bands stage fewer
  // halo rows, smaller ones give the chip more workgroups; a five-step layer holds its weights
  // in 80 registers, three workgroups per CU, and does best with few, large workgroups; a
  // one-step layer at stride 2 reads twice the rows it writes and does best with small ones)
  a.BR = steps == 5 ? 7 : (p.sh > 1 ? 2 : 4);
#ifdef BSP_ROWS_TUNE
  if (const char* e = getenv("BSP_FIRST_BR")) a.BR = atoi(e);
#endif
  a.PR = (a.BR - 1) * a.S + p.H;
  a.nbands = (p.M + a.BR - 1) / a.BR;
  a.tiles_x = (p.N + 15) / 16;
  a.Kt = fs[BSP_FIRST_KT_W];
  a.rowel = p.J * p.I;
  a.ub = a.rowel % 8 == 0 ? 16 : (a.rowel % 2 == 0 ? 4 : 2);
  a.units = a.rowel * 2 / a.ub;
  a.lead = (4 - (p.pw * p.I * 2) % 4) % 4;
  // a staged row reaches as far as the last window does
  const int reach = std::max(p.J + 2 * p.pw, (p.N - 1) * a.S + p.K);
  a.lpitch = (a.lead + reach * p.I * 2 + 3) & ~3;
  a.halo = (a.lpitch - a.rowel * 2) / 2;
  const int64_t ldsb = (int64_t)a.PR * a.lpitch;
  if (ldsb > 64 * 1024 || (int64_t)(p.H - 1) * a.lpitch + p.K * p.I * 2 >= 65536) return BSP_ERR_UNSUPPORTED;
  a.d_nbands = make_fastdiv((uint32_t)a.nbands);
  a.d_tx = make_fastdiv((uint32_t)a.tiles_x);
  a.d_units = make_fastdiv((uint32_t)a.units);
  a.d_kc = make_fastdiv((uint32_t)(p.K * p.I));
  a.d_halo = make_fastdiv((uint32_t)std::max(a.halo, 1));
  // multiply-high divisions are exact while dividend * divisor < 2^32
  const int64_t nwg = (int64_t)((p.B + 7) / 8) * a.nbands * 8;  // eight images at a time, one per XCD
  if (nwg * a.nbands >= (1ll << 32) || nwg >= (1ll << 31) || (int64_t)(a.PR * a.units + 2048) * a.units >= (1ll << 32) ||
      (int64_t)a.PR * a.halo * std::max(a.halo, 1) >= (1ll << 32))
    return BSP_ERR_UNSUPPORTED;
  dim3 grid((unsigned)nwg);
  if (NS == 4) return steps == 1 ? launch_first<4, 1>(a, grid, (size_t)ldsb, st) : launch_first<4, 5>(a, grid, (size_t)ldsb, st);
  return steps == 1 ? launch_first<2, 1>(a, grid, (size_t)ldsb, st) : launch_first<2, 5>(a, grid, (size_t)ldsb, st);
}
