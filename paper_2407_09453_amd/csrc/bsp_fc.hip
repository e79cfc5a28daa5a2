// Fully-connected layers with few output rows (batch <= 64): weight streaming.
//
// Such a layer is bound by reading its weights once from HBM, so only the kept
// blocks are read, straight from the compressed block rows (every 8x8 bf16
// block is one aligned 128-byte run): half the blocks zeroed means half the
// bytes moved (paper Section I: smaller footprint, faster communication, fewer
// operations).  One workgroup owns one strip of 16 output channels; its eight
// waves split the strip's list of kept 8-channel chunks, each wave gathering
// the matching activations (the whole X is small and stays in L2), and the
// partial 16 x batch tiles are summed through LDS before the bias is
// added and the result rounded once.  A GEMM is the 1x1 case of the
// convolution (Section III), so the same kernel serves 1x1 convolutions whose
// batch x height x width is small.
#include "bsp_launch.h"
#include "bsp_tile.h"

namespace {


// Index-table entries of one batch of steps: for this lane's group, the chunk's
// channel offset in X and the payload offsets of the block(s) it reads, or -1.
template <int U>
struct FcTab {
  int xoff[U], w0[U], w1[U];
};

template <int BO, int BI, int NT, int kFcWaves>
__global__ __launch_bounds__(kFcWaves * 64) void fc_stream_bf16(ConvParams p) {
  constexpr int U = NT <= 2 ? 4 : 2;  // MFMA steps whose loads are issued together
  __shared__ f32x4_t red[kFcWaves][NT][64];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int jn = lane & 15, g = lane >> 4;
  const int strip = blockIdx.x;
  const PlanView pv = plan_view(p.plan);
  const int c0 = pv.strip_ptr[strip], c1 = pv.strip_ptr[strip + 1];
  const int nsteps = (c1 - c0 + 3) >> 2;  // four chunks per MFMA, one per 16-lane group
  const int per = (nsteps + kFcWaves - 1) / kFcWaves;
  const int sa = wave * per, sb = min(sa + per, nsteps);

  const uint16_t* X = (const uint16_t*)p.X;
  const uint16_t* Wp = (const uint16_t*)p.payload;
  // which block of the (strip, chunk) cell this lane's output channel lies in
  const int sub = BI == 4 ? 0 : jn / BO, row = jn % BO;

  f32x4_t acc[NT];
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) acc[nt] = f32x4_t{0.f, 0.f, 0.f, 0.f};
  int xrow[NT];  // element offset of this lane's activation row, or -1 past the batch
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) xrow[nt] = nt * 16 + jn < p.P ? (nt * 16 + jn) * p.I : -1;

  // software pipeline over batches of U steps: index tables four batches ahead,
  // weight and activation loads one batch ahead, MFMAs now
  auto tables = [&](int s, FcTab<U>& t) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int ce = c0 + 4 * (s + u) + g;
      t.xoff[u] = -1;
      t.w0[u] = -1;
      t.w1[u] = -1;
      if (s + u < sb && ce < c1) {
        t.xoff[u] = pv.chunk_xc[ce] * BSP_CHUNK;
        if constexpr (BI >= 8) {
          t.w0[u] = pv.chunk_src[ce * BSP_MAXSUB + sub];
        } else {
          t.w0[u] = pv.chunk_src[ce * BSP_MAXSUB + 0];
          t.w1[u] = pv.chunk_src[ce * BSP_MAXSUB + 1];
        }
      }
    }
  };
  auto fetch = [&](const FcTab<U>& t, u32x4_t (&a)[U], u32x4_t (&b)[U][NT]) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
      a[u] = u32x4_t{0u, 0u, 0u, 0u};
      if constexpr (BI >= 8) {
        if (t.w0[u] >= 0) a[u] = *(const u32x4_t*)(Wp + t.w0[u] + row * BI);
      } else {
        if (t.w0[u] >= 0) {
          const u32x2_t lo = *(const u32x2_t*)(Wp + t.w0[u] + row * BI);
          a[u].x = lo.x;
          a[u].y = lo.y;
        }
        if (t.w1[u] >= 0) {
          const u32x2_t hi = *(const u32x2_t*)(Wp + t.w1[u] + row * BI);
          a[u].z = hi.x;
          a[u].w = hi.y;
        }
      }
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) {
        b[u][nt] = u32x4_t{0u, 0u, 0u, 0u};
        if (t.xoff[u] >= 0 && xrow[nt] >= 0) b[u][nt] = *(const u32x4_t*)(X + xrow[nt] + t.xoff[u]);
      }
    }
  };
  auto mma = [&](const u32x4_t (&a)[U], const u32x4_t (&b)[U][NT]) {
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) acc[nt] = mfma_bf16_16x16x32(a[u], b[u][nt], acc[nt]);
  };

  if (sa < sb) {
    FcTab<U> tab[4];
    u32x4_t a[2][U], b[2][U][NT];
#pragma unroll
    for (int j = 0; j < 4; ++j) tables(sa + j * U, tab[j]);
    fetch(tab[0], a[0], b[0]);
    for (int s = sa; s < sb; s += 4 * U) {
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        fetch(tab[(j + 1) & 3], a[(j + 1) & 1], b[(j + 1) & 1]);  // batch s + (j+1)U
        tables(s + (j + 4) * U, tab[j]);                          // four batches ahead
        mma(a[j & 1], b[j & 1]);                                  // batch s + jU (zeros past the end)
      }
    }
  }

  // sum the partial tiles; wave 0 finishes: + bias, one rounding, store
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) red[wave][nt][lane] = acc[nt];
  __syncthreads();
  if (wave != 0) return;
  const int ch = strip * BSP_STRIP + 4 * g;  // lane holds channels ch..ch+3 of batch row jn
  float bv[4];
#pragma unroll
  for (int r = 0; r < 4; ++r) bv[r] = (p.bias && ch + r < p.O) ? p.bias[ch + r] : 0.f;
  uint16_t* Y = (uint16_t*)p.Y;
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) {
    f32x4_t v = red[0][nt][lane];
#pragma unroll
    for (int w = 1; w < kFcWaves; ++w) v += red[w][nt][lane];
    const int pix = nt * 16 + jn;
    if (pix >= p.P) continue;
    u32x2_t o;
    o.x = pack_bf16x2(v[0] + bv[0], v[1] + bv[1]);
    o.y = pack_bf16x2(v[2] + bv[2], v[3] + bv[3]);
    uint16_t* yp = Y + (int64_t)pix * p.O + ch;
    if (p.residual || p.relu)
      o = post_bf16x4(o, p.residual ? (const uint16_t*)p.residual + (int64_t)pix * p.O + ch : nullptr,
                      p.O - ch, (p.O % 4) == 0 && ch + 3 < p.O, p.relu);
    if ((p.O % 4) == 0 && ch + 3 < p.O) {
      *(u32x2_t*)yp = o;
    } else {
      if (ch + 0 < p.O) yp[0] = (uint16_t)(o.x & 0xFFFF);
      if (ch + 1 < p.O) yp[1] = (uint16_t)(o.x >> 16);
      if (ch + 2 < p.O) yp[2] = (uint16_t)(o.y & 0xFFFF);
      if (ch + 3 < p.O) yp[3] = (uint16_t)(o.y >> 16);
    }
  }
}

template <int BO, int BI>
int launch_gran(const ConvParams& p, hipStream_t st) {
  const int nstrips = (p.O + BSP_STRIP - 1) / BSP_STRIP;
  dim3 grid((unsigned)nstrips);
  const int nt = (p.P + 15) / 16;
  switch (nt) {
    case 1: hipLaunchKernelGGL((fc_stream_bf16<BO, BI, 1, 8>), grid, dim3(512), 0, st, p); break;
    case 2: hipLaunchKernelGGL((fc_stream_bf16<BO, BI, 2, 8>), grid, dim3(512), 0, st, p); break;
    case 3:
    case 4: hipLaunchKernelGGL((fc_stream_bf16<BO, BI, 4, 8>), grid, dim3(512), 0, st, p); break;
    default: return BSP_ERR_UNSUPPORTED;
  }
  return hipGetLastError() == hipSuccess ? BSP_OK : BSP_ERR_HIP;
}

}  // namespace

// 1x1, stride 1, no padding, bf16, at most 64 output pixels in all, I a multiple of 8.
int bsp_launch_fc_stream(const ConvParams& p, int dtype, int bo, int bi, hipStream_t st) {
  if (dtype != BSP_BF16 || p.H != 1 || p.K != 1 || p.sh != 1 || p.sw != 1 || p.ph != 0 ||
      p.pw != 0 || p.P > 64 || (p.I % 8) != 0 || (int64_t)p.P * p.I > 0x7FFFFFFF)
    return BSP_ERR_UNSUPPORTED;
  if (bo == 8 && bi == 8) return launch_gran<8, 8>(p, st);
  if (bo == 4 && bi == 16) return launch_gran<4, 16>(p, st);
  if (bo == 16 && bi == 4) return launch_gran<16, 4>(p, st);
  return BSP_ERR_UNSUPPORTED;
}

// ---------------------------------------------------------------------------------------
// 8x8 blocks: streaming the compressed block rows themselves.
//
// The kept blocks of a block row lie one after the other in the payload (128 bytes each), so
// a block row is one contiguous stream and col_idx says which eight input channels each
// block multiplies (paper Section III: compressed block row storage).  One workgroup owns a
// block row (eight output channels); its eight waves split the row's kept blocks and read
// them in order, four blocks (512 contiguous bytes) per MFMA step: lane group g takes block
// n + g, lanes 0-7 of the group one 16-byte row each.  The MFMA's rows 8-15 stay zero: the
// layer is bound by reading the weights once, not by the matrix cores, and in exchange there
// is no table to look up but four column indices per step.  Partial tiles are summed through
// LDS as above.
namespace {

template <int NT>
__global__ __launch_bounds__(512) void fc_rows_bf16(ConvParams p) {
  constexpr int kWaves = 8;
  constexpr int U = NT <= 2 ? 4 : 2;  // MFMA steps whose loads are issued together
  __shared__ f32x4_t red[kWaves][NT][32];  // only lane groups 0 and 1 hold the eight real rows
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int jn = lane & 15, g = lane >> 4;
  const int brow = blockIdx.x;
  const int n0 = p.row_ptr[brow], n1 = p.row_ptr[brow + 1];
  const int nsteps = (n1 - n0 + 3) >> 2;
  const int per = (nsteps + kWaves - 1) / kWaves;
  const int sa = wave * per, sb = min(sa + per, nsteps);

  const uint16_t* X = (const uint16_t*)p.X;
  const uint16_t* Wp = (const uint16_t*)p.payload;
  f32x4_t acc[NT];
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) acc[nt] = f32x4_t{0.f, 0.f, 0.f, 0.f};
  int xrow[NT];  // element offset of this lane's activation row, or -1 past the batch
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) xrow[nt] = nt * 16 + jn < p.P ? (nt * 16 + jn) * p.I : -1;

  // block of step s for this lane's group, or -1
  auto block_of = [&](int s) {
    const int n = n0 + 4 * s + g;
    return (s < sb && n < n1) ? n : -1;
  };
  auto columns = [&](int s, int (&col)[U]) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int n = block_of(s + u);
      col[u] = n >= 0 ? p.col_idx[n] : -1;
    }
  };
  auto fetch = [&](int s, const int (&col)[U], u32x4_t (&a)[U], u32x4_t (&b)[U][NT]) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int n = block_of(s + u);
      a[u] = u32x4_t{0u, 0u, 0u, 0u};
      if (n >= 0 && jn < 8) a[u] = *(const u32x4_t*)(Wp + (int64_t)n * 64 + jn * 8);
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) {
        b[u][nt] = u32x4_t{0u, 0u, 0u, 0u};
        if (col[u] >= 0 && xrow[nt] >= 0) b[u][nt] = *(const u32x4_t*)(X + xrow[nt] + col[u] * BSP_CHUNK);
      }
    }
  };
  auto mma = [&](const u32x4_t (&a)[U], const u32x4_t (&b)[U][NT]) {
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) acc[nt] = mfma_bf16_16x16x32(a[u], b[u][nt], acc[nt]);
  };

  if (sa < sb) {
    // software pipeline over batches of U steps: column indices two batches ahead, block and
    // activation loads one batch ahead, MFMAs now
    int col[2][U];
    u32x4_t a[2][U], b[2][U][NT];
    columns(sa, col[0]);
    columns(sa + U, col[1]);
    fetch(sa, col[0], a[0], b[0]);
    for (int s = sa; s < sb; s += 2 * U) {
      fetch(s + U, col[1], a[1], b[1]);
      columns(s + 2 * U, col[0]);
      mma(a[0], b[0]);
      fetch(s + 2 * U, col[0], a[0], b[0]);
      columns(s + 3 * U, col[1]);
      mma(a[1], b[1]);
    }
  }

  // sum the partial tiles; wave 0 finishes: + bias, one rounding, store.  Lane (g, jn) holds
  // rows 4g..4g+3 of batch row jn: groups 0 and 1 are the block row's eight output channels
  if (g < 2) {
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) red[wave][nt][lane] = acc[nt];
  }
  __syncthreads();
  if (wave != 0 || g >= 2) return;
  const int ch = brow * 8 + 4 * g;
  float bv[4];
#pragma unroll
  for (int r = 0; r < 4; ++r) bv[r] = (p.bias && ch + r < p.O) ? p.bias[ch + r] : 0.f;
  uint16_t* Y = (uint16_t*)p.Y;
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) {
    f32x4_t v = red[0][nt][lane];
#pragma unroll
    for (int w = 1; w < kWaves; ++w) v += red[w][nt][lane];
    const int pix = nt * 16 + jn;
    if (pix >= p.P) continue;
    u32x2_t o;
    o.x = pack_bf16x2(v[0] + bv[0], v[1] + bv[1]);
    o.y = pack_bf16x2(v[2] + bv[2], v[3] + bv[3]);
    uint16_t* yp = Y + (int64_t)pix * p.O + ch;
    const bool vec = (p.O % 4) == 0 && ch + 3 < p.O;
    if (p.residual || p.relu)
      o = post_bf16x4(o, p.residual ? (const uint16_t*)p.residual + (int64_t)pix * p.O + ch : nullptr,
                      p.O - ch, vec, p.relu);
    if (vec) {
      *(u32x2_t*)yp = o;
    } else {
      if (ch + 0 < p.O) yp[0] = (uint16_t)(o.x & 0xFFFF);
      if (ch + 1 < p.O) yp[1] = (uint16_t)(o.x >> 16);
      if (ch + 2 < p.O) yp[2] = (uint16_t)(o.y & 0xFFFF);
      if (ch + 3 < p.O) yp[3] = (uint16_t)(o.y >> 16);
    }
  }
}

}  // namespace

// 8x8 blocks, 1x1, stride 1, no padding, bf16, at most 64 output pixels in all, I a multiple
// of 8, and enough block rows to fill the chip.
int bsp_launch_fc_rows(const ConvParams& p, int dtype, int bo, int bi, int64_t nnzb, hipStream_t st) {
  if (dtype != BSP_BF16 || bo != 8 || bi != 8 || p.H != 1 || p.K != 1 || p.sh != 1 || p.sw != 1 ||
      p.ph != 0 || p.pw != 0 || p.P > 64 || (p.I % 8) != 0 || (int64_t)p.P * p.I > 0x7FFFFFFF ||
      !p.row_ptr || !p.col_idx)
    return BSP_ERR_UNSUPPORTED;
  const int nbr = (p.O + 7) / 8;
  if (nbr < 128) return BSP_ERR_UNSUPPORTED;  // too few block rows: the strip kernel spreads better
  // An MFMA here has eight real rows, so the activations (gathered from L2) are fetched twice
  // as often per output as in the strip kernel; that pays only while the weight stream is
  // thin enough, i.e. for sparse layers.  nnzb comes with the launch (host value).
  if (nnzb * 10 > (int64_t)nbr * (p.I / 8) * 6) return BSP_ERR_UNSUPPORTED;
  dim3 grid((unsigned)nbr);
  const int nt = (p.P + 15) / 16;
  switch (nt) {
    case 1: hipLaunchKernelGGL((fc_rows_bf16<1>), grid, dim3(512), 0, st, p); break;
    case 2: hipLaunchKernelGGL((fc_rows_bf16<2>), grid, dim3(512), 0, st, p); break;
    case 3:
    case 4: hipLaunchKernelGGL((fc_rows_bf16<4>), grid, dim3(512), 0, st, p); break;
    default: return BSP_ERR_UNSUPPORTED;
  }
  return hipGetLastError() == hipSuccess ? BSP_OK : BSP_ERR_HIP;
}
