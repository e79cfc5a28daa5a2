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
#include <algorithm>
#ifdef BSP_ROWS_TUNE
#include <cstdlib>
#endif
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
  kernarg_touch<ConvParams>();
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
// 8x8 blocks: activations resident in LDS, compressed block rows streamed past them.
//
// The kernel above fetches, for every kept chunk, the eight input channels it multiplies
// from global memory; the dependent look-up (col_idx, then X) and the L2 traffic of those
// gathers, not the weight stream, is what holds it back.  Here a workgroup first copies a
// whole range of input channels of X (all of it when it fits: [pixels][channels] bf16 within
// 150 KB) into LDS, global -> LDS without passing registers, and then streams compressed
// block rows past it: a wave reads a row's kept blocks in storage order (512 contiguous bytes
// per MFMA step, lanes 0-7 of each lane group one 16-byte block row each), col_idx says which
// eight channels of the LDS image each block multiplies.  The weights are read once
// (paper Section I: half the blocks kept, half the bytes moved); X is read once per workgroup
// from L2 instead of once per block row.
//
// Work split: the input channels are cut into nseg ranges (one when X fits), the block rows
// into groups; a workgroup owns (range, group).  With at least eight rows in a group a wave
// owns whole rows; with fewer, KP = 8 / rows waves share a row's blocks and their partial tiles
// are summed through LDS.  With nseg > 1 a workgroup's sums are partial: they go to a scratch
// array [nseg][pixels][O] of floats and a second kernel adds the ranges in order, adds the
// bias, rounds once and applies the fused epilogue.  A row's blocks inside a channel range
// are one contiguous run of its compressed row (col_idx ascends); its ends are found by a
// wave-wide search of col_idx, sixty-four probes at a time.
namespace {

typedef __attribute__((address_space(1))) const void* gptr_t;
typedef __attribute__((address_space(3))) void* lptr_t;

struct FcXArgs {
  const unsigned char* X;
  const unsigned char* W;
  const int32_t* row_ptr;
  const int32_t* col_idx;
  const float* bias;
  const uint16_t* residual;
  uint16_t* Y;
  float* part;       // [nseg][P][O] when nseg > 1
  int32_t P, I, O, nbr, relu;
  int32_t segc;      // input channels per range, a multiple of 8
  int32_t nseg, ngroups, rpg;  // ranges, row groups, block rows per group
  int32_t kp, lkp;   // waves that share a row (1, 2, 4 or 8) and its log2
  int32_t pitch;     // bytes between the pixels of the LDS image (an odd number of 16-byte slots)
  int32_t red_off;   // where the partial tiles are summed
  int32_t rng_off;   // where the rows' runs inside the channel range are kept
};

// First n in [a, b) with col[n] >= cb, or b: col ascends on [a, b); a, b, cb uniform.
__device__ __forceinline__ int fcx_lower_bound(const int32_t* col, int a, int b, int cb, int lane) {
  while (b - a > 64) {
    const int step = (b - a + 63) >> 6;
    const int n = a + lane * step;
    const bool below = n < b && col[n] < cb;
    const int cnt = __popcll(__ballot(below));  // the probes below cb are the first cnt lanes
    if (cnt == 0) return a;
    const int na = a + (cnt - 1) * step + 1;
    b = min(b, a + cnt * step);
    a = na;
  }
  const int n = a + lane;
  const bool below = n < b && col[n] < cb;
  return a + __popcll(__ballot(below));
}

template <int NT>
__global__ __launch_bounds__(1024) void fc_xlds_bf16(FcXArgs q) {
  kernarg_touch<FcXArgs>();
  constexpr int R = 8;  // MFMA steps of weights in flight per wave
  extern __shared__ __align__(16) unsigned char lds[];
  const int tid = threadIdx.x, lane = tid & 63, jn = lane & 15, g = lane >> 4;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  // consecutive workgroups (different XCDs) take different channel ranges of one row group
  const int seg = blockIdx.x % q.nseg, grp = blockIdx.x / q.nseg;
  const int c0 = seg * q.segc, cw = min(q.segc, q.I - c0);  // this range's channels
  const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)lds;

  const int rows_here = min(q.rpg, q.nbr - grp * q.rpg);
  const int cb0 = c0 >> 3, cb1 = (c0 + cw) >> 3;  // block columns of the range
  int* rng = (int*)(lds + q.rng_off);             // with several ranges: [row of the group][first, end)
  // ---- X[:, c0 : c0 + cw] -> LDS: a request is 64 pieces of 16 bytes of one pixel.  With
  // several ranges the first half of the waves look the rows' runs up meanwhile and the other
  // half copy (a wave that did both would wait for its copies before it could use a probe).
  const bool split = q.nseg > 1;
  const int nw = (int)(blockDim.x >> 6), hw = nw >> 1;  // eight waves, or sixteen that own rows
  if (!split || wave >= hw) {
    const int ppx = cw >> 3;                 // pieces per pixel
    const int rpp = (ppx + 63) >> 6;         // requests per pixel
    for (int rq = split ? wave - hw : wave; rq < q.P * rpp; rq += split ? hw : nw) {
      const int px = rq / rpp, piece = (rq - px * rpp) * 64 + lane;
      if (piece < ppx)
        __builtin_amdgcn_global_load_lds((gptr_t)(q.X + ((int64_t)px * q.I + c0) * 2 + piece * 16),
                                         (lptr_t)(uintptr_t)(lds0 + (uint32_t)(px * q.pitch + (piece - lane) * 16)),
                                         16, 0, 0);
    }
  } else {
    for (int r = wave; r < rows_here; r += hw) {
      const int brow = grp * q.rpg + r;
      const int a = q.row_ptr[brow], b = q.row_ptr[brow + 1];
      const int n0 = seg > 0 ? fcx_lower_bound(q.col_idx, a, b, cb0, lane) : a;
      const int n1 = seg + 1 < q.nseg ? fcx_lower_bound(q.col_idx, n0, b, cb1, lane) : b;
      if (lane == 0) {
        rng[2 * r] = n0;
        rng[2 * r + 1] = n1;
      }
    }
  }

  // ---- this wave's share: item = (row of the group, part of the row)
  const int row_l = wave >> q.lkp, part = wave & (q.kp - 1);
  const int nitems = q.kp > 1 ? 1 : (rows_here - wave + nw - 1) / nw;  // rows wave, wave + nw, ... when a wave owns rows

  f32x4_t acc[NT];
  const uint32_t xlane = (uint32_t)jn * (uint32_t)q.pitch;
  __builtin_amdgcn_s_waitcnt(0);
  __syncthreads();  // the range is in LDS

  for (int it = 0; it < nitems; ++it) {
    const int rl = q.kp > 1 ? row_l : wave + nw * it;
    const bool real = rl < rows_here;
    const int brow = grp * q.rpg + (real ? rl : 0);
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) acc[nt] = f32x4_t{0.f, 0.f, 0.f, 0.f};
    int n0 = 0, n1 = 0;
    if (real) {
      n0 = __builtin_amdgcn_readfirstlane(split ? rng[2 * rl] : q.row_ptr[brow]);
      n1 = __builtin_amdgcn_readfirstlane(split ? rng[2 * rl + 1] : q.row_ptr[brow + 1]);
      if (q.kp > 1) {  // this wave's part of the row's steps
        const int steps = (n1 - n0 + 3) >> 2, per = (steps + q.kp - 1) >> q.lkp;
        const int sa = n0 + 4 * part * per;
        n1 = min(n1, sa + 4 * per);
        n0 = min(sa, n1);
      }
    }
    const int nsteps = (n1 - n0 + 3) >> 2;
    // ring of R steps: block rows (lanes 0-7 of a group; lanes 8-15 repeat them and drop them) and
    // the block's column.  Every lane loads at every step, past the row's end the row's last
    // block again (dropped at its use): with the same loads in every pass the wait before a
    // step is for that step's slot alone.
    if (nsteps > 0) {
      u32x4_t wa[R];
      int wc[R];
      const int nlast = n1 - 1;
      const unsigned char* wl = q.W + (jn & 7) * 16;
      auto fetch = [&](int d, int t) {
        const int n = min(n0 + 4 * t + g, nlast);
        wc[d] = q.col_idx[n];
        wa[d] = *(const u32x4_t*)(wl + (int64_t)n * 128);
      };
      // (the barriers keep the loads in slot order: the wait before a step counts on it)
#pragma unroll
      for (int d = 0; d < R; ++d) {
        fetch(d, d);
        __builtin_amdgcn_sched_barrier(0);
      }
      for (int t0 = 0; t0 < nsteps; t0 += R) {
#pragma unroll
        for (int d = 0; d < R; ++d) {
          if (t0 + d < nsteps) {
            const bool keep = jn < 8 && n0 + 4 * (t0 + d) + g < n1;
            const uint32_t xo = xlane + (uint32_t)(wc[d] * 8 - c0) * 2u;
            u32x4_t b[NT];
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) b[nt] = *(const u32x4_t*)(lds + xo + (uint32_t)(nt * 16 * q.pitch));
            const u32x4_t a = keep ? wa[d] : u32x4_t{0u, 0u, 0u, 0u};
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) acc[nt] = mfma_bf16_16x16x32(a, b[nt], acc[nt]);
          }
          __builtin_amdgcn_sched_barrier(0);
          fetch(d, t0 + d + R);
          __builtin_amdgcn_sched_barrier(0);
        }
      }
    }

    // ---- the row's tile: rows 0-7 of the MFMA tile are its eight channels (lane groups 0, 1)
    if (q.kp > 1) {
      f32x4_t* red = (f32x4_t*)(lds + q.red_off);
      if (g < 2) {
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) red[(wave * NT + nt) * 32 + lane] = acc[nt];
      }
      __syncthreads();
      if (part == 0 && g < 2) {
        for (int k = 1; k < q.kp; ++k)
#pragma unroll
          for (int nt = 0; nt < NT; ++nt) acc[nt] += red[((wave + k) * NT + nt) * 32 + lane];
      }
    }
    if (!real || part != 0 || g >= 2) continue;
    const int ch = brow * 8 + 4 * g;
    const bool vec = (q.O % 4) == 0 && ch + 3 < q.O;
    if (q.nseg > 1) {
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) {
        const int pix = nt * 16 + jn;
        if (pix >= q.P) continue;
        float* pp = q.part + ((int64_t)seg * q.P + pix) * q.O + ch;
        if (vec) {
          *(f32x4_t*)pp = acc[nt];
        } else {
#pragma unroll
          for (int r = 0; r < 4; ++r)
            if (ch + r < q.O) pp[r] = acc[nt][r];
        }
      }
      continue;
    }
    float bv[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) bv[r] = (q.bias && ch + r < q.O) ? q.bias[ch + r] : 0.f;
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
      const int pix = nt * 16 + jn;
      if (pix >= q.P) continue;
      const f32x4_t v = acc[nt];
      u32x2_t o;
      o.x = pack_bf16x2(v[0] + bv[0], v[1] + bv[1]);
      o.y = pack_bf16x2(v[2] + bv[2], v[3] + bv[3]);
      uint16_t* yp = q.Y + (int64_t)pix * q.O + ch;
      if (q.residual || q.relu)
        o = post_bf16x4(o, q.residual ? q.residual + (int64_t)pix * q.O + ch : nullptr, q.O - ch, vec, q.relu);
      if (vec) {
        *(u32x2_t*)yp = o;
      } else {
        if (ch + 0 < q.O) yp[0] = (uint16_t)(o.x & 0xFFFF);
        if (ch + 1 < q.O) yp[1] = (uint16_t)(o.x >> 16);
        if (ch + 2 < q.O) yp[2] = (uint16_t)(o.y & 0xFFFF);
        if (ch + 3 < q.O) yp[3] = (uint16_t)(o.y >> 16);
      }
    }
  }
}

// Y[pix][ch] = epilogue(sum over the channel ranges, in order, of part[range][pix][ch] + bias);
// a thread takes four consecutive channels when O is a multiple of four, one otherwise.
template <int V>
__global__ __launch_bounds__(256) void fc_xlds_sum(FcXArgs q) {
  const int64_t n = (int64_t)q.P * q.O;
  const int64_t i = ((int64_t)blockIdx.x * 256 + threadIdx.x) * V;  // (pixel, channel)
  if (i >= n) return;
  const int ch = (int)(i % q.O);
  float v[V];
#pragma unroll
  for (int k = 0; k < V; ++k) v[k] = 0.f;
  for (int s0 = 0; s0 < q.nseg; s0 += 8) {  // eight ranges' loads in flight together
    float t[8][V];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int s = min(s0 + u, q.nseg - 1);
      if (V == 4) {
        const f32x4_t w = *(const f32x4_t*)(q.part + (int64_t)s * n + i);
#pragma unroll
        for (int k = 0; k < V; ++k) t[u][k] = w[k];
      } else {
        t[u][0] = q.part[(int64_t)s * n + i];
      }
    }
#pragma unroll
    for (int u = 0; u < 8; ++u)
      if (s0 + u < q.nseg) {
#pragma unroll
        for (int k = 0; k < V; ++k) v[k] += t[u][k];
      }
  }
  uint16_t o[V];
#pragma unroll
  for (int k = 0; k < V; ++k) {
    float f = bf16_bits_to_f32(f32_to_bf16_rne(v[k] + (q.bias ? q.bias[ch + k] : 0.f)));
    if (q.residual) f += bf16_bits_to_f32(q.residual[i + k]);
    if (q.relu) f = fmaxf(f, 0.f);
    o[k] = f32_to_bf16_rne(f);
  }
  if (V == 4) {
    *(u32x2_t*)(q.Y + i) = u32x2_t{(uint32_t)o[0] | ((uint32_t)o[1] << 16), (uint32_t)o[2] | ((uint32_t)o[3] << 16)};
  } else {
    q.Y[i] = o[0];
  }
}

constexpr int kFcxLds = 150 * 1024;

}  // namespace

// 8x8 blocks, 1x1, stride 1, no padding, bf16, at most 64 output pixels, I a multiple of 8.
// `scratch` holds scratch_bytes for the partial sums of layers whose X does not fit LDS in one
// piece; BSP_ERR_CAPACITY (nothing launched) says how much is needed through *need.
int bsp_launch_fc_xlds(const ConvParams& p, int dtype, int bo, int bi, float* scratch, int64_t scratch_bytes,
                       int64_t* need, hipStream_t st) {
  if (need) *need = 0;
  if (dtype != BSP_BF16 || bo != 8 || bi != 8 || p.H != 1 || p.K != 1 || p.sh != 1 || p.sw != 1 ||
      p.ph != 0 || p.pw != 0 || p.P > 64 || p.P < 1 || (p.I % 8) != 0 || (int64_t)p.P * p.I * 2 >= (1ll << 31) ||
      !p.row_ptr || !p.col_idx)
    return BSP_ERR_UNSUPPORTED;
  const int NT = (p.P + 15) / 16 == 3 ? 4 : (p.P + 15) / 16;
  const int nbr = (p.O + 7) / 8;
  FcXArgs q{};
  // channel ranges: all of X when [NT * 16][I] bf16 (plus padding and the summing area) fits
  const int red_bytes = 8 * NT * 32 * 16;
  const int cap = ((kFcxLds - red_bytes) / (NT * 16) - 32) / 2 / 8 * 8;  // channels per range at most
  if (cap < 64) return BSP_ERR_UNSUPPORTED;
  q.nseg = (p.I + cap - 1) / cap;
  if (q.nseg > 1) q.nseg = (q.nseg + 7) / 8 * 8;  // one range per XCD, or a multiple
#ifdef BSP_ROWS_TUNE
  if (const char* e = std::getenv("BSP_FCX_NSEG")) q.nseg = std::max(q.nseg, std::atoi(e));
#endif
  q.segc = ((p.I + q.nseg - 1) / q.nseg + 7) / 8 * 8;
  q.nseg = (p.I + q.segc - 1) / q.segc;
  q.pitch = q.segc * 2 + ((q.segc / 8) % 2 == 0 ? 16 : 32);
  q.red_off = NT * 16 * q.pitch;
  q.rng_off = q.red_off + red_bytes;
  // block rows per workgroup: about one workgroup per CU; fewer than eight rows are shared by
  // 8 / rows waves each
  int rpg = (int)(((int64_t)nbr * q.nseg + 255) / 256);
  if (rpg >= 8) {
    q.kp = 1;
  } else {
    rpg = rpg >= 4 ? 4 : rpg >= 2 ? 2 : 1;
    q.kp = 8 / rpg;
  }
  q.lkp = q.kp == 8 ? 3 : q.kp == 4 ? 2 : q.kp == 2 ? 1 : 0;
  rpg = std::min(rpg, 512);  // (their runs are kept in 4 KB of LDS)
  q.rpg = rpg;
  const size_t ldsb = (size_t)q.rng_off + (size_t)rpg * 8;
  if (ldsb > (size_t)kFcxLds + 4096) return BSP_ERR_UNSUPPORTED;
  q.ngroups = (nbr + rpg - 1) / rpg;
  if ((int64_t)q.ngroups * q.nseg > 0x7FFFFFFF) return BSP_ERR_UNSUPPORTED;
  if (q.nseg > 1) {
    const int64_t bytes = (int64_t)q.nseg * p.P * p.O * 4;
    if (need) *need = bytes;
    if (!scratch || scratch_bytes < bytes) return BSP_ERR_CAPACITY;
    if (reinterpret_cast<uintptr_t>(scratch) & 15u) return BSP_ERR_ALIGN;
  }
  q.X = (const unsigned char*)p.X;
  q.W = (const unsigned char*)p.payload;
  q.row_ptr = p.row_ptr;
  q.col_idx = p.col_idx;
  q.bias = p.bias;
  q.residual = (const uint16_t*)p.residual;
  q.Y = (uint16_t*)p.Y;
  q.part = scratch;
  q.P = p.P;
  q.I = p.I;
  q.O = p.O;
  q.nbr = nbr;
  q.relu = p.relu;
  static bool raised[3] = {false, false, false};
  const void* fn = NT == 1 ? (const void*)fc_xlds_bf16<1> : NT == 2 ? (const void*)fc_xlds_bf16<2> : (const void*)fc_xlds_bf16<4>;
  bool& r = raised[NT == 1 ? 0 : NT == 2 ? 1 : 2];
  if (!r) {
    if (hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, kFcxLds + 4096) != hipSuccess) return BSP_ERR_HIP;
    r = true;
  }
  const dim3 grid((unsigned)(q.ngroups * q.nseg));
  // sixteen waves when each can own a row: more weight bytes in flight per CU, and a row's
  // start-up (its first loads' latency) paid once per workgroup instead of once per round
  const dim3 block(q.kp == 1 && rpg >= 16 ? 1024 : 512);
  switch (NT) {
    case 1: hipLaunchKernelGGL((fc_xlds_bf16<1>), grid, block, ldsb, st, q); break;
    case 2: hipLaunchKernelGGL((fc_xlds_bf16<2>), grid, block, ldsb, st, q); break;
    default: hipLaunchKernelGGL((fc_xlds_bf16<4>), grid, block, ldsb, st, q); break;
  }
  if (hipGetLastError() != hipSuccess) return BSP_ERR_HIP;
  if (q.nseg > 1) {
    const int64_t n = (int64_t)p.P * p.O;
    if (p.O % 4 == 0)
      hipLaunchKernelGGL(fc_xlds_sum<4>, dim3((unsigned)((n / 4 + 255) / 256)), dim3(256), 0, st, q);
    else
      hipLaunchKernelGGL(fc_xlds_sum<1>, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, q);
    if (hipGetLastError() != hipSuccess) return BSP_ERR_HIP;
  }
  return BSP_OK;
}
