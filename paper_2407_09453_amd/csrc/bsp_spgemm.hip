// Block-sparse x block-sparse product C = (Gamma A)(Omega B)^t, 8x8 blocks (paper Section
// III-A).  A block product is done only where both operands keep the block column.
//
// A workgroup owns a 128 x 128 tile of C: sixteen block rows of A against sixteen of B.  It
// walks the block columns in segments of 16 to 64 (as many sixteens as fit the payload area
// of LDS) and, per segment, copies the kept blocks of its 32 block rows from their compressed
// block rows into LDS (each row's blocks of the segment are one contiguous run, found through
// the per-sixteen row pointers seg_ptr) and scatters a one-byte position table per row from
// col_idx.  A wave owns one pair of A block rows and meets every pair of B block rows in
// turn (a 16 x 16 MFMA tile each).  For such a tile the columns worth multiplying are those
// kept by one of the two A rows and by one of the two B rows: the two rows' column sets are
// united, the two sides intersected (the merge of the sorted index lists of Section III-A,
// done on 64-bit column sets), and the surviving columns are compacted so that every MFMA
// 16x16x32 takes four of them; columns kept on one side only are never multiplied.
#include "bsp_device.h"
#include "bsp_launch.h"
#include <algorithm>
#ifdef BSP_ROWS_TUNE
#include <cstdlib>
#endif

namespace {

constexpr int kRows = 16;     // block rows of each operand per workgroup
constexpr int kSub = 16;      // block columns per seg_ptr entry
constexpr int kMaxSub = 4;    // a segment is one to four of those
constexpr int kCap = 592;     // blocks the payload area holds (>= 2 * kRows * kSub); slot kCap stays zero
constexpr int kTabOff = (kCap + 1) * 128;           // position tables, two sets of [32 rows][64 columns] bytes
constexpr int kTabBytes = 2 * kRows * 64;
constexpr int kLdsBytes = kTabOff + 2 * kTabBytes;
static_assert(kCap >= 2 * kRows * kSub, "one sixteen of columns must always fit");
static_assert(2 * kLdsBytes <= 160 * 1024, "two workgroups share a CU");

struct SpParams {
  const int32_t* sa;   // seg_ptr of A: [ra][nsub + 1]
  const int32_t* sb;
  const int32_t* ca;   // col_idx
  const int32_t* cb;
  const unsigned char* pa;  // [nnzb][8][8] bf16
  const unsigned char* pb;
  float* C;            // [ra*8][rb*8]
  int32_t ra, rb, nsub;
  int32_t nnzb_a, nnzb_b;   // both positive
  int32_t tiles_i, tiles_j;  // workgroup tiles along A's and B's block rows
  int32_t sbj, nsb;          // 8 x 8 groups of tiles: along j, in all
#ifdef BSP_ROWS_TUNE
  long long* trace;
#endif
};

#ifdef BSP_ROWS_TUNE
#define SP_CLOCK() wall_clock64()
#define SP_ADD(k, t0)                          \
  do {                                         \
    const long long t1_ = wall_clock64();      \
    tacc[k] += t1_ - (t0);                     \
    (t0) = t1_;                                \
  } while (0)
#else
#define SP_CLOCK() 0ll
#define SP_ADD(k, t0)
#endif

typedef __attribute__((address_space(1))) const void* gptr_t;
typedef __attribute__((address_space(3))) void* lptr_t;

// What a wave keeps of the next segment between asking for its row pointers and using them.
struct SegRows {
  int first, d[kMaxSub];
};
// A segment as every wave sees it: lane r < 32 holds row r's first block, slot in LDS and number
// of blocks; ks (the same in all lanes) is the segment's width in sixteens.
struct SegPlan {
  int first, off, cnt, ks;
};

// C = 0: an operand without a kept block.
__global__ __launch_bounds__(256) void spgemm_zero(float* C, int64_t n) {
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) C[i] = 0.f;
}

template <int U>
__global__ __launch_bounds__(512) void spgemm_nt_bf16(SpParams q) {
  kernarg_touch<SpParams>();
  extern __shared__ __align__(16) unsigned char lds[];
  const int tid = threadIdx.x, lane = tid & 63, jn = lane & 15, g = lane >> 4;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  // consecutive workgroups go to different XCDs; each XCD takes whole 8 x 8 groups of tiles so
  // that the operand rows its workgroups share stay in its L2
  const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
  const int grp = (slot >> 6) * 8 + xcd, within = slot & 63;
  if (grp >= q.nsb) return;
  const int gi = grp / q.sbj, gj = grp - gi * q.sbj;
  const int ti = gi * 8 + (within >> 3), tj = gj * 8 + (within & 7);
  if (ti >= q.tiles_i || tj >= q.tiles_j) return;
#ifdef BSP_ROWS_TUNE
  long long tacc[6] = {0, 0, 0, 0, 0, 0};
  const long long tentry = wall_clock64();
#endif
  long long tm = SP_CLOCK();

  const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)lds;
  const int half = jn >> 3, lr = jn & 7;  // which row of the pair, which row of the block
  constexpr uint32_t kZero = (uint32_t)kCap;           // the slot that holds zeros
  constexpr uint32_t kZZ = kZero | (kZero << 16);

  f32x4_t acc[8];
#pragma unroll
  for (int jp = 0; jp < 8; ++jp) acc[jp] = f32x4_t{0.f, 0.f, 0.f, 0.f};

  // Every wave plans the segments for itself (the same few loads and shuffles in each, no
  // table in LDS and no barrier for it): lane r < 32 stands for row r of the 32 (A's sixteen,
  // then B's).
  const int mrow = lane & 31;
  const bool m_isA = mrow < kRows;
  const int m_row = m_isA ? ti * kRows + mrow : tj * kRows + mrow - kRows;
  const bool m_ok = lane < 32 && m_row < (m_isA ? q.ra : q.rb);
  const int32_t* m_sp = (m_isA ? q.sa : q.sb) + (int64_t)(m_ok ? m_row : 0) * (q.nsub + 1);
  auto seg_load = [&](int x, SegRows& sr) {
    sr.first = 0;
#pragma unroll
    for (int k = 0; k < kMaxSub; ++k) sr.d[k] = 0;
    if (m_ok && x < q.nsub) {
      const int kmax = min(kMaxSub, q.nsub - x);
      sr.first = m_sp[x];
#pragma unroll
      for (int k = 0; k < kMaxSub; ++k)
        if (k < kmax) sr.d[k] = m_sp[x + k + 1];
    }
  };
  // how many sixteens fit (the same answer in every wave), where each row's blocks start and go
  auto seg_plan = [&](int x, const SegRows& sr, SegPlan& pl) {
    const int kmax = min(kMaxSub, q.nsub - x);
    int ks = 1, cnt = m_ok ? sr.d[0] - sr.first : 0;
#pragma unroll
    for (int k = 1; k < kMaxSub; ++k) {
      const int dk = (m_ok && k < kmax) ? sr.d[k] - sr.first : 0;
      int t = dk;
#pragma unroll
      for (int m = 1; m < 32; m <<= 1) t += __shfl_xor(t, m);
      t = __builtin_amdgcn_readfirstlane(t);  // lanes 0-31 hold the total of the 32 rows
      if (k < kmax && t <= kCap) {            // totals grow with k: the last k that fits wins
        ks = k + 1;
        cnt = dk;
      }
    }
    int incl = cnt;
#pragma unroll
    for (int m = 1; m < 32; m <<= 1) {
      const int v = __shfl_up(incl, m);
      if (lane >= m) incl += v;
    }
    pl.first = sr.first;
    pl.off = incl - cnt;
    pl.cnt = cnt;
    pl.ks = ks;
  };
  // wave w brings rows 4w .. 4w + 3 (waves 0-3: A's, waves 4-7: B's); the columns of their
  // blocks, asked for one segment ahead
  const int32_t* my_col = wave < 4 ? q.ca : q.cb;
  const unsigned char* my_pay = wave < 4 ? q.pa : q.pb;
  // (every lane loads, the lanes past the row's blocks an entry they do not use: a load under a
  // condition would be waited for on the spot)
  const int my_last = (wave < 4 ? q.nnzb_a : q.nnzb_b) - 1;
  auto col_load = [&](const SegPlan& pl, int (&col)[4]) {
#pragma unroll
    for (int rr = 0; rr < 4; ++rr) {
      const int first = __builtin_amdgcn_readlane(pl.first, wave * 4 + rr);
      col[rr] = my_col[min(first + lane, my_last)];
    }
  };

  // ---- before the first segment: its plan and columns, an empty table, the zero block
  if (tid < 8) ((u32x4_t*)lds)[kCap * 8 + tid] = u32x4_t{0u, 0u, 0u, 0u};
  ((uint32_t*)(lds + kTabOff))[tid] = 0xFFFFFFFFu;  // 512 threads x 4 bytes: no block anywhere
  SegRows sr;
  SegPlan pl, pn;
  int col[4], coln[4];
  seg_load(0, sr);
  seg_plan(0, sr, pl);
  pn = pl;
  col_load(pl, col);
  __syncthreads();
  SP_ADD(0, tm);

  int buf = 0;
  for (int x = 0; x < q.nsub; buf ^= 1) {
    uint8_t* tab = lds + kTabOff + buf * kTabBytes;
    const int xn = x + __builtin_amdgcn_readfirstlane(pl.ks);

    // ---- copies: the position tables first (their columns came long ago), then the blocks
#pragma unroll
    for (int rr = 0; rr < 4; ++rr) {
      const int r = wave * 4 + rr;
      const int n = __builtin_amdgcn_readlane(pl.cnt, r);
      if (lane < n) tab[r * 64 + ((col[rr] - x * kSub) & 63)] = (uint8_t)lane;
    }
#pragma unroll
    for (int rr = 0; rr < 4; ++rr) {
      const int r = wave * 4 + rr;
      const int first = __builtin_amdgcn_readlane(pl.first, r), off = __builtin_amdgcn_readlane(pl.off, r);
      const int n = __builtin_amdgcn_readlane(pl.cnt, r);
      const unsigned char* pay = my_pay + (int64_t)first * 128;
      const int pieces = n * 8;  // 16 bytes each
      for (int it = 0; it < pieces; it += 64) {
        if (it + lane < pieces)
          __builtin_amdgcn_global_load_lds((gptr_t)(pay + (it + lane) * 16),
                                           (lptr_t)(uintptr_t)(lds0 + (uint32_t)(off * 8 + it) * 16u), 16, 0, 0);
      }
    }
    // the next segment: its row pointers asked for now, its table emptied
    seg_load(xn, sr);
    ((uint32_t*)(lds + kTabOff + (buf ^ 1) * kTabBytes))[tid] = 0xFFFFFFFFu;
    SP_ADD(1, tm);
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();
    SP_ADD(2, tm);
    seg_plan(xn, sr, pn);  // past the last segment: rows without blocks, loads of entries nobody uses
    col_load(pn, coln);

    // ---- products: this wave's pair of A rows against the eight pairs of B rows
    {
      const int ra0 = 2 * wave;
      const uint32_t a0 = tab[ra0 * 64 + lane], a1 = tab[(ra0 + 1) * 64 + lane];  // this lane's column
      const uint32_t oa0 = (uint32_t)__builtin_amdgcn_readlane(pl.off, ra0);
      const uint32_t oa1 = (uint32_t)__builtin_amdgcn_readlane(pl.off, ra0 + 1);
      const unsigned long long ma = __ballot(a0 != 255u) | __ballot(a1 != 255u);
      const uint32_t mineA = (a0 == 255u ? kZero : oa0 + a0) | ((a1 == 255u ? kZero : oa1 + a1) << 16);
      const int sh = half * 16;
      const uint32_t rowb = (uint32_t)lr * 16u;
      // per pair of B rows: the columns both sides keep, compacted: lane n gets the slots of the
      // n-th such column, the lanes past their number get the zero block
      int pA[8], pB[8], cnt[8];
#pragma unroll
      for (int jp = 0; jp < 8; ++jp) {
        const int rb0 = kRows + 2 * jp;
        const uint32_t b0 = tab[rb0 * 64 + lane], b1 = tab[(rb0 + 1) * 64 + lane];
        const uint32_t ob0 = (uint32_t)__builtin_amdgcn_readlane(pl.off, rb0);
        const uint32_t ob1 = (uint32_t)__builtin_amdgcn_readlane(pl.off, rb0 + 1);
        const unsigned long long m = ma & (__ballot(b0 != 255u) | __ballot(b1 != 255u));
        cnt[jp] = __popcll(m);
        const uint32_t mineB = (b0 == 255u ? kZero : ob0 + b0) | ((b1 == 255u ? kZero : ob1 + b1) << 16);
        const int rank = (int)__builtin_amdgcn_mbcnt_hi((uint32_t)(m >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m, 0u));
        const bool isset = (m >> lane) & 1ull;
        const int dest = (isset ? rank : cnt[jp] + lane - rank) << 2;
        pA[jp] = __builtin_amdgcn_ds_permute(dest, (int)(isset ? mineA : kZZ));
        pB[jp] = __builtin_amdgcn_ds_permute(dest, (int)(isset ? mineB : kZZ));
      }
#pragma unroll
      for (int jp = 0; jp < 8; ++jp) {
        for (int s0 = 0; s0 < cnt[jp]; s0 += 4 * U) {
          uint32_t va[U], vb[U];
#pragma unroll
          for (int u = 0; u < U; ++u) {
            const int n = (s0 + 4 * u + g) & 63;
            va[u] = (uint32_t)__builtin_amdgcn_ds_bpermute(n << 2, pA[jp]);
            vb[u] = (uint32_t)__builtin_amdgcn_ds_bpermute(n << 2, pB[jp]);
          }
          u32x4_t a[U], b[U];
#pragma unroll
          for (int u = 0; u < U; ++u) {
            if (u > 0 && s0 + 4 * u >= cnt[jp]) continue;
            a[u] = *(const u32x4_t*)(lds + (((va[u] >> sh) & 0xFFFFu) * 128u + rowb));
            b[u] = *(const u32x4_t*)(lds + (((vb[u] >> sh) & 0xFFFFu) * 128u + rowb));
          }
#pragma unroll
          for (int u = 0; u < U; ++u)
            if (u == 0 || s0 + 4 * u < cnt[jp]) acc[jp] = mfma_bf16_16x16x32(a[u], b[u], acc[jp]);
        }
      }
    }
    SP_ADD(3, tm);
    __syncthreads();  // every wave is done with the tables and the blocks
    SP_ADD(4, tm);
    x = xn;
    pl = pn;
#pragma unroll
    for (int rr = 0; rr < 4; ++rr) col[rr] = coln[rr];
  }

  // lane holds C[128 ti + 16 wave + 4 g + r][128 tj + 16 jp + jn], r = 0..3
  const int ncol = q.rb * 8;
#pragma unroll
  for (int jp = 0; jp < 8; ++jp) {
    const int col = 128 * tj + 16 * jp + jn;
    if (col >= ncol) continue;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int row = 128 * ti + 16 * wave + 4 * g + r;
      if (row < q.ra * 8) q.C[(int64_t)row * ncol + col] = acc[jp][r];
    }
  }
#ifdef BSP_ROWS_TUNE
  if (q.trace && lane == 0) {
    __builtin_amdgcn_s_waitcnt(0);
    SP_ADD(5, tm);
    long long* t = q.trace + ((size_t)blockIdx.x * 8 + wave) * 8;
    t[0] = tentry;
    for (int k = 0; k < 6; ++k) t[1 + k] = tacc[k];
    t[7] = tm;
  }
#endif
}

constexpr int kU = 2;  // MFMA steps whose fragments are asked for together

template <int U>
int launch_u(const SpParams& q, unsigned grid, hipStream_t st) {
  static bool raised = false;  // dynamic LDS above 64 KB has to be allowed once per kernel
  if (!raised) {
    if (hipFuncSetAttribute((const void*)spgemm_nt_bf16<U>, hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes) !=
        hipSuccess)
      return BSP_ERR_HIP;
    raised = true;
  }
  hipLaunchKernelGGL((spgemm_nt_bf16<U>), dim3(grid), dim3(512), kLdsBytes, st, q);
  return hipGetLastError() == hipSuccess ? BSP_OK : BSP_ERR_HIP;
}

}  // namespace

extern "C" int bsp_spgemm_nt(const bsp_bcsr* A, const bsp_bcsr* B, float* C, void* stream) {
  if (!A || !B || !C) return BSP_ERR_NULL;
  if (!A->seg_ptr || !B->seg_ptr || (A->nnzb > 0 && (!A->payload || !A->col_idx)) ||
      (B->nnzb > 0 && (!B->payload || !B->col_idx)))
    return BSP_ERR_NULL;
  if (A->rows <= 0 || B->rows <= 0 || A->cols <= 0 || A->cols != B->cols || A->nnzb < 0 || B->nnzb < 0)
    return BSP_ERR_SHAPE;
  if (A->k != 8 || B->k != 8) return BSP_ERR_UNSUPPORTED;
  if (A->dtype != BSP_BF16 || B->dtype != BSP_BF16) return BSP_ERR_DTYPE;
  if ((int64_t)A->rows * 8 * B->rows * 8 > 0x7FFFFFFFll * 4 || A->nnzb > 0x7FFFFFFFll || B->nnzb > 0x7FFFFFFFll)
    return BSP_ERR_SHAPE;
  if ((reinterpret_cast<uintptr_t>(A->payload) & 15u) || (reinterpret_cast<uintptr_t>(B->payload) & 15u) ||
      (reinterpret_cast<uintptr_t>(C) & 3u))
    return BSP_ERR_ALIGN;
  if (A->nnzb == 0 || B->nnzb == 0) {
    const int64_t n = (int64_t)A->rows * 8 * B->rows * 8;
    hipLaunchKernelGGL(spgemm_zero, dim3((unsigned)std::min<int64_t>((n + 255) / 256, 4096)), dim3(256), 0,
                       (hipStream_t)stream, C, n);
    return hipGetLastError() == hipSuccess ? BSP_OK : BSP_ERR_HIP;
  }
  SpParams q;
  q.nnzb_a = (int32_t)A->nnzb;
  q.nnzb_b = (int32_t)B->nnzb;
  q.sa = A->seg_ptr;
  q.sb = B->seg_ptr;
  q.ca = A->col_idx;
  q.cb = B->col_idx;
  q.pa = (const unsigned char*)A->payload;
  q.pb = (const unsigned char*)B->payload;
  q.C = C;
  q.ra = A->rows;
  q.rb = B->rows;
  q.nsub = (A->cols + kSub - 1) / kSub;
  q.tiles_i = (A->rows + kRows - 1) / kRows;
  q.tiles_j = (B->rows + kRows - 1) / kRows;
  q.sbj = (q.tiles_j + 7) / 8;
  const int64_t nsb = (int64_t)((q.tiles_i + 7) / 8) * q.sbj;
  if (nsb * 64 > 0x7FFFFFFF) return BSP_ERR_SHAPE;
  q.nsb = (int32_t)nsb;
#ifdef BSP_ROWS_TUNE
  q.trace = nullptr;
  if (const char* e = std::getenv("BSP_PW_TRACE_PTR")) q.trace = (long long*)std::strtoull(e, nullptr, 16);
#endif
  const unsigned grid = (unsigned)(((nsb + 7) / 8) * 8 * 64);
#ifdef BSP_ROWS_TUNE
  if (const char* e = std::getenv("BSP_SP_U")) {
    const int u = std::atoi(e);
    if (u == 2) return launch_u<2>(q, grid, (hipStream_t)stream);
    if (u == 3) return launch_u<3>(q, grid, (hipStream_t)stream);
    if (u == 6) return launch_u<6>(q, grid, (hipStream_t)stream);
  }
#endif
  return launch_u<kU>(q, grid, (hipStream_t)stream);
}
