// Block-sparse x block-sparse product C = (Gamma A)(Omega B)^t, 8x8 blocks (paper Section
// III-A).  A block product is done only where both operands keep the block column.
//
// One wave owns a 32 x 32 tile of C as four 16 x 16 MFMA tiles: two halves of two block
// rows of A against two halves of two block rows of B.  It walks the block columns four at
// a time (one MFMA 16x16x32 per tile: group g of sixteen lanes takes column 4s + g); each
// lane looks up, in the operands' position tables, the blocks its rows of A and B have in
// that column.  Wave-wide votes find out, per 16 x 16 tile, whether any column of the four
// is kept on both sides; if not that tile's MFMA (and, if no tile needs it, the fragment
// load) is skipped, which is how the zero products are avoided.  Kept blocks are read straight from the payloads
// (a lane reads one 16-byte row of a block).
#include "bsp_device.h"
#include "bsp_launch.h"

namespace {

struct SpParams {
  const int32_t* ia;   // [ra][nc]
  const int32_t* ib;   // [rb][nc]
  const uint16_t* pa;  // [nnzb][8][8] bf16
  const uint16_t* pb;
  float* C;            // [ra*8][rb*8]
  int32_t ra, rb, nc;
  int32_t tiles_j;     // ceil(rb / 4)
  int32_t ntiles;
};

__global__ __launch_bounds__(256) void spgemm_nt_bf16(SpParams q) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int jn = lane & 15, g = lane >> 4;
  const int tile = blockIdx.x * 4 + wave;
  if (tile >= q.ntiles) return;
  // a wave's tile is 32 x 32: two 16-row halves of A against two 16-row halves of B, so
  // that every fragment it loads feeds two MFMAs
  const int ti = tile / q.tiles_j, tj = tile - ti * q.tiles_j;
  const int lr = jn & 7;  // this lane's row inside its block
  const int32_t* ia[2];
  const int32_t* ib[2];
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    const int ra = 4 * ti + 2 * h + (jn >> 3), rb = 4 * tj + 2 * h + (jn >> 3);
    ia[h] = ra < q.ra ? q.ia + (int64_t)ra * q.nc : nullptr;
    ib[h] = rb < q.rb ? q.ib + (int64_t)rb * q.nc : nullptr;
  }

  // Two steps (eight block columns) per round: all position look-ups first, then the votes,
  // then the block loads of the steps that have a match, then their MFMAs, so that the
  // loads of a round are in flight together.
  constexpr int U = 2;
  f32x4_t acc[2][2];
#pragma unroll
  for (int x = 0; x < 2; ++x)
#pragma unroll
    for (int y = 0; y < 2; ++y) acc[x][y] = f32x4_t{0.f, 0.f, 0.f, 0.f};
  for (int c0 = 0; c0 < q.nc; c0 += 4 * U) {
    int na[U][2], nb[U][2];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int c = c0 + 4 * u + g;
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        na[u][h] = (ia[h] && c < q.nc) ? ia[h][c] : -1;
        nb[u][h] = (ib[h] && c < q.nc) ? ib[h][c] : -1;
      }
    }
    // per 16-row half: which of the step's four columns have a block, over the sixteen rows
    bool any[U][2][2];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      unsigned long long va[2], vb[2];
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        va[h] = __ballot(na[u][h] >= 0);
        vb[h] = __ballot(nb[u][h] >= 0);
      }
#pragma unroll
      for (int x = 0; x < 2; ++x)
#pragma unroll
        for (int y = 0; y < 2; ++y) {
          any[u][x][y] = false;
#pragma unroll
          for (int k = 0; k < 4; ++k)
            any[u][x][y] |= ((va[x] >> (16 * k)) & 0xFFFFull) != 0 && ((vb[y] >> (16 * k)) & 0xFFFFull) != 0;
        }
    }
    u32x4_t a[U][2], b[U][2];
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        a[u][h] = u32x4_t{0u, 0u, 0u, 0u};
        b[u][h] = u32x4_t{0u, 0u, 0u, 0u};
        if ((any[u][h][0] || any[u][h][1]) && na[u][h] >= 0)
          a[u][h] = *(const u32x4_t*)(q.pa + (int64_t)na[u][h] * 64 + lr * 8);
        if ((any[u][0][h] || any[u][1][h]) && nb[u][h] >= 0)
          b[u][h] = *(const u32x4_t*)(q.pb + (int64_t)nb[u][h] * 64 + lr * 8);
      }
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
      for (int x = 0; x < 2; ++x)
#pragma unroll
        for (int y = 0; y < 2; ++y)
          if (any[u][x][y]) acc[x][y] = mfma_bf16_16x16x32(a[u][x], b[u][y], acc[x][y]);
  }
  // lane holds C[32 ti + 16 x + 4 g + r][32 tj + 16 y + jn], r = 0..3
#pragma unroll
  for (int x = 0; x < 2; ++x)
#pragma unroll
    for (int y = 0; y < 2; ++y) {
      const int col = 32 * tj + 16 * y + jn;
      if (col >= q.rb * 8) continue;
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int row = 32 * ti + 16 * x + 4 * g + r;
        if (row < q.ra * 8) q.C[(int64_t)row * (q.rb * 8) + col] = acc[x][y][r];
      }
    }
}

}  // namespace

extern "C" int bsp_spgemm_nt(const bsp_bcsr* A, const bsp_bcsr* B, float* C, void* stream) {
  if (!A || !B || !C) return BSP_ERR_NULL;
  if (!A->index || !B->index || (A->nnzb > 0 && !A->payload) || (B->nnzb > 0 && !B->payload))
    return BSP_ERR_NULL;
  if (A->rows <= 0 || B->rows <= 0 || A->cols <= 0 || A->cols != B->cols || A->nnzb < 0 || B->nnzb < 0)
    return BSP_ERR_SHAPE;
  if (A->k != 8 || B->k != 8) return BSP_ERR_UNSUPPORTED;
  if (A->dtype != BSP_BF16 || B->dtype != BSP_BF16) return BSP_ERR_DTYPE;
  if ((int64_t)A->rows * 8 * B->rows * 8 > 0x7FFFFFFFll * 4 || (int64_t)A->rows * A->cols > 0x7FFFFFFFll ||
      (int64_t)B->rows * B->cols > 0x7FFFFFFFll)
    return BSP_ERR_SHAPE;
  if ((reinterpret_cast<uintptr_t>(A->payload) & 15u) || (reinterpret_cast<uintptr_t>(B->payload) & 15u) ||
      (reinterpret_cast<uintptr_t>(C) & 3u))
    return BSP_ERR_ALIGN;
  SpParams q;
  q.ia = A->index;
  q.ib = B->index;
  q.pa = (const uint16_t*)A->payload;
  q.pb = (const uint16_t*)B->payload;
  q.C = C;
  q.ra = A->rows;
  q.rb = B->rows;
  q.nc = A->cols;
  q.tiles_j = (B->rows + 3) / 4;
  const int64_t ntiles = (int64_t)((A->rows + 3) / 4) * q.tiles_j;
  if (ntiles > 0x7FFFFFFF) return BSP_ERR_SHAPE;
  q.ntiles = (int32_t)ntiles;
  hipLaunchKernelGGL(spgemm_nt_bf16, dim3((unsigned)((ntiles + 3) / 4)), dim3(256), 0,
                     (hipStream_t)stream, q);
  return hipGetLastError() == hipSuccess ? BSP_OK : BSP_ERR_HIP;
}
