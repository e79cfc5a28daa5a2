// Block-sparse x block-sparse product C = (Gamma A)(Omega B)^t, 8x8 blocks (paper Section
// III-A).  A block product is done only where both operands keep the block column.
//
// One wave owns a 16 x 16 tile of C: two block rows of A against two block rows of B.  It
// walks the block columns four at a time (one MFMA 16x16x32: group g of sixteen lanes takes
// column 4s + g); each lane looks up, in the operands' position tables, the block its row of
// A and its row of B have in that column.  A wave-wide vote finds out whether any column of
// the four is kept on both sides; if not the step costs two small loads and no MFMA, which
// is how the zero products are skipped.  Kept blocks are read straight from the payloads
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
  int32_t tiles_j;     // ceil(rb / 2)
  int32_t ntiles;
};

__global__ __launch_bounds__(256) void spgemm_nt_bf16(SpParams q) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int jn = lane & 15, g = lane >> 4;
  const int tile = blockIdx.x * 4 + wave;
  if (tile >= q.ntiles) return;
  const int ti = tile / q.tiles_j, tj = tile - ti * q.tiles_j;
  const int ra = 2 * ti + (jn >> 3), rb = 2 * tj + (jn >> 3);  // this lane's block rows
  const int lr = jn & 7;                                        // its row inside the block
  const int32_t* ia = ra < q.ra ? q.ia + (int64_t)ra * q.nc : nullptr;
  const int32_t* ib = rb < q.rb ? q.ib + (int64_t)rb * q.nc : nullptr;

  f32x4_t acc = f32x4_t{0.f, 0.f, 0.f, 0.f};
  for (int c0 = 0; c0 < q.nc; c0 += 4) {
    const int c = c0 + g;
    const int na = (ia && c < q.nc) ? ia[c] : -1;
    const int nb = (ib && c < q.nc) ? ib[c] : -1;
    // which of the four columns have a block on each side, over all sixteen rows of a group
    const unsigned long long va = __ballot(na >= 0), vb = __ballot(nb >= 0);
    bool any = false;
#pragma unroll
    for (int k = 0; k < 4; ++k)
      any |= ((va >> (16 * k)) & 0xFFFFull) != 0 && ((vb >> (16 * k)) & 0xFFFFull) != 0;
    if (!any) continue;
    u32x4_t a = u32x4_t{0u, 0u, 0u, 0u}, b = u32x4_t{0u, 0u, 0u, 0u};
    if (na >= 0) a = *(const u32x4_t*)(q.pa + (int64_t)na * 64 + lr * 8);
    if (nb >= 0) b = *(const u32x4_t*)(q.pb + (int64_t)nb * 64 + lr * 8);
    acc = mfma_bf16_16x16x32(a, b, acc);
  }
  // lane holds C[16 ti + 4 g + r][16 tj + jn], r = 0..3
  const int col = 16 * tj + jn;
  if (col < q.rb * 8) {
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int row = 16 * ti + 4 * g + r;
      if (row < q.ra * 8) q.C[(int64_t)row * (q.rb * 8) + col] = acc[r];
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
  q.tiles_j = (B->rows + 1) / 2;
  const int64_t ntiles = (int64_t)((A->rows + 1) / 2) * q.tiles_j;
  if (ntiles > 0x7FFFFFFF) return BSP_ERR_SHAPE;
  q.ntiles = (int32_t)ntiles;
  hipLaunchKernelGGL(spgemm_nt_bf16, dim3((unsigned)((ntiles + 3) / 4)), dim3(256), 0,
                     (hipStream_t)stream, q);
  return hipGetLastError() == hipSuccess ? BSP_OK : BSP_ERR_HIP;
}
