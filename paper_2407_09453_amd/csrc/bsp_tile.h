// Pieces shared by the LDS-tiled bf16 kernels: tile geometry, cheap integer
// division, MFMA step helpers (library private).
#ifndef BSP_TILE_H
#define BSP_TILE_H

#include "bsp_device.h"
#include "bsp_fastdiv.h"

// (both words are read and the product is formed whatever the divisor: a select instead of a
// branch around a second load, which in a kernel's opening was one more wait for the scalar
// cache per division)
__device__ __forceinline__ uint32_t fdiv(uint32_t x, FastDiv f) {
  const uint32_t q = __umulhi(x, f.mul);
  return f.d == 1 ? x : q;
}

struct TileCfg {
  int32_t TH, TW;            // output tile, pixels
  int32_t TPH, TPW;          // staged input patch, pixels
  int32_t lsh, lsw;          // LDS pixels per output pixel step
  int32_t gsh, gsw;          // input pixels per LDS pixel step
  int32_t tiles_y, tiles_x;  // tiles per image
  int32_t row_bytes;         // LDS bytes per staged pixel (slab*2 + pad)
  int32_t pitch;             // LDS bytes per staged patch row (TPW*row_bytes + pad)
  int32_t tile2x8;           // 1: a 16-pixel tile is 2 rows x 8 columns, 0: 16 consecutive pixels
  int32_t slab, nslabs;      // channels per slab, slabs
  int32_t spc;               // strips per workgroup (4 when nslabs > 1)
  int32_t nstrips;
  int32_t ntiles;            // B * tiles_y * tiles_x
  FastDiv d_pp, d_tpw, d_tw, d_tpr, d_ntiles, d_tpi, d_tiles_x;
};

constexpr int kStageBatch = 8;  // 16-byte pieces a thread keeps in flight while staging
#ifndef BSP_WDEPTH
#define BSP_WDEPTH 8
#endif
constexpr int kWDepth = BSP_WDEPTH;  // weight fragments fetched ahead

typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
typedef __attribute__((ext_vector_type(2))) float f32x2_t;
// two fp32 -> packed bf16 pair, round to nearest even (v_cvt_pk_bf16_f32)
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  const f32x2_t v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}

// Four bf16 results (v) plus four residual values already in registers (r), the activation,
// one more rounding: post_bf16x4's arithmetic without a trip through memory.
__device__ __forceinline__ u32x2_t post_bf16x4_reg(u32x2_t v, u32x2_t r, bool has_r, int relu) {
  float f[4] = {bf16_bits_to_f32((uint16_t)(v.x & 0xFFFF)), bf16_bits_to_f32((uint16_t)(v.x >> 16)),
                bf16_bits_to_f32((uint16_t)(v.y & 0xFFFF)), bf16_bits_to_f32((uint16_t)(v.y >> 16))};
  if (has_r) {
    f[0] += bf16_bits_to_f32((uint16_t)(r.x & 0xFFFF));
    f[1] += bf16_bits_to_f32((uint16_t)(r.x >> 16));
    f[2] += bf16_bits_to_f32((uint16_t)(r.y & 0xFFFF));
    f[3] += bf16_bits_to_f32((uint16_t)(r.y >> 16));
  }
  if (relu) {
#pragma unroll
    for (int k = 0; k < 4; ++k) f[k] = fmaxf(f[k], 0.f);
  }
  return u32x2_t{pack_bf16x2(f[0], f[1]), pack_bf16x2(f[2], f[3])};
}

// The activations one step needs: every pixel tile of the wave reads its 16
// bytes at the offset the step's descriptor d (chunk, tap) selects.
template <int NT>
__device__ __forceinline__ void load_b(u32x4_t (&b)[NT], const int d, const unsigned char* lds,
                                       const int (&base)[NT], const int pitch,
                                       const int row_bytes) {
  const int xoff = ((d >> 16) & 0xFF) * pitch + ((d >> 24) & 0xFF) * row_bytes + (d & 0xFFFF) * 16;
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) b[nt] = *(const u32x4_t*)(lds + base[nt] + xoff);
}
template <int NT>
__device__ __forceinline__ void do_mma(f32x4_t (&acc)[NT], const u32x4_t a,
                                       const u32x4_t (&b)[NT]) {
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) acc[nt] = mfma_bf16_16x16x32(a, b[nt], acc[nt]);
}


// Pick the output tile for a layer (most useful pixels per MFMA pixel slot,
// least halo, no LDS bank conflicts) and the LDS paddings; false if nothing fits
// in max_lds bytes.  Fills everything in *out except spc, ntiles and the dividers.
// The tile holds nt_scale * NT pixel tiles (nt_scale waves share a strip) and the LDS
// budget also has to cover out_row_bytes per output pixel (results staging), if any.
bool bsp_choose_tile(const ConvParams& p, int slab, int64_t max_lds, int max_pieces, int nt_scale,
                     int out_row_bytes, int min_nt, int slots, int* NT, TileCfg* out);

#endif
