// Launch-plan blob shared by the host builder and the kernels (library private).
//
// The kernels tile the output channels into strips of BSP_STRIP = 16 (the
// row count of a 16x16 MFMA tile) and the input channels into chunks of
// BSP_CHUNK = 8 (what one lane feeds a bf16 MFMA).  A strip covers two 8x8
// block rows, four 4x16 block rows or one 16x4 block row; a chunk is one 8x8
// block column, half a 4x16 block column or two 16x4 block columns.  For each
// strip the plan lists, in ascending order, the chunks in which at least one
// block of the strip is kept, and for each of the up to BSP_MAXSUB blocks that
// meet in a (strip, chunk) cell the element offset of its first needed entry
// inside the payload array, or -1 if that block is zeroed.
//
// Words (int32):
//   [0..31]                header, see enum below
//   [off_strip ..]         strip_ptr[nstrips+1]    first chunk of each strip
//   [off_xc ..]            chunk_xc[nchunks]       chunk index (input channel / 8)
//   [off_src ..]           chunk_src[nchunks][4]   payload element offsets or -1
//   bf16 payloads only (the "step" section, used by the LDS-tiled kernels):
//   [off_slab ..]          slab_ptr[nstrips][nslabs+1]  first step of each (strip, slab)
//   [off_xdesc ..]         xdesc[nsteps][4]        per 16-lane group: which activation
//                                                  chunk and tap it multiplies
//   [off_wfrag ..]         wfrag[nsteps][64][8]    bf16 weights in MFMA operand order
//
// Meaning of chunk_src[c][s] by granularity (element offset of row 0, tap 0):
//   8x8   s = 0,1   block row 2*strip+s, block column xc
//   4x16  s = 0..3  block row 4*strip+s, block column xc/2, already advanced by
//                   8*(xc%2) to the half of the block this chunk covers
//   16x4  s = 0,1   block row strip, block column 2*xc+s (channels 4s..4s+3 of the chunk)
//
// Step section.  The input channels are cut into slabs of `slab` channels (what
// the kernel keeps in LDS at a time).  Inside one (strip, slab) the contraction
// index is the list of pairs (chunk, tap), chunk-major over the strip's kept
// chunks that fall in the slab; one step = four consecutive pairs = one MFMA
// 16x16x32, pair 4*step+g going to lanes 16g..16g+15.  The last step of a
// (strip, slab) is padded with null pairs (zero weights).
//   xdesc = (chunk index within the slab) | tap_row << 16 | tap_col << 24
//   wfrag[step][16g + j][0..7] = W[16*strip + j][tap][8*chunk .. 8*chunk+7] or 0
#ifndef BSP_PLAN_H
#define BSP_PLAN_H

#include <stdint.h>

enum {
  BSP_STRIP = 16,
  BSP_CHUNK = 8,
  BSP_MAXSUB = 4,
  BSP_PLAN_HEADER_WORDS = 32,
  BSP_PLAN_MAGIC = 0x42535032,
  BSP_PLAN_VERSION = 6,
};

enum {
  BSP_PLAN_MAGIC_W = 0,
  BSP_PLAN_VERSION_W = 1,
  BSP_PLAN_O_W = 2,
  BSP_PLAN_I_W = 3,
  BSP_PLAN_H_W = 4,
  BSP_PLAN_K_W = 5,
  BSP_PLAN_BO_W = 6,
  BSP_PLAN_BI_W = 7,
  BSP_PLAN_NSTRIPS_W = 8,
  BSP_PLAN_NCHUNKS_W = 9,
  BSP_PLAN_OFF_STRIP_W = 10,
  BSP_PLAN_OFF_XC_W = 11,
  BSP_PLAN_OFF_SRC_W = 12,
  BSP_PLAN_TOTAL_W = 13,
  BSP_PLAN_MAXCHUNKS_W = 14,
  BSP_PLAN_DTYPE_W = 15,
  BSP_PLAN_SLAB_W = 16,       // channels per slab
  BSP_PLAN_NSLABS_W = 17,
  BSP_PLAN_NSTEPS_W = 18,     // 0 when there is no step section
  BSP_PLAN_OFF_SLAB_W = 19,
  BSP_PLAN_OFF_XDESC_W = 20,
  BSP_PLAN_OFF_WFRAG_W = 21,
  BSP_PLAN_MAXSTEPS_W = 22,   // most steps in any one strip
  BSP_PLAN_MAXSLABSTEPS_W = 23,  // most steps in any one (strip, slab)
  BSP_PLAN_OFF_ROWS_W = 24,   // first word of the row-band section, 0 when there is none
  BSP_PLAN_OFF_FIRST_W = 25,  // first word of the thin-input section, 0 when there is none
};

// Row-band section (bf16 layers with whole 8-channel groups; read by bsp_rows.hip).
//
// Strips here are groups of block rows chosen by the builder so that rows sharing many kept
// columns sit together (a 16-row matrix-core tile multiplies one activation operand with all
// of its rows, so a strip runs the union of its rows' columns): two 8x8 block rows, four 4x16
// block rows or one 16x4 block row per strip, in any order; rstrip gives, per group of four
// tile rows, the first output channel they produce (-1: none).  The contraction of a strip is
// a list of items (unit, dx): a unit is a group of `cw` input channels (8, or 4 for 16x4
// blocks, where every kept block is then exactly one unit and nothing is zero-filled), dx a
// column of the kernel window; all H rows of the window belong to the item, which is what
// lets the kernel reuse one activation fragment for H output rows.  `32 / cw` consecutive
// items form a column step (one MFMA's K extent per window row).  Input channels are cut
// into slabs of `slab` channels; a column step never crosses a slab.
//   [0..23]                     header, see enum
//   rstrip[nstrips][4]          first output channel of tile rows 4q..4q+3, or -1
//   rslab[nstrips][nslabs+1]    first column step of each (strip, slab)
//   rdesc[ncs][4]               per lane group: its item as unit_in_slab | dx << 8 (cw 4: two
//                               items, one per 16-bit half)
//   rfrag[ncs][H][64][8]        bf16 weights, lane 16q + j of (step, window row dy):
//                               W[strip row j][dy][dx(item)][unit(item) channels] or 0
// Strips are stored heaviest first, or in window order (BSP_ROWS_WINDOW_W).
enum {
  BSP_ROWS_HEADER_WORDS = 24,
  BSP_ROWS_NSTRIPS_W = 0,
  BSP_ROWS_SLAB_W = 1,
  BSP_ROWS_NSLABS_W = 2,
  BSP_ROWS_NCS_W = 3,
  BSP_ROWS_RESERVED_W = 4,
  BSP_ROWS_OFF_STRIP_W = 5,    // offsets in words from the section start
  BSP_ROWS_OFF_SLAB_W = 6,
  BSP_ROWS_OFF_DESC_W = 7,
  BSP_ROWS_OFF_FRAG_W = 8,
  BSP_ROWS_CW_W = 9,
  BSP_ROWS_MAXSTEPS_W = 10,       // most column steps in any (strip, slab)
  BSP_ROWS_MAXSTRIPSTEPS_W = 11,  // most column steps in any strip
  BSP_ROWS_KEPT_ITEMS_W = 12,     // units in kept blocks (work the mask asks for)
  BSP_ROWS_UNION_ITEMS_W = 13,    // units the strips run (kept + zero-filled)
  BSP_ROWS_WINDOW_W = 14,         // strips per window of output channels (see bsp_rows_window), 0: none
  BSP_ROWS_ZEROS_W = 16,          // four zero words, 16-byte aligned: the source of padding pieces
  BSP_ROWS_MAXH = 7,
};

// Thin-input section (bf16 layers with at most four input channels, a network's first layer;
// read by bsp_first.hip).  Such a layer has one block column, so its mask only drops whole
// block rows; the contraction index k = (dy * K + dx) * I + i runs over the whole window,
// 32 per step, and the O / 16 strips interleave the output channels so that a lane ends up
// with 4 * NS consecutive channels of its pixel: row 4q + r of strip s is channel
// q * 4 * NS + 4 * s + r.
//   [0..7]                      header, see enum
//   frag[steps][NS][64][8]      bf16 weights, lane 16g + j of (step t, strip s):
//                               W[channel(s, j)][k = 32 t + 8 g + 0..7] or 0 (k past the window,
//                               block row dropped)
enum {
  BSP_FIRST_HEADER_WORDS = 8,
  BSP_FIRST_NS_W = 0,
  BSP_FIRST_STEPS_W = 1,
  BSP_FIRST_KT_W = 2,        // H * K * I
  BSP_FIRST_OFF_FRAG_W = 3,  // in words from the section start
};

// Channels of one slab of the row-band section: windows are staged 128 channels at a time;
// a pointwise layer keeps all its channels in LDS (one slab) as long as a unit number fits
// the descriptor's eight bits (256 units of `cw` channels).
static inline int32_t bsp_rows_slab(int32_t I, int32_t H, int32_t K, int32_t cw) {
  const int32_t i8 = (I + 7) / 8 * 8;
  const int32_t cap = (H * K > 1) ? 128 : 256 * cw;
  return i8 < cap ? i8 : cap;
}

// Strips per window of output channels.  Pointwise layers group block rows into strips only
// within windows of 64 output channels (four strips) and keep the strips in window order:
// strip s then produces channels of window s / 4 only.  Other layers group rows freely and
// order the strips heaviest first (0).
static inline int32_t bsp_rows_window(int32_t H, int32_t K) { return H * K == 1 ? 4 : 0; }

// Channels kept in LDS at a time, as a function of the layer shape alone so
// that the plan builder and the launcher agree without talking to each other.
static inline int32_t bsp_slab_channels(int32_t I, int32_t H, int32_t K) {
  const int32_t i8 = (I + 7) / 8 * 8;
  const int32_t cap = (H * K > 1) ? 64 : 256;
  return i8 < cap ? i8 : cap;
}

#endif
