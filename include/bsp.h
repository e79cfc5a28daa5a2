/*
 * bsp — block-sparse convolution / fully-connected inference for AMD MI355X
 * (gfx950).  C ABI of libbsp.so.
 *
 * Notation follows the paper (Section I): a layer computes Y = W * X + b with
 * Y of size M x N x O, X of size L x J x I, W of size O x H x K x I and b of
 * size O.  W-bar[o][i] = W[o][*][*][i] is the O x I matrix whose entries hide
 * the H x K kernel window; the mask Gamma has one entry per b_o x b_i block of
 * W-bar (Eq. (1)) and a zero entry means the whole b_o x H x K x b_i
 * sub-tensor is zero.  A leading batch dimension B is added to X and Y.
 *
 * Layouts (row-major, last index fastest):
 *   X        [B][L][J][I]          input channel innermost
 *   Y        [B][M][N][O]          M = (L + 2*pad_h - H)/stride_h + 1 (floor), N alike
 *   W        [O][H][K][I]          the layout the paper's compiler uses (Section V)
 *   Gamma    [ceil(O/b_o)][ceil(I/b_i)]  one byte per block, 1 = kept, 0 = zeroed
 *   bias     [O] float
 *
 * Block-compressed weights (compressed block row, Section III):
 *   row_ptr  [ceil(O/b_o)+1] int32   exclusive prefix sums of kept blocks per block row
 *   col_idx  [nnzb] int32            kept block columns of each row, ascending
 *   payload  [nnzb][b_o][H][K][b_i]  the kept blocks, fp32, bf16 or int8 codes; where a
 *                                    block overhangs O or I the missing entries are +0
 * For given (W, Gamma) these three arrays are unique, so they are compared
 * bit for bit.
 *
 * Every function returns an int: BSP_OK or a negative bsp_status.  Nothing
 * aborts, throws or prints.  The library allocates no device memory and every
 * buffer belongs to the caller.  The only state it keeps between calls is a
 * per-process memo of values that are pure functions of the arguments (the
 * tile shape picked for a layer shape, the device's CU count, "this kernel may
 * use more than 64 KB of LDS" set once per kernel); it reads no environment
 * variable.
 */
#ifndef BSP_H
#define BSP_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum bsp_status {
  BSP_OK = 0,
  BSP_ERR_NULL = -1,        /* a required pointer is null */
  BSP_ERR_SHAPE = -2,       /* a size is non-positive, inconsistent, or the output is empty */
  BSP_ERR_MASK = -3,        /* a Gamma byte is neither 0 nor 1 */
  BSP_ERR_INDEX = -4,       /* row_ptr not monotone / col_idx not ascending or out of range */
  BSP_ERR_DTYPE = -5,       /* unknown element type, or a combination not offered */
  BSP_ERR_UNSUPPORTED = -6, /* block granularity outside {8x8, 4x16, 16x4}; bsp_conv2d_only: the
                               layer lies outside the requested kernel family */
  BSP_ERR_CAPACITY = -7,    /* an output buffer, or the fixed scratch memory of a *_static call, is too small */
  BSP_ERR_HIP = -8,         /* the HIP runtime reported an error at launch */
  BSP_ERR_ALIGN = -9        /* a device pointer is not 16-byte aligned */
};

enum bsp_dtype { BSP_F32 = 0, BSP_BF16 = 1, BSP_I8 = 2, BSP_I32 = 3 };

/* Static, never-null description of a status code. */
const char* bsp_strerror(int code);

/* ABI revision of this header. */
int bsp_version(void);

/* ------------------------------------------------------------------ host side
 * The packer: Gamma + dense W -> block-compressed weights.  Paper Section II
 * (the kept blocks are compacted, the zeroed ones dropped), Section III
 * (compressed block row / index storage of Gamma) and Section V-B (weights are
 * compressed so that every move is a whole number of blocks, dense or sparse
 * alike).  All pointers are HOST memory.
 */

/* Number of kept blocks, so the caller can size col_idx and payload.
 * gamma: [ceil(O/bo)][ceil(I/bi)] bytes.  Errors: NULL, SHAPE, UNSUPPORTED, MASK. */
int bsp_pack_count(const uint8_t* gamma, int32_t O, int32_t I, int32_t bo, int32_t bi,
                   int64_t* nnzb);

/* Build row_ptr / col_idx / payload.
 *   W               dense weights [O][H][K][I], element type w_dtype (BSP_F32,
 *                   BSP_BF16 as raw 16-bit patterns, or BSP_I8 codes)
 *   payload_dtype   BSP_F32 or BSP_BF16.  fp32 -> bf16 rounds to nearest, ties to
 *                   even; bf16 -> fp32 widens exactly.  BSP_I8 codes are copied
 *                   (w_dtype and payload_dtype must then both be BSP_I8).
 *   row_ptr         out, ceil(O/bo)+1 entries
 *   col_idx         out, nnzb entries
 *   payload         out, nnzb*bo*H*K*bi elements of payload_dtype
 *   payload_capacity_bytes / col_capacity   sizes of the two out buffers
 * Structure follows Gamma only: a kept block of zeros is stored, a zeroed
 * block is dropped whatever W holds there.
 * Errors: NULL, SHAPE, UNSUPPORTED, MASK, DTYPE, CAPACITY. */
int bsp_pack(const void* W, int32_t w_dtype, const uint8_t* gamma,
             int32_t O, int32_t H, int32_t K, int32_t I, int32_t bo, int32_t bi,
             int32_t payload_dtype,
             int32_t* row_ptr, int32_t* col_idx, int64_t col_capacity,
             void* payload, int64_t payload_capacity_bytes);

/* Inverse of bsp_pack onto a dense [O][H][K][I] tensor of element type
 * w_dtype == payload_dtype (zeroed blocks become +0).  Validates the index
 * arrays first.  Errors: NULL, SHAPE, UNSUPPORTED, DTYPE, INDEX. */
int bsp_unpack(const int32_t* row_ptr, const int32_t* col_idx, const void* payload,
               int32_t payload_dtype,
               int32_t O, int32_t H, int32_t K, int32_t I, int32_t bo, int32_t bi,
               void* W);

/* Check row_ptr / col_idx: row_ptr[0] == 0, non-decreasing, col_idx strictly
 * ascending inside each row and < ceil(I/bi).  Errors: NULL, SHAPE,
 * UNSUPPORTED, INDEX. */
int bsp_validate(const int32_t* row_ptr, const int32_t* col_idx,
                 int32_t O, int32_t I, int32_t bo, int32_t bi);

/* Launch plan.  The kernels walk strips of 16 output channels; for each strip
 * the plan lists which 8-wide groups of input channels carry at least one kept
 * block and where in `payload` each kept block of the strip starts.  For bf16
 * it also holds a copy of the kept weights re-ordered into the exact order in
 * which the matrix-core kernels consume them (the paper's compiler likewise
 * lays weights out per sub-volume ahead of time, Sections III and V-B), so
 * that every weight read on the device is one contiguous, aligned run.  The
 * plan is derived from row_ptr / col_idx / payload alone (weights are prepared
 * once, ahead of inference), holds offsets only (position independent), and is
 * private to this library version: build it on the host, copy the bytes to
 * the device, pass the device pointer in bsp_weights.plan.
 *   payload, payload_dtype   the arrays bsp_pack produced (HOST pointers)
 * bsp_plan_size  -> bytes needed.   bsp_plan_build -> fills `plan`.
 * Errors: NULL, SHAPE, UNSUPPORTED, DTYPE, INDEX, CAPACITY. */
int bsp_plan_size(const int32_t* row_ptr, const int32_t* col_idx,
                  int32_t O, int32_t H, int32_t K, int32_t I, int32_t bo, int32_t bi,
                  int32_t payload_dtype, int64_t* bytes);
int bsp_plan_build(const int32_t* row_ptr, const int32_t* col_idx,
                   const void* payload, int32_t payload_dtype,
                   int32_t O, int32_t H, int32_t K, int32_t I, int32_t bo, int32_t bi,
                   void* plan, int64_t capacity_bytes);

/* ---------------------------------------------------------------- device side
 * Block-compressed weights as the kernels see them.  The caller fills the
 * struct (host memory) with DEVICE pointers; all of them 16-byte aligned.
 */
typedef struct bsp_weights {
  int32_t O, I, H, K;       /* layer shape (H = K = 1 for a fully-connected layer) */
  int32_t bo, bi;           /* block granularity: 8x8, 4x16 or 16x4 */
  int32_t dtype;            /* element type of payload, X and Y: BSP_F32 or BSP_BF16 */
  int32_t kernels;          /* 0: the library picks the kernel.  Otherwise a mask of
                               bsp_kernel_family bits the dispatcher may use (the
                               general-shape kernel is always allowed); for tests and timing */
  int64_t nnzb;             /* kept blocks */
  const int32_t* row_ptr;   /* device copies of bsp_pack's arrays that match `payload`, or both */
  const int32_t* col_idx;   /* null.  The kernel that streams compressed block rows (FC layers
                               with 8x8 blocks) reads them on the device when they are given;
                               with null pointers it is not used. */
  const void* payload;      /* device [nnzb][bo][H][K][bi] */
  const void* plan;         /* device copy of bsp_plan_build's output */
  int64_t plan_bytes;
  const void* plan_host;    /* the one HOST pointer: the host copy of the same plan bytes (what
                               bsp_plan_build wrote).  The launchers size tiles and LDS from the
                               plan's counts without a device round trip.  Required (NULL is
                               BSP_ERR_NULL); must stay valid during the call, not after. */
} bsp_weights;

enum bsp_kernel_family {
  BSP_KERNEL_ROWS = 1,  /* row-band kernel: activation fragments reused over window rows */
  BSP_KERNEL_LDS = 2,   /* weights and activations of a slab resident in LDS */
  BSP_KERNEL_TILE = 4,  /* weights streamed through a register ring */
  BSP_KERNEL_FC = 8,    /* weight-streaming kernels for layers with at most 64 output pixels */
  BSP_KERNEL_PW = 16,   /* pointwise layers: all input channels of a pixel tile resident in LDS */
  BSP_KERNEL_BAND = 64, /* 3x3 stride-1 layers with at most 128 input channels and rows of at most
                           64 pixels: one workgroup per band of whole image rows */
  BSP_KERNEL_CHAIN = 32, /* bsp_bottleneck only: run the fused chain even where the library
                            expects the three layers one by one to be faster */
  BSP_KERNEL_FIRST = 128 /* layers with at most four input channels (a network's first layer):
                            the whole window is the contraction */
};

/* Fully-connected layer Y[B][O] = X[B][I] . (Gamma W-bar)^T + bias, work done
 * for kept blocks only.  Paper Section III: a GEMM is handled as a 1x1
 * convolution; Section I, advantages 3-4: zero blocks are skipped and the
 * operation count is proportional to the kept blocks.
 *   X, Y     device, element type w->dtype; bias device float[O] or null (no bias)
 *   stream   a hipStream_t passed as void* (null = default stream)
 * Accumulation is fp32; bias is added in fp32; the result is rounded once
 * (nearest-even) to w->dtype.  Asynchronous: returns after the launch.
 * B = 0 is valid and does nothing (X and Y may then be null).
 * Device memory the library owns: a bf16 layer with 8x8 blocks, 1x1 window and at most 64
 * output pixels whose activations do not fit the 150 KB of LDS in one piece (I * 32 *
 * ceil(pixels / 16) bytes; VGG16's fc6 at batch 16) is cut along its input channels into
 * nseg <= ~32 ranges, and the ranges' partial sums pass through nseg * pixels * O floats of
 * scratch memory that the library allocates (hipMalloc) the first time such a layer runs,
 * keeps, and replaces by a larger one when a larger layer comes.  Such a call therefore
 * cannot be the first of its size under stream capture, and two such calls that overlap in
 * time on different streams race on that memory.  No other call allocates.
 * Errors: NULL, SHAPE, UNSUPPORTED, DTYPE, ALIGN, HIP. */
int bsp_fc(const bsp_weights* w, const void* X, const float* bias, void* Y,
           int32_t B, void* stream);

/* Convolution Y[B][M][N][O] = (Gamma W) * X[B][L][J][I] + bias (Section I),
 * cross-correlation with zero padding, work done for kept blocks only.
 * Dilation and groups are not expressible.  Same types, rounding, stream and
 * error conventions as bsp_fc; SHAPE if M or N would be < 1. */
int bsp_conv2d(const bsp_weights* w, const void* X, const float* bias, void* Y,
               int32_t B, int32_t L, int32_t J,
               int32_t stride_h, int32_t stride_w, int32_t pad_h, int32_t pad_w,
               void* stream);

/* The same layers with a fused epilogue (a step towards the fusion the paper's Section VI
 * explores for its sub-graph tiling: the element-wise work after a convolution shares its
 * pass over Y):
 *   Y = act( round(conv + bias) + residual ), rounded again to w->dtype
 *   residual   device, same shape and element type as Y (16-byte aligned), or null
 *   relu       nonzero: act = max(., 0); zero: identity
 * The sum of convolution and bias is rounded to w->dtype before the residual is added, i.e.
 * the result equals bsp_conv2d followed by an element-wise add and activation in w->dtype's
 * precision (fp32 arithmetic), without the extra pass over Y.  With residual null and relu 0
 * this is bsp_conv2d.  Errors as bsp_conv2d, plus ALIGN for the residual. */
int bsp_conv2d_fused(const bsp_weights* w, const void* X, const float* bias,
                     const void* residual, int32_t relu, void* Y,
                     int32_t B, int32_t L, int32_t J,
                     int32_t stride_h, int32_t stride_w, int32_t pad_h, int32_t pad_w,
                     void* stream);
int bsp_fc_fused(const bsp_weights* w, const void* X, const float* bias, const void* residual,
                 int32_t relu, void* Y, int32_t B, void* stream);

/* bsp_fc_fused for callers that cannot allocate device memory or let a library do it: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments, same kernels and bit-identical results; the partial sums of a layer cut along its
 * input channels (see bsp_fc) go to a fixed array of 4 MiB that is part of the library's
 * image on each GPU (held until the process ends) instead of allocated memory, and nothing
 * is allocated or freed.  A layer that needs more (nseg * B * O * 4 bytes > 4 MiB) is refused
 * with BSP_ERR_CAPACITY and nothing launched.  All calls on one GPU share that array and it
 * keeps the last call's contents (every value a call reads it has written itself, nothing
 * needs clearing): calls that overlap in time on one GPU race.
 * Errors: as bsp_fc_fused, plus CAPACITY. */
int bsp_fc_fused_static(const bsp_weights* w, const void* X, const float* bias,
                        const void* residual, int32_t relu, void* Y, int32_t B, void* stream);

/* Same layer, but always through the general-shape kernel (no shape-specialised
 * fast path).  For testing and for timing the dispatcher's choice. */
int bsp_conv2d_general(const bsp_weights* w, const void* X, const float* bias, void* Y,
                       int32_t B, int32_t L, int32_t J,
                       int32_t stride_h, int32_t stride_w, int32_t pad_h, int32_t pad_w,
                       void* stream);

/* Same layer (with the fused epilogue's arguments), but through one kernel family only:
 * family is one bsp_kernel_family bit, or 0 for the general-shape kernel.  Returns
 * BSP_ERR_UNSUPPORTED, with nothing launched, when the layer lies outside that family's limits.
 * For testing each kernel on its own and for timing the dispatcher's choice. */
int bsp_conv2d_only(const bsp_weights* w, const void* X, const float* bias, const void* residual,
                    int32_t relu, void* Y, int32_t B, int32_t L, int32_t J,
                    int32_t stride_h, int32_t stride_w, int32_t pad_h, int32_t pad_w,
                    int32_t family, void* stream);

/* Three consecutive layers on one output tile, the two intermediates kept on chip (paper
 * Section VI: depth-wise tiling of consecutive layers, tiles never leaving the chip between
 * them).  The chain is 1x1 (w1: I -> C), 3x3 with stride 1 and padding 1 (w2: C -> C), 1x1
 * (w3: C -> O):
 *   T1 = act(round(conv(X, w1) + bias1)),  T2 = act(round(conv(T1, w2) + bias2)),
 *   Y  = round(act(round(conv(T2, w3) + bias3) + residual))
 * with act = ReLU when relu != 0 and the identity otherwise: exactly what three bsp_conv2d
 * calls with the fused epilogue give (each intermediate is rounded to bf16 where it would
 * have been stored), without T1 and T2 ever reaching memory.
 *   w1, w2, w3   bf16 layers with 8x8 or 4x16 blocks and plans from bsp_plan_build
 *   X            device [B][L][J][I] bf16;  Y device [B][L][J][O] bf16
 *   bias1..3     device float or null;  residual device, shape and type of Y, or null
 * Returns BSP_ERR_UNSUPPORTED, with nothing launched, when the chain is not of this form, when
 * its intermediates do not fit the 160 KB of LDS, or when streaming the three layers' weights
 * once per output band would cost more memory traffic than keeping the intermediates on chip
 * saves (deep layers on small images); the caller then runs the layers one by one.  Setting
 * BSP_KERNEL_CHAIN in the `kernels` field of any of the three overrides the last reason.
 * Asynchronous.  Errors: NULL, SHAPE, UNSUPPORTED, DTYPE, ALIGN, HIP. */
int bsp_bottleneck(const bsp_weights* w1, const bsp_weights* w2, const bsp_weights* w3,
                   const void* X, const float* bias1, const float* bias2, const float* bias3,
                   const void* residual, int32_t relu, void* Y,
                   int32_t B, int32_t L, int32_t J, void* stream);

/* ------------------------------------------- block-sparse x block-sparse product
 * Paper Section III-A: C = (Gamma A) (Omega B)^t with k x k blocks; a block product is done
 * if and only if both blocks are kept (the paper merges the two sorted lists of kept block
 * columns; here two block rows of each operand meet in one matrix-core tile, their column
 * sets are united per side and intersected across the sides, 64 columns at a time, and only
 * the surviving columns are multiplied).
 * An operand is what bsp_pack makes of a matrix [rows*8][1][1][cols*8] with 8x8 blocks:
 * row_ptr / col_idx / payload [nnzb][8][8], plus row pointers per sixteen block columns from
 * bsp_bcsr_segments (a second level of row_ptr: it grows with rows * cols / 16, not with the
 * dense matrix).
 */
typedef struct {
  int32_t rows, cols;      /* block rows and block columns */
  int32_t k;               /* block edge; 8 */
  int32_t dtype;           /* BSP_BF16 */
  int64_t nnzb;
  const int32_t* row_ptr;  /* device, rows + 1 */
  const int32_t* col_idx;  /* device, nnzb, ascending within a block row */
  const void* payload;     /* device, [nnzb][k][k], 16-byte aligned */
  const int32_t* seg_ptr;  /* device, [rows][ceil(cols/16) + 1]: seg_ptr[r][s] = position in
                              col_idx / payload of row r's first kept block with column >= 16 s */
} bsp_bcsr;

/* Host: fill seg_ptr[rows][ceil(cols/16) + 1] from row_ptr / col_idx (validated first:
 * ascending, distinct, in range).  seg_ptr[r][0] = row_ptr[r], the last entry = row_ptr[r+1].
 * Errors: NULL, SHAPE, INDEX. */
int bsp_bcsr_segments(const int32_t* row_ptr, const int32_t* col_idx, int32_t rows, int32_t cols,
                      int32_t* seg_ptr);

/* Device: C [A.rows*k][B.rows*k] float, row-major, = A . B^t, every element written (zero
 * where no block pair matches); fp32 accumulation of bf16 products.  A.cols must equal
 * B.cols.  seg_ptr and col_idx are trusted to describe the payload (as bsp_bcsr_segments and
 * bsp_pack wrote them).  Asynchronous on `stream`.  Errors: NULL, SHAPE, DTYPE,
 * UNSUPPORTED (k != 8), ALIGN, HIP. */
int bsp_spgemm_nt(const bsp_bcsr* A, const bsp_bcsr* B, float* C, void* stream);

/* ------------------------------------------------------- choosing the mask (host)
 * Paper Section IV ("Predetermined Sparsity ratio and Full Training Ahead"): every mask
 * entry stands for one block W_i; blocks are ranked by an importance measure and the least
 * important ones are zeroed.
 */
enum bsp_importance {
  BSP_IMPORTANCE_L2 = 0,   /* sqrt(sum w^2) over the block */
  BSP_IMPORTANCE_L1 = 1,   /* sum |w| */
  BSP_IMPORTANCE_VAR = 2   /* (1/n) sum (w - mean)^2, n = bo*H*K*bi (overhang counts as zeros) */
};

/* Importance of every block of W [O][H][K][I] (float), in fp64, summed in the block's storage
 * order.  score: out, [ceil(O/bo)][ceil(I/bi)].  Errors: NULL, SHAPE, UNSUPPORTED. */
int bsp_block_importance(const float* W, int32_t O, int32_t H, int32_t K, int32_t I,
                         int32_t bo, int32_t bi, int32_t measure, double* score);

/* Gamma with round(density * n) blocks kept: blocks sorted by ascending importance (ties:
 * lower block index first) and the first n - round(density * n) zeroed; n counts the blocks
 * of the layer, or of each block row when per_row != 0.  density in [0, 1].
 * gamma: out, [ceil(O/bo)][ceil(I/bi)] bytes.  Errors: NULL, SHAPE, UNSUPPORTED. */
int bsp_select_mask(const float* W, int32_t O, int32_t H, int32_t K, int32_t I,
                    int32_t bo, int32_t bi, int32_t measure, double density, int32_t per_row,
                    uint8_t* gamma);

/* One step of the incremental schedule (Section IV, "Sparsity Ratio as Incremental"): with k
 * kept blocks still above the target round(target_density * n), zero the
 * max(ceil(0.05 k), 1) least important kept blocks (never more than k).  gamma: in/out.
 * zeroed: out, how many were zeroed (0 when the target is reached).
 * Errors: NULL, SHAPE, UNSUPPORTED, MASK. */
int bsp_mask_step(const float* W, int32_t O, int32_t H, int32_t K, int32_t I,
                  int32_t bo, int32_t bi, int32_t measure, double target_density,
                  uint8_t* gamma, int32_t* zeroed);

/* ------------------------------------------------------------- 8-bit integers
 * The paper deploys 8-bit integer layers (Section I: the sparse model is quantized to
 * 8-bit integer arithmetic; Section III: weights 8 bits, bias 32 bits; Section V, Eq. (8):
 * INT8 tensors with power-of-two scales).
 */

/* Host.  Round-to-nearest quantizer of Section V, Eq. (8):
 *   Delta = max|W| / 2^(bits-1),  code = Round(W / Delta)  (ties to even),
 * codes clamped to [-2^(bits-1), 2^(bits-1) - 1] (only +max|W| itself is clamped).
 *   W      n floats;  codes  n int8 out;  delta  out (0 when W is all zero)
 *   bits   2..8
 * Errors: NULL, SHAPE (n < 0 or bits out of range). */
int bsp_quantize(const float* W, int64_t n, int32_t bits, int8_t* codes, double* delta);

/* Device.  Integer layer on packed int8 codes (bsp_pack with w_dtype = payload_dtype =
 * BSP_I8; plan built for BSP_I8):
 *   acc = bias + sum over kept blocks of W_code * X_code          (exact, 32 bits)
 *   X       int8  [B][L][J][I];  bias  int32 [O] or null
 *   y_dtype BSP_I32: Y int32 [B][M][N][O] = acc (shift ignored)
 *           BSP_I8:  Y int8 = saturate((acc + 2^(shift-1)) >> shift), shift 0..31
 *                    (power-of-two output scale, round to nearest, ties upward)
 * Same shape, stream, B = 0 and error conventions as bsp_conv2d; DTYPE if the weights
 * are not BSP_I8 or y_dtype is neither; SHAPE if shift is out of range.  X needs 8-byte,
 * Y and the payload 16-byte alignment. */
int bsp_conv2d_i8(const bsp_weights* w, const int8_t* X, const int32_t* bias, void* Y,
                  int32_t y_dtype, int32_t shift, int32_t B, int32_t L, int32_t J,
                  int32_t stride_h, int32_t stride_w, int32_t pad_h, int32_t pad_w,
                  void* stream);

/* The 1x1 case on X[B][I] (Section III: a GEMM is a 1x1 convolution). */
int bsp_fc_i8(const bsp_weights* w, const int8_t* X, const int32_t* bias, void* Y,
              int32_t y_dtype, int32_t shift, int32_t B, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* BSP_H */
