// Internal launch entry points, one per kernel family.  Each returns a bsp_status.
#ifndef BSP_LAUNCH_H
#define BSP_LAUNCH_H

#include <hip/hip_runtime.h>

#include "bsp.h"
#include "bsp_device.h"

int bsp_launch_general(const ConvParams& p, int dtype, int bo, int bi, hipStream_t st);

// LDS-tiled bf16 kernels (need the plan's step section and I % 8 == 0).
// BSP_ERR_UNSUPPORTED means "use the general kernel", nothing was launched.
bool bsp_tile_supported(const ConvParams& p, int dtype);
int bsp_launch_tile(const ConvParams& p, int dtype, hipStream_t st);

// Weight-streaming kernel for 1x1 layers with at most 64 output pixels (FC layers).
int bsp_launch_fc_stream(const ConvParams& p, int dtype, int bo, int bi, hipStream_t st);
// The same layers with 8x8 blocks, the activations resident in LDS and the compressed block rows
// streamed past them.  Layers whose activations do not fit LDS in one piece are cut along the
// input channels and need `scratch` (device, 16-byte aligned) for the partial sums:
// BSP_ERR_CAPACITY, with nothing launched and the bytes needed in *need, when it is too small.
int bsp_launch_fc_xlds(const ConvParams& p, int dtype, int bo, int bi, float* scratch, int64_t scratch_bytes,
                       int64_t* need, hipStream_t st);

// LDS-resident kernel (weights and activations of a slab both in LDS); needs the host copy
// of the plan to size LDS.  BSP_ERR_UNSUPPORTED = not applicable, nothing launched.
int bsp_launch_lds(const ConvParams& p, int dtype, const void* plan_host, hipStream_t st);
// the same for int8 codes with int8 results (sum + bias, rounding right shift, saturation)
int bsp_launch_lds_i8(const ConvParams& p, const void* plan_host, int shift, hipStream_t st);

// Row-band kernel (bf16, 1xK and 3xK windows, strides 1 and 2; needs the plan's row-band
// section and its host copy).  BSP_ERR_UNSUPPORTED = not applicable, nothing launched.
int bsp_launch_rows(const ConvParams& p, int dtype, const void* plan_host, hipStream_t st);

// Band kernel (bf16, 3x3 stride 1 padding 1, at most 128 input channels, rows of at most 64
// pixels, strips x column tiles <= 16).  BSP_ERR_UNSUPPORTED = not applicable, nothing launched.
int bsp_launch_band(const ConvParams& p, int dtype, const void* plan_host, hipStream_t st);

// Thin-input kernel (bf16, at most four input channels, windows up to 7x7, 32 or 64 output
// channels; needs the plan's thin-input section and its host copy).  BSP_ERR_UNSUPPORTED = not
// applicable, nothing launched.
int bsp_launch_first(const ConvParams& p, int dtype, const void* plan_host, hipStream_t st);

// Pointwise kernel (bf16, 1x1 windows without padding, any stride, all input channels in one
// slab of the row-band section).  BSP_ERR_UNSUPPORTED = not applicable, nothing launched.
int bsp_launch_pw(const ConvParams& p, int dtype, const void* plan_host, hipStream_t st);

// Three-layer chain 1x1 -> 3x3 -> 1x1 with the intermediates in LDS (bsp_chain.hip).
// BSP_ERR_UNSUPPORTED = not of that form or too large for LDS, nothing launched.
int bsp_launch_chain(const bsp_weights* w1, const bsp_weights* w2, const bsp_weights* w3, const void* X,
                     const float* bias1, const float* bias2, const float* bias3, const void* residual, void* Y,
                     int B, int L, int J, int relu, hipStream_t st);

// 8-bit integer layers: X and payload int8, bias int32 (passed through ConvParams::bias),
// Y int8 after a rounding right shift (y_i8 = 1) or the int32 sums.
int bsp_launch_i8(const ConvParams& p, int y_i8, int shift, int bo, int bi, hipStream_t st);

#endif
