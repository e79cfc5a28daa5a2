/*
 * Measurement helpers of libbsp.so: three small kernels that show what this GPU sustains, so
 * that a layer's achieved bandwidth or matrix-core rate can be quoted against a measured peak
 * as well as against the published one.  They are not part of the inference path (no paper
 * passage defines them); bench.py calls them.
 *
 * All pointers are DEVICE memory owned by the caller, 16-byte aligned; `stream` is a
 * hipStream_t passed as void*.  Asynchronous: the caller times the launches with events.
 * Return BSP_OK or a negative status code: NULL, SHAPE, ALIGN or HIP.
 */
#ifndef BSP_BENCH_H
#define BSP_BENCH_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* dst[0..bytes) = src[0..bytes), 16 bytes per lane, grid-stride; bytes a multiple of 16.
 * Moves 2*bytes through HBM when the buffers exceed the caches. */
int bsp_bench_copy(void* dst, const void* src, int64_t bytes, void* stream);

/* Every wave of a grid of `waves` wavefronts (a multiple of 4) issues iters * 8 independent
 * bf16 MFMA 16x16x32 (16 384 flop each) on register operands and adds its accumulators into
 * sink[wave] (float, `waves` entries) so the work cannot be dropped.
 * Total flop = waves * iters * 8 * 16384.  clocks (device, two int64, or null): the first
 * wave stores how many shader-clock ticks and how many ticks of the constant 100 MHz
 * counter its loop took, which gives the shader clock the GPU held during the loop. */
int bsp_bench_mfma_bf16(float* sink, int32_t waves, int32_t iters, int64_t* clocks, void* stream);

/* Every wave of `waves` wavefronts reads iters * 8 conflict-free 16-byte-per-lane pieces from
 * LDS (1 KiB per read and wave) and adds them into sink[wave].  Total bytes read from LDS =
 * waves * iters * 8 * 1024. */
int bsp_bench_lds_read(float* sink, int32_t waves, int32_t iters, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* BSP_BENCH_H */
