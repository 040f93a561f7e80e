/* sd_measure.h -- measurement kernels behind the bounds quoted for the hot path (no part of the method).
 *
 * The accept / reflect, draft and advance kernels are bound by HBM, the MLP denoiser's GEMMs by the bf16
 * matrix cores.  Next to the published peaks (8 TB/s, 2.5 PFLOP/s) the benchmark reports what plain
 * hand-written kernels reach on the same chip: a streaming copy / read / fill, and a loop of nothing but
 * MFMAs on register operands.  Both are launched like the kernels they are compared with (workgroups
 * of 256 or 512 threads over all compute units) and timed by the caller with events on `stream`.
 * Pointers are device memory owned by the caller; return value 0 or a negative sd_status (sd.h).
 */
#ifndef SD_MEASURE_H
#define SD_MEASURE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* One pass over `bytes` (a multiple of 16; buffers 16-byte aligned) with 16-byte accesses, consecutive lanes
 * on consecutive addresses, workgroups striding over the buffer:
 *   mode 0  dst[i] = src[i]                      (reads bytes, writes bytes)
 *   mode 1  sums src into 4 bytes per workgroup written to dst (dst needs 4 * 4096 bytes)   (reads bytes)
 *   mode 2  dst[i] = constant                    (writes bytes)
 *   mode 3, 4, 5  the same three passes with the access pattern of the window kernels: a workgroup takes
 *           whole rows of 49152 bytes (a 12288-wide fp32 row), row after row, and a thread requests all its
 *           pieces of a row before it uses any (`bytes` a multiple of 49152)
 * workgroups = 0 picks 16 per compute unit. */
int sd_measure_stream(const void* src, void* dst, size_t bytes, int32_t mode, int32_t workgroups, void* stream);

/* `iters` rounds of 16 independent MFMAs per wavefront on register operands, 512 threads per workgroup,
 * `workgroups` workgroups (0 = one per compute unit):
 *   shape 0  v_mfma_f32_32x32x16_bf16  (32768 flop each)
 *   shape 1  v_mfma_f32_16x16x32_bf16  (16384 flop each)
 * The accumulators are summed into sink[workgroup] (sink: `workgroups` floats) so that nothing is optimised
 * away.  *flops (host, may be NULL) receives the floating-point operations of the launch. */
int sd_measure_mfma(int32_t shape, int32_t iters, int32_t workgroups, float* sink, double* flops, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* SD_MEASURE_H */
