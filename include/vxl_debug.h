/*
 * vxl_debug -- cross-check and measurement hooks of libvxl.so.
 *
 * None of these belongs to the operations of the method; they exist so that tests can run a
 * second implementation of a step on the device and so that a benchmark can time one kernel.
 * They set process-wide switches (atomic; read by every later call of any thread) and are not
 * meant for production callers.  The operations themselves are declared in vxl.h.
 */
#ifndef VXL_DEBUG_H
#define VXL_DEBUG_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

/* on != 0: BF16 calls of vxl_chunk_prefill, vxl_bilevel_decode and vxl_chunk_score_topk_mass run
 * the plain fp32 vector-ALU kernels instead of the matrix-core kernels (the workspace may then be
 * NULL).  An on-device cross-check of the matrix-core path. */
void vxl_debug_force_simple(int on);

/* Pre-filling instance: 0 = default (8 waves, 256-row bands, one workgroup per compute unit);
 * 1 = the same kernel template as two independent 4-wave workgroups per compute unit (128-row
 * bands, a 2-stage ring each).  Any other value selects 0. */
void vxl_debug_prefill_variant(int variant);

/* Step-mode decode kernel form: 0 = the library chooses (4 double-buffered waves), 8 = eight
 * single-buffered waves, 4 = force the default.  Size the decode workspace after setting it. */
void vxl_debug_decode_step_waves(int waves);

/* When both are non-NULL hipEvent_t handles, every following vxl_chunk_prefill records them on
 * its stream right before and right after its main attention kernel (the compaction pre-pass is
 * outside the bracket); (NULL, NULL) switches the recording off. */
void vxl_debug_prefill_events(void* start_event, void* stop_event);

/* Launches a register-resident stream of the matrix instruction the kernels use
 * (v_mfma_f32_32x32x16_bf16: 8 waves per workgroup, 4 independent accumulators per wave,
 * `iters` x 4 instructions per wave) on `stream`, for reading kernel rates against an attained
 * peak.  out: device float [n_workgroups * 512].  Returns the floating-point operations
 * launched, 0 on a bad argument or a failed launch. */
double vxl_debug_mfma_stream(float* out, int n_workgroups, int iters, void* stream);

/* The same stream with operands as an attention kernel sees them -- eight register sets of
 * pseudo-random bf16 values in (-1, 1), another pair in every instruction -- instead of a few
 * small integers repeated: the chip lowers its clock under it, so this, not the stream above, is
 * what a matrix-bound kernel on real data can attain.  `iters` must be even.  Same return value. */
double vxl_debug_mfma_stream_random(float* out, int n_workgroups, int iters, void* stream);

/* The tile loop of the pre-filling kernel on its own (its tile functions over four LDS-resident
 * 64-key tiles, 8 waves x 32 rows per workgroup, head_dim 128; no work items, masks, query or
 * output traffic), with one ingredient left in or taken out by `mode`, for pricing the
 * ingredients of a tile against the bare matrix-instruction stream on the same data:
 *   0 matrix instructions only   1 the full tile code   2 = 1 + ring refills by direct loads
 *   3 = 1 without the softmax arithmetic   4 = 1 with both operand streams from registers
 *   5 the full tile code written for v_mfma_f32_16x16x32_bf16 (a measured alternative that no
 *     kernel uses)   6 = 5 + ring refills   7 matrix instructions only, 16x16x32 (64 per wave, tile).
 * kv: device bf16 values (any finite data), at least vxl_debug_tile_loop_bytes(n_workgroups) bytes;
 * out: device float [n_workgroups * 512]; n_tiles even.  Returns the floating-point operations of
 * the matrix instructions launched, 0 on a bad argument or a failed launch. */
size_t vxl_debug_tile_loop_bytes(int n_workgroups);
double vxl_debug_tile_loop(int mode, const void* kv, float* out, int n_workgroups, int n_tiles, void* stream);

/* Launches a bare streaming read of `bytes` (a multiple of 16) of device memory at `src` by
 * `n_workgroups` workgroups of 256 threads on `stream`; out: device float [n_workgroups * 256].
 * What a bandwidth-bound kernel could at best take for a buffer of that size.  Returns a
 * vxl_status value (0 = launched). */
int vxl_debug_read_stream(const void* src, size_t bytes, float* out, int n_workgroups, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* VXL_DEBUG_H */
