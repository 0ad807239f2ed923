/*
 * wsvd_test.h - entry points of libwsvd.so that are NOT part of the product boundary: hooks for tests, tuning and
 * profiling.  Nothing here is needed to use the library (see wsvd.h for that); the calls exist so that measurements and
 * tests can reach into it through plain C symbols.
 */
#ifndef WSVD_TEST_H
#define WSVD_TEST_H

#include "wsvd.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * In-kernel timeline (profiling build only: the library compiled with -DWSVD_TIMELINE, `python -m
 * paper_2604_02570_amd.build --timeline` -> libwsvd_timeline.so).  The decode-attention kernels then write the chip-wide
 * 100 MHz wall clock at marked points: int64 buf[(workgroup * 16 + wave) * 16 + slot], workgroup = linear id of the
 * launch grid, written by lane 0 of each wavefront.  dev_ptr: DEVICE buffer, 16-byte aligned, owned by the caller, at
 * least workgroups * 2048 bytes (a smaller buffer switches the stamps of that launch off); NULL detaches.  Slots of the
 * decode attention: 0 kernel entry, 1 first loads issued, 2 factors staged, 3 query limbs ready, 4 first tile consumed,
 * 5 last tile consumed, 6 wave's partial result written, 7 workgroup barrier passed, 8 output stored.
 * The product build returns WSVD_E_UNSUPPORTED.
 */
wsvd_status wsvd_timeline_set_buffer(wsvd_ctx *ctx, void *dev_ptr, size_t bytes);

/*
 * Settings of wsvd_ctx_set_option (wsvd.h) that choose between alternative kernels, for tests and measurements:
 *   "fused_step":     wsvd_decode_step uses 0 = two launches (default), 1 = the single-launch kernel where one exists,
 *                     2 = the single-launch kernel or WSVD_E_UNSUPPORTED
 *   "step_deferred":  which two launches: 1 = projection launch + attention launch that finishes the row where that
 *                     pair exists (default), 2 = that pair or WSVD_E_UNSUPPORTED, 0 = always the append kernel + the
 *                     attention kernel
 *   "timeline_kernel": profiling build, wsvd_decode_step: 0 = the attention launch writes the stamps (default), 1 = the
 *                     projection launch does (slots: 0 entry, 1 loads issued, 2 hidden states staged, 3 products
 *                     done, 4 wave partials in LDS, 5 partial sums stored)
 *   "step_slices":    d_model slices of that projection launch: 0 = automatic (about one workgroup per CU), 1..4
 *   "append_helpers": helper workgroups per unit of the default append kernel: -1 = automatic, 0 or 2
 *   "linear_direct":  1 = the W4A8 linear layers read their operands straight from memory (no LDS staging)
 *   "prefill_tiled":  1 = wsvd_prefill_attn and wsvd_prefill_append take their tiled kernels also for small calls
 *   "project_shape":  kernel of the tiled prefill projection: 0 = automatic, 1 / 2 = LDS-staged with 4 / 8 waves per
 *                     workgroup, 44 / 42 / 24 / 21 = direct kernel with that many channel x token tiles per wave
 *   "static_limit_kib": wsvd_decode_attn_static treats its static array as this many KiB (0 = its real size, 8192): lets
 *                     a test see the WSVD_E_WORKSPACE rejection with buffers that are valid for the call
 */

/*
 * Measurement aid: launches once more the SECOND launch of the last deferred-row wsvd_decode_step made on this context
 * with this description (the attention that sums the step's partial sums, quantises, stores the new rows and attends
 * over them).  The partial sums and the pending words of that step are still in the workspace, the lengths of `cache`
 * must already include the step's row (any cache that went through such a step with the same hidden states will do):
 * the launch stores the same rows again and returns the same output, so a benchmark can time this kernel alone.
 * Arguments as wsvd_decode_attn.  WSVD_E_UNSUPPORTED where wsvd_decode_step has no such pair of launches.
 */
wsvd_status wsvd_test_step_attention(wsvd_ctx *ctx, const wsvd_layer_desc *desc, const void *q, const void *q_scale,
                                     const void *B_K, const void *B_V, wsvd_cache *cache, int32_t max_seq_len, void *out,
                                     void *hip_stream);

/*
 * Measurement aid, not part of the method: a kernel that only READS `bytes` bytes (DEVICE pointer, 16-byte
 * aligned) with `workgroups` workgroups of 512 threads, each streaming one contiguous share.  Benchmarks run it
 * over the buffers the attention streams to report what a pure reader reaches on the same data.
 */
wsvd_status wsvd_probe_stream_read(wsvd_ctx *ctx, const void *ptr, size_t bytes, int32_t workgroups, void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* WSVD_TEST_H */
