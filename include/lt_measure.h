/*
 * lt_measure.h -- tuning knobs and measurement aids of the LightTransfer library.
 *
 * Nothing here is part of the method (Section "LightTransfer-Test" and the decoding stage of
 * Section "Preliminary" are served by lt.h alone): these calls exist so that a benchmark can time
 * single launches on the launch stream, force a split size for a sweep, and measure the read rate
 * the device sustains.  Conventions (pointers, streams, statuses) are those of lt.h.
 */
#ifndef LT_MEASURE_H
#define LT_MEASURE_H

#include "lt.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Keys one workgroup of the split decode kernel handles in full / lazy layers (multiples of 64);
 * 0 keeps the built-in choice.  LT_ERR_CAPACITY if the workspace cannot hold the resulting splits. */
lt_status lt_set_split(lt_ctx *ctx, int32_t keys_per_block_full, int32_t keys_per_block_lazy);

/* Decode launches whose workgroups each stream 8192 keys or more leave the last eighth of every
 * (sequence, KV head) to whichever wavefronts finish their own range first (on by default); with
 * 4096 keys or more it is the last quarter when a (sequence, KV head) is spread over at least 16
 * workgroups, and the last eighth when it is spread over at least 8 and the launch runs on the
 * matrix-core kernel or has at most four query heads per KV head.  The reason: the
 * compute units do not all read memory equally fast, and a launch ends with its slowest
 * workgroup.  Which wavefront gets which keys of that part is decided at run time, so the
 * floating-point sums are taken in an order that varies from launch to launch and outputs can
 * differ in their last bits between two runs on the same inputs.  on = 0 gives every key a fixed
 * place (as a forced split, paged layers and shorter ranges always have): bit-identical outputs
 * for identical inputs, at 1.5-3.5 % more time on long contexts. */
lt_status lt_set_shared_tail(lt_ctx *ctx, int32_t on);

/* Which kernel lt_decode_attn / lt_decode_step launch.  Two kernels compute the same attention: one forms q.k and
 * p.v with vector instructions (dot products and FMAs, probabilities in fp32), the other on the matrix cores
 * (probabilities as two bf16 terms, fp32 accumulation).  LT_DECODE_AUTO (the default) takes the matrix-core one for
 * key ranges of 129..2048 keys per workgroup with four or five query heads per KV head and, with six or more, for
 * every range.  The other two values force a kernel, for tests and comparisons. */
enum { LT_DECODE_AUTO = 0, LT_DECODE_VECTOR = 1, LT_DECODE_MATRIX = 2 };
lt_status lt_set_decode_path(lt_ctx *ctx, int32_t path);

/* How the layer's most recent decode launch (lt_decode_attn, lt_decode_step, lt_decode_step_active) was laid out:
 *   plan_host   host, 4 x int32, written: [0] keys per workgroup range, [1] ranges per (sequence, KV head),
 *               [2] first key of the shared tail or -1 without one (lt_set_shared_tail), [3] 1 if the matrix-core
 *               kernel ran, 0 for the vector kernel (lt_set_decode_path)
 * For benchmarks and tests that have to name the kernel they timed.  LT_ERR_INVALID_ARG for a bad handle, layer or
 * pointer, and for a layer that no decode call has run on yet; nothing is written then. */
lt_status lt_decode_plan_read(lt_ctx *ctx, int32_t layer, int32_t *plan_host);

/* Measurement aid: one launch that reads `bytes` of `buf_dev` (rounded down to a multiple of
 * 16 KiB, and at least that) once, with the same kind of loads the decode kernel uses, and discards
 * them; timed by the caller, it gives the read rate this device sustains, the practical ceiling of
 * the decode kernels.
 *   buf_dev   device, 16-byte aligned, at least `bytes` long
 *   sink_dev  device, at least 256 bytes; practically never written */
lt_status lt_probe_read(const void *buf_dev, size_t bytes, void *sink_dev, void *stream);

enum { LT_KERNEL_DECODE_FULL = 0, LT_KERNEL_DECODE_LAZY = 1, LT_KERNEL_APPEND = 2, LT_KERNEL_COUNT = 3 };

/* Bracket every later kernel launch of this context with a pair of HIP events on the launch
 * stream (on != 0), or stop doing so (on == 0).  Enabling discards earlier measurements.  Events
 * are created as launches need them and kept for reuse until lt_destroy. */
lt_status lt_profile_enable(lt_ctx *ctx, int32_t on);

/* Wait for the recorded events and return, for one kernel kind, how many launches were measured
 * and their summed duration in milliseconds.  Launches beyond the internal event pool (65536
 * pairs) are not measured. */
lt_status lt_profile_read(lt_ctx *ctx, int32_t kernel, int64_t *launches, double *total_ms);

#ifdef __cplusplus
}
#endif
#endif /* LT_MEASURE_H */
