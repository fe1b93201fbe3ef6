/*
 * moe_measure.h - measurement and test aids of libmoe_hip.so.
 *
 * Nothing here is part of the MoE layer (include/moe.h), and the conventions
 * of that header do not hold for these calls: they keep state between calls,
 * some allocate, and some synchronise with the device.  They exist so that a
 * benchmark can time the layer's kernels on the stream they are launched on,
 * relate the results to what the board delivers (the expert FFN of the DAOP
 * paper's layer, Sec. II-A, is a dense contraction at prefill sizes and a
 * stream over the selected experts' weights at decode sizes, Table I), and so
 * that a test can reach the layer's failure reporting without a fault.
 */
#ifndef MOE_MEASURE_H
#define MOE_MEASURE_H

#include "moe.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Per-stage GPU time with HIP events
 * recorded on the caller's stream between the kernels of each entry-point
 * call made by THIS thread between begin and end.  Stages: 0 routing (gate,
 * softmax, top-k, prediction), 1 counts + permutation, 2 grouped GEMM1 +
 * SwiGLU, 3 grouped GEMM2, 4 combine, 5 the single kernel that runs a bf16
 * call of at most 16 tokens (routing when the entry point routes, both
 * GEMMs, combine).  begin allocates events for up to max_calls calls (later calls
 * are not recorded); end synchronises with the last recorded event, writes
 * the mean milliseconds per launch of each stage and the number of launches
 * averaged (either pointer may be NULL), and frees the events.
 * Errors: MOE_ERR_SHAPE (bad max_calls, begin twice, end without begin),
 * MOE_ERR_DEVICE.
 */
#define MOE_NUM_STAGES 6
int moe_stage_timing_begin(int32_t max_calls);
int moe_stage_timing_end(float* stage_ms, int32_t* stage_launches);

/*
 * The rate at which the device
 * issues v_mfma_f32_32x32x16_bf16 from registers when nothing else happens,
 * the yardstick for the grouped GEMM of the expert FFN (the paper's layer,
 * Sec. II-A, is that dense contraction).  One workgroup of 8 wavefronts per
 * compute unit runs `iterations` (64 .. 2^22) rounds of 8 independent MFMAs
 * per wavefront and touches no memory in the loop.  random_operands == 0:
 * every operand element is 1.0, the matrix cores draw little power and the
 * loop shows the issue rate at the full clock.  random_operands != 0:
 * operands with random signs and mantissas, as weights and activations have
 * them, which shows what the board's power limit leaves of that rate.
 * The kernel is launched twice on hip_stream and the second launch is timed
 * with HIP events; the call returns after it has finished.
 * Host outputs: *milliseconds = duration of the timed launch, *flop = its
 * floating-point operations (2 x 32 x 32 x 16 per MFMA), *gigahertz (may be
 * NULL) = the shader clock the loop ran at, from the cycle counter and the
 * constant 100 MHz counter read by one wavefront around its loop.  Unlike
 * the layer's entry points this call allocates (16 bytes of device memory,
 * freed before it returns) and copies its clock readings back.
 * Errors: MOE_ERR_SHAPE (iterations out of range, NULL output), MOE_ERR_DEVICE.
 */
int moe_calibrate_mfma(int32_t random_operands, int32_t iterations, float* milliseconds, double* flop,
                       float* gigahertz, void* hip_stream);

/*
 * The rate of a plain read stream
 * out of device memory, the yardstick for decode-size calls, which are bound
 * by reading each selected expert's weights once (the paper's Table I and
 * Sec. III-A: expert parameters dwarf the activations).  One workgroup per
 * compute unit reads its contiguous share of device_buffer (device memory,
 * 16-byte aligned, read only; `bytes` is rounded down to a whole number of
 * rounds of all workgroups, 16 KB each) with 16-byte loads and keeps nothing.
 * The buffer should be much larger than the 256 MB memory-side cache (a
 * layer's expert weights are).  The kernel is launched twice on hip_stream
 * and the second launch is timed with HIP events; the call returns after it
 * has finished and allocates nothing.
 * Host outputs: *milliseconds, *bytes_read = bytes the timed launch read.
 * Errors: MOE_ERR_NULL, MOE_ERR_ALIGN, MOE_ERR_SHAPE (buffer smaller than one
 * round), MOE_ERR_DEVICE.
 */
int moe_calibrate_read_stream(const void* device_buffer, size_t bytes, float* milliseconds, double* bytes_read,
                              void* hip_stream);

/*
 * Test aid: the number of polling rounds a rendezvous of the decode-size
 * kernel waits before it gives up (process-wide; default 4194304).  With 0
 * every rendezvous gives up at once, which lets a test see the failure report
 * of moe_decode_status while every kernel still runs to its end: the affected
 * calls write NaN into y and raise the status word.  Not for production use.
 * Errors: MOE_ERR_SHAPE (negative).
 */
int moe_measure_set_decode_spin_limit(int32_t polling_rounds);

#ifdef __cplusplus
}
#endif
#endif /* MOE_MEASURE_H */
