/*
 * daop_policy.h - C ABI of the count-driven policy steps of DAOP (arXiv 2501.10375) that consume
 * what the MoE layer (moe.h) produces: per-layer expert activation counts and next-layer
 * predictions.  All of it is small integer / index work that runs on the device so the counts
 * never leave HBM; every call enqueues one or two small kernels on `hip_stream` and returns.
 *
 * Conventions are those of moe.h: all pointers are DEVICE pointers (dense, row-major, 16-byte
 * aligned), the caller owns every buffer, return value MOE_OK or a negative moe_status_t,
 * arguments are validated on the host before any HIP call, nothing is enqueued on error.
 * A placement mask `on_gpu` is uint8 [n_layers, n_experts] (or [n_experts]): non-zero = the
 * expert is in the GPU expert cache.  Limits: 1 <= n_experts <= 64, 1 <= n_layers <= 1024.
 */
#ifndef DAOP_POLICY_H
#define DAOP_POLICY_H

#include <stddef.h>
#include <stdint.h>

#include "moe.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Eq. 1 (Sec. III, observation 2): similarity of two activation patterns, the mean over layers of
 * the cosine similarity between corresponding rows.  counts_p, counts_d: int32 [n_layers,
 * n_experts] (prefill and decode counts; the cosine is scale-invariant, so counts stand for the
 * paper's probabilities).  out: fp64 [1 + n_layers]: out[0] the similarity, out[1 + l] the cosine
 * of layer l.  A layer whose row is all zero in either matrix contributes 0.  Arithmetic: fp64,
 * sums in index order.
 */
int daop_similarity(int32_t n_layers, int32_t n_experts, const int32_t* counts_p, const int32_t* counts_d,
                    double* out, void* hip_stream);

/*
 * Variation of a sequence's activation pattern during decoding (Sec. VI-B "Limitation & Future
 * Work", which measures it on windows of 15 tokens): the decode steps are cut into consecutive
 * windows of `window` steps (a shorter tail is left out), every window gives an n_layers x
 * n_experts matrix of activation counts, and each window is compared with the next one by Eq. 1.
 *   idx  int32 [n_layers, steps, top_k]  in: the experts every layer selected at every decode step
 *        (moe_layer's topk_idx of step s, layer l at idx[l, s, :]); every index in [0, n_experts)
 *   out  fp64 [1 + max(steps / window - 1, 0)]  out: out[0] the mean over the window pairs (0 when
 *        there are fewer than two whole windows), out[1 + v] the similarity of windows v and v + 1
 * Arithmetic as in daop_similarity.  Limits: steps <= 1048576, 1 <= window <= 4096, 1 <= top_k <= 8.
 */
int daop_window_variation(int32_t n_layers, int32_t n_experts, int32_t steps, int32_t top_k, int32_t window,
                          const int32_t* idx, double* out, void* hip_stream);

/*
 * Algorithm 1 (Sec. IV-B, sequence-specific expert allocation), the cache update of every block
 * from the block's prefill counts.  Per layer: SwapNum = n_experts / 2; the SwapNum most active
 * experts outside the cache (ties: lower index) are paired in rank order with the SwapNum least
 * active experts inside it (ties: lower index; the shorter list bounds the pairs); a pair is
 * exchanged when hot >= swap_in_out * cold (token counts, compared in fp64) and hot > 0.
 *   counts   int32 [n_layers, n_experts]            in
 *   on_gpu   uint8 [n_layers, n_experts]            in/out: updated placement
 *   swaps    int32 [n_layers, n_experts / 2, 2]     out: (expert moved in, expert moved out) in pair
 *                                                   order, unused entries -1; may be NULL
 *   n_swaps  int32 [n_layers]                       out; may be NULL
 * The paper's threshold is swap_in_out = 1.05.  Errors: MOE_ERR_SHAPE also for swap_in_out < 0 or NaN.
 */
int daop_plan_swaps(int32_t n_layers, int32_t n_experts, const int32_t* counts, uint8_t* on_gpu,
                    double swap_in_out, int32_t* swaps, int32_t* n_swaps, void* hip_stream);

/*
 * Memory initialisation (Sec. IV-A): the initial expert cache from calibration counts.  Every
 * layer gets slots / n_layers experts, those with the most calibration tokens (ties: lower
 * index); the remaining slots (fewer than n_layers) go to the experts outside that base with the
 * highest activation frequency count / (tokens of the layer), compared exactly (ties: lower
 * layer, then lower expert).  slots is clamped to [0, n_layers * n_experts]; with the paper's
 * expert cache ratio, slots = ratio * n_layers * n_experts.
 *   calib_counts int32 [n_layers, n_experts] in;  on_gpu uint8 [n_layers, n_experts] out.
 */
int daop_memory_init(int32_t n_layers, int32_t n_experts, const int32_t* calib_counts, int32_t slots,
                     uint8_t* on_gpu, void* hip_stream);

/*
 * Prediction with graceful degradation (Sec. IV-C): the next layer's gate applied to the current
 * hidden states as in moe_predict_next, then, per token, if every selected expert is outside the
 * GPU cache, the selected expert with the lowest probability is replaced by the most probable
 * expert inside it (ties: lower index); if the cache holds none the selection is kept.  Weights
 * are the selected probabilities renormalised; the list stays in descending probability.
 *   x [tokens, hidden], w_gate_next [n_experts, hidden] in shape->dtype; gate_bias_next fp32
 *   [n_experts] or NULL; on_gpu uint8 [n_experts] (the next layer's row of the placement);
 *   pred_idx int32 [tokens, top_k] out; pred_w fp32 [tokens, top_k] out or NULL.
 * tokens == 0 is MOE_OK.
 */
int daop_predict_degraded(const moe_shape_t* shape, int32_t tokens, const void* x, const void* w_gate_next,
                          const float* gate_bias_next, const uint8_t* on_gpu, int32_t* pred_idx, float* pred_w,
                          void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* DAOP_POLICY_H */
