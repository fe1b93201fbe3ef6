/*
 * moe.h - C ABI of the MI355X (gfx950) sparse Mixture-of-Experts layer.
 *
 * The library computes the data-parallel hot path that the DAOP inference
 * engine (arXiv 2501.10375) is built around: for the hidden states of one
 * sequence it runs the gating function and top-k expert selection (Sec. II-A,
 * "MoE Structure"), counts how many of the sequence's tokens each expert
 * received (the "activity level" of Sec. IV-B / Algorithm 1 that drives expert
 * placement), predicts the next layer's experts by applying the next layer's
 * gate to the same hidden states (Sec. III observation 3; Sec. IV-C "Accuracy
 * Stabilization"), and executes the selected SwiGLU experts on their tokens
 * and combines the results with the gate weights (Sec. II-A; the local expert
 * execution step of Algorithm 1).  Model shapes follow Table III.
 *
 * Conventions common to every entry point
 *   - All tensor pointers are DEVICE pointers on the current HIP device, dense
 *     row-major with the last index contiguous, 16-byte aligned.  The caller
 *     owns every buffer, including the workspace; the library allocates
 *     nothing and keeps no state between calls.
 *     The workspace is scratch: its contents never need initialising and are
 *     undefined afterwards.  Two calls that use the same workspace must not
 *     run at the same time (order them on one stream or with events).
 *   - Every call only enqueues kernels whose arguments depend on nothing but
 *     the call's own arguments, so a call may be recorded into a HIP graph
 *     (stream capture) and replayed.
 *   - `hip_stream` is a hipStream_t passed as void* (NULL = the default
 *     stream).  Calls validate their arguments on the host, enqueue kernels on
 *     that stream and return without synchronising.  Outputs are valid once
 *     the stream has reached the end of the enqueued work.
 *   - Return value: MOE_OK or a negative moe_status_t.  Argument validation
 *     happens before the first HIP call, so every error except
 *     MOE_ERR_DEVICE can be provoked on a host without a GPU.  Nothing is
 *     enqueued when an error is returned.  No exceptions, no abort().
 *   - tokens == 0 is MOE_OK: nothing is computed; `counts` is zeroed unless
 *     `accumulate` is set.  The per-token buffers (x, topk_idx, topk_w, y,
 *     pred_idx, pred_w) may then be NULL.
 *   - Limits: 1 <= top_k <= min(n_experts, 8); n_experts <= 64; hidden and ffn
 *     are multiples of 64; tokens <= 1048576.
 *   - Expert selection: softmax over all experts in fp32, the top_k largest
 *     probabilities in descending order (equal probabilities: lower expert
 *     index first), their weights renormalised to sum to one.
 *   - bf16 calls with at most 32 tokens run their experts (at most 16 tokens:
 *     the whole layer) as one persistent kernel, one workgroup per compute
 *     unit, whose workgroups wait for one another between the two expert
 *     GEMMs.  The wait is bounded, so a call always ends, but it only
 *     succeeds when the device can hold the whole grid at once, i.e. when no
 *     other kernel (another stream, another process) occupies compute units
 *     for the duration of the call.  A workgroup whose wait runs out writes
 *     NaN into its part of y and raises a status word that moe_decode_status
 *     reads; the call itself has long returned MOE_OK by then.  (The
 *     prefill-size grouped GEMM is persistent too, but no workgroup of it
 *     ever waits for another.)
 *   - Determinism: no floating-point atomics are used; two calls on the same
 *     inputs give bitwise identical outputs.  moe_layer gives bitwise the same
 *     outputs as moe_route (+ moe_predict_next) followed by moe_expert_ffn.
 */
#ifndef MOE_H
#define MOE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    MOE_OK = 0,
    MOE_ERR_NULL = -1,      /* a required pointer is NULL                         */
    MOE_ERR_SHAPE = -2,     /* a dimension is outside the limits above            */
    MOE_ERR_DTYPE = -3,     /* dtype is not a moe_dtype_t value                   */
    MOE_ERR_WORKSPACE = -4, /* workspace_bytes is smaller than the call needs     */
    MOE_ERR_ALIGN = -5,     /* a pointer is not 16-byte aligned                   */
    MOE_ERR_DEVICE = -6,    /* a kernel launch failed (hipGetLastError != success) */
    MOE_ERR_TOO_LARGE = -7  /* moe_layer_static: the call needs more than MOE_STATIC_SCRATCH_BYTES */
} moe_status_t;

typedef enum {
    MOE_F32 = 0, /* fp32 storage, fp32 arithmetic                                          */
    MOE_BF16 = 1 /* bf16 storage, fp32 accumulation, bf16 intermediate activation and output */
} moe_dtype_t;

/* Shape of one MoE layer (Table III: Mixtral 8x7B = {4096, 14336, 8, 2}, Phi-3.5-MoE = {4096, 6400, 16, 2}). */
typedef struct {
    int32_t hidden;    /* H: width of a hidden state                         */
    int32_t ffn;       /* F: inner width of one SwiGLU expert                */
    int32_t n_experts; /* E                                                   */
    int32_t top_k;     /* k: experts activated per token                      */
    int32_t dtype;     /* moe_dtype_t of x, gate weights, expert weights, y   */
    int32_t reserved;  /* must be 0                                           */
} moe_shape_t;

/* Human-readable name of a status code (static storage, never NULL). */
const char* moe_status_string(int status);

/*
 * Workspace sizes in bytes for calls with at most `max_tokens` tokens.
 * moe_workspace_bytes covers every entry point; moe_route_workspace_bytes is
 * the smaller amount moe_route and moe_predict_next need on their own.
 * Errors: MOE_ERR_NULL, MOE_ERR_SHAPE, MOE_ERR_DTYPE.
 */
int moe_workspace_bytes(const moe_shape_t* shape, int32_t max_tokens, size_t* out_bytes);
int moe_route_workspace_bytes(const moe_shape_t* shape, int32_t max_tokens, size_t* out_bytes);

/*
 * Gating function and expert selection for the tokens of one sequence
 * (Sec. II-A), plus the per-sequence expert activation counts of Sec. IV-B /
 * Algorithm 1.
 *
 *   x         [tokens, H]  in   hidden states after self-attention, shape->dtype
 *   w_gate    [E, H]       in   gate weights, shape->dtype
 *   gate_bias [E]          in   fp32 per-expert logit offset, or NULL (the models have none;
 *                               synthetic workloads use it to skew routing)
 *   topk_idx  [tokens, k]  out  int32 selected experts, descending probability
 *   topk_w    [tokens, k]  out  fp32 renormalised gate weights (sum to 1 per token)
 *   counts    [E]          out  int32 number of (token, j) selections of each expert in this
 *                               call; sums to tokens*k.  accumulate = 0 overwrites, 1 adds to the
 *                               existing values (a decode loop building per-sequence counts).
 *   workspace               scratch of at least moe_route_workspace_bytes(shape, tokens)
 */
int moe_route(const moe_shape_t* shape, int32_t tokens, const void* x, const void* w_gate,
              const float* gate_bias, int32_t* topk_idx, float* topk_w, int32_t* counts,
              int32_t accumulate, void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Next-layer expert prediction (Sec. III observation 3; Sec. IV-C): the gate of
 * layer l+1 applied to the hidden states `x` that layer l's gate sees.  Same
 * arithmetic as moe_route with the next layer's gate.
 *
 *   pred_idx    [tokens, k] out  int32 predicted experts of the next layer
 *   pred_w      [tokens, k] out  fp32 their renormalised weights, or NULL
 *   pred_counts [E]         out  int32 histogram of pred_idx (overwritten), or NULL
 */
int moe_predict_next(const moe_shape_t* shape, int32_t tokens, const void* x,
                     const void* w_gate_next, const float* gate_bias_next, int32_t* pred_idx,
                     float* pred_w, int32_t* pred_counts, void* workspace, size_t workspace_bytes,
                     void* hip_stream);

/*
 * Expert execution and weighted combine (Sec. II-A; Algorithm 1's local expert
 * execution): for every token t
 *   y[t] = sum_j topk_w[t,j] * W2_e ( silu(W1_e x[t]) * (W3_e x[t]) ),  e = topk_idx[t,j].
 * Tokens are grouped per expert on the device so that each expert's weights
 * are applied to all of its tokens at once.
 *
 *   topk_idx, topk_w  in   as produced by moe_route (every index must be in [0, E))
 *   w1, w3  [E, F, H] in   gate- and up-projection, shape->dtype
 *   w2      [E, H, F] in   down-projection, shape->dtype
 *   y       [tokens, H] out shape->dtype
 *   workspace              scratch of at least moe_workspace_bytes(shape, tokens)
 */
int moe_expert_ffn(const moe_shape_t* shape, int32_t tokens, const void* x, const int32_t* topk_idx,
                   const float* topk_w, const void* w1, const void* w3, const void* w2, void* y,
                   void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Expert execution with pre-calculated experts (Sec. IV-C "Prediction-based
 * Expert Pre-Calculation"): an expert that was predicted one block ahead and
 * is not held on the GPU has been started on the hidden state of the block
 * before, so that selection's input is the earlier state, while every other
 * selected expert sees the block's true input.  For every token t
 *   y[t] = sum_j topk_w[t,j] * W2_e ( silu(W1_e in) * (W3_e in) ),  e = topk_idx[t,j],
 *   in = x_stale[t] where stale[t,j] != 0, else x[t].
 * One pass over the experts' weights and one rounding of y, as in
 * moe_expert_ffn, which this call equals bit for bit when stale is all zero.
 * The paper does not say which gate's weights combine the outputs; the caller
 * passes them (the harness uses the predicted gate's).
 *
 *   x_stale [tokens, H]  in  the hidden states the pre-calculated experts saw, shape->dtype
 *   stale   [tokens, k]  in  uint8, non-zero = selection (t, j) was evaluated on x_stale
 *   the other arguments, the workspace and the errors as in moe_expert_ffn
 */
int moe_expert_ffn_precalc(const moe_shape_t* shape, int32_t tokens, const void* x, const void* x_stale,
                           const uint8_t* stale, const int32_t* topk_idx, const float* topk_w, const void* w1,
                           const void* w3, const void* w2, void* y, void* workspace, size_t workspace_bytes,
                           void* hip_stream);

/*
 * One whole MoE layer: moe_route, then (if w_gate_next is not NULL)
 * moe_predict_next into pred_idx, then moe_expert_ffn, with x read once for
 * both gates.  pred_idx may be NULL only when w_gate_next is NULL.
 */
int moe_layer(const moe_shape_t* shape, int32_t tokens, const void* x, const void* w_gate,
              const float* gate_bias, const void* w_gate_next, const float* gate_bias_next,
              const void* w1, const void* w3, const void* w2, void* y, int32_t* topk_idx,
              float* topk_w, int32_t* counts, int32_t accumulate, int32_t* pred_idx, void* workspace,
              size_t workspace_bytes, void* hip_stream);

/*
 * moe_layer for callers that cannot provide or allocate a workspace: code
 * under HIP graph capture, tight serving loops, harnesses that forbid device
 * allocation.  Same arguments, kernels and results as moe_layer (bit for bit),
 * but the scratch memory is a static device array of MOE_STATIC_SCRATCH_BYTES
 * inside the library (each GPU the library runs on holds one until the process
 * ends), so the call allocates nothing, neither on the host nor on the device.
 * A call whose moe_workspace_bytes(shape, tokens) exceeds that size returns
 * MOE_ERR_TOO_LARGE and enqueues nothing: the buffer is sized for decode steps
 * (every bf16 call of at most 32 tokens at the shapes of Table III fits, and
 * fp32 calls of a few hundred tokens at small widths; bf16 calls of more than
 * 32 tokens never fit, their K-split pieces alone take 64 MiB).
 * All calls on one GPU share that GPU's array, whatever the stream or thread:
 * two moe_layer_static calls that overlap in time on one GPU race.  Order them
 * on one stream or with events.  Nothing in the array needs clearing between
 * calls (the kernels reset what they need, as with a caller's workspace).
 * The first call on a device looks up the array's device address (no
 * allocation); do that once before a stream capture begins.
 * moe_decode_status(NULL, 0, ...) reads the status word of this array.
 */
#define MOE_STATIC_SCRATCH_BYTES (16u << 20)
int moe_layer_static(const moe_shape_t* shape, int32_t tokens, const void* x, const void* w_gate,
                     const float* gate_bias, const void* w_gate_next, const float* gate_bias_next,
                     const void* w1, const void* w3, const void* w2, void* y, int32_t* topk_idx,
                     float* topk_w, int32_t* counts, int32_t accumulate, int32_t* pred_idx, void* hip_stream);

/*
 * Whether a decode-size call on `workspace` gave up a rendezvous (see the
 * conventions above: bf16 calls of at most 32 tokens need the whole grid
 * resident at once; a workgroup whose bounded wait runs out stores NaN instead
 * of its part of y and raises a status word in the workspace, which stays
 * raised until it is reset).  Copies that word back: *gave_up (HOST pointer) =
 * 1 if some call since the last reset gave up, else 0; reset != 0 also clears
 * the word.  Unlike the layer's calls this one synchronises hip_stream, so it
 * cannot be recorded into a graph.  A workspace that was never used by a
 * decode-size call holds arbitrary bytes there; they read as "gave up" only
 * if they equal a 32-bit magic value.
 * workspace == NULL (workspace_bytes ignored) means the static scratch of
 * moe_layer_static on the current device.
 * Errors: MOE_ERR_NULL, MOE_ERR_ALIGN, MOE_ERR_WORKSPACE (fewer than 4096
 * bytes), MOE_ERR_DEVICE.
 */
int moe_decode_status(void* workspace, size_t workspace_bytes, int32_t reset, int32_t* gave_up, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* MOE_H */
