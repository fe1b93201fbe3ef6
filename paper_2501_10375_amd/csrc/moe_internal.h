// Internal declarations shared by the HIP translation units of libmoe_hip.so.
// Nothing here is part of the public ABI (see include/moe.h).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "moe.h"
#include "moe_measure.h"

namespace moe {

// Tokens handled by one workgroup of the routing / histogram / permute kernels.
constexpr int kRouteTokensPerBlock = 16;
// Calls with at most this many tokens take the decode path: one persistent
// weight-streaming kernel that routes, groups tokens per expert on the fly
// (no permutation in the workspace) and runs both expert GEMMs.
constexpr int kDecodeMaxTokens = 16;
// bf16 calls with at most this many tokens still stream the weights with that kernel's two GEMM
// phases (routing, counts and prediction then come from the prefill-size routing kernels): below
// this size the layer is bound by reading each selected expert once and the streaming kernel beats
// the 256-row MFMA tiles (measured: 617 vs 737 us at 32 tokens; at 64 tokens it loses, 863 vs 782 us).
constexpr int kStreamMaxTokens = 32;

// Rows (tokens) per M-tile of the grouped GEMMs; an M-tile never spans two experts.
constexpr int kTileTokensF32 = 64;
constexpr int kTileTokensBf16 = 256;

// The two blocks of flags and counters come first, at offsets that depend on nothing: calls of any
// size on one workspace then never put other data where a decode-size call keeps its launch count
// and arrival flags.
struct WorkspaceLayout {
    size_t dec_flags;    // uint32 [kDecodeFlagInts]  arrival flags, launch count and status word of the decode kernel's two grid-wide rendezvous
    size_t sync;         // int32 [kSyncInts]    tile hand-out and split-tile arrival counters of the two grouped GEMMs
    size_t hist;         // int32 [n_blocks, E]  per-block selection histogram
    size_t hist_next;    // int32 [n_blocks, E]  same for the next-layer gate
    size_t offs;         // int32 [E + 1]        exclusive scan of counts
    size_t row_of_slot;  // int32 [A]            slot -> assignment index t*k + j
    size_t slot_of;      // int32 [A]            assignment index -> slot
    size_t route_end;    // bytes needed by routing-only calls
    size_t act;          // dtype [A, F]         silu(W1 x) * (W3 x)
    size_t out;          // fp32  [A, H]         per-assignment expert output
    size_t partial;      // fp32  [8 * 32, 256, 256]  pieces of K-split tiles (bf16 prefill path only)
    size_t total;        // bytes needed by the whole layer
};

WorkspaceLayout workspace_layout(const moe_shape_t& s, int tokens);

inline int route_blocks(int tokens) {
    return (tokens + kRouteTokensPerBlock - 1) / kRouteTokensPerBlock;
}

// One gate evaluated by the routing kernel.
struct GateArgs {
    const void* w;     // [E, H]
    const float* bias; // [E] or null
    int32_t* idx;      // [T, k]
    float* wts;        // [T, k] or null
    int32_t* hist;     // [n_blocks, E] or null
};

// Stage ids of the optional per-stage timing (moe_stage_timing_begin/end in moe_measure.h).
enum Stage {
    kStageRoute = 0, kStagePermute = 1, kStageGemm1 = 2, kStageGemm2 = 3, kStageCombine = 4,
    kStageFused = 5,  // the single kernel of a decode-size bf16 call
};
static_assert(kStageFused + 1 == MOE_NUM_STAGES, "moe_measure.h lists the stages");
// Records "stage `stage` ends here" on `stream`; a no-op unless timing is active on this thread.
void stage_mark(hipStream_t stream, int stage);

// ---- launchers (each returns hipGetLastError() after enqueueing) ----------

// Gate GEMM + softmax + top-k for up to two gates that share x.  Per-block
// histograms go to gate.hist.
hipError_t launch_route(const moe_shape_t& s, int tokens, const void* x, const GateArgs* gates,
                        int n_gates, hipStream_t stream);

// Per-block histogram of caller-provided indices (moe_expert_ffn entry).
hipError_t launch_hist_from_idx(const moe_shape_t& s, int tokens, const int32_t* idx, int32_t* hist,
                                hipStream_t stream);

// Sum block histograms into counts (counts may be null), and when
// row_of_slot/slot_of are given build offs and the stable token->expert
// permutation.
// Counters and scratch of the persistent grouped GEMMs (see grouped_gemm_bf16.h): per launch 8 tile
// hand-out counters (one per XCD) + 8 x 32 split-tile arrival counters, and one 256 x 256 fp32 piece per workgroup.
constexpr int kGemmSyncInts = 8 + 8 * 32;
constexpr int kSyncInts = 2 * kGemmSyncInts;  // gemm1 and gemm2
constexpr size_t kGemmScratchBytes = (size_t)8 * 32 * 256 * 256 * sizeof(float);
// `sync` (may be null) is a block of kSyncInts counters that is cleared for the GEMMs that follow.
// For long calls the histograms in `hist` are replaced by their per-block prefixes.
hipError_t launch_finalize(const moe_shape_t& s, int tokens, int32_t* hist, const int32_t* idx,
                           int32_t* counts, int accumulate, int32_t* offs, int32_t* row_of_slot,
                           int32_t* slot_of, int32_t* sync, hipStream_t stream);

// Decode path (tokens <= kDecodeMaxTokens): routing for up to two gates with
// counts written directly, in one workgroup.
hipError_t launch_route_small(const moe_shape_t& s, int tokens, const void* x, const GateArgs* gates,
                              int n_gates, int32_t* counts, int accumulate, int32_t* counts_next,
                              hipStream_t stream);

// Expert execution with pre-calculated selections (moe_expert_ffn_precalc): selection a = t * k + j
// reads its input row from x_stale instead of x when stale[a] != 0.  Both null: the plain layer.
struct StaleInput {
    const void* x_stale;   // [T, H], storage type of x
    const uint8_t* stale;  // [T, k]
};

// Grouped expert FFN, fp32 storage.
hipError_t launch_ffn_f32(const moe_shape_t& s, int tokens, const float* x, const float* topk_w,
                          const float* w1, const float* w3, const float* w2, float* y,
                          const int32_t* offs, const int32_t* row_of_slot, const int32_t* slot_of,
                          float* act, float* out, const StaleInput& alt, hipStream_t stream);

// Grouped expert FFN, bf16 storage, MFMA (prefill-size calls).
hipError_t launch_ffn_bf16(const moe_shape_t& s, int tokens, const void* x, const float* topk_w,
                           const void* w1, const void* w3, const void* w2, void* y,
                           const int32_t* offs, const int32_t* row_of_slot, const int32_t* slot_of,
                           void* act, float* out, int32_t* sync, float* partial, const StaleInput& alt,
                           hipStream_t stream);

// Number of compute units of the current device (cached per device).
int compute_units();

// Decode-size bf16 calls (tokens <= kDecodeMaxTokens): one persistent kernel streams the selected
// experts' weights.  With `route` it first evaluates the gate (and writes indices, weights and
// counts); without, it takes topk_idx / topk_w.  `flags` are kDecodeFlagInts words of workspace
// whose contents need not be initialised (two arrays of 256 arrival flags, one per workgroup and
// rendezvous, and the launch count the flags' epoch is derived from; the grid is at most 256 workgroups).
constexpr int kDecodeFlagInts = 2 * 256 + 16;
// Word of that block that a rendezvous which gave up sets to kDecodeGaveUp (read by moe_decode_status).
constexpr int kDecodeStatusWord = 2 * 256 + 1;
constexpr uint32_t kDecodeGaveUp = 0xDEC0DEADu;
// Polling rounds a rendezvous of the decode kernel waits before it gives up (2^22 unless a test
// lowered it through moe_measure_set_decode_spin_limit).
int decode_spin_limit();
struct DecodeRoute {
    const void* w_gate;
    const float* bias;
    int32_t* idx;
    float* wts;
    int32_t* counts;
    int accumulate;
    // optional prediction (the next layer's gate on the same hidden states): evaluated by one
    // workgroup after its share of the experts; pred_idx [tokens, top_k]
    const void* w_gate_next;
    const float* bias_next;
    int32_t* pred_idx;
};
// Without `route` the selections come in topk_idx / topk_w; `counts` (may be null) then receives their
// histogram (added to what it holds with `accumulate`), written by the kernel's first workgroup.
hipError_t launch_decode_layer(const moe_shape_t& s, int tokens, const void* x, const DecodeRoute* route,
                               const int32_t* topk_idx, const float* topk_w, const void* w1, const void* w3,
                               const void* w2, void* y, void* act, uint32_t* flags, const StaleInput& alt,
                               hipStream_t stream, int32_t* counts = nullptr, int accumulate = 0);

}  // namespace moe
