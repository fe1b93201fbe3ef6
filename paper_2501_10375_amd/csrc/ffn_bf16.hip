// Grouped SwiGLU expert FFN for bf16 storage on the CDNA4 matrix cores
// (expert execution of DAOP Sec. II-A / Algorithm 1's parallel local expert
// execution; expert = W2 ( silu(W1 x) * (W3 x) ), shapes of Table III).
//
// Two grouped GEMMs, both "row . row" contractions with K contiguous in each
// operand, so operands go from HBM to LDS to MFMA registers without transposes:
//   gemm1: act[slot, f] = silu(x[tok(slot)] . w1[e, f]) * (x[tok(slot)] . w3[e, f])   K = H
//   gemm2: out[slot, h] = act[slot] . w2[e, h]                                        K = F
// followed by the gate-weighted combine over a token's k slots.
//
// The GEMM kernel itself (tiling, LDS pipeline, MFMA layout) is in grouped_gemm_bf16.h.
#include "grouped_gemm_bf16.h"
#include "moe_internal.h"

namespace moe {
namespace {

// Tile and pipeline shapes of the two GEMMs (slot rows per tile, K step, LDS stages).  Both move whole
// 128-byte lines per global->LDS load instruction (K step 64); they differ in how much of a K step's
// operand traffic can be in flight:
//   full flavour:  256 slots x 256 weight rows, three 32 KB weight stages and two 32 KB slot stages.  The
//       larger tile moves the fewest operand bytes per flop, which is what counts when the MFMAs are the
//       work.  In the first GEMM a ragged tile issues only the MFMAs of its valid 32-slot fragments.
//   ragged flavour (few routed rows per expert): 128 slots x 256 weight rows, three 48 KB stages, and
//       empty slot fragments skipped.  Two K steps of both operands in flight hide the load latency that
//       bounds a tile with little arithmetic, and half-height tiles pad cold experts less.
// Each GEMM picks its flavour from the mean number of routed rows per expert (the counts themselves are
// only known on the device).  Measured on the Mixtral- and Phi-shaped layers, 256 to 4096 tokens: the
// first GEMM is faster in the full flavour from about 96-128 rows per expert on (7 % at 512 tokens of
// the Mixtral shape, 10 % at 1536), the second from about 320 on (17 % at 1536 tokens), and slower
// below (the second GEMM by up to 25 %).
constexpr int kRaggedRowsPerExpert1 = 128;  // mean routed rows per expert below which gemm1 runs ragged
constexpr int kRaggedRowsPerExpert2 = 320;  // ... and gemm2
constexpr int kWT = 2, kWW = 4;  // wavefront grid: slot groups x weight-row groups

// y[t, :] = bf16( sum_j w[t, j] * out[slot_of[t, j], :] ), j ascending, fp32 sum, one rounding.
__global__ __launch_bounds__(256) void combine_bf16(const float* __restrict__ out, const float* __restrict__ w,
                                                    const int32_t* __restrict__ slot_of, int k, int H,
                                                    uint16_t* __restrict__ y) {
    const int t = blockIdx.x;
    for (int h = threadIdx.x * 8; h < H; h += 256 * 8) {
        float s[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        for (int j = 0; j < k; ++j) {
            const float wj = w[(size_t)t * k + j];
            const float* src = out + (size_t)slot_of[(size_t)t * k + j] * H + h;
            const float4 a = *reinterpret_cast<const float4*>(src);
            const float4 b = *reinterpret_cast<const float4*>(src + 4);
            s[0] = fmaf(wj, a.x, s[0]); s[1] = fmaf(wj, a.y, s[1]);
            s[2] = fmaf(wj, a.z, s[2]); s[3] = fmaf(wj, a.w, s[3]);
            s[4] = fmaf(wj, b.x, s[4]); s[5] = fmaf(wj, b.y, s[5]);
            s[6] = fmaf(wj, b.z, s[6]); s[7] = fmaf(wj, b.w, s[7]);
        }
        uint4 pk;
        pk.x = pack_bf16x2(s[0], s[1]);
        pk.y = pack_bf16x2(s[2], s[3]);
        pk.z = pack_bf16x2(s[4], s[5]);
        pk.w = pack_bf16x2(s[6], s[7]);
        *reinterpret_cast<uint4*>(y + (size_t)t * H + h) = pk;
    }
}

// Raises a kernel's dynamic LDS limit once (idempotent; a race only repeats it).
template <typename Kernel>
hipError_t allow_lds(Kernel k, int bytes, bool& configured) {
    if (configured) return hipSuccess;
    const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(k), hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    configured = e == hipSuccess;
    return e;
}

// One persistent workgroup per CU (a multiple of the 8 XCDs); the kernels size their own work from `offs`.
int persistent_grid() { return max(gg::kXcds, compute_units() / gg::kXcds * gg::kXcds); }

// gemm1 (+ SwiGLU) in one pipeline shape.
template <int BK, int STAGES, bool SKIP, int BT = gg::kBT, bool W3 = false>
hipError_t launch_gemm1(const moe_shape_t& s, const uint16_t* x, const uint16_t* w1, const uint16_t* w3,
                        const int32_t* offs, const int32_t* row_of_slot, void* act, int32_t* sync, float* partial,
                        const StaleInput& alt, hipStream_t stream) {
    using G1 = gg::Gemm<2, BK, STAGES, kWT, kWW, SKIP, BT, false, W3>;
    auto k1 = gg::grouped_gemm_kernel<2, BK, STAGES, kWT, kWW, SKIP, BT, W3>;
    auto k1_alt = gg::grouped_gemm1_alt_kernel<BK, STAGES, kWT, kWW, SKIP, BT, W3>;
    static bool configured = false, configured_alt = false;
    hipError_t e = allow_lds(k1, G1::kLdsBytes, configured);
    if (e != hipSuccess) return e;
    e = allow_lds(k1_alt, G1::kLdsBytes, configured_alt);
    if (e != hipSuccess) return e;
    if (alt.stale != nullptr)
        k1_alt<<<persistent_grid(), G1::kThreads, G1::kLdsBytes, stream>>>(
            x, static_cast<const uint16_t*>(alt.x_stale), alt.stale, w1, w3, offs, row_of_slot, s.n_experts, s.top_k, s.ffn,
            s.hidden, act, sync, partial);
    else
        k1<<<persistent_grid(), G1::kThreads, G1::kLdsBytes, stream>>>(x, w1, w3, offs, row_of_slot, s.n_experts, s.top_k,
                                                                       s.ffn, s.hidden, act, sync, partial);
    stage_mark(stream, kStageGemm1);
    return hipGetLastError();
}

// gemm2 in one pipeline shape.
template <int BK, int STAGES, bool SKIP, int BT = gg::kBT, bool W3 = false>
hipError_t launch_gemm2(const moe_shape_t& s, const uint16_t* act_in, const uint16_t* w2, const int32_t* offs,
                        const int32_t* row_of_slot, float* out, int32_t* sync, float* partial, hipStream_t stream) {
    using G2 = gg::Gemm<1, BK, STAGES, kWT, kWW, SKIP, BT, false, W3>;
    auto k2 = gg::grouped_gemm_kernel<1, BK, STAGES, kWT, kWW, SKIP, BT, W3>;
    static bool configured = false;
    const hipError_t e = allow_lds(k2, G2::kLdsBytes, configured);
    if (e != hipSuccess) return e;
    k2<<<persistent_grid(), G2::kThreads, G2::kLdsBytes, stream>>>(act_in, w2, nullptr, offs, row_of_slot, s.n_experts,
                                                                   s.top_k, s.hidden, s.ffn, out, sync + gg::kSyncInts, partial);
    stage_mark(stream, kStageGemm2);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_ffn_bf16(const moe_shape_t& s, int tokens, const void* x, const float* topk_w, const void* w1,
                           const void* w3, const void* w2, void* y, const int32_t* offs,
                           const int32_t* row_of_slot, const int32_t* slot_of, void* act, float* out,
                           int32_t* sync, float* partial, const StaleInput& alt, hipStream_t stream) {
    static_assert(gg::kSyncInts == kGemmSyncInts && gg::kScratchBytes == kGemmScratchBytes, "workspace layout");
    const uint16_t* xs = static_cast<const uint16_t*>(x);
    const uint16_t* a16 = static_cast<const uint16_t*>(act);
    const uint16_t *p1 = static_cast<const uint16_t*>(w1), *p3 = static_cast<const uint16_t*>(w3),
                   *p2 = static_cast<const uint16_t*>(w2);
    hipError_t e;
    const long routed = (long)tokens * s.top_k;
    e = routed < (long)s.n_experts * kRaggedRowsPerExpert1
            ? launch_gemm1<64, 3, true, 128>(s, xs, p1, p3, offs, row_of_slot, act, sync, partial, alt, stream)
            : launch_gemm1<64, 2, false, 256, true>(s, xs, p1, p3, offs, row_of_slot, act, sync, partial, alt, stream);
    if (e != hipSuccess) return e;
    e = routed < (long)s.n_experts * kRaggedRowsPerExpert2
            ? launch_gemm2<64, 3, true, 128>(s, a16, p2, offs, row_of_slot, out, sync, partial, stream)
            : launch_gemm2<64, 2, false, 256, true>(s, a16, p2, offs, row_of_slot, out, sync, partial, stream);
    if (e != hipSuccess) return e;
    combine_bf16<<<tokens, 256, 0, stream>>>(out, topk_w, slot_of, s.top_k, s.hidden, static_cast<uint16_t*>(y));
    stage_mark(stream, kStageCombine);
    return hipGetLastError();
}

}  // namespace moe

