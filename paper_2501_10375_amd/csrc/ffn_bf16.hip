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

// Pipeline shape of the two GEMMs: K step and number of LDS stages (STAGES * 512 rows * BK * 2 bytes of LDS).
#ifndef MOE_GEMM_BK
#define MOE_GEMM_BK 32
#endif
#ifndef MOE_GEMM_STAGES
#define MOE_GEMM_STAGES 4
#endif
constexpr int kBK = MOE_GEMM_BK;
constexpr int kStages = MOE_GEMM_STAGES;
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

}  // namespace

hipError_t launch_ffn_bf16(const moe_shape_t& s, int tokens, const void* x, const float* topk_w, const void* w1,
                           const void* w3, const void* w2, void* y, const int32_t* offs,
                           const int32_t* row_of_slot, const int32_t* slot_of, void* act, float* out,
                           int32_t* sync, float* partial, hipStream_t stream) {
    static_assert(gg::kSyncInts == kGemmSyncInts && gg::kScratchBytes == kGemmScratchBytes, "workspace layout");
    using G1 = gg::Gemm<2, kBK, kStages, kWT, kWW>;
    using G2 = gg::Gemm<1, kBK, kStages, kWT, kWW>;
    auto k1 = gg::grouped_gemm_kernel<2, kBK, kStages, kWT, kWW>;
    auto k2 = gg::grouped_gemm_kernel<1, kBK, kStages, kWT, kWW>;
    static bool configured = false;  // raising the dynamic LDS limit is idempotent; a race only repeats it
    if (!configured) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(k1),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, G1::kLdsBytes);
        if (e != hipSuccess) return e;
        e = hipFuncSetAttribute(reinterpret_cast<const void*>(k2), hipFuncAttributeMaxDynamicSharedMemorySize,
                                G2::kLdsBytes);
        if (e != hipSuccess) return e;
        configured = true;
    }
    // One persistent workgroup per CU (a multiple of the 8 XCDs); the kernels size their own work from `offs`.
    const int grid = max(gg::kXcds, compute_units() / gg::kXcds * gg::kXcds);
    k1<<<grid, G1::kThreads, G1::kLdsBytes, stream>>>(static_cast<const uint16_t*>(x), static_cast<const uint16_t*>(w1),
                                                      static_cast<const uint16_t*>(w3), offs, row_of_slot, s.n_experts,
                                                      s.top_k, s.ffn, s.hidden, act, sync, partial);
    stage_mark(stream, kStageGemm1);
    k2<<<grid, G2::kThreads, G2::kLdsBytes, stream>>>(static_cast<const uint16_t*>(act), static_cast<const uint16_t*>(w2),
                                                      nullptr, offs, row_of_slot, s.n_experts, s.top_k, s.hidden, s.ffn,
                                                      out, sync + gg::kSyncInts, partial);
    stage_mark(stream, kStageGemm2);
    combine_bf16<<<tokens, 256, 0, stream>>>(out, topk_w, slot_of, s.top_k, s.hidden, static_cast<uint16_t*>(y));
    stage_mark(stream, kStageCombine);
    return hipGetLastError();
}

}  // namespace moe
