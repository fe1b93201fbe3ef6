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
// Tiling: a workgroup owns 128 slots of ONE expert x 128 output features
// (gemm1: of both w1 and w3), K in steps of 64.  Four wavefronts in a 2 x 2
// arrangement each own 64 features x 64 slots as 2 x 2 v_mfma_f32_32x32x16_bf16
// tiles (weights are the MFMA "A" operand, token rows the "B" operand, so a
// lane ends up with 4 consecutive output features of one slot).  LDS tiles are
// [rows][64] bf16 with the 16-byte chunk index XOR-ed by (row & 7), which makes
// both the staging stores and the MFMA operand reads bank-conflict free.
// Global loads for step k+1 are issued into registers before the MFMAs of
// step k.  Workgroup ids are remapped so each of the 8 XCDs walks a contiguous
// range of tiles ordered (expert, feature tile, slot tile): workgroups that are
// resident together on one XCD share weight tiles through its L2.
#include "moe_internal.h"

namespace moe {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;

constexpr int BT = kTileTokensBf16;  // slots per tile
constexpr int BF = 128;              // output features per tile
constexpr int BK = 64;               // K elements per step (128 bytes per row)
constexpr int kXcds = 8;

__device__ inline uint16_t f32_to_bf16_rne(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40u);  // quiet NaN
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

// Tile id -> (expert, first slot, valid rows, feature tile).  Order: expert, feature tile, slot tile.
__device__ inline bool locate_tile(const int32_t* __restrict__ offs, int E, int n_ftiles, int id, int& e,
                                   int& slot0, int& rows, int& ft) {
    int acc = 0;
    for (int i = 0; i < E; ++i) {
        const int c = offs[i + 1] - offs[i];
        const int mt = (c + BT - 1) / BT;
        const int tiles = mt * n_ftiles;
        if (id < acc + tiles) {
            const int local = id - acc;
            ft = local / mt;
            const int m = local - ft * mt;
            e = i;
            slot0 = offs[i] + m * BT;
            rows = min(BT, c - m * BT);
            return true;
        }
        acc += tiles;
    }
    return false;
}

__device__ inline int lds_off(int row, int chunk) { return row * (BK * 2) + ((chunk ^ (row & 7)) << 4); }

// DUAL = true : gemm1 (two weight matrices, SwiGLU epilogue, bf16 output act[slot, F])
// DUAL = false: gemm2 (one weight matrix, fp32 output out[slot, N])
//   tok_base: x (DUAL, rows gathered through row_of_slot / k) or act (rows = slots), row length K
//   wa, wb  : [E, N, K] weights; wb used only when DUAL
template <bool DUAL>
__global__ __launch_bounds__(256) void grouped_gemm_bf16(const uint16_t* __restrict__ tok_base,
                                                         const uint16_t* __restrict__ wa,
                                                         const uint16_t* __restrict__ wb,
                                                         const int32_t* __restrict__ offs,
                                                         const int32_t* __restrict__ row_of_slot, int E, int topk,
                                                         int N, int K, int tiles_per_xcd, void* __restrict__ dst) {
    constexpr int NW = DUAL ? 2 : 1;
    __shared__ __attribute__((aligned(16))) unsigned char lds_tok[BT * BK * 2];
    __shared__ __attribute__((aligned(16))) unsigned char lds_w[NW][BF * BK * 2];

    const int logical = (blockIdx.x % kXcds) * tiles_per_xcd + blockIdx.x / kXcds;
    int e, slot0, rows, ft;
    if (!locate_tile(offs, E, (N + BF - 1) / BF, logical, e, slot0, rows, ft)) return;
    const int n0 = ft * BF;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wf = wave & 1, wt = wave >> 1;  // feature half, slot half of this wavefront

    // Staging: thread -> 16-byte chunk (tid & 7) of rows (tid >> 3) + 32 i, i = 0..3.
    const int sc = tid & 7, sr = tid >> 3;
    const uint16_t* tp[4];
    const uint16_t* wp[NW][4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int r = sr + 32 * i;
        const int slot = slot0 + min(r, rows - 1);  // rows past the end re-read the last valid row
        const int src_row = DUAL ? row_of_slot[slot] / topk : slot;
        tp[i] = tok_base + (size_t)src_row * K + sc * 8;
        const int wrow = min(n0 + r, N - 1);  // N is a multiple of 64: the last feature tile may be half full
        wp[0][i] = wa + ((size_t)e * N + wrow) * K + sc * 8;
        if (DUAL) wp[NW - 1][i] = wb + ((size_t)e * N + wrow) * K + sc * 8;
    }
    u32x4 treg[4], wreg[NW][4];
#define MOE_FETCH(k0_)                                                                        \
    _Pragma("unroll") for (int i = 0; i < 4; ++i) {                                           \
        treg[i] = *reinterpret_cast<const u32x4*>(tp[i] + (k0_));                            \
        _Pragma("unroll") for (int m = 0; m < NW; ++m)                                        \
            wreg[m][i] = *reinterpret_cast<const u32x4*>(wp[m][i] + (k0_));                  \
    }
#define MOE_STASH()                                                                           \
    _Pragma("unroll") for (int i = 0; i < 4; ++i) {                                           \
        const int off = lds_off(sr + 32 * i, sc);                                             \
        *reinterpret_cast<u32x4*>(lds_tok + off) = treg[i];                                  \
        _Pragma("unroll") for (int m = 0; m < NW; ++m)                                        \
            *reinterpret_cast<u32x4*>(lds_w[m] + off) = wreg[m][i];                          \
    }

    f32x16 acc[NW][2][2];  // [matrix][feature tile][slot tile]
#pragma unroll
    for (int m = 0; m < NW; ++m)
#pragma unroll
        for (int a = 0; a < 2; ++a)
#pragma unroll
            for (int b = 0; b < 2; ++b)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[m][a][b][r] = 0.f;

    const int frow = lane & 31, fhalf = lane >> 5;
    MOE_FETCH(0)
    for (int k0 = 0; k0 < K; k0 += BK) {
        if (k0 > 0) __syncthreads();
        MOE_STASH()
        __syncthreads();
        if (k0 + BK < K) {
            MOE_FETCH(k0 + BK)
        }
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks) {
            const int chunk = ks * 2 + fhalf;
            bf16x8 tf[2], wfr[NW][2];
#pragma unroll
            for (int b = 0; b < 2; ++b)
                tf[b] = *reinterpret_cast<const bf16x8*>(lds_tok + lds_off(wt * 64 + b * 32 + frow, chunk));
#pragma unroll
            for (int m = 0; m < NW; ++m)
#pragma unroll
                for (int a = 0; a < 2; ++a)
                    wfr[m][a] = *reinterpret_cast<const bf16x8*>(lds_w[m] + lds_off(wf * 64 + a * 32 + frow, chunk));
#pragma unroll
            for (int m = 0; m < NW; ++m)
#pragma unroll
                for (int a = 0; a < 2; ++a)
#pragma unroll
                    for (int b = 0; b < 2; ++b)
                        acc[m][a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wfr[m][a], tf[b], acc[m][a][b], 0, 0, 0);
        }
    }

    // MFMA 32x32 result: lane holds column (slot) lane & 31 and rows (features)
    // 8 * (r / 4) + 4 * (lane / 32) + (r % 4), r = 0..15.
#pragma unroll
    for (int b = 0; b < 2; ++b) {
        const int row = wt * 64 + b * 32 + frow;
        if (row >= rows) continue;
        const size_t slot = (size_t)(slot0 + row);
#pragma unroll
        for (int a = 0; a < 2; ++a) {
#pragma unroll
            for (int rg = 0; rg < 4; ++rg) {
                const int n = n0 + wf * 64 + a * 32 + rg * 8 + fhalf * 4;
                if (n >= N) continue;
                if (DUAL) {
                    uint16_t o[4];
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const float g = acc[0][a][b][rg * 4 + i];
                        const float u = acc[NW - 1][a][b][rg * 4 + i];
                        o[i] = f32_to_bf16_rne(g / (1.f + __expf(-g)) * u);
                    }
                    uint2 pk;
                    pk.x = (uint32_t)o[0] | ((uint32_t)o[1] << 16);
                    pk.y = (uint32_t)o[2] | ((uint32_t)o[3] << 16);
                    *reinterpret_cast<uint2*>(static_cast<uint16_t*>(dst) + slot * N + n) = pk;
                } else {
                    f32x4 v;
#pragma unroll
                    for (int i = 0; i < 4; ++i) v[i] = acc[0][a][b][rg * 4 + i];
                    *reinterpret_cast<f32x4*>(static_cast<float*>(dst) + slot * N + n) = v;
                }
            }
        }
    }
}

#undef MOE_FETCH
#undef MOE_STASH

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
        pk.x = (uint32_t)f32_to_bf16_rne(s[0]) | ((uint32_t)f32_to_bf16_rne(s[1]) << 16);
        pk.y = (uint32_t)f32_to_bf16_rne(s[2]) | ((uint32_t)f32_to_bf16_rne(s[3]) << 16);
        pk.z = (uint32_t)f32_to_bf16_rne(s[4]) | ((uint32_t)f32_to_bf16_rne(s[5]) << 16);
        pk.w = (uint32_t)f32_to_bf16_rne(s[6]) | ((uint32_t)f32_to_bf16_rne(s[7]) << 16);
        *reinterpret_cast<uint4*>(y + (size_t)t * H + h) = pk;
    }
}

}  // namespace

hipError_t launch_ffn_bf16(const moe_shape_t& s, int tokens, const void* x, const float* topk_w, const void* w1,
                           const void* w3, const void* w2, void* y, const int32_t* offs,
                           const int32_t* row_of_slot, const int32_t* slot_of, void* act, float* out,
                           hipStream_t stream) {
    const int A = tokens * s.top_k;
    const int max_mtiles = (A + BT - 1) / BT + s.n_experts;
    {
        const int tiles = max_mtiles * ((s.ffn + BF - 1) / BF);
        const int per_xcd = (tiles + kXcds - 1) / kXcds;
        grouped_gemm_bf16<true><<<per_xcd * kXcds, 256, 0, stream>>>(
            static_cast<const uint16_t*>(x), static_cast<const uint16_t*>(w1), static_cast<const uint16_t*>(w3), offs,
            row_of_slot, s.n_experts, s.top_k, s.ffn, s.hidden, per_xcd, act);
        stage_mark(stream, kStageGemm1);
    }
    {
        const int tiles = max_mtiles * ((s.hidden + BF - 1) / BF);
        const int per_xcd = (tiles + kXcds - 1) / kXcds;
        grouped_gemm_bf16<false><<<per_xcd * kXcds, 256, 0, stream>>>(
            static_cast<const uint16_t*>(act), static_cast<const uint16_t*>(w2), nullptr, offs, row_of_slot,
            s.n_experts, s.top_k, s.hidden, s.ffn, per_xcd, out);
        stage_mark(stream, kStageGemm2);
    }
    combine_bf16<<<tokens, 256, 0, stream>>>(out, topk_w, slot_of, s.top_k, s.hidden, static_cast<uint16_t*>(y));
    stage_mark(stream, kStageCombine);
    return hipGetLastError();
}

}  // namespace moe
