// Expert FFN for decode-size calls (a handful of tokens), bf16 storage.
//
// With the experts resident in HBM, a decode step of the MoE layer is a weight
// stream: each selected expert's three matrices are read once and multiplied
// by a few hidden states (the paper's Table I discussion: expert parameters
// dwarf the activations by four orders of magnitude).  These two kernels are
// therefore organised around the HBM stream, not around the arithmetic:
//
//   * no permutation and no LDS staging of weights: every weight byte is used
//     by exactly one wavefront, so it is loaded straight into MFMA operand
//     registers with 16-byte loads;
//   * every load instruction covers 8 weight rows x 128 contiguous bytes (whole
//     cache lines; 64-byte pieces stream measurably slower).  The natural
//     operand layout of v_mfma_f32_16x16x32_bf16 would give 16 rows x 64 bytes,
//     so the 16 operand rows are used as 8 weight rows x 2 halves of a 64-wide
//     K step instead: a second load fetches the next 8 weight rows with the
//     halves swapped, a per-lane select recombines the two loads into one
//     operand holding the lower K half of all 16 weight rows and one holding
//     the upper half (with rows i and i ^ 8 exchanged), and two MFMAs with the
//     matching halves of the tokens accumulate them; the two accumulators are
//     added, after undoing the row exchange with a cross-lane move, when the
//     tile is finished;
//   * the tokens of an expert form the 16 columns of the MFMA, so up to 16
//     tokens share one pass over the weights; lanes whose column has no token
//     issue no load;
//   * each wavefront keeps P steps of loads in flight in a rotating register
//     window (software pipeline unrolled P times) that runs across tile
//     boundaries, and the barrier at a tile's end waits for LDS only, so the
//     stream never drains;
//   * the 8 wavefronts of a workgroup split K, and their partial 16 x 16 tiles
//     are summed through LDS in a fixed order (deterministic);
//   * the token groups are rebuilt by every workgroup from topk_idx (at most
//     128 integers), which is cheaper than another kernel launch.
//
//   dec_gemm1: act[a, f] = silu(x[t] . w1[e, f]) * (x[t] . w3[e, f])   a = t*k + j, e = idx[a]
//   dec_gemm2: y[t, h]   = sum over the token's experts (ascending expert id) of
//                          w[a] * (act[a] . w2[e, h]),  fp32, one rounding to bf16
#include "bf16_utils.h"
#include "moe_internal.h"

namespace moe {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;

// Pipeline depths (k32 steps of loads in flight per wavefront) of the two kernels.
#ifndef MOE_DEC_P1
#define MOE_DEC_P1 4
#endif
#ifndef MOE_DEC_P2
#define MOE_DEC_P2 8
#endif

constexpr int kWaves = 8;
constexpr int kThreads = kWaves * 64;
constexpr int kMaxTok = kDecodeMaxTokens;
static_assert(kMaxTok == 16, "an expert's tokens are the 16 columns of one 16x16x32 MFMA");

struct Groups {
    int n_active;
    int expert[64];         // active experts, ascending id
    int cnt[64];            // tokens of that expert (<= 16)
    int assign[64][kMaxTok];  // their assignment ids t*k + j, ascending
};

// Builds the per-expert token lists; call with all threads, ends with a barrier.
__device__ void build_groups(Groups& g, const int32_t* __restrict__ idx, int A, int E) {
    const int tid = threadIdx.x;
    if (tid < 64) {
        int c = 0;
        if (tid < E) {
            for (int a = 0; a < A; ++a) {
                const int e = min(max(idx[a], 0), E - 1);
                if (e == tid && c < kMaxTok) ++c;
            }
        }
        const uint64_t present = __ballot(c > 0);
        const int ord = __popcll(present & ((1ull << tid) - 1ull));
        if (tid == 0) g.n_active = __popcll(present);
        if (c > 0) {
            g.expert[ord] = tid;
            g.cnt[ord] = c;
            int n = 0;
            for (int a = 0; a < A; ++a) {
                const int e = min(max(idx[a], 0), E - 1);
                if (e == tid && n < kMaxTok) g.assign[ord][n++] = a;
            }
        }
    }
    __syncthreads();
}

typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

__device__ inline u32x4 load16(const uint16_t* p, bool on) {
    u32x4 v = {0u, 0u, 0u, 0u};
    if (on) v = *reinterpret_cast<const u32x4*>(p);
    return v;
}

__device__ inline bf16x8 pick(bool first, u32x4 a, u32x4 b) {
    u32x4 v;
#pragma unroll
    for (int i = 0; i < 4; ++i) v[i] = first ? a[i] : b[i];
    return __builtin_bit_cast(bf16x8, v);
}

// Barrier that orders LDS traffic only: loads from global memory stay in flight across it.
__device__ inline void lds_barrier() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// acc1 holds MFMA row i = weight row i, acc2 holds MFMA row i = weight row i ^ 8; MFMA rows
// 4 * (lane / 16) + r sit in lane, so row i ^ 8 is the same register of lane ^ 32.
__device__ inline f32x4 fold_halves(f32x4 acc1, f32x4 acc2) {
    f32x4 r;
#pragma unroll
    for (int i = 0; i < 4; ++i) r[i] = acc1[i] + __shfl_xor(acc2[i], 32, 64);
    return r;
}

// Per-lane element offsets inside a tile of 16 weight rows and a 64-element K step.
struct LaneMap {
    int row_lo, row_hi;  // weight rows (within the tile) of the two loads
    int k_lo, k_hi;      // element offset of this lane's 8 elements inside the K step
    int kq8;             // element offset of the lane's token operand inside each 32-element half
    bool upper;
    __device__ explicit LaneMap(int lane) {
        const int i = lane & 15, kq = lane >> 4;
        upper = i >= 8;
        row_lo = i & 7;
        row_hi = 8 + (i & 7);
        k_lo = ((upper ? 4 : 0) + kq) * 8;
        k_hi = ((upper ? 0 : 4) + kq) * 8;
        kq8 = kq * 8;
    }
};

template <int P>
__global__ __launch_bounds__(kThreads) void dec_gemm1(const uint16_t* __restrict__ x,
                                                       const int32_t* __restrict__ idx,
                                                       const uint16_t* __restrict__ w1,
                                                       const uint16_t* __restrict__ w3, int T, int k, int E, int H,
                                                       int F, uint16_t* __restrict__ act) {
    __shared__ Groups g;
    __shared__ f32x4 red[2][kWaves][2][64];
    build_groups(g, idx, T * k, E);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int col = lane & 15;
    const LaneMap lm(lane);

    const int tiles_per_expert = F / 16;
    const int total_tiles = g.n_active * tiles_per_expert;
    const int tiles_per_wg = (total_tiles + gridDim.x - 1) / gridDim.x;
    const int t0 = blockIdx.x * tiles_per_wg;
    const int t1 = min(total_tiles, t0 + tiles_per_wg);
    if (t0 >= t1) return;

    // K split: 64-element steps dealt to the wavefronts in contiguous runs.
    const int k_steps = H / 64;
    const int per = (k_steps + kWaves - 1) / kWaves;
    const int s_begin = wave * per;
    const int n_valid = max(0, min(k_steps, s_begin + per) - s_begin);
    const int spt = (per + P - 1) / P * P;  // steps per tile, padded to the pipeline depth
    const long total_q = (long)(t1 - t0) * spt;

    u32x4 lo1[P], hi1[P], lo3[P], hi3[P], xa[P], xb[P];
    // Issue-side state: the next step to request and the row bases of its tile.
    int is = 0, itile = t0;
    size_t wlo = 0, whi = 0, xbase = 0;
    bool xcol = false;
    auto enter_tile = [&]() {
        const int d = itile / tiles_per_expert;
        const int f0 = (itile - d * tiles_per_expert) * 16;
        const size_t row0 = (size_t)g.expert[d] * F + f0;
        const size_t k0 = (size_t)s_begin * 64;
        wlo = (row0 + lm.row_lo) * H + k0 + lm.k_lo;
        whi = (row0 + lm.row_hi) * H + k0 + lm.k_hi;
        xcol = col < g.cnt[d];
        xbase = (size_t)(xcol ? g.assign[d][col] / k : 0) * H + k0 + lm.kq8;
    };
    enter_tile();
    auto issue = [&](int i) {
        const bool on = is < n_valid;
        lo1[i] = load16(w1 + wlo + is * 64, on);
        hi1[i] = load16(w1 + whi + is * 64, on);
        lo3[i] = load16(w3 + wlo + is * 64, on);
        hi3[i] = load16(w3 + whi + is * 64, on);
        xa[i] = load16(x + xbase + is * 64, on && xcol);
        xb[i] = load16(x + xbase + is * 64 + 32, on && xcol);
        if (++is == spt) {
            is = 0;
            if (++itile < t1) enter_tile();
        }
    };
#pragma unroll
    for (int i = 0; i < P; ++i) issue(i);  // total_q >= spt >= P

    const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
    f32x4 g1 = zero, g2 = zero, u1 = zero, u2 = zero;
    int cs = 0, ctile = t0;
    for (long q = 0; q < total_q; q += P) {
#pragma unroll
        for (int i = 0; i < P; ++i) {
            const bf16x8 b1 = __builtin_bit_cast(bf16x8, xa[i]);
            const bf16x8 b2 = __builtin_bit_cast(bf16x8, xb[i]);
            g1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(pick(lm.upper, hi1[i], lo1[i]), b1, g1, 0, 0, 0);
            g2 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(pick(lm.upper, lo1[i], hi1[i]), b2, g2, 0, 0, 0);
            u1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(pick(lm.upper, hi3[i], lo3[i]), b1, u1, 0, 0, 0);
            u2 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(pick(lm.upper, lo3[i], hi3[i]), b2, u2, 0, 0, 0);
            if (q + P + i < total_q) issue(i);
        }
        cs += P;
        if (cs == spt) {
            // Tile done: fold the 8 K-slices.  MFMA 16x16 result: lane holds column (token)
            // lane & 15 and rows (features) 4 * (lane / 16) + r, r = 0..3.
            const int par = (ctile - t0) & 1;
            red[par][wave][0][lane] = fold_halves(g1, g2);
            red[par][wave][1][lane] = fold_halves(u1, u2);
            lds_barrier();
            if (tid < 256) {
                const int p = tid & 63, r = tid >> 6;
                const int d = ctile / tiles_per_expert;
                const int f0 = (ctile - d * tiles_per_expert) * 16;
                const int c = p & 15;
                if (c < g.cnt[d]) {
                    float gs = 0.f, us = 0.f;
#pragma unroll
                    for (int w = 0; w < kWaves; ++w) {
                        gs += red[par][w][0][p][r];
                        us += red[par][w][1][p][r];
                    }
                    act[(size_t)g.assign[d][c] * F + f0 + 4 * (p >> 4) + r] = to_bf16(swiglu(gs, us));
                }
            }
            g1 = g2 = u1 = u2 = zero;
            cs = 0;
            ++ctile;
        }
    }
}

template <int P>
__global__ __launch_bounds__(kThreads) void dec_gemm2(const uint16_t* __restrict__ act,
                                                       const int32_t* __restrict__ idx,
                                                       const float* __restrict__ topk_w,
                                                       const uint16_t* __restrict__ w2, int T, int k, int E, int H,
                                                       int F, uint16_t* __restrict__ y) {
    __shared__ Groups g;
    __shared__ f32x4 red[2][kWaves][64];
    __shared__ float yacc[kMaxTok][16];
    build_groups(g, idx, T * k, E);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int col = lane & 15;
    const LaneMap lm(lane);
    const int h0 = blockIdx.x * 16;
    if (tid < kMaxTok * 16) yacc[tid >> 4][tid & 15] = 0.f;

    const int k_steps = F / 64;
    const int per = (k_steps + kWaves - 1) / kWaves;
    const int s_begin = wave * per;
    const int n_valid = max(0, min(k_steps, s_begin + per) - s_begin);
    const int spt = (per + P - 1) / P * P;
    const int D = g.n_active;
    const long total_q = (long)D * spt;

    u32x4 lo[P], hi[P], aa[P], ab[P];
    int is = 0, id = 0;
    size_t wlo = 0, whi = 0, abase = 0;
    bool acol = false;
    auto enter_expert = [&]() {
        const size_t row0 = (size_t)g.expert[id] * H + h0;
        const size_t k0 = (size_t)s_begin * 64;
        wlo = (row0 + lm.row_lo) * F + k0 + lm.k_lo;
        whi = (row0 + lm.row_hi) * F + k0 + lm.k_hi;
        acol = col < g.cnt[id];
        abase = (size_t)(acol ? g.assign[id][col] : 0) * F + k0 + lm.kq8;
    };
    if (D > 0) enter_expert();
    auto issue = [&](int i) {
        const bool on = is < n_valid;
        lo[i] = load16(w2 + wlo + is * 64, on);
        hi[i] = load16(w2 + whi + is * 64, on);
        aa[i] = load16(act + abase + is * 64, on && acol);
        ab[i] = load16(act + abase + is * 64 + 32, on && acol);
        if (++is == spt) {
            is = 0;
            if (++id < D) enter_expert();
        }
    };
    if (D > 0) {
#pragma unroll
        for (int i = 0; i < P; ++i) issue(i);
    }
    const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
    f32x4 acc1 = zero, acc2 = zero;
    int cs = 0, cd = 0;
    for (long q = 0; q < total_q; q += P) {
#pragma unroll
        for (int i = 0; i < P; ++i) {
            acc1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(pick(lm.upper, hi[i], lo[i]),
                                                           __builtin_bit_cast(bf16x8, aa[i]), acc1, 0, 0, 0);
            acc2 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(pick(lm.upper, lo[i], hi[i]),
                                                           __builtin_bit_cast(bf16x8, ab[i]), acc2, 0, 0, 0);
            if (q + P + i < total_q) issue(i);
        }
        cs += P;
        if (cs == spt) {
            const int par = cd & 1;
            red[par][wave][lane] = fold_halves(acc1, acc2);
            lds_barrier();
            if (tid < 256) {
                const int p = tid & 63, r = tid >> 6;
                const int c = p & 15;
                if (c < g.cnt[cd]) {
                    float s = 0.f;
#pragma unroll
                    for (int w = 0; w < kWaves; ++w) s += red[par][w][p][r];
                    const int a = g.assign[cd][c];
                    yacc[a / k][4 * (p >> 4) + r] += topk_w[a] * s;
                }
            }
            acc1 = acc2 = zero;
            cs = 0;
            ++cd;
        }
    }
    __syncthreads();
    if (tid < T * 16) {
        const int t = tid >> 4, r = tid & 15;
        y[(size_t)t * H + h0 + r] = to_bf16(yacc[t][r]);
    }
}

}  // namespace

hipError_t launch_ffn_bf16_decode(const moe_shape_t& s, int tokens, const void* x, const int32_t* topk_idx,
                                  const float* topk_w, const void* w1, const void* w3, const void* w2, void* y,
                                  void* act, hipStream_t stream) {
    const int max_tiles = min(s.n_experts, tokens * s.top_k) * (s.ffn / 16);
    const int grid1 = min(compute_units(), max_tiles);
    dec_gemm1<MOE_DEC_P1><<<grid1, kThreads, 0, stream>>>(static_cast<const uint16_t*>(x), topk_idx,
                                                 static_cast<const uint16_t*>(w1), static_cast<const uint16_t*>(w3),
                                                 tokens, s.top_k, s.n_experts, s.hidden, s.ffn,
                                                 static_cast<uint16_t*>(act));
    stage_mark(stream, kStageGemm1);
    dec_gemm2<MOE_DEC_P2><<<s.hidden / 16, kThreads, 0, stream>>>(static_cast<const uint16_t*>(act), topk_idx, topk_w,
                                                          static_cast<const uint16_t*>(w2), tokens, s.top_k,
                                                          s.n_experts, s.hidden, s.ffn, static_cast<uint16_t*>(y));
    stage_mark(stream, kStageGemm2);
    return hipGetLastError();
}

}  // namespace moe
