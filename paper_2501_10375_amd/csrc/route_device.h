// Device code of the gating function shared by the routing kernels and the
// fused decode kernel (DAOP paper Sec. II-A "MoE Structure": gate logits,
// softmax over all experts, top-k with renormalised weights; the same
// computation with the next layer's gate gives the prediction of Sec. III
// observation 3 / Sec. IV-C).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace moe {

__device__ inline void load8(const float* p, float (&v)[8]) {
    const float4 a = *reinterpret_cast<const float4*>(p);
    const float4 b = *reinterpret_cast<const float4*>(p + 4);
    v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w;
    v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
}

__device__ inline void load8(const uint16_t* p, float (&v)[8]) {
    const uint4 q = *reinterpret_cast<const uint4*>(p);
    const uint32_t w[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        v[2 * i] = __uint_as_float(w[i] << 16);
        v[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
    }
}

// Eight consecutive elements as loaded (16 or 32 bytes), converted to fp32 only when they are used,
// so that a group of loads can be issued back to back before the first conversion.
template <typename scalar_t>
struct Raw8;
template <>
struct Raw8<float> {
    float4 a, b;
    __device__ inline void load(const float* p) {
        a = *reinterpret_cast<const float4*>(p);
        b = *reinterpret_cast<const float4*>(p + 4);
    }
    __device__ inline void get(float (&v)[8]) const {
        v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w;
        v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
    }
};
template <>
struct Raw8<uint16_t> {
    uint4 q;
    __device__ inline void load(const uint16_t* p) { q = *reinterpret_cast<const uint4*>(p); }
    __device__ inline void get(float (&v)[8]) const {
        const uint32_t w[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            v[2 * i] = __uint_as_float(w[i] << 16);
            v[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
        }
    }
};

// Reductions over the 64 lanes, the result in every lane.  Within a row of 16 lanes the partners
// come through the data-parallel-primitive path (exchange with the neighbour, the neighbouring
// pair, the mirrored half row and the mirrored row: four register-to-register moves), the four row
// results are then read out as scalars.  An LDS-routed shuffle per step would cost about a hundred
// cycles each, and the softmax and top-k chain some twenty of these reductions one after another.
// Every lane performs the same operations on the same values in the same order, so all lanes hold
// bit-identical results (the additions of wave_sum are: pairs, quads, half rows, rows, then the
// four rows in ascending order).
template <int CTRL>
__device__ inline float dpp_move(float v) {
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xF, 0xF, false));
}
__device__ inline float lane_value(float v, int lane) {  // lane is a compile-time constant at every use
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), lane));
}
constexpr int kDppSwapNeighbours = 0xB1;   // quad_perm [1, 0, 3, 2]
constexpr int kDppSwapPairs = 0x4E;        // quad_perm [2, 3, 0, 1]
constexpr int kDppHalfRowMirror = 0x141;   // lane i of each 8 <- lane 7 - i
constexpr int kDppRowMirror = 0x140;       // lane i of each 16 <- lane 15 - i

__device__ inline float wave_max(float v) {
    v = fmaxf(v, dpp_move<kDppSwapNeighbours>(v));
    v = fmaxf(v, dpp_move<kDppSwapPairs>(v));
    v = fmaxf(v, dpp_move<kDppHalfRowMirror>(v));
    v = fmaxf(v, dpp_move<kDppRowMirror>(v));
    const float r0 = lane_value(v, 0), r1 = lane_value(v, 16), r2 = lane_value(v, 32), r3 = lane_value(v, 48);
    return fmaxf(fmaxf(r0, r1), fmaxf(r2, r3));
}

__device__ inline float wave_sum(float v) {
    v += dpp_move<kDppSwapNeighbours>(v);
    v += dpp_move<kDppSwapPairs>(v);
    v += dpp_move<kDppHalfRowMirror>(v);
    v += dpp_move<kDppRowMirror>(v);
    const float r0 = lane_value(v, 0), r1 = lane_value(v, 16), r2 = lane_value(v, 32), r3 = lane_value(v, 48);
    return ((r0 + r1) + r2) + r3;
}

// Softmax over the E logits held one per lane (z of lane e is expert e's logit, -inf beyond E),
// then k passes of arg-max across the lanes, the lowest lane among equals winning.  Every lane
// takes part; on return lane j < k holds selection j (expert and renormalised weight), in
// descending probability.
//
// With `degrade` (graceful degradation, Sec. IV-C "Accuracy Stabilization" / "Graceful
// Degradation"; `resident` = this lane's expert is in the GPU expert cache): if no selected expert
// is resident, the last selection (the lowest probability) is replaced by the most probable
// resident expert, if there is one; it cannot outrank the k - 1 selections that stay, so the
// order is preserved.
__device__ inline void select_topk_lanes(float z, int lane, int E, int k, int& my_sel, float& my_w,
                                         bool degrade = false, bool resident = false) {
    const float zmax = wave_max(z);
    float p = lane < E ? expf(z - zmax) : 0.f;
    p = p / wave_sum(p);
    bool taken = lane >= E;
    float my_p = 0.f, wsum = 0.f;
    my_sel = 0;
    for (int j = 0; j < k; ++j) {
        const float cand = taken ? -1.f : p;
        float best = wave_max(cand);
        uint64_t m = __ballot(!taken && cand == best);
        if (m == 0) {  // only with non-finite inputs: still select a valid, distinct expert
            m = __ballot(!taken);
            best = 0.f;
        }
        const int sel = __ffsll((long long)m) - 1;
        if (lane == sel) taken = true;
        if (lane == j) {
            my_sel = sel;
            my_p = best;
        }
        wsum += best;
    }
    if (degrade) {
        const bool selected = taken && lane < E;
        if (__ballot(selected && resident) == 0) {
            const bool cand = !taken && resident;
            const float best = wave_max(cand ? p : -1.f);
            const uint64_t m = __ballot(cand && p == best);
            if (m != 0) {
                if (lane == k - 1) {
                    my_sel = __ffsll((long long)m) - 1;
                    my_p = best;
                }
                wsum = 0.f;
                for (int j = 0; j < k; ++j) wsum += __shfl(my_p, j, 64);
            }
        }
    }
    my_w = my_p / wsum;
}

// ---- routing of a decode-size call (at most 16 tokens) by one workgroup of 8 wavefronts ----

constexpr int kSmallRouteThreads = 512;
constexpr int kSmallRouteMaxTokens = 16;

struct RouteSmem {
    int idx[kSmallRouteMaxTokens * 8];
    float w[kSmallRouteMaxTokens * 8];
};
// Floats of LDS scratch route_tokens_wg needs: [wavefront][token][expert] partial logits.
constexpr int kRoutePartFloats = 8 * kSmallRouteMaxTokens * 64;

// Sums acc[0..8) over the 64 lanes with a halving exchange: after the three exchange steps each
// lane carries one of the 8 values (which one is given by lane bits 5, 4, 3), after three more
// butterfly steps lanes with (lane & 7) == 0 hold the full sum of value
// 4 * bit5 + 2 * bit4 + bit3.  10 shuffles instead of 48, in a fixed order.
__device__ inline float reduce8_scatter(const float (&acc)[8], int lane) {
    const bool b5 = (lane & 32) != 0, b4 = (lane & 16) != 0, b3 = (lane & 8) != 0;
    float v4[4], v2[2];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const float keep = b5 ? acc[4 + i] : acc[i];
        const float give = b5 ? acc[i] : acc[4 + i];
        v4[i] = keep + __shfl_xor(give, 32, 64);
    }
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const float keep = b4 ? v4[2 + i] : v4[i];
        const float give = b4 ? v4[i] : v4[2 + i];
        v2[i] = keep + __shfl_xor(give, 16, 64);
    }
    const float keep = b3 ? v2[1] : v2[0];
    const float give = b3 ? v2[0] : v2[1];
    float v = keep + __shfl_xor(give, 8, 64);
    v += __shfl_xor(v, 4, 64);
    v += __shfl_xor(v, 2, 64);
    v += __shfl_xor(v, 1, 64);
    return v;
}

// Routes tokens 0..T (T <= 16) against one gate; every thread of the 512-thread workgroup calls
// it.  On return (after a workgroup barrier) sm.idx[t*k + j] / sm.w[t*k + j] hold expert and
// renormalised weight of selection j of token t, in descending probability, ties to the lower
// index.  The arithmetic depends only on (T, H, E, k), never on the workgroup, so any number of
// workgroups computing the same call agree bit for bit.  `part` is kRoutePartFloats of LDS.
// With `on_gpu` (uint8 [E]) the selection is degraded gracefully, see select_topk_lanes.
//
// The 8 wavefronts split the hidden dimension in interleaved 512-element chunks, so the gate and
// x are read once per workgroup whatever T is; a wavefront walks the tokens two at a time over
// its chunks (the gate pieces of later tokens come from the vector cache).  Per-wavefront partial
// logits are summed in wavefront order through LDS; the softmax and the k arg-max passes run
// across the lanes of one wavefront, lane e holding expert e.
template <typename scalar_t>
__device__ inline void route_tokens_wg(const scalar_t* __restrict__ x, const scalar_t* __restrict__ wg,
                                       const float* __restrict__ bias, int T, int H, int E, int k, RouteSmem& sm,
                                       float* part, const uint8_t* __restrict__ on_gpu = nullptr) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    // requested first so that it arrives together with the gate rows
    const float my_bias = (bias != nullptr && lane < E) ? bias[lane] : 0.f;
    const bool resident = on_gpu != nullptr && lane < E && on_gpu[lane] != 0;
    const int n_blocks = (E + 7) / 8;
    const int esub = ((lane >> 5) & 1) * 4 + ((lane >> 4) & 1) * 2 + ((lane >> 3) & 1);
    for (int t = 0; t < T; t += 2) {
        const bool two = t + 1 < T;
        const scalar_t* x0 = x + (size_t)t * H;
        const scalar_t* x1 = x + (size_t)(two ? t + 1 : t) * H;
        for (int eb = 0; eb < n_blocks; ++eb) {
            const int ne = min(8, E - eb * 8);
            const scalar_t* wrow = wg + (size_t)eb * 8 * H;
            float acc0[8], acc1[8];
#pragma unroll
            for (int r = 0; r < 8; ++r) acc0[r] = acc1[r] = 0.f;
            for (int h = (wave * 64 + lane) * 8; h < H; h += 8 * 512) {
                // All loads of the step first, unconditionally (rows past the last expert re-read it;
                // their sums are never looked at), and nothing else scheduled between them: a load
                // under a branch, or one the scheduler leaves next to its use, costs a memory round
                // trip of its own, ten in a row instead of one.
                Raw8<scalar_t> xr0, xr1, wr[8];
                xr0.load(x0 + h);
                xr1.load(x1 + h);
#pragma unroll
                for (int r = 0; r < 8; ++r) wr[r].load(wrow + (size_t)min(r, ne - 1) * H + h);
                __builtin_amdgcn_sched_barrier(0);
                float xv0[8], xv1[8];
                xr0.get(xv0);
                xr1.get(xv1);
#pragma unroll
                for (int r = 0; r < 8; ++r) {
                    float wv[8];
                    wr[r].get(wv);
#pragma unroll
                    for (int i = 0; i < 8; ++i) {
                        acc0[r] = fmaf(xv0[i], wv[i], acc0[r]);
                        acc1[r] = fmaf(xv1[i], wv[i], acc1[r]);
                    }
                }
            }
            const float v0 = reduce8_scatter(acc0, lane);
            const float v1 = reduce8_scatter(acc1, lane);
            if ((lane & 7) == 0) {
                part[(wave * T + t) * 64 + eb * 8 + esub] = v0;
                if (two) part[(wave * T + t + 1) * 64 + eb * 8 + esub] = v1;
            }
        }
    }
    __syncthreads();
    for (int t = wave; t < T; t += 8) {
        float z = -INFINITY;
        if (lane < E) {
            float s = 0.f;
            for (int w = 0; w < 8; ++w) s += part[(w * T + t) * 64 + lane];
            z = s + my_bias;
        }
        int my_sel;
        float my_w;
        select_topk_lanes(z, lane, E, k, my_sel, my_w, on_gpu != nullptr, resident);
        if (lane < k) {
            sm.idx[t * k + lane] = my_sel;
            sm.w[t * k + lane] = my_w;
        }
    }
    __syncthreads();
}

}  // namespace moe
