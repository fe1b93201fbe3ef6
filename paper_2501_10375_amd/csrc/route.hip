// Gating function, softmax, top-k selection and selection histograms
// (DAOP paper Sec. II-A "MoE Structure"; activity counts of Sec. IV-B /
// Algorithm 1; next-layer prediction of Sec. III observation 3 / Sec. IV-C,
// which is the same computation with the next layer's gate on the same x).
//
// One wavefront (or, for decode-size calls, a group of up to 16 wavefronts)
// owns one token.  The lanes split the hidden dimension in 16-byte pieces,
// keep one fp32 partial sum per expert, and fold the partials with a butterfly
// of wavefront shuffles (then through LDS across the wavefronts of a group),
// after which every lane holds all E logits and the softmax / top-k run
// redundantly in registers.  Up to two gates (this layer's and the next
// layer's) are evaluated per token so x comes from HBM once; the second pass
// over the row hits the vector cache.
#include "moe_internal.h"

namespace moe {
namespace {

struct RouteParams {
    const void* x;
    int tokens, hidden, n_experts, top_k, n_gates;
    GateArgs gate[2];
    int32_t* counts;       // decode path only
    int32_t* counts_next;  // decode path only
    int accumulate;
};

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

// Partial logits of one token against one gate over the 16-byte pieces
// (piece index = (i * n_slices + slice) * 64 + lane) of the hidden dimension.
// Returns with every lane holding the wavefront's sums in acc[0..E).
template <typename scalar_t, int EPAD>
__device__ inline void gate_partial(const scalar_t* __restrict__ xrow, const scalar_t* __restrict__ wg, int H, int E,
                                    int slice, int n_slices, int lane, float (&acc)[EPAD]) {
#pragma unroll
    for (int r = 0; r < EPAD; ++r) acc[r] = 0.f;
    for (int h = (slice * 64 + lane) * 8; h < H; h += n_slices * 64 * 8) {
        float xv[8];
        load8(xrow + h, xv);
#pragma unroll
        for (int r = 0; r < EPAD; ++r) {
            if (r < E) {
                float wv[8];
                load8(wg + (size_t)r * H + h, wv);
#pragma unroll
                for (int i = 0; i < 8; ++i) acc[r] = fmaf(xv[i], wv[i], acc[r]);
            }
        }
    }
#pragma unroll
    for (int r = 0; r < EPAD; ++r) {
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) acc[r] += __shfl_xor(acc[r], off, 64);
    }
}

// Softmax over the E logits in acc, k passes of arg-max, renormalised weights.
// Every lane computes the same values; lane 0 writes them and bumps the LDS histogram.
// `bias` is the gate's bias vector (global memory or a copy in LDS) or null.
template <int EPAD>
__device__ inline void select_topk(float (&acc)[EPAD], const GateArgs& g, const float* bias, int E, int k, int t,
                                   int lane, int* lds_hist) {
#pragma unroll
    for (int r = 0; r < EPAD; ++r)
        if (bias != nullptr && r < E) acc[r] += bias[r];
    float zmax = -INFINITY;
#pragma unroll
    for (int r = 0; r < EPAD; ++r)
        if (r < E) zmax = fmaxf(zmax, acc[r]);
    float denom = 0.f;
#pragma unroll
    for (int r = 0; r < EPAD; ++r) {
        acc[r] = (r < E) ? expf(acc[r] - zmax) : 0.f;
        denom += acc[r];
    }
#pragma unroll
    for (int r = 0; r < EPAD; ++r) acc[r] = acc[r] / denom;

    // strict '>' while scanning upward keeps the lower index on ties
    uint64_t taken = 0;
    int sel[8];
    float selp[8];
    float wsum = 0.f;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        sel[j] = 0;
        selp[j] = 0.f;
        if (j < k) {
            int best = -1;
            float bp = -1.f;
#pragma unroll
            for (int r = 0; r < EPAD; ++r) {
                if (r < E && !((taken >> r) & 1ull) && acc[r] > bp) {
                    bp = acc[r];
                    best = r;
                }
            }
            if (best < 0) {  // only with non-finite inputs: still return a valid, distinct expert
                best = __ffsll((long long)~taken) - 1;
                bp = 0.f;
            }
            taken |= 1ull << best;
            sel[j] = best;
            selp[j] = bp;
            wsum += bp;
        }
    }
    if (lane == 0) {
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            if (j < k) {
                g.idx[(size_t)t * k + j] = sel[j];
                if (g.wts != nullptr) g.wts[(size_t)t * k + j] = selp[j] / wsum;
                atomicAdd(&lds_hist[sel[j]], 1);
            }
        }
    }
}

// 16 wavefronts per workgroup.  WPT wavefronts share one token (each takes an
// interleaved slice of the hidden dimension; partial logits are summed through
// LDS in slice order), so a workgroup covers 16 / WPT tokens.
//   SMALL = false: WPT = 1, grid = ceil(T / 16); per-workgroup histograms go to gate.hist.
//   SMALL = true : one workgroup holds the whole call (T <= 16 / WPT); counts are written directly.
//                  The call is a chain of memory latencies, so the bias vectors and the old counts
//                  are requested before the gate rows and parked in LDS while those arrive.
template <typename scalar_t, int EPAD, int WPT, bool SMALL>
__global__ __launch_bounds__(1024) void route_kernel(RouteParams p) {
    constexpr bool kViaLds = WPT > 1 || SMALL;
    __shared__ int hist[2][64];
    __shared__ float part[kViaLds ? 16 : 1][2][EPAD];
    __shared__ float sbias[2][64];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int H = p.hidden, E = p.n_experts;
    float my_bias = 0.f;
    int old_count = 0;
    if (SMALL) {
        if (tid < 128 && (tid >> 6) < p.n_gates && (tid & 63) < E && p.gate[tid >> 6].bias != nullptr)
            my_bias = p.gate[tid >> 6].bias[tid & 63];
        if (tid < E && p.accumulate && p.counts != nullptr) old_count = p.counts[tid];
    }
    if (tid < 128) hist[tid >> 6][tid & 63] = 0;
    __syncthreads();
    const int t = blockIdx.x * (16 / WPT) + wave / WPT;
    const int slice = wave % WPT;
    const bool live = t < p.tokens;
    const scalar_t* xrow = static_cast<const scalar_t*>(p.x) + (size_t)(live ? t : 0) * H;
    float acc[EPAD];
    for (int g = 0; g < p.n_gates; ++g) {
        if (live) {
            gate_partial<scalar_t, EPAD>(xrow, static_cast<const scalar_t*>(p.gate[g].w), H, E, slice, WPT, lane, acc);
            if (!kViaLds) {
                select_topk<EPAD>(acc, p.gate[g], p.gate[g].bias, E, p.top_k, t, lane, hist[g]);
            } else if (lane == 0) {
#pragma unroll
                for (int r = 0; r < EPAD; ++r) part[wave][g][r] = acc[r];
            }
        }
    }
    if (kViaLds) {
        if (SMALL && tid < 128) sbias[tid >> 6][tid & 63] = my_bias;
        __syncthreads();
        if (live && slice == 0) {
            for (int g = 0; g < p.n_gates; ++g) {
#pragma unroll
                for (int r = 0; r < EPAD; ++r) {
                    float s = 0.f;
#pragma unroll
                    for (int w = 0; w < WPT; ++w) s += part[wave + w][g][r];
                    acc[r] = s;
                }
                const float* bias = p.gate[g].bias;
                if (SMALL && bias != nullptr) bias = sbias[g];
                select_topk<EPAD>(acc, p.gate[g], bias, E, p.top_k, t, lane, hist[g]);
            }
        }
    }
    __syncthreads();
    if (tid < E) {
        if (SMALL) {
            if (p.counts != nullptr) p.counts[tid] = old_count + hist[0][tid];
            if (p.counts_next != nullptr) p.counts_next[tid] = hist[1][tid];
        } else {
            for (int g = 0; g < p.n_gates; ++g)
                if (p.gate[g].hist != nullptr) p.gate[g].hist[(size_t)blockIdx.x * E + tid] = hist[g][tid];
        }
    }
}

template <typename scalar_t, int EPAD>
void launch_epad(const RouteParams& p, bool small, hipStream_t stream) {
    if (!small) {
        route_kernel<scalar_t, EPAD, 1, false><<<route_blocks(p.tokens), 1024, 0, stream>>>(p);
    } else if (p.tokens <= 1) {
        route_kernel<scalar_t, EPAD, 16, true><<<1, 1024, 0, stream>>>(p);
    } else if (p.tokens <= 2) {
        route_kernel<scalar_t, EPAD, 8, true><<<1, 1024, 0, stream>>>(p);
    } else if (p.tokens <= 4) {
        route_kernel<scalar_t, EPAD, 4, true><<<1, 1024, 0, stream>>>(p);
    } else if (p.tokens <= 8) {
        route_kernel<scalar_t, EPAD, 2, true><<<1, 1024, 0, stream>>>(p);
    } else {
        route_kernel<scalar_t, EPAD, 1, true><<<1, 1024, 0, stream>>>(p);
    }
}

template <typename scalar_t>
void launch_by_epad(const RouteParams& p, bool small, hipStream_t stream) {
    const int E = p.n_experts;
    if (E <= 8) launch_epad<scalar_t, 8>(p, small, stream);
    else if (E <= 16) launch_epad<scalar_t, 16>(p, small, stream);
    else if (E <= 32) launch_epad<scalar_t, 32>(p, small, stream);
    else launch_epad<scalar_t, 64>(p, small, stream);
}

RouteParams make_params(const moe_shape_t& s, int tokens, const void* x, const GateArgs* gates, int n_gates) {
    RouteParams p{};
    p.x = x;
    p.tokens = tokens;
    p.hidden = s.hidden;
    p.n_experts = s.n_experts;
    p.top_k = s.top_k;
    p.n_gates = n_gates;
    for (int g = 0; g < n_gates; ++g) p.gate[g] = gates[g];
    return p;
}

}  // namespace

hipError_t launch_route(const moe_shape_t& s, int tokens, const void* x, const GateArgs* gates, int n_gates,
                        hipStream_t stream) {
    RouteParams p = make_params(s, tokens, x, gates, n_gates);
    if (s.dtype == MOE_F32) launch_by_epad<float>(p, false, stream);
    else launch_by_epad<uint16_t>(p, false, stream);
    return hipGetLastError();
}

hipError_t launch_route_small(const moe_shape_t& s, int tokens, const void* x, const GateArgs* gates,
                              int n_gates, int32_t* counts, int accumulate, int32_t* counts_next,
                              hipStream_t stream) {
    RouteParams p = make_params(s, tokens, x, gates, n_gates);
    p.counts = counts;
    p.counts_next = counts_next;
    p.accumulate = accumulate;
    if (s.dtype == MOE_F32) launch_by_epad<float>(p, true, stream);
    else launch_by_epad<uint16_t>(p, true, stream);
    return hipGetLastError();
}

}  // namespace moe
