// Gating function, softmax, top-k selection and selection histograms
// (DAOP paper Sec. II-A "MoE Structure"; activity counts of Sec. IV-B /
// Algorithm 1; next-layer prediction of Sec. III observation 3 / Sec. IV-C,
// which is the same computation with the next layer's gate on the same x).
//
// One wavefront owns one token at a time.  The 64 lanes split the hidden
// dimension in 16-byte pieces, keep one fp32 partial sum per expert, and fold
// the partials with a butterfly of wavefront shuffles, after which every lane
// holds all E logits and the softmax / top-k run redundantly in registers.
// Up to two gates (this layer's and the next layer's) are evaluated per token
// so x comes from HBM once; the second pass over the row hits the vector cache.
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

// Routes token `t` through one gate.  All lanes of the wavefront take part;
// lane 0 writes the result and bumps the workgroup histogram in LDS.
template <typename scalar_t, int EPAD>
__device__ void route_token(const scalar_t* __restrict__ xrow, const RouteParams& p, const GateArgs& g,
                            int t, int lane, int* lds_hist) {
    const int H = p.hidden, E = p.n_experts, k = p.top_k;
    const scalar_t* __restrict__ wg = static_cast<const scalar_t*>(g.w);
    float acc[EPAD];
#pragma unroll
    for (int r = 0; r < EPAD; ++r) acc[r] = 0.f;
    for (int h = lane * 8; h < H; h += 64 * 8) {
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
        if (g.bias != nullptr && r < E) acc[r] += g.bias[r];
    }
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

    // k passes of arg-max; strict '>' while scanning upward keeps the lower index on ties.
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

template <typename scalar_t, int EPAD>
__global__ __launch_bounds__(256) void route_kernel(RouteParams p) {
    __shared__ int hist[2][64];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    if (tid < 128) hist[tid >> 6][tid & 63] = 0;
    __syncthreads();
    const scalar_t* x = static_cast<const scalar_t*>(p.x);
    for (int i = wave; i < kRouteTokensPerBlock; i += 4) {
        const int t = blockIdx.x * kRouteTokensPerBlock + i;
        if (t < p.tokens) {
            for (int g = 0; g < p.n_gates; ++g)
                route_token<scalar_t, EPAD>(x + (size_t)t * p.hidden, p, p.gate[g], t, lane, hist[g]);
        }
    }
    __syncthreads();
    if (tid < p.n_experts) {
        for (int g = 0; g < p.n_gates; ++g)
            if (p.gate[g].hist != nullptr) p.gate[g].hist[(size_t)blockIdx.x * p.n_experts + tid] = hist[g][tid];
    }
}

// Decode path: every token of the call in one workgroup of 16 wavefronts; the
// counts are final when the workgroup ends, so no second kernel is needed.
template <typename scalar_t, int EPAD>
__global__ __launch_bounds__(1024) void route_small_kernel(RouteParams p) {
    __shared__ int hist[2][64];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    if (tid < 128) hist[tid >> 6][tid & 63] = 0;
    __syncthreads();
    const scalar_t* x = static_cast<const scalar_t*>(p.x);
    for (int t = wave; t < p.tokens; t += 16) {
        for (int g = 0; g < p.n_gates; ++g)
            route_token<scalar_t, EPAD>(x + (size_t)t * p.hidden, p, p.gate[g], t, lane, hist[g]);
    }
    __syncthreads();
    if (tid < p.n_experts) {
        if (p.counts != nullptr) p.counts[tid] = (p.accumulate ? p.counts[tid] : 0) + hist[0][tid];
        if (p.counts_next != nullptr) p.counts_next[tid] = hist[1][tid];
    }
}

template <typename scalar_t>
void launch_by_epad(const RouteParams& p, bool small, hipStream_t stream) {
    const int E = p.n_experts;
    if (small) {
        if (E <= 8) route_small_kernel<scalar_t, 8><<<1, 1024, 0, stream>>>(p);
        else if (E <= 16) route_small_kernel<scalar_t, 16><<<1, 1024, 0, stream>>>(p);
        else if (E <= 32) route_small_kernel<scalar_t, 32><<<1, 1024, 0, stream>>>(p);
        else route_small_kernel<scalar_t, 64><<<1, 1024, 0, stream>>>(p);
    } else {
        const int nb = route_blocks(p.tokens);
        if (E <= 8) route_kernel<scalar_t, 8><<<nb, 256, 0, stream>>>(p);
        else if (E <= 16) route_kernel<scalar_t, 16><<<nb, 256, 0, stream>>>(p);
        else if (E <= 32) route_kernel<scalar_t, 32><<<nb, 256, 0, stream>>>(p);
        else route_kernel<scalar_t, 64><<<nb, 256, 0, stream>>>(p);
    }
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
