// Gating function, softmax, top-k selection and selection histograms
// (DAOP paper Sec. II-A "MoE Structure"; activity counts of Sec. IV-B /
// Algorithm 1; next-layer prediction of Sec. III observation 3 / Sec. IV-C,
// which is the same computation with the next layer's gate on the same x).
//
// Prefill-size calls, bf16 storage: a 16-token x 16-expert MFMA tile per
// workgroup with the hidden dimension split over 16 wavefronts
// (route_mfma_kernel); x comes from HBM once for both this layer's and the next
// layer's gate.  fp32 storage (the small parity configuration) keeps a plain
// kernel: one wavefront owns one token, the lanes split the hidden dimension
// in 16-byte pieces with one fp32 partial sum per expert, folded by a butterfly
// of wavefront shuffles, and the softmax / top-k run redundantly in registers.
//
// Decode-size calls (at most 16 tokens) are a chain of memory latencies rather
// than a stream: one workgroup routes the whole call with the hidden dimension
// split over its wavefronts (route_device.h) and writes the counts itself.
#include "moe_internal.h"
#include "route_device.h"

namespace moe {
namespace {

struct RouteParams {
    const void* x;
    int tokens, hidden, n_experts, top_k, n_gates;
    GateArgs gate[2];
    int32_t* counts;       // decode-size calls only
    int32_t* counts_next;  // decode-size calls only
    int accumulate;
};

// Partial logits of one token against one gate over the 16-byte pieces
// (piece index = i * 64 + lane) of the hidden dimension.
// Returns with every lane holding the wavefront's sums in acc[0..E).
template <typename scalar_t, int EPAD>
__device__ inline void gate_partial(const scalar_t* __restrict__ xrow, const scalar_t* __restrict__ wg, int H, int E,
                                    int lane, float (&acc)[EPAD]) {
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
    }
}

// Softmax over the E logits in acc, k passes of arg-max, renormalised weights.
// Every lane computes the same values; lane 0 writes them and bumps the LDS histogram.
template <int EPAD>
__device__ inline void select_topk(float (&acc)[EPAD], const GateArgs& g, int E, int k, int t, int lane,
                                   int* lds_hist) {
#pragma unroll
    for (int r = 0; r < EPAD; ++r)
        if (g.bias != nullptr && r < E) acc[r] += g.bias[r];
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

// 16 wavefronts per workgroup, one token each; grid = ceil(T / 16).  Per-workgroup selection
// histograms go to gate.hist.
template <typename scalar_t, int EPAD>
__global__ __launch_bounds__(1024) void route_kernel(RouteParams p) {
    __shared__ int hist[2][64];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    if (tid < 128) hist[tid >> 6][tid & 63] = 0;
    __syncthreads();
    const int H = p.hidden, E = p.n_experts;
    const int t = blockIdx.x * kRouteTokensPerBlock + wave;
    if (t < p.tokens) {
        const scalar_t* xrow = static_cast<const scalar_t*>(p.x) + (size_t)t * H;
        float acc[EPAD];
        for (int g = 0; g < p.n_gates; ++g) {
            gate_partial<scalar_t, EPAD>(xrow, static_cast<const scalar_t*>(p.gate[g].w), H, E, lane, acc);
            select_topk<EPAD>(acc, p.gate[g], E, p.top_k, t, lane, hist[g]);
        }
    }
    __syncthreads();
    if (tid < E)
        for (int g = 0; g < p.n_gates; ++g)
            if (p.gate[g].hist != nullptr) p.gate[g].hist[(size_t)blockIdx.x * E + tid] = hist[g][tid];
}

// bf16 storage: the gate GEMM on the matrix cores.  One workgroup of 16 wavefronts owns 16 tokens:
// they are the 16 rows of a v_mfma_f32_16x16x32_bf16 whose 16 columns are a block of 16 experts,
// and the wavefronts split the hidden dimension in contiguous runs of 32-element steps.  x is the
// streamed operand (each byte read once, 8 steps of it kept in registers while all gates and expert
// blocks are applied); the gate rows come from cache, once per 16 tokens.  The wavefronts' partial
// 16 x 16 tiles are summed in wavefront order through LDS, gate by gate; then wavefront i takes
// token i with expert e on lane e for the softmax and the top-k.
// NBG = number of 16-expert blocks per gate.
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

template <int NBG>
__global__ __launch_bounds__(1024) void route_mfma_kernel(RouteParams p) {
    constexpr int kChunk = NBG == 1 ? 8 : 4;  // K steps whose x fragments are held in registers at a time
    __shared__ int hist[2][64];
    __shared__ f32x4 part[16][NBG][64];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    if (tid < 128) hist[tid >> 6][tid & 63] = 0;
    const int H = p.hidden, E = p.n_experts, T = p.tokens;
    const int t0 = blockIdx.x * kRouteTokensPerBlock;
    const int row = lane & 15, kq = lane >> 4;
    const uint16_t* x = static_cast<const uint16_t*>(p.x);
    const bool xrow_on = t0 + row < T;
    const uint16_t* xrow = x + (size_t)(xrow_on ? t0 + row : 0) * H + kq * 8;

    const int k_steps = H / 32;
    const int per = (k_steps + 15) / 16;
    const int s_begin = wave * per;
    const int s_end = min(k_steps, s_begin + per);

    const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
    f32x4 acc[2][NBG];
#pragma unroll
    for (int g = 0; g < 2; ++g)
#pragma unroll
        for (int nb = 0; nb < NBG; ++nb) acc[g][nb] = zero;

    for (int s0 = s_begin; s0 < s_end; s0 += kChunk) {
        u32x4 xa[kChunk];
#pragma unroll
        for (int i = 0; i < kChunk; ++i) {
            xa[i] = u32x4{0u, 0u, 0u, 0u};
            if (xrow_on && s0 + i < s_end) xa[i] = *reinterpret_cast<const u32x4*>(xrow + (size_t)(s0 + i) * 32);
        }
#pragma unroll
        for (int g = 0; g < 2; ++g) {
            if (g < p.n_gates) {
                const uint16_t* wg = static_cast<const uint16_t*>(p.gate[g].w);
#pragma unroll
                for (int nb = 0; nb < NBG; ++nb) {
                    const int e = nb * 16 + row;  // this lane's column of the B operand
                    const uint16_t* wrow = wg + (size_t)(e < E ? e : 0) * H + kq * 8;
                    u32x4 wb[kChunk];
#pragma unroll
                    for (int i = 0; i < kChunk; ++i) {
                        wb[i] = u32x4{0u, 0u, 0u, 0u};
                        if (e < E && s0 + i < s_end)
                            wb[i] = *reinterpret_cast<const u32x4*>(wrow + (size_t)(s0 + i) * 32);
                    }
#pragma unroll
                    for (int i = 0; i < kChunk; ++i)
                        acc[g][nb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, xa[i]),
                                                                             __builtin_bit_cast(bf16x8, wb[i]),
                                                                             acc[g][nb], 0, 0, 0);
                }
            }
        }
    }

    // MFMA result: lane holds column (expert in block) lane & 15 and rows (tokens) 4 * (lane / 16) + r.
    const int t = t0 + wave;  // the token this wavefront selects for
    for (int g = 0; g < p.n_gates; ++g) {
        __syncthreads();  // hist is cleared / the previous gate's partial tiles have been read
#pragma unroll
        for (int nb = 0; nb < NBG; ++nb) part[wave][nb][lane] = g == 0 ? acc[0][nb] : acc[1][nb];
        __syncthreads();
        if (t < T) {
            float z = -INFINITY;
            if (lane < E) {
                const int nb = lane >> 4, src = (wave >> 2) * 16 + (lane & 15), r = wave & 3;
                float sum = 0.f;
#pragma unroll
                for (int w = 0; w < 16; ++w) sum += part[w][nb][src][r];
                z = sum + (p.gate[g].bias != nullptr ? p.gate[g].bias[lane] : 0.f);
            }
            int my_sel;
            float my_w;
            select_topk_lanes(z, lane, E, p.top_k, my_sel, my_w);
            if (lane < p.top_k) {
                p.gate[g].idx[(size_t)t * p.top_k + lane] = my_sel;
                if (p.gate[g].wts != nullptr) p.gate[g].wts[(size_t)t * p.top_k + lane] = my_w;
                atomicAdd(&hist[g][my_sel], 1);
            }
        }
    }
    __syncthreads();
    if (tid < E)
        for (int g = 0; g < p.n_gates; ++g)
            if (p.gate[g].hist != nullptr) p.gate[g].hist[(size_t)blockIdx.x * E + tid] = hist[g][tid];
}

// One workgroup routes a decode-size call against up to two gates and writes indices, weights
// and counts.
template <typename scalar_t>
__global__ __launch_bounds__(kSmallRouteThreads) void route_small_kernel(RouteParams p) {
    __shared__ RouteSmem sm;
    __shared__ float part[kRoutePartFloats];
    const int tid = threadIdx.x;
    const int E = p.n_experts, A = p.tokens * p.top_k;
    int old_count = 0;  // requested before the gate rows so that its latency is hidden
    if (tid < E && p.accumulate && p.counts != nullptr) old_count = p.counts[tid];
    for (int g = 0; g < p.n_gates; ++g) {
        route_tokens_wg<scalar_t>(static_cast<const scalar_t*>(p.x), static_cast<const scalar_t*>(p.gate[g].w),
                                  p.gate[g].bias, p.tokens, p.hidden, E, p.top_k, sm, part);
        if (tid < A) {
            p.gate[g].idx[tid] = sm.idx[tid];
            if (p.gate[g].wts != nullptr) p.gate[g].wts[tid] = sm.w[tid];
        }
        int32_t* counts = g == 0 ? p.counts : p.counts_next;
        if (tid < E && counts != nullptr) {
            int c = 0;
            for (int a = 0; a < A; ++a) c += sm.idx[a] == tid;
            counts[tid] = (g == 0 ? old_count : 0) + c;
        }
        __syncthreads();  // sm is reused by the next gate
    }
}

template <typename scalar_t>
void launch_by_epad(const RouteParams& p, hipStream_t stream) {
    const int E = p.n_experts;
    const int grid = route_blocks(p.tokens);
    if (E <= 8) route_kernel<scalar_t, 8><<<grid, 1024, 0, stream>>>(p);
    else if (E <= 16) route_kernel<scalar_t, 16><<<grid, 1024, 0, stream>>>(p);
    else if (E <= 32) route_kernel<scalar_t, 32><<<grid, 1024, 0, stream>>>(p);
    else route_kernel<scalar_t, 64><<<grid, 1024, 0, stream>>>(p);
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
    const int grid = route_blocks(tokens);
    if (s.dtype == MOE_F32) launch_by_epad<float>(p, stream);
    else if (s.n_experts <= 16) route_mfma_kernel<1><<<grid, 1024, 0, stream>>>(p);
    else if (s.n_experts <= 32) route_mfma_kernel<2><<<grid, 1024, 0, stream>>>(p);
    else route_mfma_kernel<4><<<grid, 1024, 0, stream>>>(p);
    return hipGetLastError();
}

hipError_t launch_route_small(const moe_shape_t& s, int tokens, const void* x, const GateArgs* gates,
                              int n_gates, int32_t* counts, int accumulate, int32_t* counts_next,
                              hipStream_t stream) {
    RouteParams p = make_params(s, tokens, x, gates, n_gates);
    p.counts = counts;
    p.counts_next = counts_next;
    p.accumulate = accumulate;
    if (s.dtype == MOE_F32) route_small_kernel<float><<<1, kSmallRouteThreads, 0, stream>>>(p);
    else route_small_kernel<uint16_t><<<1, kSmallRouteThreads, 0, stream>>>(p);
    return hipGetLastError();
}

}  // namespace moe
