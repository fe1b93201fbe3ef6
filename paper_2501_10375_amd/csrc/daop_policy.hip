// Count-driven policy steps of DAOP on the device (see include/daop_policy.h for the contract):
// Eq. 1 similarity of activation patterns, its windowed form over a sequence's decode steps
// (Sec. VI-B), the cache update of Algorithm 1, the calibrated initial cache of Sec. IV-A and
// next-layer prediction with graceful degradation (Sec. IV-C).  The data is
// a few kilobytes of integers; each call is one small kernel so the counts the MoE layer leaves in
// HBM are consumed where they are.
#include "daop_policy.h"
#include "moe_internal.h"
#include "route_device.h"

namespace moe {
namespace {

constexpr int kMaxLayers = 1024;

// ---- Eq. 1 ------------------------------------------------------------------------------------
// One wavefront; lane l takes layers l, l + 64, ...; all sums run in index order in fp64 (the
// operands are integers below 2^53, so products and sums are exact and only sqrt, the product of
// the norms and the division round).
__global__ __launch_bounds__(64) void similarity_kernel(int L, int E, const int32_t* __restrict__ P,
                                                        const int32_t* __restrict__ D, double* __restrict__ out) {
    for (int l = threadIdx.x; l < L; l += 64) {
        double dot = 0.0, pp = 0.0, dd = 0.0;
        for (int e = 0; e < E; ++e) {
            const double p = (double)P[(size_t)l * E + e], d = (double)D[(size_t)l * E + e];
            dot += p * d;
            pp += p * p;
            dd += d * d;
        }
        out[1 + l] = (pp > 0.0 && dd > 0.0) ? dot / (sqrt(pp) * sqrt(dd)) : 0.0;
    }
    __threadfence_block();
    __syncthreads();
    if (threadIdx.x == 0) {
        double total = 0.0;
        for (int l = 0; l < L; ++l) total += out[1 + l];
        out[0] = total / (double)L;
    }
}

// ---- windowed variation (Sec. VI-B) -------------------------------------------------------------
// Workgroup v compares decode window v with window v + 1: thread l takes layers l, l + 256, ... and
// forms the three sums of the cosine directly from the selections (for every expert, how often it
// occurs in either window), in expert order, in fp64: the counts are small integers, so the sums are
// exact and only the roots, their product and the quotient round, as in the similarity kernel.
__global__ __launch_bounds__(256) void window_pairs_kernel(int L, int E, int S, int k, int window,
                                                           const int32_t* __restrict__ idx, double* __restrict__ out) {
    __shared__ double cosine[kMaxLayers];
    const int v = blockIdx.x;
    for (int l = threadIdx.x; l < L; l += 256) {
        const int32_t* a = idx + ((size_t)l * S + (size_t)v * window) * k;        // window v of layer l
        const int32_t* b = a + (size_t)window * k;                                // window v + 1
        double dot = 0.0, aa = 0.0, bb = 0.0;
        for (int e = 0; e < E; ++e) {
            int ca = 0, cb = 0;
            for (int i = 0; i < window * k; ++i) {
                ca += a[i] == e ? 1 : 0;
                cb += b[i] == e ? 1 : 0;
            }
            dot += (double)ca * (double)cb;
            aa += (double)ca * (double)ca;
            bb += (double)cb * (double)cb;
        }
        cosine[l] = (aa > 0.0 && bb > 0.0) ? dot / (sqrt(aa) * sqrt(bb)) : 0.0;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        double total = 0.0;
        for (int l = 0; l < L; ++l) total += cosine[l];
        out[1 + v] = total / (double)L;
    }
}

// out[0] = mean of out[1 .. n_pairs], summed in index order (0 when there is no pair).
__global__ void window_mean_kernel(int n_pairs, double* __restrict__ out) {
    if (threadIdx.x != 0 || blockIdx.x != 0) return;
    double total = 0.0;
    for (int v = 0; v < n_pairs; ++v) total += out[1 + v];
    out[0] = n_pairs > 0 ? total / (double)n_pairs : 0.0;
}

// ---- Algorithm 1 ------------------------------------------------------------------------------
// One wavefront per layer, lane e = expert e.  Ranks come from counting the experts of the same
// side that precede in (activity, index) order.
__global__ __launch_bounds__(64) void plan_swaps_kernel(int E, const int32_t* __restrict__ counts,
                                                        uint8_t* __restrict__ on_gpu, double swap_in_out,
                                                        int32_t* __restrict__ swaps, int32_t* __restrict__ n_swaps) {
    __shared__ int cnt[64];
    __shared__ int res[64];
    __shared__ int hot[32], cold[32];
    const int l = blockIdx.x, e = threadIdx.x;
    const int swap_num = E / 2;
    const bool live = e < E;
    const int c = live ? counts[(size_t)l * E + e] : 0;
    const bool g = live && on_gpu[(size_t)l * E + e] != 0;
    cnt[e] = c;
    res[e] = g ? 1 : 0;
    __syncthreads();
    const int n_gpu = __popcll(__ballot(live && g)), n_cpu = __popcll(__ballot(live && !g));
    const int n_pairs = min(swap_num, min(n_gpu, n_cpu));
    int rank = 0;
    for (int o = 0; o < E; ++o) {
        if (o == e || (res[o] != 0) != g) continue;
        const int co = cnt[o];
        const bool before = g ? (co < c || (co == c && o < e))    // cold list: least active first
                              : (co > c || (co == c && o < e));   // hot list: most active first
        rank += before ? 1 : 0;
    }
    if (live && rank < n_pairs) (g ? cold : hot)[rank] = e;
    __syncthreads();
    bool swap = false;
    int h = -1, cd = -1;
    if (e < n_pairs) {
        h = hot[e];
        cd = cold[e];
        swap = cnt[h] > 0 && (double)cnt[h] >= swap_in_out * (double)cnt[cd];
    }
    const uint64_t m = __ballot(swap);
    if (swap) {
        const int pos = __popcll(m & ((1ull << e) - 1ull));
        if (swaps != nullptr) {
            swaps[((size_t)l * swap_num + pos) * 2] = h;
            swaps[((size_t)l * swap_num + pos) * 2 + 1] = cd;
        }
        on_gpu[(size_t)l * E + h] = 1;
        on_gpu[(size_t)l * E + cd] = 0;
    }
    const int total = __popcll(m);
    if (swaps != nullptr && e >= total && e < swap_num) {
        swaps[((size_t)l * swap_num + e) * 2] = -1;
        swaps[((size_t)l * swap_num + e) * 2 + 1] = -1;
    }
    if (n_swaps != nullptr && e == 0) n_swaps[l] = total;
}

// ---- memory initialisation --------------------------------------------------------------------
// One workgroup.  Step 1: per layer, the slots / L most active experts.  Step 2: the `left` cells
// outside that base that come first in (frequency descending, layer, expert) order; a cell's
// position in that order is the number of other candidate cells that precede it.  Frequencies
// count / row are compared exactly as 128-bit cross products.
__global__ __launch_bounds__(256) void memory_init_kernel(int L, int E, const int32_t* __restrict__ calib, int slots,
                                                          uint8_t* __restrict__ on_gpu) {
    __shared__ long long row[kMaxLayers];
    const int tid = threadIdx.x;
    const int n = L * E;
    const int per_layer = slots / L, left = slots - per_layer * L;
    for (int l = tid; l < L; l += 256) {
        long long s = 0;
        for (int e = 0; e < E; ++e) s += calib[(size_t)l * E + e];
        row[l] = s;
    }
    for (int i = tid; i < n; i += 256) {
        const int l = i / E, e = i - l * E;
        const int c = calib[i];
        int rank = 0;
        for (int o = 0; o < E; ++o) {
            const int co = calib[(size_t)l * E + o];
            rank += (co > c || (co == c && o < e)) ? 1 : 0;
        }
        on_gpu[i] = rank < per_layer ? 1 : 0;
    }
    __syncthreads();  // base masks and row sums are visible to the whole workgroup
    if (left == 0) return;
    for (int i = tid; i < n; i += 256) {
        if (on_gpu[i] == 1) continue;
        const int l = i / E;
        // frequency as a fraction; a layer without tokens has frequency 0
        const unsigned __int128 n1 = row[l] > 0 ? (unsigned __int128)calib[i] : 0;
        const unsigned __int128 d1 = row[l] > 0 ? (unsigned __int128)row[l] : 1;
        int rank = 0;
        for (int j = 0; j < n && rank < left; ++j) {
            if (j == i || on_gpu[j] == 1) continue;
            const int lj = j / E;
            const unsigned __int128 n2 = row[lj] > 0 ? (unsigned __int128)calib[j] : 0;
            const unsigned __int128 d2 = row[lj] > 0 ? (unsigned __int128)row[lj] : 1;
            const unsigned __int128 a = n2 * d1, b = n1 * d2;  // freq_j vs freq_i
            rank += (a > b || (a == b && j < i)) ? 1 : 0;
        }
        if (rank < left) on_gpu[i] = 2;  // marked, not yet counted as resident by the other threads
    }
    __syncthreads();
    for (int i = tid; i < n; i += 256)
        if (on_gpu[i] == 2) on_gpu[i] = 1;
}

// ---- prediction with graceful degradation --------------------------------------------------------
// One workgroup per 16 tokens, the decode-size routing code with the placement mask.
template <typename scalar_t>
__global__ __launch_bounds__(kSmallRouteThreads) void predict_degraded_kernel(const scalar_t* __restrict__ x,
                                                                               const scalar_t* __restrict__ wg,
                                                                               const float* __restrict__ bias,
                                                                               const uint8_t* __restrict__ on_gpu,
                                                                               int T, int H, int E, int k,
                                                                               int32_t* __restrict__ idx,
                                                                               float* __restrict__ w) {
    __shared__ RouteSmem sm;
    __shared__ float part[kRoutePartFloats];
    const int t0 = blockIdx.x * kSmallRouteMaxTokens;
    const int n = min(kSmallRouteMaxTokens, T - t0);
    route_tokens_wg<scalar_t>(x + (size_t)t0 * H, wg, bias, n, H, E, k, sm, part, on_gpu);
    const int tid = threadIdx.x;
    if (tid < n * k) {
        idx[(size_t)t0 * k + tid] = sm.idx[tid];
        if (w != nullptr) w[(size_t)t0 * k + tid] = sm.w[tid];
    }
}

bool misaligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }

int check_dims(int32_t n_layers, int32_t n_experts) {
    if (n_layers < 1 || n_layers > kMaxLayers || n_experts < 1 || n_experts > 64) return MOE_ERR_SHAPE;
    return MOE_OK;
}

int done() { return hipGetLastError() == hipSuccess ? MOE_OK : MOE_ERR_DEVICE; }

}  // namespace
}  // namespace moe

using namespace moe;

extern "C" {

int daop_similarity(int32_t n_layers, int32_t n_experts, const int32_t* counts_p, const int32_t* counts_d,
                    double* out, void* hip_stream) {
    if (int rc = check_dims(n_layers, n_experts)) return rc;
    if (counts_p == nullptr || counts_d == nullptr || out == nullptr) return MOE_ERR_NULL;
    if (misaligned16(counts_p) || misaligned16(counts_d) || misaligned16(out)) return MOE_ERR_ALIGN;
    similarity_kernel<<<1, 64, 0, static_cast<hipStream_t>(hip_stream)>>>(n_layers, n_experts, counts_p, counts_d, out);
    return done();
}

int daop_window_variation(int32_t n_layers, int32_t n_experts, int32_t steps, int32_t top_k, int32_t window,
                          const int32_t* idx, double* out, void* hip_stream) {
    if (int rc = check_dims(n_layers, n_experts)) return rc;
    if (steps < 0 || steps > (1 << 20) || top_k < 1 || top_k > 8 || top_k > n_experts) return MOE_ERR_SHAPE;
    if (window < 1 || window > 4096) return MOE_ERR_SHAPE;
    if (out == nullptr || (steps > 0 && idx == nullptr)) return MOE_ERR_NULL;
    if (misaligned16(out) || (idx != nullptr && misaligned16(idx))) return MOE_ERR_ALIGN;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const int n_pairs = steps / window - 1;
    if (n_pairs > 0)
        window_pairs_kernel<<<n_pairs, 256, 0, stream>>>(n_layers, n_experts, steps, top_k, window, idx, out);
    window_mean_kernel<<<1, 64, 0, stream>>>(n_pairs > 0 ? n_pairs : 0, out);
    return done();
}

int daop_plan_swaps(int32_t n_layers, int32_t n_experts, const int32_t* counts, uint8_t* on_gpu, double swap_in_out,
                    int32_t* swaps, int32_t* n_swaps, void* hip_stream) {
    if (int rc = check_dims(n_layers, n_experts)) return rc;
    if (!(swap_in_out >= 0.0)) return MOE_ERR_SHAPE;
    if (counts == nullptr || on_gpu == nullptr) return MOE_ERR_NULL;
    if (misaligned16(counts) || misaligned16(on_gpu) || (swaps != nullptr && misaligned16(swaps)) ||
        (n_swaps != nullptr && misaligned16(n_swaps)))
        return MOE_ERR_ALIGN;
    plan_swaps_kernel<<<n_layers, 64, 0, static_cast<hipStream_t>(hip_stream)>>>(n_experts, counts, on_gpu, swap_in_out,
                                                                                swaps, n_swaps);
    return done();
}

int daop_memory_init(int32_t n_layers, int32_t n_experts, const int32_t* calib_counts, int32_t slots, uint8_t* on_gpu,
                     void* hip_stream) {
    if (int rc = check_dims(n_layers, n_experts)) return rc;
    if (calib_counts == nullptr || on_gpu == nullptr) return MOE_ERR_NULL;
    if (misaligned16(calib_counts) || misaligned16(on_gpu)) return MOE_ERR_ALIGN;
    const int total = n_layers * n_experts;
    const int clamped = slots < 0 ? 0 : (slots > total ? total : slots);
    memory_init_kernel<<<1, 256, 0, static_cast<hipStream_t>(hip_stream)>>>(n_layers, n_experts, calib_counts, clamped,
                                                                           on_gpu);
    return done();
}

int daop_predict_degraded(const moe_shape_t* shape, int32_t tokens, const void* x, const void* w_gate_next,
                          const float* gate_bias_next, const uint8_t* on_gpu, int32_t* pred_idx, float* pred_w,
                          void* hip_stream) {
    if (shape == nullptr) return MOE_ERR_NULL;
    if (shape->dtype != MOE_F32 && shape->dtype != MOE_BF16) return MOE_ERR_DTYPE;
    if (shape->reserved != 0 || shape->hidden <= 0 || shape->hidden % 64 != 0) return MOE_ERR_SHAPE;
    if (shape->n_experts < 1 || shape->n_experts > 64) return MOE_ERR_SHAPE;
    if (shape->top_k < 1 || shape->top_k > 8 || shape->top_k > shape->n_experts) return MOE_ERR_SHAPE;
    if (tokens < 0 || tokens > (1 << 20)) return MOE_ERR_SHAPE;
    if (w_gate_next == nullptr || on_gpu == nullptr) return MOE_ERR_NULL;
    if (tokens > 0 && (x == nullptr || pred_idx == nullptr)) return MOE_ERR_NULL;
    const void* const ptrs[] = {x, w_gate_next, gate_bias_next, on_gpu, pred_idx, pred_w};
    for (const void* p : ptrs)
        if (p != nullptr && misaligned16(p)) return MOE_ERR_ALIGN;
    if (tokens == 0) return MOE_OK;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const int grid = (tokens + kSmallRouteMaxTokens - 1) / kSmallRouteMaxTokens;
    if (shape->dtype == MOE_F32)
        predict_degraded_kernel<float><<<grid, kSmallRouteThreads, 0, stream>>>(
            static_cast<const float*>(x), static_cast<const float*>(w_gate_next), gate_bias_next, on_gpu, tokens,
            shape->hidden, shape->n_experts, shape->top_k, pred_idx, pred_w);
    else
        predict_degraded_kernel<uint16_t><<<grid, kSmallRouteThreads, 0, stream>>>(
            static_cast<const uint16_t*>(x), static_cast<const uint16_t*>(w_gate_next), gate_bias_next, on_gpu, tokens,
            shape->hidden, shape->n_experts, shape->top_k, pred_idx, pred_w);
    return done();
}

}  // extern "C"
