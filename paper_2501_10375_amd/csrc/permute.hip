// Expert activation counts and the token -> expert permutation.
//
// The counts are the per-sequence "activity level" of each expert that DAOP's
// sequence-specific allocation consumes (Sec. IV-B, Algorithm 1: tokens
// assigned to each expert).  The permutation groups the (token, j) selections
// by expert so that each expert processes all of its tokens together
// (Algorithm 1's parallel local expert execution).
//
// Everything is integer work and fully deterministic: each workgroup of the
// routing kernel leaves a histogram of its 16 tokens; here every workgroup
// re-derives, from those histograms, the expert totals and the number of
// selections that precede its own tokens, then ranks its own selections in
// token order.  The resulting order inside an expert is by (token, j).
#include "moe_internal.h"

namespace moe {
namespace {

__global__ __launch_bounds__(64) void hist_from_idx_kernel(const int32_t* __restrict__ idx, int tokens, int k,
                                                           int E, int32_t* __restrict__ hist) {
    __shared__ int h[64];
    const int tid = threadIdx.x;
    h[tid] = 0;
    __syncthreads();
    const int a0 = blockIdx.x * kRouteTokensPerBlock * k;
    const int a1 = min(tokens * k, a0 + kRouteTokensPerBlock * k);
    for (int a = a0 + tid; a < a1; a += 64) {
        const int e = min(max(idx[a], 0), E - 1);
        atomicAdd(&h[e], 1);
    }
    __syncthreads();
    if (tid < E) hist[(size_t)blockIdx.x * E + tid] = h[tid];
}

// grid = max(1, n_blocks) workgroups of 256 threads.
__global__ __launch_bounds__(256) void finalize_kernel(const int32_t* __restrict__ hist, int n_blocks, int E,
                                                       int k, int tokens, const int32_t* __restrict__ idx,
                                                       int32_t* __restrict__ counts, int accumulate,
                                                       int32_t* __restrict__ offs,
                                                       int32_t* __restrict__ row_of_slot,
                                                       int32_t* __restrict__ slot_of, int32_t* __restrict__ sync) {
    __shared__ int total[64];
    __shared__ int before[64];
    __shared__ int base[64];
    __shared__ int local_e[kRouteTokensPerBlock * 8];
    const int tid = threadIdx.x;
    const int blk = blockIdx.x;
    if (tid < 64) {
        total[tid] = 0;
        before[tid] = 0;
    }
    __syncthreads();
    // Coalesced sweep over all block histograms (integer sums, so the order is immaterial).  When E
    // divides the workgroup size a thread always meets the same expert and sums in registers.
    const int n_cells = n_blocks * E;
    const int my_first = blk * E;
    if (256 % E == 0) {
        int tot = 0, bef = 0;
#pragma unroll 4
        for (int i = tid; i < n_cells; i += 256) {
            const int v = hist[i];
            tot += v;
            bef += i < my_first ? v : 0;
        }
        if (tot != 0) atomicAdd(&total[tid % E], tot);
        if (bef != 0) atomicAdd(&before[tid % E], bef);
    } else {
        for (int i = tid; i < n_cells; i += 256) {
            const int v = hist[i];
            if (v != 0) {
                atomicAdd(&total[i % E], v);
                if (i < my_first) atomicAdd(&before[i % E], v);
            }
        }
    }
    __syncthreads();
    if (tid == 0) {
        int run = 0;
        for (int e = 0; e < E; ++e) {
            base[e] = run + before[e];
            if (blk == 0 && offs != nullptr) offs[e] = run;
            run += total[e];
        }
        if (blk == 0 && offs != nullptr) offs[E] = run;
    }
    if (blk == 0 && counts != nullptr && tid < E) counts[tid] = (accumulate ? counts[tid] : 0) + total[tid];
    if (blk == 0 && sync != nullptr)
        for (int i = tid; i < kSyncInts; i += 256) sync[i] = 0;
    if (row_of_slot == nullptr) return;
    const int a0 = blk * kRouteTokensPerBlock * k;
    const int n_local = min(tokens * k, a0 + kRouteTokensPerBlock * k) - a0;
    if (tid < n_local) local_e[tid] = min(max(idx[a0 + tid], 0), E - 1);
    __syncthreads();
    if (tid < n_local) {
        const int e = local_e[tid];
        int rank = 0;
        for (int i = 0; i < tid; ++i) rank += (local_e[i] == e);
        const int slot = base[e] + rank;
        slot_of[a0 + tid] = slot;
        row_of_slot[slot] = a0 + tid;
    }
}

// ---- long calls: the fused kernel above sweeps all block histograms in every workgroup, which is
// quadratic in the number of blocks.  Beyond kFusedBlocks blocks one workgroup turns the histograms
// into per-block exclusive prefixes in place (and writes counts / offs), then one workgroup per
// block ranks its selections from its own row.
constexpr int kFusedBlocks = 1024;

// 1024 threads = 16 block ranges x 64 expert lanes.
__global__ __launch_bounds__(1024) void scan_blocks_kernel(int32_t* __restrict__ hist, int n_blocks, int E,
                                                           int32_t* __restrict__ counts, int accumulate,
                                                           int32_t* __restrict__ offs, int32_t* __restrict__ sync) {
    __shared__ int part[16][64];
    __shared__ int total[64];
    const int tid = threadIdx.x, e = tid & 63, g = tid >> 6;
    const int per = (n_blocks + 15) / 16;
    const int b0 = g * per, b1 = min(n_blocks, b0 + per);
    int sum = 0;
    if (e < E)
        for (int b = b0; b < b1; ++b) sum += hist[(size_t)b * E + e];
    part[g][e] = sum;
    __syncthreads();
    if (g == 0) {
        int run = 0;
        for (int i = 0; i < 16; ++i) {
            const int v = part[i][e];
            part[i][e] = run;
            run += v;
        }
        total[e] = run;
    }
    __syncthreads();
    if (e < E) {
        int run = part[g][e];
        for (int b = b0; b < b1; ++b) {
            const int v = hist[(size_t)b * E + e];
            hist[(size_t)b * E + e] = run;
            run += v;
        }
    }
    if (tid == 0 && offs != nullptr) {
        int run = 0;
        for (int i = 0; i < E; ++i) {
            offs[i] = run;
            run += total[i];
        }
        offs[E] = run;
    }
    if (tid < E && counts != nullptr) counts[tid] = (accumulate ? counts[tid] : 0) + total[tid];
    if (sync != nullptr)
        for (int i = tid; i < kSyncInts; i += 1024) sync[i] = 0;
}

// prefix: the histograms after scan_blocks_kernel; offs from the same kernel.
__global__ __launch_bounds__(256) void rank_kernel(const int32_t* __restrict__ prefix, const int32_t* __restrict__ offs,
                                                   int E, int k, int tokens, const int32_t* __restrict__ idx,
                                                   int32_t* __restrict__ row_of_slot, int32_t* __restrict__ slot_of) {
    __shared__ int base[64];
    __shared__ int local_e[kRouteTokensPerBlock * 8];
    const int tid = threadIdx.x, blk = blockIdx.x;
    if (tid < E) base[tid] = offs[tid] + prefix[(size_t)blk * E + tid];
    const int a0 = blk * kRouteTokensPerBlock * k;
    const int n_local = min(tokens * k, a0 + kRouteTokensPerBlock * k) - a0;
    if (tid < n_local) local_e[tid] = min(max(idx[a0 + tid], 0), E - 1);
    __syncthreads();
    if (tid < n_local) {
        const int e = local_e[tid];
        int rank = 0;
        for (int i = 0; i < tid; ++i) rank += (local_e[i] == e);
        const int slot = base[e] + rank;
        slot_of[a0 + tid] = slot;
        row_of_slot[slot] = a0 + tid;
    }
}

}  // namespace

hipError_t launch_hist_from_idx(const moe_shape_t& s, int tokens, const int32_t* idx, int32_t* hist,
                                hipStream_t stream) {
    const int nb = route_blocks(tokens);
    if (nb > 0) hist_from_idx_kernel<<<nb, 64, 0, stream>>>(idx, tokens, s.top_k, s.n_experts, hist);
    return hipGetLastError();
}

hipError_t launch_finalize(const moe_shape_t& s, int tokens, int32_t* hist, const int32_t* idx,
                           int32_t* counts, int accumulate, int32_t* offs, int32_t* row_of_slot,
                           int32_t* slot_of, int32_t* sync, hipStream_t stream) {
    const int nb = route_blocks(tokens);
    if (row_of_slot != nullptr && nb > kFusedBlocks) {
        scan_blocks_kernel<<<1, 1024, 0, stream>>>(hist, nb, s.n_experts, counts, accumulate, offs, sync);
        rank_kernel<<<nb, 256, 0, stream>>>(hist, offs, s.n_experts, s.top_k, tokens, idx, row_of_slot, slot_of);
        return hipGetLastError();
    }
    const int grid = (row_of_slot != nullptr && nb > 0) ? nb : 1;
    finalize_kernel<<<grid, 256, 0, stream>>>(hist, nb, s.n_experts, s.top_k, tokens, idx, counts, accumulate,
                                              offs, row_of_slot, slot_of, sync);
    return hipGetLastError();
}

}  // namespace moe
