// Grouped SwiGLU expert FFN and weighted combine for fp32 storage
// (expert execution of DAOP Sec. II-A / Algorithm 1's local expert execution,
// with the Mixtral expert  y = W2 ( silu(W1 x) * (W3 x) )  the paper builds on).
//
// This is the exact-arithmetic configuration: fp32 in, fp32 FMA accumulation,
// nothing narrowed.  Plain LDS-tiled kernels, 64 x 64 output tile, 4 x 4
// outputs per thread; rows of an M-tile are gathered through the permutation
// and never span two experts.
#include "moe_internal.h"

namespace moe {
namespace {

constexpr int BM = kTileTokensF32;  // tokens (slots) per tile
constexpr int BN = 64;              // output features per tile
constexpr int BK = 16;

// Maps a linear M-tile index to (expert, first slot, valid rows).  Uniform per workgroup.
__device__ inline bool find_mtile(const int32_t* __restrict__ offs, int E, int mt, int& e, int& slot0, int& rows) {
    int acc = 0;
    for (int i = 0; i < E; ++i) {
        const int c = offs[i + 1] - offs[i];
        const int nt = (c + BM - 1) / BM;
        if (mt < acc + nt) {
            const int local = (mt - acc) * BM;
            e = i;
            slot0 = offs[i] + local;
            rows = min(BM, c - local);
            return true;
        }
        acc += nt;
    }
    return false;
}

// Loads a [64 rows x 16 k] tile, one float4 per thread, and stores it k-major in LDS.
__device__ inline void stage_tile(float (*dst)[BM + 4], const float* __restrict__ rowptr, int kq, int r) {
    const float4 v = *reinterpret_cast<const float4*>(rowptr + kq * 4);
    dst[kq * 4 + 0][r] = v.x;
    dst[kq * 4 + 1][r] = v.y;
    dst[kq * 4 + 2][r] = v.z;
    dst[kq * 4 + 3][r] = v.w;
}

// act[slot, f] = silu(x_row . w1[e,f,:]) * (x_row . w3[e,f,:])
__global__ __launch_bounds__(256) void gemm1_swiglu_f32(const float* __restrict__ x, const float* __restrict__ w1,
                                                        const float* __restrict__ w3,
                                                        const int32_t* __restrict__ offs,
                                                        const int32_t* __restrict__ row_of_slot, int E, int k, int H,
                                                        int F, float* __restrict__ act,
                                                        const float* __restrict__ x_stale,
                                                        const uint8_t* __restrict__ stale) {
    __shared__ float As[BK][BM + 4];
    __shared__ float B1s[BK][BN + 4];
    __shared__ float B3s[BK][BN + 4];
    int e, slot0, rows;
    if (!find_mtile(offs, E, blockIdx.x, e, slot0, rows)) return;
    const int f0 = blockIdx.y * BN;
    const int tid = threadIdx.x;
    const int lr = tid >> 2, kq = tid & 3;  // staging: row 0..63, k quarter 0..3
    const int srow = min(lr, rows - 1);     // rows past the end re-read a valid row; never stored
    const int assignment = row_of_slot[slot0 + srow];  // t * k + j
    const int token = assignment / k;
    // a pre-calculated selection reads the earlier hidden state of its token
    const float* xa = ((stale != nullptr && stale[assignment] != 0) ? x_stale : x) + (size_t)token * H;
    const float* b1 = w1 + ((size_t)e * F + f0 + lr) * H;
    const float* b3 = w3 + ((size_t)e * F + f0 + lr) * H;
    const int tm = (tid >> 4) * 4, tn = (tid & 15) * 4;
    float g[4][4] = {}, u[4][4] = {};
    for (int k0 = 0; k0 < H; k0 += BK) {
        stage_tile(As, xa + k0, kq, lr);
        stage_tile(B1s, b1 + k0, kq, lr);
        stage_tile(B3s, b3 + k0, kq, lr);
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < BK; ++kk) {
            float a[4], p[4], q[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                a[i] = As[kk][tm + i];
                p[i] = B1s[kk][tn + i];
                q[i] = B3s[kk][tn + i];
            }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    g[i][j] = fmaf(a[i], p[j], g[i][j]);
                    u[i][j] = fmaf(a[i], q[j], u[i][j]);
                }
        }
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        if (tm + i < rows) {
            float4 o;
            float* op = &o.x;
#pragma unroll
            for (int j = 0; j < 4; ++j) op[j] = g[i][j] / (1.f + expf(-g[i][j])) * u[i][j];
            *reinterpret_cast<float4*>(act + (size_t)(slot0 + tm + i) * F + f0 + tn) = o;
        }
    }
}

// out[slot, h] = act[slot, :] . w2[e, h, :]
__global__ __launch_bounds__(256) void gemm2_f32(const float* __restrict__ act, const float* __restrict__ w2,
                                                 const int32_t* __restrict__ offs, int E, int H, int F,
                                                 float* __restrict__ out) {
    __shared__ float As[BK][BM + 4];
    __shared__ float Bs[BK][BN + 4];
    int e, slot0, rows;
    if (!find_mtile(offs, E, blockIdx.x, e, slot0, rows)) return;
    const int h0 = blockIdx.y * BN;
    const int tid = threadIdx.x;
    const int lr = tid >> 2, kq = tid & 3;
    const int srow = min(lr, rows - 1);
    const float* aa = act + (size_t)(slot0 + srow) * F;
    const float* bb = w2 + ((size_t)e * H + h0 + lr) * F;
    const int tm = (tid >> 4) * 4, tn = (tid & 15) * 4;
    float c[4][4] = {};
    for (int k0 = 0; k0 < F; k0 += BK) {
        stage_tile(As, aa + k0, kq, lr);
        stage_tile(Bs, bb + k0, kq, lr);
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < BK; ++kk) {
            float a[4], p[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                a[i] = As[kk][tm + i];
                p[i] = Bs[kk][tn + i];
            }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) c[i][j] = fmaf(a[i], p[j], c[i][j]);
        }
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        if (tm + i < rows)
            *reinterpret_cast<float4*>(out + (size_t)(slot0 + tm + i) * H + h0 + tn) =
                make_float4(c[i][0], c[i][1], c[i][2], c[i][3]);
    }
}

// y[t, :] = sum_j w[t, j] * out[slot_of[t, j], :], j ascending, fp32.
__global__ __launch_bounds__(256) void combine_f32(const float* __restrict__ out, const float* __restrict__ w,
                                                   const int32_t* __restrict__ slot_of, int k, int H,
                                                   float* __restrict__ y) {
    const int t = blockIdx.x;
    for (int h = threadIdx.x * 4; h < H; h += 256 * 4) {
        float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
        for (int j = 0; j < k; ++j) {
            const float wj = w[(size_t)t * k + j];
            const float4 v = *reinterpret_cast<const float4*>(out + (size_t)slot_of[(size_t)t * k + j] * H + h);
            s.x = fmaf(wj, v.x, s.x);
            s.y = fmaf(wj, v.y, s.y);
            s.z = fmaf(wj, v.z, s.z);
            s.w = fmaf(wj, v.w, s.w);
        }
        *reinterpret_cast<float4*>(y + (size_t)t * H + h) = s;
    }
}

}  // namespace

hipError_t launch_ffn_f32(const moe_shape_t& s, int tokens, const float* x, const float* topk_w, const float* w1,
                          const float* w3, const float* w2, float* y, const int32_t* offs,
                          const int32_t* row_of_slot, const int32_t* slot_of, float* act, float* out,
                          const StaleInput& alt, hipStream_t stream) {
    const int A = tokens * s.top_k;
    const int max_mtiles = (A + BM - 1) / BM + s.n_experts;
    gemm1_swiglu_f32<<<dim3(max_mtiles, s.ffn / BN), 256, 0, stream>>>(x, w1, w3, offs, row_of_slot, s.n_experts,
                                                                       s.top_k, s.hidden, s.ffn, act,
                                                                       static_cast<const float*>(alt.x_stale), alt.stale);
    stage_mark(stream, kStageGemm1);
    gemm2_f32<<<dim3(max_mtiles, s.hidden / BN), 256, 0, stream>>>(act, w2, offs, s.n_experts, s.hidden, s.ffn,
                                                                  out);
    stage_mark(stream, kStageGemm2);
    combine_f32<<<tokens, 256, 0, stream>>>(out, topk_w, slot_of, s.top_k, s.hidden, y);
    stage_mark(stream, kStageCombine);
    return hipGetLastError();
}

}  // namespace moe
