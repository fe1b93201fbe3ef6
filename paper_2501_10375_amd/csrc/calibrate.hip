// Measurement aid: the rate at which this chip issues bf16 MFMAs when nothing else happens.
//
// The published peak (2.5 PFLOP/s dense bf16) assumes 2.4 GHz.  Under the board's power limit the
// clock depends on what the matrix cores multiply: operands that never change draw little power and
// the loop below holds the full clock, operands with random mantissas and signs (what real weights
// and activations look like) pull it down.  Timing the same register-only loop both ways gives the
// matrix-core rate a GEMM could reach on this board if every operand were already in registers,
// which is the yardstick the measured GEMM rates are read against.  No memory is touched in the loop.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "moe_measure.h"
#include "moe_internal.h"

namespace moe {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

constexpr int kProbeThreads = 512;       // 8 wavefronts per workgroup, one workgroup per CU: two per SIMD
constexpr int kProbeAccumulators = 8;    // independent 32 x 32 accumulators per wavefront
constexpr double kFlopPerMfma = 2.0 * 32 * 32 * 16;

__device__ inline uint32_t mix(uint32_t v) {
    v ^= v >> 16; v *= 0x7feb352du; v ^= v >> 15; v *= 0x846ca68bu; v ^= v >> 16;
    return v;
}
// Two bf16 values of magnitude in [0.5, 2) with random sign and mantissa.
__device__ inline uint32_t random_bf16_pair(uint32_t seed) {
    const uint32_t h = mix(seed);
    const uint32_t lo = 0x3f00u | (h & 0x80ffu) | ((h >> 8) & 0x0080u);
    const uint32_t hi = 0x3f00u | ((h >> 16) & 0x80ffu) | ((h >> 24) & 0x0080u);
    return lo | (hi << 16);
}

// clocks[0] = shader cycles, clocks[1] = ticks of the constant 100 MHz counter that the loop of
// workgroup 0 took (their ratio is the shader clock the loop ran at).
template <bool RANDOM>
__global__ __launch_bounds__(kProbeThreads) void mfma_rate_kernel(int iters, unsigned long long* clocks) {
    f32x16 acc[kProbeAccumulators];
    for (int a = 0; a < kProbeAccumulators; ++a)
        for (int r = 0; r < 16; ++r) acc[a][r] = 0.f;
    bf16x8 x[4], y[4];
    for (int n = 0; n < 4; ++n) {
        u32x4 xv, yv;
        for (int i = 0; i < 4; ++i) {
            const uint32_t seed = (blockIdx.x * (uint32_t)kProbeThreads + threadIdx.x) * 64u + n * 8u + i;
            xv[i] = RANDOM ? random_bf16_pair(seed) : 0x3f803f80u;       // 1.0, 1.0
            yv[i] = RANDOM ? random_bf16_pair(seed + 4u) : 0x3f803f80u;
        }
        x[n] = __builtin_bit_cast(bf16x8, xv);
        y[n] = __builtin_bit_cast(bf16x8, yv);
    }
    const unsigned long long c0 = __builtin_readcyclecounter(), w0 = wall_clock64();
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int a = 0; a < kProbeAccumulators; ++a)
            acc[a] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(x[a % 4], y[(a / 2) % 4], acc[a], 0, 0, 0);
        if ((it & 63) == 63) {  // keep the sums finite: scale them down now and then (both flavours alike)
#pragma unroll
            for (int a = 0; a < kProbeAccumulators; ++a)
                for (int r = 0; r < 16; ++r) acc[a][r] *= 0.001f;
        }
    }
    float s = 0.f;
    for (int a = 0; a < kProbeAccumulators; ++a)
        for (int r = 0; r < 16; ++r) s += acc[a][r];
    asm volatile("" ::"v"(s));  // the sums exist before the clocks are read again
    const unsigned long long c1 = __builtin_readcyclecounter(), w1 = wall_clock64();
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        clocks[0] = c1 - c0;
        clocks[1] = w1 - w0;
    }
    asm volatile("" ::"v"(s));  // the sums are the loop's only result: keep them (and with them the loop) alive
}

// Plain read stream: every workgroup reads its contiguous share of the buffer with 16-byte loads,
// consecutive lanes on consecutive addresses, eight loads (8 KB per workgroup) in flight per
// wavefront, and keeps nothing.  What this reaches is what a kernel that only has to pull bytes out
// of HBM gets on this device, the yardstick for the decode-size calls of the layer.
constexpr int kStreamUnroll = 8;
__global__ __launch_bounds__(kProbeThreads) void read_stream_kernel(const u32x4* __restrict__ data, size_t n16) {
    const size_t per_wg = n16 / gridDim.x;  // 16-byte pieces of this workgroup (the host passes a multiple)
    const u32x4* mine = data + (size_t)blockIdx.x * per_wg;
    u32x4 acc = {0u, 0u, 0u, 0u};
    for (size_t i = threadIdx.x; i < per_wg; i += (size_t)kProbeThreads * kStreamUnroll) {
        u32x4 v[kStreamUnroll];
#pragma unroll
        for (int u = 0; u < kStreamUnroll; ++u) v[u] = mine[min(i + (size_t)u * kProbeThreads, per_wg - 1)];
#pragma unroll
        for (int u = 0; u < kStreamUnroll; ++u) acc ^= v[u];
    }
    asm volatile("" ::"v"(acc));  // the loads are the point
}

}  // namespace
}  // namespace moe

extern "C" int moe_calibrate_read_stream(const void* device_buffer, size_t bytes, float* milliseconds,
                                         double* bytes_read, void* hip_stream) {
    using namespace moe;
    if (device_buffer == nullptr || milliseconds == nullptr || bytes_read == nullptr) return MOE_ERR_NULL;
    if ((reinterpret_cast<uintptr_t>(device_buffer) & 15u) != 0) return MOE_ERR_ALIGN;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const int grid = compute_units();
    const size_t unit = (size_t)grid * kProbeThreads * kStreamUnroll * 16;  // one round of every workgroup
    const size_t n16 = bytes / unit * (unit / 16);
    if (n16 == 0) return MOE_ERR_SHAPE;
    hipEvent_t e0, e1;
    if (hipEventCreate(&e0) != hipSuccess) return MOE_ERR_DEVICE;
    if (hipEventCreate(&e1) != hipSuccess) {
        (void)hipEventDestroy(e0);
        return MOE_ERR_DEVICE;
    }
    const u32x4* data = static_cast<const u32x4*>(device_buffer);
    read_stream_kernel<<<grid, kProbeThreads, 0, stream>>>(data, n16);
    hipError_t e = hipEventRecord(e0, stream);
    read_stream_kernel<<<grid, kProbeThreads, 0, stream>>>(data, n16);
    if (e == hipSuccess) e = hipEventRecord(e1, stream);
    if (e == hipSuccess) e = hipEventSynchronize(e1);
    float ms = 0.f;
    if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
    if (e == hipSuccess) e = hipGetLastError();
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (e != hipSuccess) return MOE_ERR_DEVICE;
    *milliseconds = ms;
    *bytes_read = (double)n16 * 16.0;
    return MOE_OK;
}

extern "C" int moe_calibrate_mfma(int32_t random_operands, int32_t iterations, float* milliseconds,
                                  double* flop, float* gigahertz, void* hip_stream) {
    using namespace moe;
    if (iterations < 64 || iterations > (1 << 22) || milliseconds == nullptr || flop == nullptr) return MOE_ERR_SHAPE;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const int grid = compute_units();
    unsigned long long* clocks = nullptr;  // a calibration call may allocate: 16 bytes, freed before it returns
    if (hipMalloc(&clocks, 2 * sizeof(unsigned long long)) != hipSuccess) return MOE_ERR_DEVICE;
    hipEvent_t e0, e1;
    if (hipEventCreate(&e0) != hipSuccess) {
        (void)hipFree(clocks);
        return MOE_ERR_DEVICE;
    }
    if (hipEventCreate(&e1) != hipSuccess) {
        (void)hipEventDestroy(e0);
        (void)hipFree(clocks);
        return MOE_ERR_DEVICE;
    }
    auto launch = [&]() {
        if (random_operands) mfma_rate_kernel<true><<<grid, kProbeThreads, 0, stream>>>(iterations, clocks);
        else mfma_rate_kernel<false><<<grid, kProbeThreads, 0, stream>>>(iterations, clocks);
    };
    launch();  // the first launch also brings the clocks to where the second one finds them
    hipError_t e = hipEventRecord(e0, stream);
    launch();
    if (e == hipSuccess) e = hipEventRecord(e1, stream);
    if (e == hipSuccess) e = hipEventSynchronize(e1);
    float ms = 0.f;
    if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
    if (e == hipSuccess) e = hipGetLastError();
    unsigned long long host_clocks[2] = {0, 0};
    if (e == hipSuccess) e = hipMemcpy(host_clocks, clocks, sizeof(host_clocks), hipMemcpyDeviceToHost);
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    (void)hipFree(clocks);
    if (e != hipSuccess) return MOE_ERR_DEVICE;
    if (gigahertz != nullptr) *gigahertz = host_clocks[1] > 0 ? (float)((double)host_clocks[0] / (double)host_clocks[1] * 0.1) : 0.f;
    *milliseconds = ms;
    *flop = (double)grid * (kProbeThreads / 64) * (double)iterations * kProbeAccumulators * kFlopPerMfma;
    return MOE_OK;
}
