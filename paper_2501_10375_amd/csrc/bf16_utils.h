// bf16 helpers shared by the bf16 kernels (device code).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace moe {

// Two fp32 values -> two bf16 in one dword (a in the low half), round-to-nearest-even in hardware
// (v_cvt_pk_bf16_f32).
__device__ inline uint32_t pack_bf16x2(float a, float b) {
    typedef __attribute__((ext_vector_type(2))) float f32x2_t;
    typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
    const f32x2_t v = {a, b};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}

__device__ inline uint16_t to_bf16(float a) { return (uint16_t)(pack_bf16x2(a, 0.f) & 0xffffu); }

// silu(g) * u in fp32 with the hardware exp2 / reciprocal (about 1 ulp each; the result is rounded
// to bf16 afterwards).
__device__ inline float swiglu(float g, float u) { return g * __builtin_amdgcn_rcpf(1.f + __expf(-g)) * u; }

}  // namespace moe
