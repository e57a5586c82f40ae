// Output stage shared by the product kernels: four consecutive features of one row, either as fp32 (the accumulator
// itself) or rounded to bf16 (round to nearest, ties to even, on the bit pattern: no floating-point instruction).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace patch {

typedef float ep_f32x4 __attribute__((ext_vector_type(4)));

// bf16 bit pattern of an fp32 value, round to nearest even; a NaN stays a (quiet) NaN
__device__ __forceinline__ uint32_t bf16_rne_bits(float f) {
    const uint32_t u = __float_as_uint(f);
    const uint32_t nan = (u >> 16) | 0x40u, rne = (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;   // both computed: a select, no branch
    return (u & 0x7FFFFFFFu) > 0x7F800000u ? nan : rne;
}

typedef unsigned int ep_u32x2 __attribute__((ext_vector_type(2)));
#define PATCH_EP_GLOBAL __attribute__((address_space(1)))

// Store v at element offset `elem` of Y: fp32 (16 bytes) or bf16 (8 bytes).  `elem` is a multiple of 4.
// Y is device memory by contract; the store says so (address space 1).  The kernels pick Y with scalar selects from a
// by-value struct, after which the compiler no longer knows the address space and would emit flat stores.
__device__ __forceinline__ void store4(float* Y, int64_t elem, ep_f32x4 v, int ybf16) {
    if (ybf16) {
        ep_u32x2 p;
        p[0] = bf16_rne_bits(v[0]) | (bf16_rne_bits(v[1]) << 16);
        p[1] = bf16_rne_bits(v[2]) | (bf16_rne_bits(v[3]) << 16);
        PATCH_EP_GLOBAL uint16_t* Yh = reinterpret_cast<PATCH_EP_GLOBAL uint16_t*>(reinterpret_cast<uintptr_t>(Y));
        *reinterpret_cast<PATCH_EP_GLOBAL ep_u32x2*>(Yh + elem) = p;
    } else {
        PATCH_EP_GLOBAL float* Yg = reinterpret_cast<PATCH_EP_GLOBAL float*>(reinterpret_cast<uintptr_t>(Y));
        *reinterpret_cast<PATCH_EP_GLOBAL ep_f32x4*>(Yg + elem) = v;
    }
}

}  // namespace patch
