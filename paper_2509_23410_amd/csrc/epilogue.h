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
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (u >> 16) | 0x40u;
    return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}

// Store v at element offset `elem` of Y: fp32 (16 bytes) or bf16 (8 bytes).  `elem` is a multiple of 4.
__device__ __forceinline__ void store4(float* Y, int64_t elem, ep_f32x4 v, int ybf16) {
    if (ybf16) {
        uint2 p;
        p.x = bf16_rne_bits(v[0]) | (bf16_rne_bits(v[1]) << 16);
        p.y = bf16_rne_bits(v[2]) | (bf16_rne_bits(v[3]) << 16);
        *reinterpret_cast<uint2*>(reinterpret_cast<uint16_t*>(Y) + elem) = p;
    } else {
        *reinterpret_cast<ep_f32x4*>(Y + elem) = v;
    }
}

}  // namespace patch
