// Device-side parts shared by the prefill kernels that work on 32 x 32 output blocks (gemm_prefill.hip, and the 4-bit
// prefill kernel in quant4.hip): operand types, the swizzled X tile in LDS, the global -> LDS copy and the one asm block
// that multiplies a half-step of a 32-feature block on either tile type (Section 4 / Appendix A of the paper: one
// uniform choice of the dense or the 2:4 instruction per tile).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "epilogue.h"

namespace patch {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

union A8 { u32x4 raw; bf16x8 v; };
union B16 { u32x4 raw[2]; bf16x8 h[2]; bf16x16 v; };

// X tile in LDS: row m holds 8 chunks of 16 bytes (64 columns); chunk p of row m sits at physical chunk
// p ^ ((m >> 1) & 7), so that 16 consecutive rows reading the same logical chunk hit 16 distinct 16-byte
// bank groups.
__device__ __forceinline__ int xs_off(int m, int p) { return m * 128 + ((p ^ ((m >> 1) & 7)) << 4); }

typedef const __attribute__((address_space(1))) void* gptr_t;
typedef __attribute__((address_space(3))) void* lptr_t;

__device__ __forceinline__ void g2l16(const void* g, void* l) {
    // 16 bytes per lane, global -> LDS, no registers: LDS address = (wave-uniform) l + lane * 16
    __builtin_amdgcn_global_load_lds((gptr_t)g, (lptr_t)l, 16, 0, 0);
}

// One 32-column half-step of a 32-feature block against two 32-row blocks, in place:
//   2:4   : c0 += A0 (*) B0, c1 += A0 (*) B1                         (v_smfmac_f32_32x32x32_bf16, positions idx)
//   dense : c0 += A0 B0.lo + A1 B0.hi, c1 += A0 B1.lo + A1 B1.hi     (v_mfma_f32_32x32x16_bf16)
// The wavefront-uniform choice is a scalar branch INSIDE the asm block.  Written with the compiler builtins
// and an if/else, the accumulators of the two arms end up in different registers (the register allocator
// splits the 16-register tuples at the branch), which doubles the accumulator footprint and spills to
// scratch; here the compiler sees straight-line code and every accumulator tile stays in one place.
// It does not see the matrix instructions either: the epilogue pads the matrix-pipe -> memory read hazard.
__device__ __forceinline__ void mma_step(f32x16& c0, f32x16& c1, const bf16x8& a0, const bf16x8& a1, const B16& b0,
                                         const B16& b1, int idx, int sparse) {
    asm volatile(
        "s_cmp_eq_u32 %[sp], 0\n\t"
        "s_cbranch_scc1 .Ldense%=\n\t"
        "v_smfmac_f32_32x32x32_bf16 %[c0], %[a0], %[b0], %[idx]\n\t"
        "v_smfmac_f32_32x32x32_bf16 %[c1], %[a0], %[b1], %[idx]\n\t"
        "s_branch .Ldone%=\n"
        ".Ldense%=:\n\t"
        "v_mfma_f32_32x32x16_bf16 %[c0], %[a0], %[b0lo], %[c0]\n\t"
        "v_mfma_f32_32x32x16_bf16 %[c1], %[a0], %[b1lo], %[c1]\n\t"
        "v_mfma_f32_32x32x16_bf16 %[c0], %[a1], %[b0hi], %[c0]\n\t"
        "v_mfma_f32_32x32x16_bf16 %[c1], %[a1], %[b1hi], %[c1]\n"
        ".Ldone%=:"
        : [c0] "+v"(c0), [c1] "+v"(c1)
        : [a0] "v"(a0), [a1] "v"(a1), [b0] "v"(b0.v), [b1] "v"(b1.v), [b0lo] "v"(b0.h[0]), [b0hi] "v"(b0.h[1]),
          [b1lo] "v"(b1.h[0]), [b1hi] "v"(b1.h[1]), [idx] "v"(idx), [sp] "s"(sparse)
        : "scc");
}

// Output of one 32-row block of a wavefront's 32 features.  acc[i]: feature 8 (i / 4) + 4 q + i % 4, row i32 (lane =
// 32 q + i32).  Stored from there, an instruction would write 32 rows x 32 bytes (quarter cache lines), which a
// compute unit's store path takes at a fraction of its rate (the output stage of prefill_kernel_wreg has the
// measurements).  The block is turned through 4 KB of LDS of the wavefront's own (`stg`) - written as it lies in the
// registers, read back as 8 rows x 128 contiguous bytes per instruction; a wavefront's LDS instructions execute in
// order, so no barrier lies between the two.  16-byte chunk c of row r sits at chunk c ^ (r / 2 % 8): two rows fill
// the 64 banks, and sixteen lanes that write one chunk of sixteen rows, or read two whole rows, touch every bank once.
// `elem` = element offset of (row 0 of the block, first feature of the wavefront) in Y, `rows` = rows of the block
// that exist (the others are not stored).
__device__ __forceinline__ void store_block_rows(uint8_t* stg, const f32x16& acc, int lane, float* Y, int64_t elem, int64_t N,
                                                 int64_t rows, int ybf16) {
    const int i32 = lane & 31, q = lane >> 5;
    const int rr = lane >> 3, ch = lane & 7;   // as a reader: row rr of every eight, chunk ch = features 4 ch .. 4 ch + 3
#pragma unroll
    for (int g = 0; g < 4; ++g) {
        const f32x4 v = {acc[4 * g], acc[4 * g + 1], acc[4 * g + 2], acc[4 * g + 3]};
        *reinterpret_cast<f32x4*>(stg + i32 * 128 + ((((2 * g + q) ^ (i32 >> 1)) & 7) << 4)) = v;
    }
    f32x4 o[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int r = 8 * j + rr;
        o[j] = *reinterpret_cast<const f32x4*>(stg + r * 128 + (((ch ^ (r >> 1)) & 7) << 4));
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int r = 8 * j + rr;
        if (r < rows) store4(Y, elem + (int64_t)r * N + 4 * ch, o[j], ybf16);
    }
}

}  // namespace patch
