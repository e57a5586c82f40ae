// 4-bit weight-only storage of the hybrid dense / 2:4 weight and its decode-shaped product (Section 5.2 of the paper,
// "Quantization": the pruned model is composed with 4-bit weight-only quantization; the table there counts 4 bits per
// element of a dense tile and 2 x 4 + 4 bits per group of four of a 2:4 tile).  The paper names no quantizer; this
// library's: symmetric, 15 levels, one scale per row of a tile,
//     s = bf16(max|w| / 7),   q = clamp(rint(w / s), -7, 7)   (both in fp32, correctly rounded division, ties to even),
// and the weight the product uses is bf16(q s): the exact product rounded once.  A pruned weight keeps code 0, so a
// 2:4 tile stays 2:4; its kept positions are those of the unquantized matrix.
//
// Layout (tiles row-major, each on a 256-byte granule, table entry = offset / 256 << 1 | is 2:4, as for bf16):
//   dense tile : code fragments in (strip, K-step) order, 512 B each: lane l holds two dwords, the 8 codes of
//                W[row0 + l % 16][k0 + 8 (l / 16) + e] and those 32 columns further (the two operands of
//                v_mfma_f32_16x16x32_bf16), code e in bits [4e+3 : 4e], two's complement
//   2:4 tile   : code fragments of 256 B: lane l holds the 8 kept codes of W[row0 + l % 16][k0 + 16 (l / 16) .. + 15]
//                (the operand of v_smfmac_f32_16x16x64_bf16); then the positions, uint16 [strip][lane][K-step] as in the
//                bf16 layout
//   scales     : an array of their own, bf16 [strip of 16 rows][tile column][row in strip]: the scales a strip needs
//                along K are contiguous and no cache line is shared between strips (strips of one tile run in
//                workgroups on different XCDs; inside the tile every line of scales was fetched by four L2s)
// The product kernel dequantizes in registers (8 codes -> 8 bf16 with integer rounding) and then runs the same matrix
// instructions as the bf16 decode kernel: a workgroup owns one to three strips of 16 features, its wavefronts split K,
// partial sums meet in LDS in wavefront order (bit-reproducible); several weights sharing X run as one launch
// (patch_gemm4_many).  That kernel takes up to 64 rows of X (one, two or four blocks of 16) per pass over the weight;
// for more rows mask tile 128 has a prefill-shaped kernel that keeps the weight in 4 bits (prefill4_kernel below,
// patch_gemm4_ex), and any weight can be dequantized once and packed as bf16 (patch_pack_from4).
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <string.h>

#include <new>
#include <vector>

#include "../../include/patch.h"
#include "epilogue.h"
#include "kernels.h"
#include "layout.h"
#include "prefill_parts.h"
#include "saved.h"

namespace patch {

typedef __bf16 q4_bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 q4_bf16x16 __attribute__((ext_vector_type(16)));
typedef float q4_f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int q4_u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int q4_u32x2 __attribute__((ext_vector_type(2)));
union Q4A { q4_u32x4 raw; q4_bf16x8 v; };
union Q4B { q4_u32x4 raw[2]; q4_bf16x8 h[2]; q4_bf16x16 v; };

__host__ __device__ constexpr int q4_dense_codes(int t) { return t * t / 2; }
__host__ __device__ constexpr int q4_sparse_codes(int t) { return t * t / 4; }
__host__ __device__ constexpr int q4_sparse_pos(int t) { return t * t / 8; }
__host__ __device__ constexpr int q4_round_up(int b) { return (b + kGranule - 1) / kGranule * kGranule; }
__host__ __device__ constexpr int q4_dense_tile(int t) { return q4_round_up(q4_dense_codes(t)); }
__host__ __device__ constexpr int q4_sparse_tile(int t) { return q4_round_up(q4_sparse_codes(t) + q4_sparse_pos(t)); }
// scale of row r (0..15) of strip `strip` (over the whole matrix) for tile column tk
__host__ __device__ constexpr int64_t q4_scale_index(int64_t strip, int Tk, int tk, int r) { return (strip * Tk + tk) * 16 + r; }

__device__ __forceinline__ float q4_bf16_to_float(uint32_t bits) { return __uint_as_float(bits << 16); }

// 4-bit code of w for scale s (s > 0), as a nibble
__device__ __forceinline__ uint32_t q4_code(uint16_t w_bits, float s) {
    float r = rintf(__fdiv_rn(q4_bf16_to_float(w_bits), s));
    r = fminf(fmaxf(r, -7.0f), 7.0f);
    return (uint32_t)((int)r) & 0xFu;
}

// 8 codes of a dword -> 8 bf16 values bf16(q s), element e from bits [4e+3 : 4e].  v_cvt_off_f32_i4 turns the low nibble
// of a byte (selected by SDWA; the odd nibbles come from the dword shifted by 4) into the float q / 16 in one
// instruction - a bit-field extract and an integer conversion otherwise; q / 16 times 16 s is q s, exact in fp32
// (4 x 8 bits), and the conversion of a float pair to bf16 rounds to nearest, ties to even (v_cvt_pk_bf16_f32).
typedef __bf16 q4_bf16x2 __attribute__((ext_vector_type(2)));
typedef float q4_f32x2 __attribute__((ext_vector_type(2)));
#define PATCH_Q4_NIBBLE(dst, src, byte) \
    asm("v_cvt_off_f32_i4_sdwa %0, %1 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:BYTE_" #byte : "=v"(dst) : "v"(src))
__device__ __forceinline__ q4_u32x4 q4_dequant8(uint32_t codes, float s) {
    const float s16 = s * 16.0f;
    const uint32_t odd = codes >> 4;
    float lo[4], hi[4];
    PATCH_Q4_NIBBLE(lo[0], codes, 0); PATCH_Q4_NIBBLE(lo[1], codes, 1); PATCH_Q4_NIBBLE(lo[2], codes, 2); PATCH_Q4_NIBBLE(lo[3], codes, 3);
    PATCH_Q4_NIBBLE(hi[0], odd, 0); PATCH_Q4_NIBBLE(hi[1], odd, 1); PATCH_Q4_NIBBLE(hi[2], odd, 2); PATCH_Q4_NIBBLE(hi[3], odd, 3);
    q4_u32x4 out;
#pragma unroll
    for (int p = 0; p < 4; ++p) {
        const q4_f32x2 f = {lo[p] * s16, hi[p] * s16};
        const q4_bf16x2 r = __builtin_convertvector(f, q4_bf16x2);
        out[p] = *reinterpret_cast<const uint32_t*>(&r);
    }
    return out;
}
#undef PATCH_Q4_NIBBLE

__device__ __forceinline__ bool q4_nonzero(uint16_t h) { return (h & 0x7FFFu) != 0; }

// One workgroup per tile: scales, then codes (and, for a 2:4 tile, the kept positions of the unquantized weights).
__global__ __launch_bounds__(256) void pack4_kernel(const uint16_t* __restrict__ W, int64_t K, const uint32_t* __restrict__ table, int Tk,
                                                    int tile, uint8_t* __restrict__ payload, uint16_t* __restrict__ scales,
                                                    int* __restrict__ err) {
    __shared__ float sc[128];
    const int t = blockIdx.x;
    const int tn = t / Tk, tk = t % Tk;
    const uint32_t e = table[t];
    const bool sparse = entry_sparse(e);
    uint8_t* base = payload + entry_offset(e);
    const int64_t n0 = (int64_t)tn * tile, k0 = (int64_t)tk * tile;
    const int KPT = tile / kStepCols, SPT = tile / kStripRows;
    for (int r = threadIdx.x; r < tile; r += blockDim.x) {
        const uint16_t* row = W + (n0 + r) * K + k0;
        uint32_t amax = 0;   // |w| compares like its bit pattern
        for (int k = 0; k < tile; k += 8) {
            union { q4_u32x4 v; uint16_t h[8]; } in;
            in.v = *reinterpret_cast<const q4_u32x4*>(row + k);
#pragma unroll
            for (int i = 0; i < 8; ++i) { const uint32_t a = in.h[i] & 0x7FFFu; amax = a > amax ? a : amax; }
        }
        const uint32_t sb = bf16_rne_bits(__fdiv_rn(q4_bf16_to_float(amax), 7.0f));
        scales[q4_scale_index((int64_t)tn * SPT + r / 16, Tk, tk, r % 16)] = (uint16_t)sb;
        sc[r] = q4_bf16_to_float(sb);
    }
    __syncthreads();
    if (!sparse) {
        const int nchunks = tile * tile / 16;   // one lane of one fragment: 16 elements -> 2 dwords
        for (int c = threadIdx.x; c < nchunks; c += blockDim.x) {
            const int lane = c & 63, sj = c >> 6;
            const int j = sj % KPT, s = sj / KPT, i = lane & 15, q = lane >> 4;
            const float scl = sc[16 * s + i];
            uint32_t d[2];
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                union { q4_u32x4 v; uint16_t hh[8]; } in;
                in.v = *reinterpret_cast<const q4_u32x4*>(W + (n0 + 16 * s + i) * K + k0 + 64 * j + 32 * h + 8 * q);
                uint32_t w = 0;
#pragma unroll
                for (int el = 0; el < 8; ++el) w |= (scl > 0.f ? q4_code(in.hh[el], scl) : 0u) << (4 * el);
                d[h] = w;
            }
            *reinterpret_cast<uint2*>(base + (size_t)c * 8) = uint2{d[0], d[1]};
        }
    } else {
        const int nchunks = tile * tile / 16;   // one lane of one fragment: 16 elements -> 8 kept codes
        uint16_t* meta = reinterpret_cast<uint16_t*>(base + q4_sparse_codes(tile));
        bool ok = true;
        for (int c = threadIdx.x; c < nchunks; c += blockDim.x) {
            const int lane = c & 63, sj = c >> 6;
            const int j = sj % KPT, s = sj / KPT, i = lane & 15, qa = lane >> 4;
            const float scl = sc[16 * s + i];
            union { q4_u32x4 v[2]; uint16_t h[16]; } in;
            const uint16_t* src = W + (n0 + 16 * s + i) * K + k0 + 64 * j + 16 * qa;
            in.v[0] = *reinterpret_cast<const q4_u32x4*>(src);
            in.v[1] = *reinterpret_cast<const q4_u32x4*>(src + 8);
            uint32_t codes = 0, idx = 0;
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                // kept positions: the nonzeros, padded with the lowest-index zeros (the rule of the bf16 packer)
                bool keep[4];
                int nnz = 0;
#pragma unroll
                for (int p = 0; p < 4; ++p) { keep[p] = q4_nonzero(in.h[4 * g + p]); nnz += keep[p] ? 1 : 0; }
                if (nnz > 2) ok = false;
#pragma unroll
                for (int p = 0; p < 4; ++p)
                    if (!keep[p] && nnz < 2) { keep[p] = true; ++nnz; }
                int p0 = -1, p1 = -1;
#pragma unroll
                for (int p = 0; p < 4; ++p)
                    if (keep[p]) { if (p0 < 0) p0 = p; else if (p1 < 0) p1 = p; }
                if (p1 < 0) { p0 = 0; p1 = 1; }
                const uint32_t c0 = scl > 0.f ? q4_code(in.h[4 * g + p0], scl) : 0u, c1 = scl > 0.f ? q4_code(in.h[4 * g + p1], scl) : 0u;
                codes |= (c0 | (c1 << 4)) << (8 * g);
                idx |= (uint32_t)(p0 | (p1 << 2)) << (4 * g);
            }
            *reinterpret_cast<uint32_t*>(base + (size_t)c * 4) = codes;
            meta[(s * 64 + lane) * KPT + j] = (uint16_t)idx;
        }
        if (!ok) atomicOr(err, 1);
    }
}

// The inverse: the dequantized bf16 matrix and / or the codes (int8, 0 at dropped positions) and scales in matrix order.
__global__ __launch_bounds__(256) void unpack4_kernel(const uint8_t* __restrict__ payload, const uint16_t* __restrict__ scales,
                                                      const uint32_t* __restrict__ table, int Tk, int tile, int64_t K,
                                                      uint16_t* __restrict__ W_deq, int8_t* __restrict__ codes_out,
                                                      uint16_t* __restrict__ scales_out) {
    const int t = blockIdx.x;
    const int tn = t / Tk, tk = t % Tk;
    const uint32_t e = table[t];
    const bool sparse = entry_sparse(e);
    const uint8_t* base = payload + entry_offset(e);
    const int64_t n0 = (int64_t)tn * tile, k0 = (int64_t)tk * tile;
    const int KPT = tile / kStepCols, SPT = tile / kStripRows;
    if (scales_out)
        for (int r = threadIdx.x; r < tile; r += blockDim.x)
            scales_out[(n0 + r) * Tk + tk] = scales[q4_scale_index((int64_t)tn * SPT + r / 16, Tk, tk, r % 16)];
    const int nchunks = tile * tile / 16;
    const uint16_t* meta = reinterpret_cast<const uint16_t*>(base + q4_sparse_codes(tile));
    for (int c = threadIdx.x; c < nchunks; c += blockDim.x) {
        const int lane = c & 63, sj = c >> 6;
        const int j = sj % KPT, s = sj / KPT, i = lane & 15, q = lane >> 4;
        const float scl = q4_bf16_to_float(scales[q4_scale_index((int64_t)tn * SPT + s, Tk, tk, i)]);
        int qv[16];
        int64_t kk[16];
        if (!sparse) {
            const uint2 d = *reinterpret_cast<const uint2*>(base + (size_t)c * 8);
#pragma unroll
            for (int el = 0; el < 8; ++el) {
                qv[el] = ((int)(d.x << (28 - 4 * el))) >> 28;
                qv[8 + el] = ((int)(d.y << (28 - 4 * el))) >> 28;
                kk[el] = 64 * j + 8 * q + el;
                kk[8 + el] = 64 * j + 32 + 8 * q + el;
            }
        } else {
            const uint32_t d = *reinterpret_cast<const uint32_t*>(base + (size_t)c * 4);
            const uint32_t idx = meta[(s * 64 + lane) * KPT + j];
#pragma unroll
            for (int el = 0; el < 16; ++el) { qv[el] = 0; kk[el] = 64 * j + 16 * q + el; }
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int p0 = (idx >> (4 * g)) & 3, p1 = (idx >> (4 * g + 2)) & 3;
                const int c0 = ((int)(d << (28 - 8 * g))) >> 28, c1 = ((int)(d << (24 - 8 * g))) >> 28;
#pragma unroll
                for (int p = 0; p < 4; ++p) {
                    if (p == p0) qv[4 * g + p] = c0;
                    if (p == p1) qv[4 * g + p] = c1;
                }
            }
        }
#pragma unroll
        for (int el = 0; el < 16; ++el) {
            const int64_t at = (n0 + 16 * s + i) * K + k0 + kk[el];
            if (W_deq) W_deq[at] = (uint16_t)bf16_rne_bits((float)qv[el] * scl);
            if (codes_out) codes_out[at] = (int8_t)qv[el];
        }
    }
}

// Up to 16 RB rows of X (RB = 1, 2 or 4 blocks of 16 rows) against the 4-bit weight in one pass over it.  A workgroup
// owns R consecutive strips of 16 features (the registers hold R x RB accumulators and RB X operands per step: R <= 3
// with one row block, R <= 2 with more); its KW wavefronts take contiguous runs of 64-column steps.  A wavefront loads
// the X operand of a step once and uses it for all R strips (at 4 bits per weight X is the larger stream, so this
// reuse is what bounds the traffic), works in batches of NB steps (2; 1 when RB > 1) - table entries, then every load
// of the batch, then the arithmetic - and issues the next batch's loads before it consumes the current one.  Two batch
// buffers alternate; no copies.
constexpr int kQ4MaxR = 3;
constexpr int kQ4Rows = 64;   // rows of X per launch at most

template <int R, int RB, int NB>
struct Q4Batch {
    uint32_t e[NB][R];
    q4_u32x2 d[NB][R];         // dense: both dwords; 2:4: [0] = codes, [1] = positions
    uint32_t sc[NB][R];        // scale bits
    q4_u32x4 x[NB][RB][2];
};

// The product kernel's pointers carry their address space: the weight pointers reach it inside a by-value struct and
// pass through scalar selects, after which the compiler no longer knows that they are global (it then emits flat
// loads) nor that the table is not written by the kernel (it then reads entries with vector loads).  Table entries
// are read through the constant address space (scalar loads), everything else through the global one.
#define PATCH_Q4_GLOBAL __attribute__((address_space(1)))
#define PATCH_Q4_CONST __attribute__((address_space(4)))
typedef const PATCH_Q4_CONST uint32_t* q4_table_ptr;
typedef const PATCH_Q4_GLOBAL uint8_t* q4_bytes_ptr;
typedef const PATCH_Q4_GLOBAL uint16_t* q4_u16_ptr;

template <int R>
struct Q4Strips {
    q4_table_ptr row[R];      // table entries of the strip's tile row
    q4_bytes_ptr pay[R];      // payload of the strip's weight
    int s[R];                 // strip within the tile
    q4_u16_ptr scl[R];        // this lane's scale of the strip for tile column 0 (the next column is 16 scales on)
};

// Steps past the wavefront's run repeat its last step (in bounds; discarded by q4_compute).
template <int TILE, int R, int RB, int NB>
__device__ __forceinline__ void q4_loads(Q4Batch<R, RB, NB>& b, const Q4Strips<R>& st, const q4_u16_ptr (&xrow)[RB], const bool (&xvalid)[RB],
                                         int lane, int step0, int last) {
    constexpr int KPT = TILE / kStepCols;
#pragma unroll
    for (int i = 0; i < NB; ++i) {
        const int step = step0 + i < last ? step0 + i : last;
#pragma unroll
        for (int r = 0; r < R; ++r) b.e[i][r] = st.row[r][step / KPT];
    }
#pragma unroll
    for (int i = 0; i < NB; ++i) {
        const int step = step0 + i < last ? step0 + i : last;
        const int j = step % KPT;
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) {
            b.x[i][rb][0] = q4_u32x4{0u, 0u, 0u, 0u};
            b.x[i][rb][1] = q4_u32x4{0u, 0u, 0u, 0u};
            if (xvalid[rb]) {
                b.x[i][rb][0] = *reinterpret_cast<const PATCH_Q4_GLOBAL q4_u32x4*>(xrow[rb] + (int64_t)step * kStepCols);
                b.x[i][rb][1] = *reinterpret_cast<const PATCH_Q4_GLOBAL q4_u32x4*>(xrow[rb] + (int64_t)step * kStepCols + 32);
            }
        }
#pragma unroll
        for (int r = 0; r < R; ++r) {
            q4_bytes_ptr base = st.pay[r] + entry_offset(b.e[i][r]);
            const int s = st.s[r];
            b.sc[i][r] = st.scl[r][(step / KPT) * 16];
            if (!entry_sparse(b.e[i][r])) {
                b.d[i][r] = *reinterpret_cast<const PATCH_Q4_GLOBAL q4_u32x2*>(base + (size_t)(s * KPT + j) * 512 + lane * 8);
            } else {
                b.d[i][r][0] = *reinterpret_cast<const PATCH_Q4_GLOBAL uint32_t*>(base + (size_t)(s * KPT + j) * 256 + lane * 4);
                b.d[i][r][1] = *reinterpret_cast<q4_u16_ptr>(base + q4_sparse_codes(TILE) + ((s * 64 + lane) * KPT + j) * 2);
            }
        }
    }
}

template <int R, int RB, int NB>
__device__ __forceinline__ void q4_compute(const Q4Batch<R, RB, NB>& b, q4_f32x4 (&acc)[R][RB], int step0, int end) {
#pragma unroll
    for (int i = 0; i < NB; ++i) {
        if (step0 + i >= end) break;   // uniform
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const float scl = q4_bf16_to_float(b.sc[i][r]);
            if (!entry_sparse(b.e[i][r])) {
                Q4A a0, a1;
                a0.raw = q4_dequant8(b.d[i][r][0], scl);
                a1.raw = q4_dequant8(b.d[i][r][1], scl);
#pragma unroll
                for (int rb = 0; rb < RB; ++rb) {
                    Q4B x;
                    x.raw[0] = b.x[i][rb][0];
                    x.raw[1] = b.x[i][rb][1];
                    acc[r][rb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a0.v, x.h[0], acc[r][rb], 0, 0, 0);
                    acc[r][rb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a1.v, x.h[1], acc[r][rb], 0, 0, 0);
                }
            } else {
                Q4A a;
                a.raw = q4_dequant8(b.d[i][r][0], scl);
#pragma unroll
                for (int rb = 0; rb < RB; ++rb) {
                    Q4B x;
                    x.raw[0] = b.x[i][rb][0];
                    x.raw[1] = b.x[i][rb][1];
                    acc[r][rb] = __builtin_amdgcn_smfmac_f32_16x16x64_bf16(a.v, x.v, acc[r][rb], (int)b.d[i][r][1], 0, 0);
                }
            }
        }
    }
}

// Up to MAXC 4-bit weights that share one X (same K, same tile) in one launch.  The launch numbers the 16-feature strips
// across all weights (first[i] = first strip of weight i, total = their number); a workgroup takes R consecutive
// strips, which may belong to two weights.
template <int MAXC>
struct Q4Set {
    static constexpr int kMax = MAXC;
    const uint8_t* payload[MAXC];
    const uint16_t* scales[MAXC];
    const uint32_t* table[MAXC];
    float* Y[MAXC];
    int64_t N[MAXC];
    int first[MAXC];
    int count, total;
};

// A set of one: 40 bytes of kernel arguments.
struct Q4One {
    const uint8_t* payload;
    const uint16_t* scales;
    const uint32_t* table;
    float* Y;
    int64_t N;
};

struct Q4Weight {
    uint64_t payload, scales, table, Y;
    int64_t N;
    int first;
};

// The weight that strip g of the launch belongs to (g uniform): scalar selects over the candidates, so that every
// pointer stays in scalar registers.
template <typename SetT>
__device__ __forceinline__ Q4Weight q4_weight_of(const SetT& set, int g) {
    Q4Weight wt;
    if constexpr (sizeof(SetT) == sizeof(Q4One)) {
        wt = Q4Weight{reinterpret_cast<uint64_t>(set.payload), reinterpret_cast<uint64_t>(set.scales), reinterpret_cast<uint64_t>(set.table),
                      reinterpret_cast<uint64_t>(set.Y), set.N, 0};
    } else {
        wt = Q4Weight{reinterpret_cast<uint64_t>(set.payload[0]), reinterpret_cast<uint64_t>(set.scales[0]),
                      reinterpret_cast<uint64_t>(set.table[0]), reinterpret_cast<uint64_t>(set.Y[0]), set.N[0], 0};
#pragma unroll
        for (int i = 1; i < SetT::kMax; ++i) {
            const bool here = i < set.count && g >= set.first[i];
            wt.payload = here ? reinterpret_cast<uint64_t>(set.payload[i]) : wt.payload;
            wt.scales = here ? reinterpret_cast<uint64_t>(set.scales[i]) : wt.scales;
            wt.table = here ? reinterpret_cast<uint64_t>(set.table[i]) : wt.table;
            wt.Y = here ? reinterpret_cast<uint64_t>(set.Y[i]) : wt.Y;
            wt.N = here ? set.N[i] : wt.N;
            wt.first = here ? set.first[i] : wt.first;
        }
    }
    return wt;
}

// Every kernel argument is requested in the kernel's first instructions and waited for once (the compiler otherwise
// fetches an argument where it is first used, e.g. behind a branch: one more, if short, round trip before the first
// weight load).  What costs far more is losing the address spaces (see PATCH_Q4_GLOBAL above): with flat loads and
// table entries read by vector loads the same launch took 8.0 us instead of 6.2.
#define PATCH_Q4_ARGS_NOW(...) asm volatile("" ::__VA_ARGS__)

// wavefronts per workgroup at most: 16, or 8 with four or more accumulators and X operands of several row blocks
// (whose registers do not fit 16 times into a compute unit)
constexpr int q4_max_waves(int R, int RB) { return RB == 4 || R * RB > 4 || (RB == 2 && R > 1) ? 8 : 16; }

template <int TILE, int R, int RB, typename SetT>
__global__ __launch_bounds__(64 * q4_max_waves(R, RB)) void decode4_kernel(const uint16_t* __restrict__ X, int64_t m0, int rows, int64_t K, int Tk, int KW,
                                                       const SetT set) {
    constexpr bool kOne = sizeof(SetT) == sizeof(Q4One);
    constexpr int KPT = TILE / kStepCols, SPT = TILE / kStripRows;
    constexpr int NB = RB > 1 ? 1 : 2;   // steps per batch
    constexpr int CH = R * RB < 8 ? R * RB : 8;   // items per round of the final reduction
    __shared__ q4_f32x4 red[CH][q4_max_waves(R, RB)][64];
    const int tid = threadIdx.x, lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);   // of KW wavefronts: an argument (the launch size is a hidden one, fetched apart)
    const int col = lane & 15, q = lane >> 4;
    int total_strips;
    if constexpr (kOne) total_strips = (int)(set.N / kStripRows);
    else total_strips = set.total;
    const int g0 = (int)blockIdx.x * R;
    Q4Strips<R> st;
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const int g = g0 + r < total_strips ? g0 + r : total_strips - 1;   // a strip past the end repeats the last one (not stored)
        const Q4Weight wt = q4_weight_of(set, g);
        PATCH_Q4_ARGS_NOW("s"(wt.payload), "s"(wt.scales), "s"(wt.table), "s"(wt.first));
        const int strip = g - wt.first;
        st.row[r] = reinterpret_cast<q4_table_ptr>(wt.table) + (int64_t)(strip / SPT) * Tk;
        st.pay[r] = reinterpret_cast<q4_bytes_ptr>(wt.payload);
        st.s[r] = strip % SPT;
        st.scl[r] = reinterpret_cast<q4_u16_ptr>(wt.scales) + q4_scale_index(strip, Tk, 0, col);
    }
    // the first (strip, row block) this wavefront adds up and stores at the end (it takes items w, w + KW, ...)
    {
        const int gw = g0 + (w < R * RB ? w / RB : 0);
        const Q4Weight wy = q4_weight_of(set, gw < total_strips ? gw : total_strips - 1);
        PATCH_Q4_ARGS_NOW("s"(X), "s"(m0), "s"(rows), "s"(K), "s"(Tk), "s"(KW), "s"(wy.Y), "s"(wy.N), "s"(wy.first));
    }
    const int total = Tk * KPT, per = (total + KW - 1) / KW;
    const int begin = w * per, end = begin + per < total ? begin + per : total;
    bool xvalid[RB];
    q4_u16_ptr xrow[RB];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
        xvalid[rb] = 16 * rb + col < rows;
        xrow[rb] = reinterpret_cast<q4_u16_ptr>(reinterpret_cast<uintptr_t>(X)) + (m0 + (xvalid[rb] ? 16 * rb + col : 0)) * K + 8 * q;
    }
    q4_f32x4 acc[R][RB];
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) acc[r][rb] = q4_f32x4{0.f, 0.f, 0.f, 0.f};
    if (begin < end) {
        Q4Batch<R, RB, NB> b0, b1;
        q4_loads<TILE, R, RB, NB>(b0, st, xrow, xvalid, lane, begin, end - 1);
        for (int step0 = begin; step0 < end; step0 += 2 * NB) {
            const bool have1 = step0 + NB < end, have2 = step0 + 2 * NB < end;   // uniform
            if (have1) q4_loads<TILE, R, RB, NB>(b1, st, xrow, xvalid, lane, step0 + NB, end - 1);
            q4_compute<R, RB, NB>(b0, acc, step0, end);
            if (have2) q4_loads<TILE, R, RB, NB>(b0, st, xrow, xvalid, lane, step0 + 2 * NB, end - 1);
            if (have1) q4_compute<R, RB, NB>(b1, acc, step0 + NB, end);
        }
    }
    // Partial sums meet in LDS, CH (strip, row block) items at a time (all of them unless R RB > 8): wavefront w adds
    // up the items w, w + KW, ... of the chunk in wavefront order and stores them.
#pragma unroll
    for (int c0 = 0; c0 < R * RB; c0 += CH) {
        if (c0 > 0) __syncthreads();
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
            for (int rb = 0; rb < RB; ++rb)
                if (r * RB + rb >= c0 && r * RB + rb < c0 + CH) red[r * RB + rb - c0][w][lane] = acc[r][rb];
        __syncthreads();
        for (int i0 = w; i0 < CH && c0 + i0 < R * RB; i0 += KW) {
            const int item = c0 + i0, gw = g0 + item / RB, wrb = item % RB;
            if (gw >= total_strips) break;
            const Q4Weight wy = q4_weight_of(set, gw);
            q4_f32x4 sum = red[i0][0][lane];
            for (int i = 1; i < KW; ++i) {
                const q4_f32x4 v = red[i0][i][lane];
                sum[0] += v[0]; sum[1] += v[1]; sum[2] += v[2]; sum[3] += v[3];
            }
            PATCH_Q4_GLOBAL float* Yg = reinterpret_cast<PATCH_Q4_GLOBAL float*>(wy.Y);
            if (16 * wrb + col < rows)
                *reinterpret_cast<PATCH_Q4_GLOBAL q4_f32x4*>(Yg + (m0 + 16 * wrb + col) * wy.N + (int64_t)(gw - wy.first) * 16 + 4 * q) = sum;
        }
    }
}

template <int TILE, int R, int RB, typename SetT>
static void launch_decode4(const uint16_t* X, int64_t m0, int rows, int64_t K, int Tk, const SetT& set, int groups, int kw, hipStream_t s) {
    hipLaunchKernelGGL((decode4_kernel<TILE, R, RB, SetT>), dim3((unsigned)groups), dim3((unsigned)(kw * 64)), 0, s, X, m0, rows, K, Tk, kw,
                       set);
}

// up to 3 strips per workgroup with one or four blocks of 16 rows, up to 4 with two
template <int TILE, typename SetT>
static void launch_decode4_r(int R, int RB, const uint16_t* X, int64_t m0, int rows, int64_t K, int Tk, const SetT& set, int groups, int kw,
                             hipStream_t s) {
#define PATCH_Q4_CASE(r, rb) \
    if (R == r && RB == rb) return launch_decode4<TILE, r, rb, SetT>(X, m0, rows, K, Tk, set, groups, kw, s)
    PATCH_Q4_CASE(1, 1); PATCH_Q4_CASE(2, 1); PATCH_Q4_CASE(3, 1);
    PATCH_Q4_CASE(1, 2); PATCH_Q4_CASE(2, 2); PATCH_Q4_CASE(3, 2); PATCH_Q4_CASE(4, 2);
    PATCH_Q4_CASE(1, 4); PATCH_Q4_CASE(2, 4); PATCH_Q4_CASE(3, 4);
#undef PATCH_Q4_CASE
}

// Strips per workgroup for a pass of `rows` rows over `strips` strips: the R that minimises an estimate of the pass,
//     rounds(workgroups) x (x + R),
// in units of one strip's share of a wavefront's work.  x is what a workgroup spends on its X operands (it loads all of
// X whatever R is; fitted: 0.15 + 0.045 rows up to 16 rows, 1.7 for 32, 4.5 for 64 - at 4 bits per weight 64 rows of X
// are 16 times a strip's codes); rounds = workgroups / compute units, rounded up while at most two rounds are resident at
// once (then the busiest compute unit decides), with half a round for the tail beyond.  More strips per workgroup
// share X further but must not leave compute units idle: 688 strips on 256 units run as 230 workgroups of 3 (one
// round) rather than 344 of 2.  R <= 3 (one or four row blocks) or 4 (two): what the registers hold.
static int q4_strips_per_group(int strips, int n_cus, int rows) {
    const int max_r = rows > 16 && rows <= 32 ? 4 : kQ4MaxR;
    const double x = rows <= 16 ? 0.15 + 0.045 * rows : rows <= 32 ? 1.7 : 4.5;
    int best = 1;
    double best_cost = 0.0;
    for (int r = 1; r <= max_r; ++r) {
        const int groups = (strips + r - 1) / r;
        const double rounds = groups <= 2 * n_cus ? (double)((groups + n_cus - 1) / n_cus) : (double)groups / n_cus + 0.5;
        const double cost = rounds * (x + r);
        if (r == 1 || cost <= best_cost) { best = r; best_cost = cost; }
    }
    return best;
}

// ------------------------------------------------------------------------------------------------------
// Prefill-shaped product from the 4-bit storage: the structure of prefill_kernel_areg - blocks of 256
// features x 128 or 256 rows, a wavefront owns 32 features x all rows, X through two LDS stages - with the weight operands
// dequantized in registers.  A lane loads the codes of its pieces of the stored fragments one step ahead (dense: two
// 8-byte loads, fragment lanes fl and fl + 32, each holding the codes of both half-steps; 2:4: two 4-byte loads), the
// scale of its row once per tile and the position dwords once per tile; at the top of a step the codes of that step
// become bf16 operands (q4_dequant8) and the step runs as in the bf16 kernel.  The weight is read once per 128 rows of
// X, at 4 bits per kept weight, and no bf16 copy of it exists anywhere.
// ------------------------------------------------------------------------------------------------------
constexpr int kP4BN = 256;

typedef const __attribute__((address_space(1))) uint32_t* p4_g4_t;
typedef const __attribute__((address_space(1))) uint16_t* p4_g2_t;
typedef const __attribute__((address_space(1))) q4_u32x2* p4_g8_t;

// One step's codes of a wavefront.  Named by use (an array indexed by the tile type would live in scratch memory):
// half-step u multiplies the operands dequantized from (a_u, b_u); a 2:4 tile uses a_0 and a_1 only.
struct P4Codes {
    uint32_t a0, a1, b0, b1;
};

template <int TILE, int BM, bool SPLIT>
__global__ __launch_bounds__(512) void prefill4_kernel(const uint16_t* __restrict__ X, int64_t M, int64_t N, int64_t K,
                                                       const uint8_t* __restrict__ payload, const uint16_t* __restrict__ scales,
                                                       const uint32_t* __restrict__ table, int Tk_all, int tiles_n, int tiles_m,
                                                       float* __restrict__ Y) {
    constexpr int KPT = TILE / kStepCols;      // K-steps per tile: 2 or 1
    constexpr int NB = BM / 32;                // 32-row blocks: 4 or 8
    constexpr int XP = BM / 64;                // 1 KB pieces of the X tile per wavefront
    constexpr int kP4Stage = BM * 128;         // 16 or 32 KB
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
    const int tid = threadIdx.x, lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int fo = 32 * w;                 // first feature of the wavefront inside the block
    const int w4 = fo / TILE;              // tile row of the block its features lie in
    // block -> (n, m): one contiguous run of the grouped order (4 row blocks x all feature blocks) per XCD
    const int nblk = tiles_n * tiles_m;
    int bid = blockIdx.x;
    {
        const int per = (nblk + 7) / 8;
        const int x = bid & 7, i = bid >> 3;
        const int t = x * per + i;
        bid = (i < per && t < nblk) ? t : -1;
    }
    if (bid < 0) return;
    int bn, bm;
    {
        constexpr int GM = 4;
        const int full = (tiles_m / GM) * GM * tiles_n;
        if (bid < full) {
            const int g = bid / (GM * tiles_n), rem = bid % (GM * tiles_n);
            bn = rem / GM;
            bm = g * GM + rem % GM;
        } else {
            const int gm = tiles_m % GM, rem = bid - full;
            bn = rem / gm;
            bm = (tiles_m / GM) * GM + rem % gm;
        }
    }
    const int64_t n0 = (int64_t)bn * kP4BN, m0 = (int64_t)bm * BM;
    // N is a multiple of the tile, not necessarily of 256: a wavefront of a missing tile row works on the last live one's
    // weights (valid addresses) and stores nothing
    const int live = (int)((N - n0) / TILE) < kP4BN / TILE ? (int)((N - n0) / TILE) : kP4BN / TILE;
    const int trw = w4 < live ? w4 : live - 1;
    const int t_begin = SPLIT ? (int)((int64_t)blockIdx.y * Tk_all / gridDim.y) : 0;
    const int Tk = SPLIT ? (int)((int64_t)(blockIdx.y + 1) * Tk_all / gridDim.y) - t_begin : Tk_all;
    const uint32_t* trow = table + ((int64_t)(n0 / TILE) + trw) * Tk_all + t_begin;

    const uint8_t* xsrc[XP];
#pragma unroll
    for (int i = 0; i < XP; ++i) {
        const int c = (w + 8 * i) * 64 + lane;
        const int m = c >> 3, pp = c & 7, pl = pp ^ ((m >> 1) & 7);
        int64_t row = m0 + m;
        if (row >= M) row = M - 1;
        xsrc[i] = reinterpret_cast<const uint8_t*>(X + row * K + pl * 8 + (int64_t)t_begin * TILE);
    }
    auto load_x = [&](int ks, int stage) {
#pragma unroll
        for (int i = 0; i < XP; ++i) g2l16(xsrc[i] + (size_t)ks * 128, lds + stage * kP4Stage + (w + 8 * i) * 1024);
    };

    const int i32 = lane & 31, q = lane >> 5;
    // this lane's pieces: strip (32 w % TILE) / 16 + i32 / 16 of the tile, fragment lanes fl and fl + 32
    const int strip = (fo % TILE) / 16 + (i32 >> 4);
    const int fl = 16 * q + (i32 & 15);
    // scale of the lane's row for the first tile of this K slice; the next tile's is 16 scales on
    const uint16_t* sc = scales + q4_scale_index(((n0 + (int64_t)trw * TILE) / 16) + strip, Tk_all, t_begin, i32 & 15);
    auto load_codes = [&](P4Codes& d, uint32_t e, int j) {
        const uint8_t* tb = payload + entry_offset(e);
        if (entry_sparse(e)) {
            const uint8_t* f = tb + (size_t)(strip * KPT + j) * 256;
            d.a0 = *(p4_g4_t)(f + fl * 4);
            d.a1 = *(p4_g4_t)(f + (fl + 32) * 4);
        } else {
            const uint8_t* f = tb + (size_t)(strip * KPT + j) * 512;
            const q4_u32x2 lo = *(p4_g8_t)(f + fl * 8), hi = *(p4_g8_t)(f + (fl + 32) * 8);
            d.a0 = lo[0];
            d.a1 = lo[1];
            d.b0 = hi[0];
            d.b1 = hi[1];
        }
    };
    // per tile: the position words of fragment lanes fl and fl + 32 (mask tile 128: a dword holding both K-steps; mask
    // tile 64: 16 bits), and the scale
    auto load_tile = [&](uint32_t& d0, uint32_t& d1, uint32_t& scl, uint32_t e, int tk) {
        scl = *(p4_g2_t)(sc + (size_t)tk * 16);
        if (entry_sparse(e)) {
            const uint8_t* pb = payload + entry_offset(e) + q4_sparse_codes(TILE) + (size_t)(strip * 64 + fl) * (2 * KPT);
            if constexpr (KPT == 2) {
                d0 = *(p4_g4_t)(pb);
                d1 = *(p4_g4_t)(pb + 32 * 4);
            } else {
                d0 = *(p4_g2_t)(pb);
                d1 = *(p4_g2_t)(pb + 32 * 2);
            }
        }
    };

    f32x16 acc[NB];
#pragma unroll
    for (int b = 0; b < NB; ++b)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[b][i] = 0.f;

    auto step_begin = [&](int ks, int pf_ks) {
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        load_x(pf_ks, (ks & 1) ^ 1);
    };
    auto step_mma = [&](int ks, const P4Codes& c, uint32_t p0, uint32_t p1, uint32_t sbits, int sp, int j) {
        const float scl = q4_bf16_to_float(sbits);
        A8 h0a, h0b, h1a, h1b;
        h0a.raw = q4_dequant8(c.a0, scl);
        h1a.raw = q4_dequant8(c.a1, scl);
        h0b.raw = h0a.raw;                                 // a 2:4 step does not use the second operands
        h1b.raw = h1a.raw;
        if (!sp) {
            h0b.raw = q4_dequant8(c.b0, scl);
            h1b.raw = q4_dequant8(c.b1, scl);
        }
        const uint8_t* bs = lds + (ks & 1) * kP4Stage;
        B16 xa[3], xb[3];
        auto fetch = [&](int p, int buf) {
            const int u = p / (NB / 2), b0 = 2 * (p % (NB / 2));
#pragma unroll
            for (int cc = 0; cc < 2; ++cc) {
                xa[buf].raw[cc] = *reinterpret_cast<const u32x4*>(bs + xs_off(32 * b0 + i32, 2 * (2 * u + cc) + q));
                xb[buf].raw[cc] = *reinterpret_cast<const u32x4*>(bs + xs_off(32 * (b0 + 1) + i32, 2 * (2 * u + cc) + q));
            }
        };
        fetch(0, 0);
        fetch(1, 1);
#pragma unroll
        for (int p = 0; p < NB; ++p) {
            if (p + 2 < NB) fetch(p + 2, (p + 2) % 3);
            const int u = p / (NB / 2), b0 = 2 * (p % (NB / 2)), buf = p % 3;
            mma_step(acc[b0], acc[b0 + 1], u ? h1a.v : h0a.v, u ? h1b.v : h0b.v, xa[buf], xb[buf], (int)((u ? p1 : p0) >> (16 * j)), sp);
        }
    };

    if constexpr (KPT == 2) {
        P4Codes c0, c1;              // codes of the even / odd step of a tile
        c0.b0 = c0.b1 = c1.b0 = c1.b1 = 0u;
        uint32_t p0 = 0u, p1 = 0u, sb = 0u, pn0 = 0u, pn1 = 0u, sbn = 0u;
        uint32_t e = trow[0];
        load_x(0, 0);
        load_codes(c0, e, 0);
        load_tile(pn0, pn1, sbn, e, 0);
        __builtin_assume(Tk > 0);
        for (int tk = 0; tk < Tk; ++tk) {
            const int more = tk + 1 < Tk ? 1 : 0;
            const uint32_t en = trow[tk + more];
            const int sp = (int)(e & 1u);
            step_begin(2 * tk, 2 * tk + 1);
            // this tile's position dwords and scale were loaded a step ago and have landed; an opaque copy, so that it does
            // not become a copy on the loop's back edge right behind the loads
            asm volatile("v_mov_b32 %0, %3\n\tv_mov_b32 %1, %4\n\tv_mov_b32 %2, %5" : "=&v"(p0), "=&v"(p1), "=&v"(sb) : "v"(pn0), "v"(pn1), "v"(sbn));
            load_codes(c1, e, 1);
            step_mma(2 * tk, c0, p0, p1, sb, sp, 0);
            step_begin(2 * tk + 1, 2 * tk + 1 + more);
            load_codes(c0, en, 0);
            load_tile(pn0, pn1, sbn, en, tk + more);
            step_mma(2 * tk + 1, c1, p0, p1, sb, sp, 1);
            e = en;
        }
    } else {
        // Mask tile 64: every step is a tile of its own, with its own scale and position words.  Steps go in pairs (the
        // buffers alternate without a copy), table entries are read two steps ahead; past the end the last step is
        // fetched again, and the second step of the last pair is skipped when the count is odd.
        const int S = Tk;
        P4Codes c0, c1;
        c0.b0 = c0.b1 = c1.b0 = c1.b1 = 0u;
        uint32_t a0 = 0u, a1 = 0u, as_ = 0u, b0_ = 0u, b1_ = 0u, bs_ = 0u;   // position words and scale of c0 / c1
        uint32_t e0 = trow[0], e1 = trow[S > 1 ? 1 : 0];
        load_x(0, 0);
        load_codes(c0, e0, 0);
        load_tile(a0, a1, as_, e0, 0);
        __builtin_assume(S > 0);
        for (int s_ = 0; s_ < S; s_ += 2) {
            const int s1 = s_ + 1 < S ? s_ + 1 : S - 1, s2 = s_ + 2 < S ? s_ + 2 : S - 1, s3 = s_ + 3 < S ? s_ + 3 : S - 1;
            const uint32_t e2 = trow[s2], e3 = trow[s3];
            step_begin(s_, s1);
            load_codes(c1, e1, 0);
            load_tile(b0_, b1_, bs_, e1, s1);
            step_mma(s_, c0, a0, a1, as_, (int)(e0 & 1u), 0);
            if (s_ + 1 < S) {
                step_begin(s_ + 1, s2);
                load_codes(c0, e2, 0);
                load_tile(a0, a1, as_, e2, s2);
                step_mma(s_ + 1, c1, b0_, b1_, bs_, (int)(e1 & 1u), 0);
            }
            e0 = e2;
            e1 = e3;
        }
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    asm volatile("s_nop 15\n\ts_nop 15\n\ts_nop 15" ::: "memory");
    // acc[b][i]: feature n0 + fo + 8 (i/4) + 4 q + i%4, row m0 + 32 b + i32.  The X stages are free once every wavefront
    // has left the loop: each block of 32 rows is turned through 4 KB of them and stored in whole rows
    // (store_block_rows).
    __syncthreads();
    if (w4 < live) {
#pragma unroll
        for (int b = 0; b < NB; ++b)
            store_block_rows(lds + w * 4096, acc[b], lane, Y, (SPLIT ? (int64_t)blockIdx.y * M * N : 0) + (m0 + 32 * b) * N + n0 + fo, N,
                             M - (m0 + 32 * b), 0);
    }
}

}  // namespace patch

using namespace patch;

struct patch_packed4 {
    int64_t N = 0, K = 0;
    int tile = 0, Tn = 0, Tk = 0;
    int64_t n_sparse = 0;
    size_t algorithmic_bytes = 0;   // codes + positions + scales, without alignment padding
    size_t payload_bytes = 0;
    uint8_t* d_payload = nullptr;   // codes and positions
    uint16_t* d_scales = nullptr;   // N x Tk bf16, strip-major
    uint32_t* d_table = nullptr;
    std::vector<uint8_t> tile_map;  // host copy, 1 = dense
    int n_cus = 256;
};

static bool q4_aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

extern "C" {

void patch_free4(patch_packed4* P) {
    if (!P) return;
    if (P->d_payload) (void)hipFree(P->d_payload);
    if (P->d_scales) (void)hipFree(P->d_scales);
    if (P->d_table) (void)hipFree(P->d_table);
    delete P;
}

// The host side of a 4-bit packed weight and its device buffers: table uploaded on `s`, payload zeroed (its alignment
// padding reads as zero), codes and scales not yet written.  Shared by patch_pack4 and patch_deserialize4.
static patch_status new_packed4(int64_t N, int64_t K, const uint8_t* tile_map, int tile, hipStream_t s, patch_packed4** out) {
    patch_packed4* P = new (std::nothrow) patch_packed4();
    if (!P) return PATCH_ERR_ALLOC;
    P->N = N; P->K = K; P->tile = tile;
    P->Tn = (int)(N / tile); P->Tk = (int)(K / tile);
    const size_t T = (size_t)P->Tn * (size_t)P->Tk;
    std::vector<uint32_t> table;
    try { table.resize(T); P->tile_map.resize(T); } catch (...) { delete P; return PATCH_ERR_ALLOC; }
    uint64_t off = 0;
    for (size_t i = 0; i < T; ++i) {
        const bool sparse = tile_map[i] == 0;
        P->tile_map[i] = sparse ? 0 : 1;
        table[i] = make_entry(off, sparse);
        off += sparse ? q4_sparse_tile(tile) : q4_dense_tile(tile);
        P->algorithmic_bytes += sparse ? q4_sparse_codes(tile) + q4_sparse_pos(tile) + 2 * tile : q4_dense_codes(tile) + 2 * tile;
        if (sparse) ++P->n_sparse;
    }
    P->payload_bytes = off;
    if ((off / kGranule) >> 31) { delete P; return PATCH_ERR_SHAPE; }
    int dev = 0;
    hipDeviceProp_t prop;
    if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess) {
        patch_note_hip_error((int)hipGetLastError());
        delete P;
        return PATCH_ERR_HIP;
    }
    P->n_cus = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;
    const bool ok = hipMalloc(&P->d_payload, P->payload_bytes) == hipSuccess && hipMalloc(&P->d_table, T * sizeof(uint32_t)) == hipSuccess &&
                    hipMalloc(&P->d_scales, (size_t)N * P->Tk * sizeof(uint16_t)) == hipSuccess;
    if (!ok) {
        (void)hipGetLastError();
        patch_free4(P);
        return PATCH_ERR_ALLOC;
    }
    hipError_t e = hipMemcpyAsync(P->d_table, table.data(), T * sizeof(uint32_t), hipMemcpyHostToDevice, s);
    if (e == hipSuccess) e = hipMemsetAsync(P->d_payload, 0, P->payload_bytes, s);
    const hipError_t e_sync = hipStreamSynchronize(s);   // the host table goes out of scope here
    if (e == hipSuccess) e = e_sync;
    if (e != hipSuccess) {
        patch_note_hip_error((int)e);
        patch_free4(P);
        return PATCH_ERR_HIP;
    }
    *out = P;
    return PATCH_OK;
}

patch_status patch_pack4(const void* W_hat, int64_t N, int64_t K, const uint8_t* tile_map, int tile, void* stream, patch_packed4** out) {
    if (!W_hat || !tile_map || !out || N <= 0 || K <= 0) return PATCH_ERR_ARG;
    if ((tile != 64 && tile != 128) || N % tile || K % tile || N / tile > (1 << 20) || K / tile > (1 << 20)) return PATCH_ERR_SHAPE;
    if (!q4_aligned16(W_hat)) return PATCH_ERR_ARG;
    hipStream_t s = static_cast<hipStream_t>(stream);
    patch_packed4* P = nullptr;
    const patch_status st = new_packed4(N, K, tile_map, tile, s, &P);
    if (st != PATCH_OK) return st;
    const size_t T = (size_t)P->Tn * (size_t)P->Tk;
    int* d_err = nullptr;
    if (hipMalloc(&d_err, sizeof(int)) != hipSuccess) {
        (void)hipGetLastError();
        patch_free4(P);
        return PATCH_ERR_ALLOC;
    }
    hipError_t e = hipMemsetAsync(d_err, 0, sizeof(int), s);
    if (e == hipSuccess) {
        hipLaunchKernelGGL(pack4_kernel, dim3((unsigned)T), dim3(256), 0, s, static_cast<const uint16_t*>(W_hat), K, P->d_table, P->Tk, tile,
                           P->d_payload, P->d_scales, d_err);
        e = hipGetLastError();
    }
    int h_err = 0;
    if (e == hipSuccess) e = hipMemcpyAsync(&h_err, d_err, sizeof(int), hipMemcpyDeviceToHost, s);
    const hipError_t e_sync = hipStreamSynchronize(s);
    if (e == hipSuccess) e = e_sync;
    (void)hipFree(d_err);
    if (e != hipSuccess) {
        patch_note_hip_error((int)e);
        patch_free4(P);
        return PATCH_ERR_HIP;
    }
    if (h_err) {
        patch_free4(P);
        return PATCH_ERR_NOT_24;
    }
    *out = P;
    return PATCH_OK;
}

// ---- the 4-bit storage saved to and loaded from host memory (saved.h): header, tile map, codes and positions, scales
size_t patch_serialized4_bytes(const patch_packed4* P) {
    if (!P) return 0;
    return saved_round(sizeof(SavedHeader)) + saved_round(P->tile_map.size()) + saved_round(P->payload_bytes) +
           (size_t)P->N * P->Tk * sizeof(uint16_t);
}

patch_status patch_serialize4(const patch_packed4* P, void* buf, size_t bytes, void* stream) {
    if (!P || !buf) return PATCH_ERR_ARG;
    if (bytes < patch_serialized4_bytes(P)) return PATCH_ERR_SIZE;
    uint8_t* b = static_cast<uint8_t*>(buf);
    const size_t scales_bytes = (size_t)P->N * P->Tk * sizeof(uint16_t);
    const size_t map_at = saved_round(sizeof(SavedHeader)), pay_at = map_at + saved_round(P->tile_map.size());
    const size_t sc_at = pay_at + saved_round(P->payload_bytes);
    memset(b, 0, pay_at);
    memset(b + pay_at + P->payload_bytes, 0, sc_at - pay_at - P->payload_bytes);
    memcpy(b + map_at, P->tile_map.data(), P->tile_map.size());
    hipStream_t s = static_cast<hipStream_t>(stream);
    hipError_t e = hipMemcpyAsync(b + pay_at, P->d_payload, P->payload_bytes, hipMemcpyDeviceToHost, s);
    if (e == hipSuccess) e = hipMemcpyAsync(b + sc_at, P->d_scales, scales_bytes, hipMemcpyDeviceToHost, s);
    const hipError_t e_sync = hipStreamSynchronize(s);
    if (e == hipSuccess) e = e_sync;
    if (e != hipSuccess) { patch_note_hip_error((int)e); return PATCH_ERR_HIP; }
    SavedHeader h = {};
    memcpy(h.magic, kSavedMagic4, 8);
    h.layout = kSavedLayout;
    h.tile = (uint32_t)P->tile;
    h.N = P->N;
    h.K = P->K;
    h.map_bytes = P->tile_map.size();
    h.payload_bytes = P->payload_bytes;
    h.aux_bytes = scales_bytes;
    h.checksum = fnv1a(b + sc_at, scales_bytes, fnv1a(b + pay_at, P->payload_bytes, fnv1a(b + map_at, P->tile_map.size(), kFnvBasis)));
    memcpy(b, &h, sizeof(h));
    return PATCH_OK;
}

patch_status patch_deserialize4(const void* buf, size_t bytes, void* stream, patch_packed4** out) {
    if (!buf || !out) return PATCH_ERR_ARG;
    if (bytes < saved_round(sizeof(SavedHeader))) return PATCH_ERR_SIZE;
    const uint8_t* b = static_cast<const uint8_t*>(buf);
    SavedHeader h;
    memcpy(&h, b, sizeof(h));
    if (memcmp(h.magic, kSavedMagic4, 8) != 0 || h.layout != kSavedLayout) return PATCH_ERR_ARG;
    if (h.N <= 0 || h.K <= 0) return PATCH_ERR_ARG;
    if ((h.tile != 64 && h.tile != 128) || h.N % h.tile || h.K % h.tile || h.N / h.tile > (1 << 20) || h.K / h.tile > (1 << 20))
        return PATCH_ERR_SHAPE;
    const uint64_t Tk = (uint64_t)(h.K / h.tile), T = (uint64_t)(h.N / h.tile) * Tk;
    if (h.map_bytes != T || h.aux_bytes != (uint64_t)h.N * Tk * sizeof(uint16_t)) return PATCH_ERR_ARG;
    const size_t map_at = saved_round(sizeof(SavedHeader)), pay_at = map_at + saved_round((size_t)T);
    if (bytes < pay_at || h.payload_bytes > bytes - pay_at) return PATCH_ERR_SIZE;
    const size_t sc_at = pay_at + saved_round((size_t)h.payload_bytes);
    if (bytes < sc_at || h.aux_bytes > bytes - sc_at) return PATCH_ERR_SIZE;
    for (uint64_t i = 0; i < T; ++i)
        if (b[map_at + i] > 1) return PATCH_ERR_ARG;
    if (fnv1a(b + sc_at, (size_t)h.aux_bytes, fnv1a(b + pay_at, (size_t)h.payload_bytes, fnv1a(b + map_at, (size_t)T, kFnvBasis))) != h.checksum)
        return PATCH_ERR_ARG;
    hipStream_t s = static_cast<hipStream_t>(stream);
    patch_packed4* P = nullptr;
    const patch_status st = new_packed4(h.N, h.K, b + map_at, (int)h.tile, s, &P);
    if (st != PATCH_OK) return st;
    if (P->payload_bytes != h.payload_bytes) {   // the map decides the size: a header that disagrees is not ours
        patch_free4(P);
        return PATCH_ERR_ARG;
    }
    hipError_t e = hipMemcpyAsync(P->d_payload, b + pay_at, P->payload_bytes, hipMemcpyHostToDevice, s);
    if (e == hipSuccess) e = hipMemcpyAsync(P->d_scales, b + sc_at, (size_t)h.aux_bytes, hipMemcpyHostToDevice, s);
    const hipError_t e_sync = hipStreamSynchronize(s);   // the caller's buffer is free to go when the call returns
    if (e == hipSuccess) e = e_sync;
    if (e != hipSuccess) {
        patch_note_hip_error((int)e);
        patch_free4(P);
        return PATCH_ERR_HIP;
    }
    *out = P;
    return PATCH_OK;
}

patch_status patch_unpack4(const patch_packed4* P, void* W_deq, void* codes, void* scales, void* stream) {
    if (!P || (!W_deq && !codes && !scales)) return PATCH_ERR_ARG;
    if ((W_deq && !q4_aligned16(W_deq)) || (scales && (reinterpret_cast<uintptr_t>(scales) & 1u))) return PATCH_ERR_ARG;
    hipLaunchKernelGGL(unpack4_kernel, dim3((unsigned)(P->Tn * P->Tk)), dim3(256), 0, static_cast<hipStream_t>(stream), P->d_payload, P->d_scales,
                       P->d_table, P->Tk, P->tile, P->K, static_cast<uint16_t*>(W_deq), static_cast<int8_t*>(codes), static_cast<uint16_t*>(scales));
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) { patch_note_hip_error((int)e); return PATCH_ERR_HIP; }
    return PATCH_OK;
}

patch_status patch_gemm4_many(const void* X, int64_t M, const patch_packed4* const* P, void* const* Y, int count, void* stream) {
    if (!X || !P || !Y || M < 0 || count < 1 || count > PATCH_MAX_MANY) return PATCH_ERR_ARG;
    static_assert(PATCH_MAX_MANY == kMaxMany, "header and kernels disagree");
    if (!q4_aligned16(X)) return PATCH_ERR_ARG;
    for (int i = 0; i < count; ++i) {
        if (!P[i] || !Y[i] || !q4_aligned16(Y[i])) return PATCH_ERR_ARG;
        if (P[i]->K != P[0]->K || P[i]->tile != P[0]->tile) return PATCH_ERR_SHAPE;
    }
    if (M == 0) return PATCH_OK;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const patch_packed4* P0 = P[0];
    const int total = P0->Tk * (P0->tile / kStepCols);
    int first[kMaxMany], total_strips = 0;
    for (int i = 0; i < count; ++i) {
        first[i] = total_strips;
        total_strips += (int)(P[i]->N / kStripRows);
    }
    // One launch per pass of up to 64 rows (1, 2 or 4 blocks of 16), R strips per workgroup (q4_strips_per_group).
    auto run = [&](const auto& set) {
        for (int64_t m0 = 0; m0 < M; m0 += kQ4Rows) {
            const int rows = (int)(M - m0 < kQ4Rows ? M - m0 : kQ4Rows);
            const int RB = rows <= 16 ? 1 : rows <= 32 ? 2 : 4;
            const int R = q4_strips_per_group(total_strips, P0->n_cus, rows);
            const int groups = (total_strips + R - 1) / R;
            // wavefronts per workgroup: about 4 steps each, at least 4, at most 16 (8 with many registers); with more
            // workgroups than compute units half of that, so that two workgroups share a compute unit (its registers
            // hold 16 of these wavefronts) instead of running one after the other
            int kw = (total + 3) / 4;
            if (kw > q4_max_waves(R, RB)) kw = q4_max_waves(R, RB);
            if (groups > P0->n_cus && kw > 8) kw = 8;
            if (kw < 4) kw = 4;
            if (P0->tile == 128) launch_decode4_r<128>(R, RB, static_cast<const uint16_t*>(X), m0, rows, P0->K, P0->Tk, set, groups, kw, s);
            else launch_decode4_r<64>(R, RB, static_cast<const uint16_t*>(X), m0, rows, P0->K, P0->Tk, set, groups, kw, s);
        }
    };
    auto fill = [&](auto& set) {
        for (int i = 0; i < count; ++i) {
            set.payload[i] = P[i]->d_payload;
            set.scales[i] = P[i]->d_scales;
            set.table[i] = P[i]->d_table;
            set.Y[i] = static_cast<float*>(Y[i]);
            set.N[i] = P[i]->N;
            set.first[i] = first[i];
        }
        set.count = count;
        set.total = total_strips;
    };
    // the fewer kernel arguments the better: a set of one, of up to three (q / k / v, gate / up), of up to eight
    if (count == 1) {
        run(Q4One{P0->d_payload, P0->d_scales, P0->d_table, static_cast<float*>(Y[0]), P0->N});
    } else if (count <= 3) {
        Q4Set<3> set = {};
        fill(set);
        run(set);
    } else {
        Q4Set<kMaxMany> set = {};
        fill(set);
        run(set);
    }
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) { patch_note_hip_error((int)e); return PATCH_ERR_HIP; }
    return PATCH_OK;
}

patch_status patch_gemm4(const void* X, int64_t M, const patch_packed4* P, void* Y, void* stream) {
    return patch_gemm4_ex(X, M, P, Y, nullptr, 0, stream);
}

// Passes of up to 64 rows (the decode-shaped kernel) or the prefill-shaped kernel?  Both sides are
// estimated from measured rates, as for the bf16 kernels:
//   pass of r rows   rounds x (x(r) + R) x 0.05 us x 64-column steps, the terms of q4_strips_per_group (a workgroup
//                    loads all of X whatever R is); 64 rows: 4096^2 17.8 us, 11008 x 4096 21.9, 13824 x 5120 44.5
//   prefill kernel   rounds x steps per workgroup x (t0 + t1 fill) us + 3, fill = min(1, workgroups / compute units),
//                    for blocks of 128 and of 256 rows (the dequantization makes a step 0.2 - 0.4 us longer than the
//                    bf16 kernel's), + for a split 3 + (2 split + 1) M N 4 B / 5.5 TB/s; splits of at most 8 slices of at
//                    least 512 columns
// Returns the split to launch the prefill kernel with (and the block height), or 0 for passes.
static double q4_pass_us(int strips, int n_cus, int rows, int steps) {
    const int R = q4_strips_per_group(strips, n_cus, rows);
    const int groups = (strips + R - 1) / R;
    const double x = rows <= 16 ? 0.15 + 0.045 * rows : rows <= 32 ? 1.7 : 1.7 + 2.8 * (rows - 32) / 32.0;   // 4.5 at 64 rows
    const double rounds = groups <= 2 * n_cus ? (double)((groups + n_cus - 1) / n_cus) : (double)groups / n_cus + 0.5;
    return rounds * (x + R) * 0.05 * steps;
}

static int q4_prefill_split(int64_t M, const patch_packed4* P, const GemmArgs& a, int* bm_out) {
    *bm_out = 128;
    if (M <= 16) return 0;
    const int kpt = P->tile / 64, steps = P->Tk * kpt, strips = (int)(P->N / 16);
    const int64_t full = M / kQ4Rows;
    const int rest = (int)(M % kQ4Rows);
    const double passes_us = (double)full * q4_pass_us(strips, P->n_cus, kQ4Rows, steps) + (rest ? q4_pass_us(strips, P->n_cus, rest, steps) : 0.0);
    const size_t per_slice = (size_t)M * (size_t)P->N * sizeof(float);
    const int fit = a.ws ? (int)(a.ws_bytes / per_slice < 8 ? a.ws_bytes / per_slice : 8) : 1;
    const int longest = P->Tk * P->tile / 512;
    int best_split = 1;
    double best = 0.0;
    bool first = true;
    for (int bm : {128, 256}) {
        const int blocks = (int)((P->N + kP4BN - 1) / kP4BN) * (int)((M + bm - 1) / bm);
        // a step of 256 rows dequantizes the same codes for twice the rows: 1.2 + 0.47 fill us against 0.88 + 0.2 fill
        // (fitted to unsplit launches of 16 .. 256 workgroups); it pays once 128-row blocks would need a second round
        const double t0 = bm == 128 ? 0.88 : 1.2, t1 = bm == 128 ? 0.2 : 0.47;
        for (int sp = 1; sp <= 8 && (sp == 1 || (sp <= fit && sp <= longest)); ++sp) {
            const int wgs = blocks * sp;
            const int rounds = (wgs + P->n_cus - 1) / P->n_cus;
            const double fill = wgs < P->n_cus ? (double)wgs / P->n_cus : 1.0;
            double us = rounds * ((P->Tk + sp - 1) / sp) * kpt * (t0 + t1 * fill) + 3.0;
            if (sp > 1) us += 3.0 + (2.0 * sp + 1.0) * (double)per_slice / 5.5e6;
            if (first || us < best) { best = us; best_split = sp; *bm_out = bm; first = false; }
        }
    }
    return best < passes_us ? best_split : 0;
}

patch_status patch_gemm4_ex(const void* X, int64_t M, const patch_packed4* P, void* Y, void* workspace, size_t workspace_bytes,
                            void* stream) {
    if (!X || !P || !Y || M < 0) return PATCH_ERR_ARG;
    if (!q4_aligned16(X) || !q4_aligned16(Y) || (workspace && !q4_aligned16(workspace))) return PATCH_ERR_ARG;
    if (M == 0) return PATCH_OK;
    const bool ws = workspace && workspace_bytes >= 2 * (size_t)M * (size_t)P->N * sizeof(float);
    GemmArgs a = {};
    a.M = M; a.N = P->N; a.K = P->K;
    a.tile = P->tile; a.Tn = P->Tn; a.Tk = P->Tk;
    a.n_cus = P->n_cus;
    if (ws) { a.ws = static_cast<float*>(workspace); a.ws_bytes = workspace_bytes; }
    int bm = 128;
    const int split = q4_prefill_split(M, P, a, &bm);
    if (split == 0) return patch_gemm4_many(X, M, &P, &Y, 1, stream);
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int tiles_n = (int)((P->N + kP4BN - 1) / kP4BN), tiles_m = (int)((M + bm - 1) / bm);
    const int grid = ((tiles_n * tiles_m + 7) / 8) * 8;
    const int lds_bytes = 2 * bm * 128;
    const uint16_t* Xp = static_cast<const uint16_t*>(X);
    auto launch = [&](auto whole, auto sliced) {
        if (split == 1) {
            hipLaunchKernelGGL(whole, dim3(grid), dim3(512), lds_bytes, s, Xp, M, P->N, P->K, P->d_payload, P->d_scales, P->d_table, P->Tk, tiles_n,
                               tiles_m, static_cast<float*>(Y));
        } else {
            hipLaunchKernelGGL(sliced, dim3(grid, split), dim3(512), lds_bytes, s, Xp, M, P->N, P->K, P->d_payload, P->d_scales, P->d_table, P->Tk,
                               tiles_n, tiles_m, a.ws);
            wr_reduce(a.ws, (size_t)M * (size_t)P->N / 4, split, static_cast<float*>(Y), 0, s);
        }
    };
    if (P->tile == 128 && bm == 128) launch(prefill4_kernel<128, 128, false>, prefill4_kernel<128, 128, true>);
    else if (P->tile == 128) launch(prefill4_kernel<128, 256, false>, prefill4_kernel<128, 256, true>);
    else if (bm == 128) launch(prefill4_kernel<64, 128, false>, prefill4_kernel<64, 128, true>);
    else launch(prefill4_kernel<64, 256, false>, prefill4_kernel<64, 256, true>);
    const hipError_t err = hipGetLastError();
    if (err != hipSuccess) { patch_note_hip_error((int)err); return PATCH_ERR_HIP; }
    return PATCH_OK;
}

patch_status patch_pack_from4(const patch_packed4* P4, void* stream, patch_packed** out) {
    if (!P4 || !out) return PATCH_ERR_ARG;
    uint16_t* W_deq = nullptr;
    if (hipMalloc(&W_deq, (size_t)P4->N * (size_t)P4->K * sizeof(uint16_t)) != hipSuccess) {
        (void)hipGetLastError();
        return PATCH_ERR_ALLOC;
    }
    patch_status st = patch_unpack4(P4, W_deq, nullptr, nullptr, stream);
    // patch_pack runs on the same stream behind the dequantization and waits for the stream before it returns
    if (st == PATCH_OK) st = patch_pack(W_deq, P4->N, P4->K, P4->tile_map.data(), P4->tile, stream, out);
    else (void)hipStreamSynchronize(static_cast<hipStream_t>(stream));
    (void)hipFree(W_deq);
    return st;
}

size_t patch_packed4_bytes(const patch_packed4* P) { return P ? P->algorithmic_bytes : 0; }

patch_status patch_packed4_dims(const patch_packed4* P, int64_t* N, int64_t* K, int* tile, int64_t* n_sparse_tiles) {
    if (!P) return PATCH_ERR_ARG;
    if (N) *N = P->N;
    if (K) *K = P->K;
    if (tile) *tile = P->tile;
    if (n_sparse_tiles) *n_sparse_tiles = P->n_sparse;
    return PATCH_OK;
}

}  // extern "C"
