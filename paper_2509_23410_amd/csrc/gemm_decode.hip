// Decode-shaped hybrid GEMM (at most 16 rows of X per launch) with split-K across the wavefronts of a
// workgroup and a fixed-order fp32 reduction through LDS.  This is the product Y = X * W_hat^T of Section 4 /
// Appendix A of the paper for the decoding input (batch x K), with "split-K" as the schedule Appendix A names.
//
// Mapping.  The weight is the A operand (the sparse operand of the gfx950 sparse matrix instruction is A),
// so the kernel computes Y^T = W_hat * X^T.  A workgroup owns one strip of 16 output features; its
// wavefronts split K into contiguous slices of NK 64-column steps.  The path is HBM-bound, so it is built
// around the memory system: a wavefront first issues ALL weight loads of its slice (128-bit, non-temporal,
// register-order storage from layout.h, so every byte is requested exactly once and as early as possible),
// interleaved with the loads of its slice of X (L2 hits), and only then runs its matrix instructions.
// Fewer, fatter wavefronts (16 KB of weights in flight each) measured faster than many thin ones.
// Per 64-column step the wavefront takes ONE scalar branch on the tile type:
//   dense : 2 x v_mfma_f32_16x16x32_bf16
//   2:4   : 1 x v_smfmac_f32_16x16x64_bf16
// The partial accumulators of the wavefronts meet in LDS and are summed in slice order, so results are
// bit-reproducible; there is no global workspace, no atomics and no second launch.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "epilogue.h"
#include "kernels.h"
#include "layout.h"

namespace patch {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

union AFrag { u32x4 raw; bf16x8 v; };
union BFrag { u32x4 raw[2]; bf16x8 h[2]; bf16x16 v; };

__device__ __forceinline__ uint64_t uniform64(uint64_t v) {
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v), hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
    return ((uint64_t)hi << 32) | lo;
}

// dst[lane] = v[lane + S] within each row of 16 lanes (S = 0 .. 15): a DPP row rotation (row_ror:n delivers
// src[lane - n], measured), one instruction per dword.
template <int S>
__device__ __forceinline__ u32x4 rows_up(u32x4 v) {
    if constexpr (S == 0) return v;
    u32x4 r;
#pragma unroll
    for (int i = 0; i < 4; ++i) r[i] = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v[i], 0x120 + ((16 - S) & 15), 0xF, 0xF, false);
    return r;
}
__device__ __forceinline__ u32x4 rows_up(u32x4 v, int s) {   // s is a constant once the caller's loop is unrolled
    switch (s) {
        case 1: return rows_up<1>(v);
        case 2: return rows_up<2>(v);
        case 3: return rows_up<3>(v);
        case 4: return rows_up<4>(v);
        case 5: return rows_up<5>(v);
        case 6: return rows_up<6>(v);
        case 7: return rows_up<7>(v);
        case 8: return rows_up<8>(v);
        case 9: return rows_up<9>(v);
        case 10: return rows_up<10>(v);
        case 11: return rows_up<11>(v);
        case 12: return rows_up<12>(v);
        case 13: return rows_up<13>(v);
        case 14: return rows_up<14>(v);
        case 15: return rows_up<15>(v);
        default: return v;
    }
}

// RB = blocks of 16 rows of X per launch (1, 2 or 4): the weights are streamed once for up to 64 rows.
// SetT = DecodeSet (up to 8 weights sharing X) or WeightOne (a single weight: short kernel arguments, no selection).
// XR = 16: every step loads its two X operands with two instructions, in the lanes the matrix instruction reads
//      them from (16 columns = rows of X, 4 lane groups = 8 elements of K each).
// XR = 1, 2, 4, 8 (at most XR rows, RB = 1): with few rows most of those lanes are idle, and a load instruction costs
//      its turn in the memory pipeline however few lanes it has.  The 16 columns then hold 16 / XR operands of XR rows
//      each - column c = operand c / XR (K-step (c / XR) / 2 of the load, half (c / XR) % 2), row c % XR - so one
//      instruction fetches X for 8 / XR steps, and each step rotates its two operands down to columns 0 .. XR - 1
//      (four DPP moves each).  Columns XR .. 15 of the product are then other steps' leftovers; they are never stored.
template <int TILE, int NK, int MAXW, int RB, typename SetT, int XR = 16>
__global__ __launch_bounds__(MAXW * 64) void decode_kernel(const uint16_t* __restrict__ X, int64_t m0, int rows, int64_t K, int Tk,
                                                           const SetT set, int ybf16) {
    constexpr bool kOne = sizeof(SetT) == sizeof(WeightOne);
    constexpr int KPT = TILE / kStepCols, SPT = TILE / kStripRows;
    constexpr bool kWide = XR < 16;
    static_assert(!kWide || RB == 1, "several steps per X load: one row block only");
    constexpr int SPL = kWide ? 8 / XR : 1;               // steps served by one X load
    constexpr int NL = kWide ? (NK + SPL - 1) / SPL : 1;   // X loads per pass
    __shared__ f32x4 red[MAXW][RB][64];

    const int tid = threadIdx.x, lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int KW = blockDim.x >> 6;
    // which weight of the set this strip belongs to: scalar selects over the (at most 8) candidates, so that every
    // pointer stays in scalar registers
    const uint8_t* __restrict__ payload;
    const uint32_t* __restrict__ table;
    float* __restrict__ Y;
    int64_t N;
    int first = 0;
    if constexpr (kOne) {
        payload = set.payload;
        table = set.table;
        Y = set.Y;
        N = set.N;
    } else {
        payload = set.payload[0];
        table = set.table[0];
        Y = set.Y[0];
        N = set.N[0];
        if (set.count > 1)
#pragma unroll
        for (int i = 1; i < kMaxMany; ++i) {
            const bool here = i < set.count && (int)blockIdx.x >= set.first[i];
            payload = here ? set.payload[i] : payload;
            table = here ? set.table[i] : table;
            Y = here ? set.Y[i] : Y;
            N = here ? set.N[i] : N;
            first = here ? set.first[i] : first;
        }
        // the selects above are wavefront-uniform; say so (the weight addresses below must be scalar)
        payload = reinterpret_cast<const uint8_t*>(uniform64(reinterpret_cast<uint64_t>(payload)));
        table = reinterpret_cast<const uint32_t*>(uniform64(reinterpret_cast<uint64_t>(table)));
        Y = reinterpret_cast<float*>(uniform64(reinterpret_cast<uint64_t>(Y)));
        N = (int64_t)uniform64((uint64_t)N);
    }
    const int strip = (int)blockIdx.x - __builtin_amdgcn_readfirstlane(first);
    const int tn = strip / SPT, s = strip % SPT;
    const int col = lane & 15, q = lane >> 4;
    const bool xvalid = col < rows;   // row block 0; block rb holds rows 16 rb + col
    const uint32_t* trow = table + (int64_t)tn * Tk;
    const int total = Tk * KPT;
    // per-lane byte offsets, fixed for the whole kernel; every address below is a scalar base plus one of these
    const uint32_t voff = lane * 16, voffm = lane * KPT * 2;
    const uint32_t voffx = (uint32_t)(((xvalid ? col : 0) * K + 8 * q) * 2);
    const uint8_t* xbase = reinterpret_cast<const uint8_t*>(X + m0 * K);
    // lanes whose column is a row of X; the other lanes never load X and never store
    const uint64_t xmask = __builtin_amdgcn_ballot_w64(xvalid);

    // several steps per load: this lane's operand (step xs of the load, half xh) and row xr
    const int xcw = col / (kWide ? XR : 16), xr = col % (kWide ? XR : 16);
    const int xs = xcw >> 1;
    const uint32_t voffxw = (uint32_t)(((xr < rows ? xr : 0) * K + xs * kStepCols + (xcw & 1) * 32 + 8 * q) * 2);

    // the same for the further row blocks (RB > 1)
    uint32_t voffx_r[RB];
    uint64_t xmask_r[RB];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
        const bool v = 16 * rb + col < rows;
        voffx_r[rb] = (uint32_t)(((v ? 16 * rb + col : 0) * K + 8 * q) * 2);
        xmask_r[rb] = __builtin_amdgcn_ballot_w64(v);
    }
    f32x4 acc[RB];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) acc[rb] = f32x4{0.f, 0.f, 0.f, 0.f};
    for (int base = w * NK; base < total; base += KW * NK) {
        const int n = (total - base < NK) ? total - base : NK;
        uint32_t ent[NK];
#pragma unroll
        for (int g = 0; g < NK; ++g) {
            // scalar load by hand: the table pointer comes out of a select, and the compiler would fall back to
            // vector loads (and vector registers for everything derived from the entries)
            const uint32_t off = (uint32_t)(((g < n) ? base + g : base) / KPT) * 4u;
            asm volatile("s_load_dword %0, %1, %2" : "=s"(ent[g]) : "s"(trow), "s"(off));
        }
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
        for (int g = 0; g < NK; ++g) asm volatile("" : "+s"(ent[g]));

        // ---- every byte of the slice is requested now, weights and X interleaved step by step (issuing the X
        // loads after all the weight loads measured 1.2 us slower).  One asm block per step: the compiler can
        // neither sink these loads into the branches that consume them nor wait for them one by one.  A load
        // the step does not need (second half of a 2:4 step, positions of a dense step, anything past the end of
        // K) is jumped over by a scalar branch inside the block and leaves the zero its destination was initialised
        // with (issuing it with an empty EXEC mask instead still costs an instruction's turn in the memory pipeline:
        // all-2:4 maps at M = 1 went from 6.5 to 6.0 us on 4096 x 4096 and from 13.4 to 11.6 us on 11008 x 4096); X is loaded by the lanes that have a row only.
        u32x4 a[NK][2], b[kWide ? 1 : NK][RB][2], xl[NL];
        uint32_t idx[NK];
        // several steps per X load: these loads go first, so that they are the oldest in flight and their operands
        // can be moved into place while the weights are still on their way.  Lanes whose step lies past the end of K
        // or whose row does not exist are masked out and keep their zero; nothing is issued when no lane is left.
#pragma unroll
        for (int i = 0; i < NL; ++i) {
            xl[i] = u32x4{0u, 0u, 0u, 0u};
            if constexpr (kWide) {
                const uint64_t xm = __builtin_amdgcn_ballot_w64(xr < rows && i * SPL + xs < n);
                uint64_t saved;
                asm volatile(
                    "s_mov_b64 %[sv], exec\n\t"
                    "s_mov_b64 exec, %[xm]\n\t"
                    "s_cbranch_execz 1f\n\t"
                    "global_load_dwordx4 %[x0], %[vx], %[sbx]\n\t"
                    "1:\n\t"
                    "s_mov_b64 exec, %[sv]"
                    : [x0] "+v"(xl[i]), [sv] "=&s"(saved)
                    : [vx] "v"(voffxw), [sbx] "s"(xbase + (size_t)(base + i * SPL) * (kStepCols * 2)), [xm] "s"(xm)
                    : "memory");
            }
        }
#pragma unroll
        for (int g = 0; g < NK; ++g) {
            const int k = (g < n) ? base + g : base;
            const int j = k % KPT;
            const uint32_t e = ent[g];
            const int kind = (g < n) ? (int)(e & 1u) + 1 : 0;  // 0 = past the end, 1 = dense, 2 = 2:4
            const uint8_t* tb = payload + entry_offset(e);
            const uint8_t* sb0 = tb + (size_t)(s * KPT + j) * ((e & 1u) ? kSparseFragBytes : kDenseFragBytes);
            // positions: one 16-bit word per lane and step; with two steps per tile the even step fetches the
            // lane's dword for both (a fully used 256-byte row) and the odd step takes its upper half
            const uint8_t* sbm = tb + sparse_vals_bytes(TILE) + (s * 64 * KPT) * 2;
            const int mkind = (KPT == 2 && (g & 1)) ? 0 : kind;
            const uint8_t* sbx = xbase + (size_t)k * (kStepCols * 2);
            u32x4 v0 = {0u, 0u, 0u, 0u}, v1 = {0u, 0u, 0u, 0u}, x0 = {0u, 0u, 0u, 0u}, x1 = {0u, 0u, 0u, 0u};
            uint32_t vi = 0;
            uint64_t saved;
// One step's loads.  LDM is the mnemonic of the positions load (16 or 32 bits per lane).
#define PATCH_DECODE_WEIGHT_LOADS(LDM)                                                                            \
        "s_cmp_eq_u32 %[kind], 0\n\t"                                                                             \
        "s_cbranch_scc1 3f\n\t"                                                                                   \
        "global_load_dwordx4 %[v0], %[vo], %[sb0] nt\n\t"                                                         \
        "s_cmp_eq_u32 %[kind], 1\n\t"                                                                             \
        "s_cbranch_scc0 1f\n\t"                                                                                   \
        "global_load_dwordx4 %[v1], %[vo], %[sb0] offset:1024 nt\n\t"                                             \
        "1:\n\t"                                                                                                  \
        "s_cmp_eq_u32 %[mkind], 2\n\t"                                                                            \
        "s_cbranch_scc0 2f\n\t"                                                                                   \
        LDM " %[vi], %[vm], %[sbm] nt\n\t"                                                                        \
        "2:\n\t"
#define PATCH_DECODE_STEP_LOADS(LDM)                                                                              \
    asm volatile(                                                                                                 \
        PATCH_DECODE_WEIGHT_LOADS(LDM)                                                                            \
        "s_mov_b64 %[sv], exec\n\t"                                                                               \
        "s_mov_b64 exec, %[xm]\n\t"                                                                               \
        "global_load_dwordx4 %[x0], %[vx], %[sbx]\n\t"                                                            \
        "global_load_dwordx4 %[x1], %[vx], %[sbx] offset:64\n\t"                                                  \
        "s_mov_b64 exec, %[sv]\n\t"                                                                               \
        "3:"                                                                                                       \
        : [v0] "+v"(v0), [v1] "+v"(v1), [vi] "+v"(vi), [x0] "+v"(x0), [x1] "+v"(x1), [sv] "=&s"(saved)            \
        : [vo] "v"(voff), [vm] "v"(voffm), [vx] "v"(voffx), [sb0] "s"(sb0), [sbm] "s"(sbm), [sbx] "s"(sbx),       \
          [kind] "s"(kind), [mkind] "s"(mkind), [xm] "s"(xmask)                                                   \
        : "memory", "scc")
// The same without X (several steps per X load: issued ahead of the steps).
#define PATCH_DECODE_STEP_LOADS_W(LDM)                                                                            \
    asm volatile(                                                                                                 \
        PATCH_DECODE_WEIGHT_LOADS(LDM)                                                                            \
        "3:"                                                                                                       \
        : [v0] "+v"(v0), [v1] "+v"(v1), [vi] "+v"(vi)                                                             \
        : [vo] "v"(voff), [vm] "v"(voffm), [sb0] "s"(sb0), [sbm] "s"(sbm), [kind] "s"(kind), [mkind] "s"(mkind)   \
        : "memory", "scc")
            if constexpr (kWide) {
                if constexpr (KPT == 2) { PATCH_DECODE_STEP_LOADS_W("global_load_dword"); }
                else { PATCH_DECODE_STEP_LOADS_W("global_load_ushort"); }
            } else {
                if constexpr (KPT == 2) { PATCH_DECODE_STEP_LOADS("global_load_dword"); }
                else { PATCH_DECODE_STEP_LOADS("global_load_ushort"); }
                b[g][0][0] = x0;
                b[g][0][1] = x1;
            }
#undef PATCH_DECODE_STEP_LOADS
#undef PATCH_DECODE_STEP_LOADS_W
#undef PATCH_DECODE_WEIGHT_LOADS
            a[g][0] = v0;
            a[g][1] = v1;
            idx[g] = vi;
            // X of the further row blocks: same step, same scalar base, the block's own lanes and rows
#pragma unroll
            for (int rb = 1; rb < RB; ++rb) {
                u32x4 y0 = {0u, 0u, 0u, 0u}, y1 = {0u, 0u, 0u, 0u};
                asm volatile(
                    "s_mov_b64 %[sv], exec\n\t"
                    "s_cmp_lg_u32 %[kind], 0\n\t"
                    "s_cselect_b64 exec, %[xm], 0\n\t"
                    "global_load_dwordx4 %[x0], %[vx], %[sbx]\n\t"
                    "global_load_dwordx4 %[x1], %[vx], %[sbx] offset:64\n\t"
                    "s_mov_b64 exec, %[sv]"
                    : [x0] "+v"(y0), [x1] "+v"(y1), [sv] "=&s"(saved)
                    : [vx] "v"(voffx_r[rb]), [sbx] "s"(sbx), [kind] "s"(kind), [xm] "s"(xmask_r[rb])
                    : "memory", "scc");
                b[g][rb][0] = y0;
                b[g][rb][1] = y1;
            }
        }
        // ---- wait for the loads (the compiler does not know about them), then tie every destination to this
        // point so that no use can be scheduled above the wait
        u32x4 bw[kWide ? NK : 1][2];
        if constexpr (kWide) {
            // every live step has issued at least one weight load since: once no more than NK loads are outstanding
            // the X loads (the oldest) have landed.  Their operands move into place under the weights' latency.
            if (n == NK) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(NK) : "memory");
            else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
#pragma unroll
            for (int i = 0; i < NL; ++i) asm volatile("" : "+v"(xl[i]));
#pragma unroll
            for (int g = 0; g < NK; ++g) {
                bw[g][0] = rows_up(xl[g / SPL], 2 * (g % SPL) * XR);
                bw[g][1] = rows_up(xl[g / SPL], (2 * (g % SPL) + 1) * XR);
                asm volatile("" : "+v"(bw[g][0]), "+v"(bw[g][1]));
            }
        }
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
#pragma unroll
        for (int g = 0; g < NK; ++g)
        {
            asm volatile("" : "+v"(a[g][0]), "+v"(a[g][1]), "+v"(idx[g]));
            if constexpr (!kWide) {
#pragma unroll
                for (int rb = 0; rb < RB; ++rb) asm volatile("" : "+v"(b[g][rb][0]), "+v"(b[g][rb][1]));
            }
        }

#pragma unroll
        for (int g = 0; g < NK; ++g) {
            AFrag a0, a1;
            a0.raw = a[g][0];
            a1.raw = a[g][1];
            if (g < n) {
                // two steps per tile: the even step's dword holds both position words
                const uint32_t pos = (KPT == 2 && (g & 1)) ? (idx[g - 1] >> 16) : idx[g];
                const bool sp = entry_sparse(ent[g]);
#pragma unroll
                for (int rb = 0; rb < RB; ++rb) {
                    BFrag bb;
                    if constexpr (kWide) {
                        bb.raw[0] = bw[g][0];
                        bb.raw[1] = bw[g][1];
                    } else {
                        bb.raw[0] = b[g][rb][0];
                        bb.raw[1] = b[g][rb][1];
                    }
                    if (sp) {
                        acc[rb] = __builtin_amdgcn_smfmac_f32_16x16x64_bf16(a0.v, bb.v, acc[rb], (int)pos, 0, 0);
                    } else {
                        acc[rb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a0.v, bb.h[0], acc[rb], 0, 0, 0);
                        acc[rb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a1.v, bb.h[1], acc[rb], 0, 0, 0);
                    }
                }
            }
        }
    }

    // fixed-order reduction of the partials; acc[rb][r] = Y^T[strip*16 + 4 q + r][16 rb + col]
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) red[w][rb][lane] = acc[rb];
    __syncthreads();
    if (w == 0) {
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) {
            f32x4 sum = red[0][rb][lane];
            for (int i = 1; i < KW; ++i) {
                const f32x4 v = red[i][rb][lane];
                sum[0] += v[0]; sum[1] += v[1]; sum[2] += v[2]; sum[3] += v[3];
            }
            if (16 * rb + col < rows) store4(Y, (m0 + 16 * rb + col) * N + (int64_t)strip * 16 + 4 * q, sum, ybf16);
        }
    }
}

template <int TILE, typename SetT>
static void launch_decode_s(const GemmArgs& a, const SetT& set, int units, int64_t m0, int rows, int nk, int kw, int xr, hipStream_t stream) {
    dim3 grid((unsigned)units), block((unsigned)(kw * 64));
    if (rows > 32) hipLaunchKernelGGL((decode_kernel<TILE, 4, 8, 4, SetT>), grid, block, 0, stream, a.X, m0, rows, a.K, a.Tk, set, a.ybf16);
    else if (rows > 16) hipLaunchKernelGGL((decode_kernel<TILE, 4, 8, 2, SetT>), grid, block, 0, stream, a.X, m0, rows, a.K, a.Tk, set, a.ybf16);
    else if (xr == 16 && nk == 8) hipLaunchKernelGGL((decode_kernel<TILE, 8, 8, 1, SetT>), grid, block, 0, stream, a.X, m0, rows, a.K, a.Tk, set, a.ybf16);
    else if (xr == 16) hipLaunchKernelGGL((decode_kernel<TILE, 4, 16, 1, SetT>), grid, block, 0, stream, a.X, m0, rows, a.K, a.Tk, set, a.ybf16);
#define PATCH_DECODE_WIDE(XR_)                                                                                                               \
    else if (xr == XR_ && nk == 8)                                                                                                           \
        hipLaunchKernelGGL((decode_kernel<TILE, 8, 8, 1, SetT, XR_>), grid, block, 0, stream, a.X, m0, rows, a.K, a.Tk, set, a.ybf16);       \
    else if (xr == XR_)                                                                                                                      \
        hipLaunchKernelGGL((decode_kernel<TILE, 4, 16, 1, SetT, XR_>), grid, block, 0, stream, a.X, m0, rows, a.K, a.Tk, set, a.ybf16);
    PATCH_DECODE_WIDE(1)
    PATCH_DECODE_WIDE(4)
    PATCH_DECODE_WIDE(8)
#undef PATCH_DECODE_WIDE
}

template <int TILE>
static void launch_decode_t(const GemmArgs& a, const DecodeSet& set, int64_t m0, int rows, int nk, int kw, int xr, hipStream_t stream) {
    if (set.count == 1) {
        const WeightOne one = {set.payload[0], set.table[0], set.Y[0], set.N[0]};
        launch_decode_s<TILE>(a, one, set.units, m0, rows, nk, kw, xr, stream);
    } else {
        launch_decode_s<TILE>(a, set, set.units, m0, rows, nk, kw, xr, stream);
    }
}

// Schedule: NK = 64-column steps per wavefront and pass (8 or 4), KW = wavefronts per workgroup.
// split_k > 0 forces KW; variant 2 / 3 forces NK = 8 / 4.
// Default (measured, M = 1):
//   two or more workgroups per compute unit (N >= 8192): NK = 8, KW = 4 - three small workgroups share a compute unit
//     and overlap one's reduction and exit with the others' loads (11008 x 4096: 17.6 vs 19.9 us; 13824 x 5120:
//     25.8 vs 26.9 us);
//   about one workgroup per compute unit and a long K (>= 128 steps): NK = 4, KW = 16 - more, shorter passes per
//     wavefront (4096 x 11008: 16.3 vs 17.7 us);
//   else NK = 8 if that still leaves about four wavefronts per compute unit, else 4.
int launch_decode(const GemmArgs& a, int64_t m0, int rows, int split_k, int variant, hipStream_t stream) {
    DecodeSet set = {};
    set.payload[0] = a.payload;
    set.table[0] = a.table;
    set.Y[0] = a.Y;
    set.N[0] = a.N;
    set.count = 1;
    set.units = (int)(a.N / 16);
    return launch_decode_set(a, set, m0, rows, split_k, variant, stream);
}

int launch_decode_set(const GemmArgs& a, const DecodeSet& set, int64_t m0, int rows, int split_k, int variant, hipStream_t stream) {
    const int64_t strips = set.units;
    const int total = a.Tk * (a.tile / kStepCols);
    int nk = 0;
    if (variant == 2) nk = 8;
    else if (variant == 3) nk = 4;
    if (nk == 0 && split_k > 0) nk = ((total + split_k - 1) / split_k > 4) ? 8 : 4;
    int kw_default = 0;
    if (nk == 0 && rows <= 16) {
        if (strips >= 2 * (int64_t)a.n_cus) { nk = 8; kw_default = 4; }
        else if (total >= 128) nk = 4;
    }
    if (nk == 0) {
        int kw8 = (total + 7) / 8;
        if (kw8 > 8) kw8 = 8;
        nk = (strips * kw8 >= (int64_t)a.n_cus * 4) ? 8 : 4;
    }
    if (rows > 16) nk = 4;   // 17 .. 64 rows: 4 steps and 8 wavefronts (registers hold X for up to four row blocks)
    const int maxw = (nk == 4 && rows <= 16) ? 16 : 8;
    int kw = split_k > 0 ? split_k : kw_default > 0 ? kw_default : (total + nk - 1) / nk;
    if (kw > maxw) kw = maxw;
    if (kw < 1) kw = 1;
    // up to 8 rows: X of several steps per load instruction where 2:4 tiles are at least a quarter of the map (on an
    // all-dense map the X loads are a small part of the instructions and the two schedules measured equal within the
    // noise, at 5 .. 8 rows the old one 2 - 3 % ahead; all-2:4 maps gain 3 - 13 %, half-2:4 maps 0 - 6 %).  Variant 5
    // keeps the two loads per step, variant 6 asks for the new schedule whatever the map.
    const bool wide = rows <= 8 && variant != 5 && (variant == 6 || a.sparse_pct >= 25);
    const int xr = !wide ? 16 : rows == 1 ? 1 : rows <= 4 ? 4 : 8;
    if (a.tile == 128) launch_decode_t<128>(a, set, m0, rows, nk, kw, xr, stream);
    else launch_decode_t<64>(a, set, m0, rows, nk, kw, xr, stream);
    return kw;
}

}  // namespace patch
