// Hybrid GEMM for batched decoding: up to 64 rows of X per launch, meant for 12 and more (the product
// Y = X * W_hat^T of Section 4 / Appendix A of the paper between its decoding input, a few rows, and its prefill
// input, thousands).
//
// With more than 16 rows the decode mapping (one 16-feature strip per workgroup) re-reads X once per strip: at 64
// rows that is four times the weight bytes through every vector L1, and the L1 fill rate is what bounds these
// kernels.  Here a wavefront owns FOUR strips (64 features) and up to four 16-row blocks of X: every X operand it
// loads is used by four strips, so X costs as many bytes as the weights, not four times as many.
//
// Mapping.  Workgroup (g, c) = 64-feature group g x K-chunk c (whole tiles).  Its eight wavefronts take the chunk's
// steps in turn, two 64-column steps per pass; per pass a wavefront issues all its loads first (weights straight
// into registers in the stored register order, X from L2), then the matrix instructions: per strip one scalar
// branch on the tile type, dense 2 x v_mfma_f32_16x16x32_bf16 or 2:4 1 x v_smfmac_f32_16x16x64_bf16 per row block.
// The wavefronts' partial sums meet in LDS and are added in wavefront order.  With one chunk (gridDim.y = 1) the
// result goes to Y; with several, chunk c writes rows x N partial sums to the workspace slice c and
// wr_reduce_kernel (gemm_prefill_wreg.hip) adds the slices in order: bit-reproducible either way.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "epilogue.h"
#include "kernels.h"
#include "layout.h"

namespace patch {

typedef __bf16 mid_bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 mid_bf16x16 __attribute__((ext_vector_type(16)));
typedef float mid_f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int mid_u32x4 __attribute__((ext_vector_type(4)));

union MidA { mid_u32x4 raw; mid_bf16x8 v; };
union MidB { mid_u32x4 raw[2]; mid_bf16x8 h[2]; mid_bf16x16 v; };

constexpr int kMidSB = 4;   // strips (16 features) per wavefront
constexpr int kMidNK = 2;   // 64-column steps per pass
constexpr int kMidKW = 8;   // wavefronts per workgroup: two per SIMD, one's loads overlap the other's matrix instructions

__device__ __forceinline__ uint64_t mid_uniform64(uint64_t v) {
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v), hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
    return ((uint64_t)hi << 32) | lo;
}

// RB = 16-row blocks of X (1: up to 16 rows, 2: up to 32, 4: up to 64).  SPLIT: gridDim.y K-chunks, partial sums to a workspace.
// Two 64-column steps per pass, all their loads in flight together; the register budget is held to two wavefronts
// per SIMD (243 registers at RB = 4), so a second workgroup's loads overlap this one's matrix instructions.
template <int TILE, int RB, bool SPLIT>
__global__ __launch_bounds__(kMidKW * 64) __attribute__((amdgpu_waves_per_eu(2, 2))) void mid_kernel(const uint16_t* __restrict__ X, int64_t m0, int rows, int64_t K, int Tk,
                                                          const WeightSet set, int ybf16) {
    constexpr int KPT = TILE / kStepCols, SPT = TILE / kStripRows, GPT = SPT / kMidSB;  // groups per tile row
    constexpr int SB = kMidSB, NK = kMidNK, KW = kMidKW;
    constexpr int KH = KW / 2;
    __shared__ mid_f32x4 red[KH][SB * RB][64];  // 64 KB at RB = 4: half of the wavefronts at a time

    const int tid = threadIdx.x, lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    // which weight of the set this group belongs to: scalar selects, made explicitly uniform
    const uint8_t* __restrict__ payload = set.payload[0];
    const uint32_t* __restrict__ table = set.table[0];
    float* __restrict__ Y = set.Y[0];
    int64_t N = set.N[0];
    int first = 0;
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
    payload = reinterpret_cast<const uint8_t*>(mid_uniform64(reinterpret_cast<uint64_t>(payload)));
    table = reinterpret_cast<const uint32_t*>(mid_uniform64(reinterpret_cast<uint64_t>(table)));
    Y = reinterpret_cast<float*>(mid_uniform64(reinterpret_cast<uint64_t>(Y)));
    N = (int64_t)mid_uniform64((uint64_t)N);
    const int grp = (int)blockIdx.x - __builtin_amdgcn_readfirstlane(first);
    const int tn = grp / GPT, s0 = (grp % GPT) * SB;  // tile row, first strip inside the tile
    const int col = lane & 15, q = lane >> 4;
    const uint32_t* trow = table + (int64_t)tn * Tk;
    // this workgroup's K-chunk, in whole tiles
    const int t_begin = SPLIT ? (int)((int64_t)blockIdx.y * Tk / gridDim.y) : 0;
    const int t_end = SPLIT ? (int)((int64_t)(blockIdx.y + 1) * Tk / gridDim.y) : Tk;
    const int c0 = t_begin * KPT, c1 = t_end * KPT;
    // per-lane byte offsets, fixed for the whole kernel; every address below is a scalar base plus one of these
    const uint32_t voff = lane * 16, voffm = lane * KPT * 2;
    const uint8_t* xbase = reinterpret_cast<const uint8_t*>(X + m0 * K);
    uint32_t voffx[RB];
    uint64_t xmask[RB];  // lanes whose column is a row of X; the others never load X and never store
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
        const bool v = 16 * rb + col < rows;
        voffx[rb] = (uint32_t)(((v ? 16 * rb + col : 0) * K + 8 * q) * 2);
        xmask[rb] = __builtin_amdgcn_ballot_w64(v);
    }
    mid_f32x4 acc[SB][RB];
#pragma unroll
    for (int sb = 0; sb < SB; ++sb)
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) acc[sb][rb] = mid_f32x4{0.f, 0.f, 0.f, 0.f};

    for (int base = c0 + w * NK; base < c1; base += KW * NK) {
        const int n = (c1 - base < NK) ? c1 - base : NK;
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

        // ---- every byte of the pass is requested now.  A load the step does not need (second half of a 2:4 step,
        // positions of a dense step, anything past the end of the chunk) is jumped over by a scalar branch inside
        // the asm block and leaves the zero its destination was initialised with; X is loaded by the lanes that
        // have a row only.
        mid_u32x4 a[NK][SB][2], b[NK][RB][2];
        uint32_t idx[NK][SB];
#pragma unroll
        for (int g = 0; g < NK; ++g) {
            const int k = (g < n) ? base + g : base;
            const int j = k % KPT;
            const uint32_t e = ent[g];
            const int kind = (g < n) ? (int)(e & 1u) + 1 : 0;  // 0 = past the end, 1 = dense, 2 = 2:4
            // positions: one 16-bit word per lane and step; with two steps per tile the even step fetches the
            // lane's dword for both and the odd step of the pass takes its upper half (a pass starts on an even step)
            const int mkind = (KPT == 2 && (g & 1)) ? 0 : kind;
            const uint8_t* tb = payload + entry_offset(e);
            uint64_t saved;
#pragma unroll
            for (int sb = 0; sb < SB; ++sb) {
                const int s = s0 + sb;
                const uint8_t* sbw = tb + (size_t)(s * KPT + j) * ((e & 1u) ? kSparseFragBytes : kDenseFragBytes);
                const uint8_t* sbm = tb + sparse_vals_bytes(TILE) + (s * 64 * KPT) * 2;
                mid_u32x4 v0 = {0u, 0u, 0u, 0u}, v1 = {0u, 0u, 0u, 0u};
                uint32_t vi = 0;
#define PATCH_MID_WEIGHT_LOADS(LDM)                                                                               \
    asm volatile(                                                                                                 \
        "s_cmp_eq_u32 %[kind], 0\n\t"                                                                             \
        "s_cbranch_scc1 3f\n\t"                                                                                   \
        "global_load_dwordx4 %[v0], %[vo], %[sbw] nt\n\t"                                                         \
        "s_cmp_eq_u32 %[kind], 1\n\t"                                                                             \
        "s_cbranch_scc0 1f\n\t"                                                                                   \
        "global_load_dwordx4 %[v1], %[vo], %[sbw] offset:1024 nt\n\t"                                             \
        "s_branch 3f\n\t"                                                                                         \
        "1:\n\t"                                                                                                  \
        "s_cmp_eq_u32 %[mkind], 2\n\t"                                                                            \
        "s_cbranch_scc0 3f\n\t"                                                                                   \
        LDM " %[vi], %[vm], %[sbm] nt\n\t"                                                                        \
        "3:"                                                                                                       \
        : [v0] "+v"(v0), [v1] "+v"(v1), [vi] "+v"(vi)                                                             \
        : [vo] "v"(voff), [vm] "v"(voffm), [sbw] "s"(sbw), [sbm] "s"(sbm), [kind] "s"(kind), [mkind] "s"(mkind)   \
        : "memory", "scc")
                if constexpr (KPT == 2) { PATCH_MID_WEIGHT_LOADS("global_load_dword"); }
                else { PATCH_MID_WEIGHT_LOADS("global_load_ushort"); }
#undef PATCH_MID_WEIGHT_LOADS
                a[g][sb][0] = v0;
                a[g][sb][1] = v1;
                idx[g][sb] = vi;
            }
            const uint8_t* sbx = xbase + (size_t)k * (kStepCols * 2);
#pragma unroll
            for (int rb = 0; rb < RB; ++rb) {
                mid_u32x4 x0 = {0u, 0u, 0u, 0u}, x1 = {0u, 0u, 0u, 0u};
                asm volatile(
                    "s_cmp_eq_u32 %[kind], 0\n\t"
                    "s_cbranch_scc1 1f\n\t"
                    "s_mov_b64 %[sv], exec\n\t"
                    "s_mov_b64 exec, %[xm]\n\t"
                    "global_load_dwordx4 %[x0], %[vx], %[sbx]\n\t"
                    "global_load_dwordx4 %[x1], %[vx], %[sbx] offset:64\n\t"
                    "s_mov_b64 exec, %[sv]\n\t"
                    "1:"
                    : [x0] "+v"(x0), [x1] "+v"(x1), [sv] "=&s"(saved)
                    : [vx] "v"(voffx[rb]), [sbx] "s"(sbx), [kind] "s"(kind), [xm] "s"(xmask[rb])
                    : "memory", "scc");
                b[g][rb][0] = x0;
                b[g][rb][1] = x1;
            }
        }
        // ---- wait for the loads (the compiler does not know about them), then tie every destination to this
        // point so that no use can be scheduled above the wait
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
#pragma unroll
        for (int g = 0; g < NK; ++g) {
#pragma unroll
            for (int sb = 0; sb < SB; ++sb) asm volatile("" : "+v"(a[g][sb][0]), "+v"(a[g][sb][1]), "+v"(idx[g][sb]));
#pragma unroll
            for (int rb = 0; rb < RB; ++rb) asm volatile("" : "+v"(b[g][rb][0]), "+v"(b[g][rb][1]));
        }

#pragma unroll
        for (int g = 0; g < NK; ++g) {
            if (g < n) {
                const bool sp = entry_sparse(ent[g]);
#pragma unroll
                for (int sb = 0; sb < SB; ++sb) {
                    MidA a0, a1;
                    a0.raw = a[g][sb][0];
                    a1.raw = a[g][sb][1];
                    const uint32_t pos = (KPT == 2 && (g & 1)) ? (idx[g - 1][sb] >> 16) : idx[g][sb];
#pragma unroll
                    for (int rb = 0; rb < RB; ++rb) {
                        MidB bb;
                        bb.raw[0] = b[g][rb][0];
                        bb.raw[1] = b[g][rb][1];
                        if (sp) {
                            acc[sb][rb] = __builtin_amdgcn_smfmac_f32_16x16x64_bf16(a0.v, bb.v, acc[sb][rb], (int)pos, 0, 0);
                        } else {
                            acc[sb][rb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a0.v, bb.h[0], acc[sb][rb], 0, 0, 0);
                            acc[sb][rb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a1.v, bb.h[1], acc[sb][rb], 0, 0, 0);
                        }
                    }
                }
            }
        }
    }

    // fixed-order sum of the wavefronts' partials; acc[sb][rb][r] = Y^T[64 grp + 16 sb + 4 q + r][16 rb + col].
    // First wavefront w + KH hands its partials to wavefront w, then the KH sums meet in LDS again and wavefront w
    // adds and stores the accumulator tiles t = w, w + KW, ... (t = sb * RB + rb): ((p0 + p4) + (p1 + p5)) + ...
    if (w >= KH) {
#pragma unroll
        for (int sb = 0; sb < SB; ++sb)
#pragma unroll
            for (int rb = 0; rb < RB; ++rb) red[w - KH][sb * RB + rb][lane] = acc[sb][rb];
    }
    __syncthreads();
    if (w < KH) {
#pragma unroll
        for (int sb = 0; sb < SB; ++sb)
#pragma unroll
            for (int rb = 0; rb < RB; ++rb) {
                const mid_f32x4 v = red[w][sb * RB + rb][lane];
                acc[sb][rb][0] += v[0]; acc[sb][rb][1] += v[1]; acc[sb][rb][2] += v[2]; acc[sb][rb][3] += v[3];
                red[w][sb * RB + rb][lane] = acc[sb][rb];  // the same lane wrote and reads this slot: no barrier between
            }
    }
    __syncthreads();
    // SPLIT: Y is the workspace, slices of rows x N fp32; else row m0 of Y (fp32 or bf16 elements)
    float* dst = SPLIT ? Y + (int64_t)blockIdx.y * rows * N : ybf16 ? reinterpret_cast<float*>(reinterpret_cast<uint16_t*>(Y) + m0 * N) : Y + m0 * N;
    for (int t = w; t < SB * RB; t += KW) {
        const int sb = t / RB, rb = t % RB;
        mid_f32x4 sum = red[0][t][lane];
#pragma unroll
        for (int i = 1; i < KH; ++i) {
            const mid_f32x4 v = red[i][t][lane];
            sum[0] += v[0]; sum[1] += v[1]; sum[2] += v[2]; sum[3] += v[3];
        }
        if (16 * rb + col < rows)   // partial sums of a K-chunk stay fp32; the sum over the chunks is rounded
            store4(dst, (int64_t)(16 * rb + col) * N + (int64_t)grp * 64 + 16 * sb + 4 * q, sum, SPLIT ? 0 : ybf16);
    }
}

// K-chunks per 64-feature group: as many as bring the workgroup count closest to one per compute unit, each at
// least two tiles long, at most 8, and no more than the workspace a.ws holds partial sums for (rows x N fp32 each).
// 1 = no split (no workspace needed).
int mid_split(const GemmArgs& a, int rows, int requested) {
    const int64_t groups = a.N / 64;
    int s = requested;
    if (s <= 0) {
        s = (int)((a.n_cus + groups / 2) / groups);
        // every chunk at least 512 columns long: with a short K (896 x 896) the strip kernel is faster than chunks of
        // 256 columns plus the second launch (7.7 against 8.6 us at 64 rows)
        const int longest = (int)((int64_t)a.Tk * a.tile / 512);
        if (s > longest) s = longest;
        if (s > 8) s = 8;
    }
    if (s > a.Tk) s = a.Tk;
    const size_t per_slice = (size_t)rows * (size_t)a.N * sizeof(float);
    const size_t fit = (a.ws && per_slice) ? a.ws_bytes / per_slice : 0;
    if ((size_t)s > fit) s = (int)fit;
    return s < 2 ? 1 : s;
}

template <int TILE>
static void launch_mid_t(const GemmArgs& a, const WeightSet& set, int64_t m0, int rows, int split, hipStream_t stream) {
    const dim3 block(kMidKW * 64);
    if (split > 1) {
        WeightSet part = set;
        part.Y[0] = a.ws;
        const dim3 grid((unsigned)set.units, (unsigned)split);
        if (rows <= 16) hipLaunchKernelGGL((mid_kernel<TILE, 1, true>), grid, block, 0, stream, a.X, m0, rows, a.K, a.Tk, part, 0);
        else if (rows <= 32) hipLaunchKernelGGL((mid_kernel<TILE, 2, true>), grid, block, 0, stream, a.X, m0, rows, a.K, a.Tk, part, 0);
        else hipLaunchKernelGGL((mid_kernel<TILE, 4, true>), grid, block, 0, stream, a.X, m0, rows, a.K, a.Tk, part, 0);
        float* y0 = a.ybf16 ? reinterpret_cast<float*>(reinterpret_cast<uint16_t*>(set.Y[0]) + m0 * set.N[0]) : set.Y[0] + m0 * set.N[0];
        wr_reduce(a.ws, (size_t)rows * (size_t)set.N[0] / 4, split, y0, a.ybf16, stream);
    } else {
        const dim3 grid((unsigned)set.units);
        if (rows <= 16) hipLaunchKernelGGL((mid_kernel<TILE, 1, false>), grid, block, 0, stream, a.X, m0, rows, a.K, a.Tk, set, a.ybf16);
        else if (rows <= 32) hipLaunchKernelGGL((mid_kernel<TILE, 2, false>), grid, block, 0, stream, a.X, m0, rows, a.K, a.Tk, set, a.ybf16);
        else hipLaunchKernelGGL((mid_kernel<TILE, 4, false>), grid, block, 0, stream, a.X, m0, rows, a.K, a.Tk, set, a.ybf16);
    }
}

// Up to 64 rows of X starting at row m0.  set.units / first[] count 64-feature groups.  A K split (split > 1) needs
// a single weight and a.ws with room for split x rows x N floats.
void launch_mid_set(const GemmArgs& a, const WeightSet& set, int64_t m0, int rows, int split, hipStream_t stream) {
    if (set.count != 1) split = 1;
    if (a.tile == 128) launch_mid_t<128>(a, set, m0, rows, split, stream);
    else launch_mid_t<64>(a, set, m0, rows, split, stream);
}

}  // namespace patch
