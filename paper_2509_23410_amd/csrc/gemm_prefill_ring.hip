// Prefill-shaped hybrid GEMM, main kernel for tile = 128 (Section 4 / Appendix A of the paper: the product for
// the prefill input, dense and 2:4 tiles mixed inside one launch).
//
// Workgroup = 256 output features (two tile rows) x 256 rows of X, 4 wavefronts (one per SIMD), K walked in
// 32-column steps through a ring of FOUR LDS stages filled by direct global->LDS loads three steps ahead:
//
//   step s:  wait until the loads of steps s and s+1 have landed | barrier | issue the loads of step s+3 into the
//            stage step s-1 just left | multiply stage s | meanwhile read the first operands of step s+1 from LDS
//
// so a step never starts by waiting for LDS, one barrier per step covers both the visibility of new data and the
// reuse of the old stage, and three stages (96 KB per CU) of loads are in flight.
//
// Every wavefront owns 64 features of tile row 0 AND 64 features of tile row 1 of the block (x 128 rows of X):
// whatever the types of the two tiles at a step, all four wavefronts carry the same matrix-instruction count, so
// the dense / 2:4 mix cannot unbalance the workgroup between two barriers.  The 16 accumulator tiles (32 x 32
// fp32 each) fill the 256 accumulation registers; all other state lives in the 256 ordinary vector registers.
//
// Per (32 features x 32 columns x 4 x 32 rows) one asm block holds the wavefront-uniform scalar branch:
//   2:4   : 4 x v_smfmac_f32_32x32x32_bf16
//   dense : 8 x v_mfma_f32_32x32x16_bf16
// in place (two-address), see mma_block4.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "kernels.h"
#include "layout.h"

namespace patch {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

union RA8 { u32x4 raw; bf16x8 v; };
union RB16 { u32x4 raw[2]; bf16x8 h[2]; bf16x16 v; };

constexpr int kRgBN = 256, kRgBM = 256;
constexpr int kRgStep = 32;                    // columns per step
constexpr int kRgAStage = 2 * 8 * 1024;        // [tile row][strip][1024 B]; a 2:4 tile row packs its strips at 512 B
constexpr int kRgBStage = kRgBM * 64;          // 256 rows x 64 B, swizzled
constexpr int kRgStage = kRgAStage + kRgBStage;
constexpr int kRgMeta = 2 * 2 * 2048;          // [tile parity][tile row][2 KB of position words]
constexpr int kRgLds = 4 * kRgStage + kRgMeta; // 136 KB

typedef const __attribute__((address_space(1))) void* rg_gptr_t;
typedef __attribute__((address_space(3))) void* rg_lptr_t;

__device__ __forceinline__ void rg_g2l16(const void* g, void* l) {
    // 16 bytes per lane, global -> LDS, no registers: LDS address = (wave-uniform) l + lane * 16
    __builtin_amdgcn_global_load_lds((rg_gptr_t)g, (rg_lptr_t)l, 16, 0, 0);
}

// X tile of one step in LDS: row m holds 4 chunks of 16 bytes (32 columns); chunk p sits at physical chunk
// p ^ ((m >> 2) & 3), so 16 consecutive rows reading the same logical chunk hit 16 distinct 16-byte bank groups.
__device__ __forceinline__ int xs32_off(int m, int p) { return m * 64 + ((p ^ ((m >> 2) & 3)) << 4); }

// One 32-feature block x 32 columns against four 32-row blocks, in place:
//   2:4   : c_i += A0 (*) B_i                       (positions idx)
//   dense : c_i += A0 B_i.lo + A1 B_i.hi
// The branch is inside the asm block: written with the builtins and an if/else, the register allocator splits the
// 16-register accumulator tuples at the branch and doubles the accumulator footprint.  The compiler does not see
// the matrix instructions: the epilogue pads the matrix-pipe -> memory read hazard itself.
__device__ __forceinline__ void mma_block4(f32x16& c0, f32x16& c1, f32x16& c2, f32x16& c3, const bf16x8& a0, const bf16x8& a1,
                                           const RB16& b0, const RB16& b1, const RB16& b2, const RB16& b3, int idx, int sparse) {
    asm volatile(
        "s_cmp_eq_u32 %[sp], 0\n\t"
        "s_cbranch_scc1 .Ldense%=\n\t"
        "v_smfmac_f32_32x32x32_bf16 %[c0], %[a0], %[b0], %[idx]\n\t"
        "v_smfmac_f32_32x32x32_bf16 %[c1], %[a0], %[b1], %[idx]\n\t"
        "v_smfmac_f32_32x32x32_bf16 %[c2], %[a0], %[b2], %[idx]\n\t"
        "v_smfmac_f32_32x32x32_bf16 %[c3], %[a0], %[b3], %[idx]\n\t"
        "s_branch .Ldone%=\n"
        ".Ldense%=:\n\t"
        "v_mfma_f32_32x32x16_bf16 %[c0], %[a0], %[b0l], %[c0]\n\t"
        "v_mfma_f32_32x32x16_bf16 %[c1], %[a0], %[b1l], %[c1]\n\t"
        "v_mfma_f32_32x32x16_bf16 %[c2], %[a0], %[b2l], %[c2]\n\t"
        "v_mfma_f32_32x32x16_bf16 %[c3], %[a0], %[b3l], %[c3]\n\t"
        "v_mfma_f32_32x32x16_bf16 %[c0], %[a1], %[b0h], %[c0]\n\t"
        "v_mfma_f32_32x32x16_bf16 %[c1], %[a1], %[b1h], %[c1]\n\t"
        "v_mfma_f32_32x32x16_bf16 %[c2], %[a1], %[b2h], %[c2]\n\t"
        "v_mfma_f32_32x32x16_bf16 %[c3], %[a1], %[b3h], %[c3]\n"
        ".Ldone%=:"
        : [c0] "+a"(c0), [c1] "+a"(c1), [c2] "+a"(c2), [c3] "+a"(c3)
        : [a0] "v"(a0), [a1] "v"(a1), [b0] "v"(b0.v), [b1] "v"(b1.v), [b2] "v"(b2.v), [b3] "v"(b3.v), [b0l] "v"(b0.h[0]),
          [b0h] "v"(b0.h[1]), [b1l] "v"(b1.h[0]), [b1h] "v"(b1.h[1]), [b2l] "v"(b2.h[0]), [b2h] "v"(b2.h[1]), [b3l] "v"(b3.h[0]),
          [b3h] "v"(b3.h[1]), [idx] "v"(idx), [sp] "s"(sparse)
        : "scc");
}

// Half of mma_block4 (two row blocks): short enough that the few LDS reads the compiler places between two pieces
// issue while the matrix pipe is still busy with the previous piece.
__device__ __forceinline__ void mma_piece2(f32x16& c0, f32x16& c1, const bf16x8& a0, const bf16x8& a1, const RB16& b0,
                                           const RB16& b1, int idx, int sparse) {
    asm volatile(
        "s_cmp_eq_u32 %[sp], 0\n\t"
        "s_cbranch_scc1 .Ldense%=\n\t"
        "v_smfmac_f32_32x32x32_bf16 %[c0], %[a0], %[b0], %[idx]\n\t"
        "v_smfmac_f32_32x32x32_bf16 %[c1], %[a0], %[b1], %[idx]\n\t"
        "s_branch .Ldone%=\n"
        ".Ldense%=:\n\t"
        "v_mfma_f32_32x32x16_bf16 %[c0], %[a0], %[b0l], %[c0]\n\t"
        "v_mfma_f32_32x32x16_bf16 %[c1], %[a0], %[b1l], %[c1]\n\t"
        "v_mfma_f32_32x32x16_bf16 %[c0], %[a1], %[b0h], %[c0]\n\t"
        "v_mfma_f32_32x32x16_bf16 %[c1], %[a1], %[b1h], %[c1]\n"
        ".Ldone%=:"
        : [c0] "+a"(c0), [c1] "+a"(c1)
        : [a0] "v"(a0), [a1] "v"(a1), [b0] "v"(b0.v), [b1] "v"(b1.v), [b0l] "v"(b0.h[0]), [b0h] "v"(b0.h[1]), [b1l] "v"(b1.h[0]),
          [b1h] "v"(b1.h[1]), [idx] "v"(idx), [sp] "s"(sparse)
        : "scc");
}

// LDS reads issued from asm so that the waits can be exact.  (The compiler waits with lgkmcnt(0) in this kernel,
// i.e. also for the operands it has just requested for the NEXT block, which exposes an LDS round trip per block.)
// The destination is only valid after a later rg_lds_wait<N>() with a small enough N and a tie of the register.
__device__ __forceinline__ void rg_lds_read128(u32x4& dst, uint32_t addr) {
    asm volatile("ds_read_b128 %0, %1" : "=v"(dst) : "v"(addr));
}
__device__ __forceinline__ void rg_lds_read128_512(u32x4& dst, uint32_t addr) {
    asm volatile("ds_read_b128 %0, %1 offset:512" : "=v"(dst) : "v"(addr));
}
__device__ __forceinline__ void rg_lds_read32(uint32_t& dst, uint32_t addr) {
    asm volatile("ds_read_b32 %0, %1" : "=v"(dst) : "v"(addr));
}
template <int N>
__device__ __forceinline__ void rg_lds_wait() {
    asm volatile("s_waitcnt lgkmcnt(%0)" ::"n"(N) : "memory");
}
__device__ __forceinline__ uint32_t rg_lds_addr(const void* p) {
    return (uint32_t)(size_t)((rg_lptr_t)p);
}

struct RgAOps {  // operands of one 32-feature block at one step
    RA8 a0, a1;
    uint32_t pw;
};

__global__ __launch_bounds__(256) void prefill_kernel_ring(const uint16_t* __restrict__ X, int64_t M, int64_t N, int64_t K,
                                                           const uint8_t* __restrict__ payload, const uint32_t* __restrict__ table,
                                                           int Tk, int tiles_n, int tiles_m, float* __restrict__ Y) {
    constexpr int TILE = 128;
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
    uint8_t* const Ms = lds + 4 * kRgStage;

    const int tid = threadIdx.x, lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wh = w & 1, wm = w >> 1;  // 64-feature half of both tile rows, 128-row half of the block
    const int i32 = lane & 31, q = lane >> 5;

    // ---- block -> (n, m) tile of the output.  Consecutive blocks go to different XCDs (hardware round-robin),
    // each with its own L2, so every XCD gets a contiguous run of the tile order below, and that order walks
    // groups of 4 row blocks x all feature blocks: the workgroups an XCD runs at a time then cover about
    // 8 feature blocks x 4 row blocks and share both operands in L2.
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
    const int64_t n0 = (int64_t)bn * kRgBN, m0 = (int64_t)bm * kRgBM;
    const bool two_rows = n0 + TILE < N;  // N is a multiple of 128, not necessarily of 256
    const uint32_t* trow0 = table + (int64_t)(n0 / TILE) * Tk;
    const uint32_t* trow1 = trow0 + (two_rows ? Tk : 0);  // a missing second tile row recomputes the first, unstored

    // ---- per-lane sources of the X copy: wavefront w copies 1 KB pieces w, w+4, w+8, w+12 of the 16 KB stage.
    // Byte offsets from X + step * 64 (a scalar base); the host keeps M * K * 2 below 4 GB for this kernel.
    uint32_t xoff[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int c = (w + 4 * i) * 64 + lane;  // physical 16-byte chunk of the X stage
        const int m = c >> 2, pp = c & 3, pl = pp ^ ((m >> 2) & 3);
        int64_t row = m0 + m;
        if (row >= M) row = M - 1;  // rows past M: any valid row, their outputs are not stored
        xoff[i] = (uint32_t)((row * K + pl * 8) * 2);
    }
    const uint8_t* const xbase = reinterpret_cast<const uint8_t*>(X);
    // ---- per-lane LDS read offsets
    const int swz = (i32 >> 2) & 3;
    const int xlo = wm * 128 * 64 + i32 * 64 + ((q ^ swz) << 4);        // + 32 mb * 64 per row block
    const int xhi = wm * 128 * 64 + i32 * 64 + (((2 + q) ^ swz) << 4);
    const int alane = (16 * q + (i32 & 15)) * 16;                        // inside a strip
    const int astrip = 4 * wh + (i32 >> 4);                              // + 2 hb: strip of the lane's row in the tile
    const int mlane = (16 * q + (i32 & 15)) * 4;                         // position dword inside a strip's 256 B; + 32*4 u

    const int nsteps = (int)(K / kRgStep);

    // Filling one LDS stage with step s (tile s/4, K-step j = (s/2)%2, half u = s%2) takes 6-10 loads per
    // wavefront (4 of X, 1-2 per tile row, the position words of a new 2:4 tile).  They are issued one or two at
    // a time between the matrix pieces of a step (slot 0..7): with one wavefront per SIMD every instruction that
    // is not a matrix instruction must hide in the shadow of one.
    auto issue_slot = [&](int slot, int s, uint32_t e0, uint32_t e1) {
        const int tk = s >> 2, j = (s >> 1) & 1, u = s & 1;
        uint8_t* sb = lds + (s & 3) * kRgStage;
        if (slot < 4) {  // X piece `slot`
            rg_g2l16(xbase + (size_t)s * 64 + xoff[slot], sb + kRgAStage + (w + 4 * slot) * 1024);
            return;
        }
        const int rr = (slot - 4) >> 1, t = (slot - 4) & 1;  // tile row, first / second load of the row
        const uint32_t e = rr ? e1 : e0;
        const uint8_t* tb = payload + entry_offset(e);
        uint8_t* dst = sb + rr * 8192;
        if (entry_sparse(e)) {
            if (t == 0) {
                // strips 2w (lanes 0-31) and 2w+1 (lanes 32-63): 512 B each, packed at 512 B in LDS
                const int strip = 2 * w + (lane >> 5);
                rg_g2l16(tb + (size_t)(strip * 2 + j) * kSparseFragBytes + u * 512 + (lane & 31) * 16, dst + w * 1024);
            } else if ((s & 3) == 0 && w < 2) {
                // first step of a tile: its 2 KB of position words, 1 KB per wavefront 0 / 1
                rg_g2l16(tb + sparse_vals_bytes(TILE) + w * 1024 + lane * 16, Ms + (tk & 1) * 4096 + rr * 2048 + w * 1024);
            }
        } else {
            const int strip = 2 * w + t;
            rg_g2l16(tb + (size_t)(strip * 2 + j) * kDenseFragBytes + u * 1024 + lane * 16, dst + strip * 1024);
        }
    };
    auto issue = [&](int s, uint32_t e0, uint32_t e1) {
#pragma unroll
        for (int slot = 0; slot < 8; ++slot) issue_slot(slot, s, e0, e1);
    };

    f32x16 acc[4][4];  // [feature block: 0,1 = tile row 0; 2,3 = tile row 1][row block]
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < 4; ++b)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[a][b][i] = 0.f;

    // LDS -> register fetches (asm-issued, see rg_lds_read128).  stage: ring slot; sp: type of the block's tile;
    // all offsets are lane constants plus compile-time or wavefront-uniform terms.  fetch_a issues 3 LDS
    // operations, fetch_b 2: the wait counts below depend on that.
    const uint32_t lds0 = rg_lds_addr(lds);
    auto fetch_a = [&](RgAOps& o, int stage, int nb, int sp, int tkpar, int u) {
        const int rr = nb >> 1, hb = nb & 1;
        const int strip = astrip + 2 * hb;
        const uint32_t p = lds0 + stage * kRgStage + rr * 8192 + strip * (sp ? 512 : 1024) + alane;
#ifndef LAB_NO_LDSREAD
        rg_lds_read128(o.a0.raw, p);
        rg_lds_read128_512(o.a1.raw, p);  // second dense operand; unused by a 2:4 block
        rg_lds_read32(o.pw, lds0 + 4 * kRgStage + tkpar * 4096 + rr * 2048 + strip * 256 + u * 128 + mlane);
#endif
    };
    auto fetch_b = [&](u32x4& lo, u32x4& hi, int stage, int mb) {
        const uint32_t p = lds0 + stage * kRgStage + kRgAStage + mb * 32 * 64;
#ifndef LAB_NO_LDSREAD
        rg_lds_read128(lo, p + xlo);
        rg_lds_read128(hi, p + xhi);
#endif
    };
    auto tie_a = [&](RgAOps& o) { asm volatile("" : "+v"(o.a0.raw), "+v"(o.a1.raw), "+v"(o.pw)); };

    // ---- prologue: three steps in flight, then the operands of step 0 / block 0
    uint32_t e0 = trow0[0], e1 = trow1[0];
    issue(0, e0, e1);
    issue(nsteps > 1 ? 1 : 0, e0, e1);
    issue(nsteps > 2 ? 2 : 0, e0, e1);
    asm volatile("s_waitcnt vmcnt(6)" ::: "memory");  // all but (at most) the newest step have landed
    __builtin_amdgcn_s_barrier();                     // bare barrier: __syncthreads() would wait for ALL loads
    asm volatile("" ::: "memory");
    // X fragments of the current / next step as separate halves (a dense instruction takes a half, a 2:4
    // instruction the pair); operands of the current / next feature block
    u32x4 xl[2][4], xh[2][4];
    RgAOps ao[2];
#pragma unroll
    for (int mb = 0; mb < 4; ++mb) fetch_b(xl[0][mb], xh[0][mb], 0, mb);
    fetch_a(ao[0], 0, 0, (int)(e0 & 1u), 0, 0);
    rg_lds_wait<0>();
#pragma unroll
    for (int mb = 0; mb < 4; ++mb) asm volatile("" : "+v"(xl[0][mb]), "+v"(xh[0][mb]));
    tie_a(ao[0]);

    for (int tk = 0; tk < Tk; ++tk) {
        const int tkn = (tk + 1 < Tk) ? tk + 1 : tk;
        const uint32_t e0n = trow0[tkn], e1n = trow1[tkn];  // read a tile ahead of their first use
        const int sp0 = (int)(e0 & 1u), sp1 = (int)(e1 & 1u);
#pragma unroll
        for (int ss = 0; ss < 4; ++ss) {
            const int s = 4 * tk + ss;
            const int j = ss >> 1, u = ss & 1, par = ss & 1;
            if (s > 0) {
                // loads of steps s and s+1 were issued at least two steps ago; everything older than the newest
                // six loads (a step issues at least six) has landed
                asm volatile("s_waitcnt vmcnt(6)" ::: "memory");
                __builtin_amdgcn_s_barrier();
                asm volatile("" ::: "memory");
            }
            // refill the stage step s-1 just left, slot by slot below; past the end re-fetch the last step (keeps
            // the load counts uniform)
            const int s3 = (s + 3 < nsteps) ? s + 3 : nsteps - 1;
            const bool next_tile = (ss + 3) >= 4 && (s + 3 < nsteps);
            const uint32_t pe0 = next_tile ? e0n : e0, pe1 = next_tile ? e1n : e1;
            // next step: its tile, its types
            const bool nt = ss == 3;
            const int spn0 = nt ? (int)(e0n & 1u) : sp0;
            const int tkparn = nt ? ((tk + 1) & 1) : (tk & 1);
            const int un = (ss + 1) & 1;
#pragma unroll
            for (int nb = 0; nb < 4; ++nb) {
                const int sp = (nb < 2) ? sp0 : sp1;
                // LDS operations in flight, oldest first, when block nb starts:
                //   [A(nb): 3, issued before the first piece of block nb-1] [X'(nb-1): 2, issued between its pieces]
                // (for nb = 0 read "block 3 of the previous step"; after the tile loop's full wait: none).
                // Now the operands of the next block are requested (3 more) and the wait below lets exactly those
                // stay in flight.
                if (nb < 3) fetch_a(ao[(nb + 1) & 1], ss, nb + 1, (nb + 1 < 2) ? sp0 : sp1, tk & 1, u);
                else fetch_a(ao[0], (ss + 1) & 3, 0, spn0, tkparn, un);
                rg_lds_wait<3>();
                tie_a(ao[nb & 1]);
                if (nb == 0) {
#pragma unroll
                    for (int mb = 0; mb < 4; ++mb) asm volatile("" : "+v"(xl[par][mb]), "+v"(xh[par][mb]));
                }
                const int idx = (int)(ao[nb & 1].pw >> (16 * j));
                RB16 b0, b1, b2, b3;
                b0.raw[0] = xl[par][0]; b0.raw[1] = xh[par][0];
                b1.raw[0] = xl[par][1]; b1.raw[1] = xh[par][1];
                b2.raw[0] = xl[par][2]; b2.raw[1] = xh[par][2];
                b3.raw[0] = xl[par][3]; b3.raw[1] = xh[par][3];
#ifndef LAB_NO_LOADS
                issue_slot(2 * nb, s3, pe0, pe1);
#endif
#ifndef LAB_NO_MMA
                mma_piece2(acc[nb][0], acc[nb][1], ao[nb & 1].a0.v, ao[nb & 1].a1.v, b0, b1, idx, sp);
#endif
                // one X fragment of the next step (next ring slot, visible since this step's barrier)
                fetch_b(xl[par ^ 1][nb], xh[par ^ 1][nb], (ss + 1) & 3, nb);
#ifndef LAB_NO_LOADS
                issue_slot(2 * nb + 1, s3, pe0, pe1);
#endif
#ifndef LAB_NO_MMA
                mma_piece2(acc[nb][2], acc[nb][3], ao[nb & 1].a0.v, ao[nb & 1].a1.v, b2, b3, idx, sp);
#else
                acc[nb][0][0] += (float)(ao[nb & 1].a0.raw[0] + ao[nb & 1].a1.raw[1] + b0.raw[0][0] + b1.raw[1][1] + b2.raw[0][1] + b3.raw[1][0] + idx + sp);
#endif
            }
        }
        // Values fetched by asm and carried over the loop edge must have landed before the compiler may copy them.
        rg_lds_wait<0>();
#pragma unroll
        for (int mb = 0; mb < 4; ++mb) asm volatile("" : "+v"(xl[0][mb]), "+v"(xh[0][mb]));
        tie_a(ao[0]);
        e0 = e0n;
        e1 = e1n;
    }

    // outstanding (re-fetched) loads must land before this workgroup's LDS can be handed on
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    // the last matrix instructions may still be writing their accumulators: 16-pass results need up to 18 wait
    // states before another unit may read them
    asm volatile("s_nop 15\n\ts_nop 15\n\ts_nop 15" ::: "memory");

    // acc[nb][mb][i]: feature n0 + 128 (nb/2) + 64 wh + 32 (nb%2) + 8 (i/4) + 4 q + i%4, row m0 + 128 wm + 32 mb + i32
#pragma unroll
    for (int mb = 0; mb < 4; ++mb) {
        const int64_t m = m0 + 128 * wm + 32 * mb + i32;
        if (m >= M) continue;
#pragma unroll
        for (int nb = 0; nb < 4; ++nb) {
            if (nb >= 2 && !two_rows) continue;
            const int64_t n = n0 + 128 * (nb >> 1) + 64 * wh + 32 * (nb & 1) + 4 * q;
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                f32x4 v = {acc[nb][mb][4 * g], acc[nb][mb][4 * g + 1], acc[nb][mb][4 * g + 2], acc[nb][mb][4 * g + 3]};
#ifdef LAB_NO_STORE
                if (v[0] == 1.2345f)
#endif
                *reinterpret_cast<f32x4*>(Y + m * N + n + 8 * g) = v;
            }
        }
    }
}

void launch_prefill_ring(const GemmArgs& a, hipStream_t stream) {
    static const hipError_t granted = hipFuncSetAttribute(reinterpret_cast<const void*>(&prefill_kernel_ring),
                                                          hipFuncAttributeMaxDynamicSharedMemorySize, kRgLds);
    (void)granted;
    const int tiles_n = (int)((a.N + kRgBN - 1) / kRgBN), tiles_m = (int)((a.M + kRgBM - 1) / kRgBM);
    const int nblk = tiles_n * tiles_m;
    const int grid = ((nblk + 7) / 8) * 8;
    hipLaunchKernelGGL(prefill_kernel_ring, dim3(grid), dim3(256), kRgLds, stream, a.X, a.M, a.N, a.K, a.payload, a.table, a.Tk, tiles_n,
                       tiles_m, a.Y);
}

}  // namespace patch
