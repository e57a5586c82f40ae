// Prefill-shaped hybrid GEMM (any M): Y = X * W_hat^T of Section 4 / Appendix A of the paper for the
// prefill input (batch * sequence x K), dense and 2:4 tiles mixed inside one launch.
//
// As in the decode kernel the weight is the A operand (Y^T = W_hat * X^T).  A workgroup owns 128 output
// features x BM rows of X; per 64-column K-step the compressed weight fragments are copied verbatim
// (they already are in register order, see layout.h) and the X tile is copied with an XOR swizzle into LDS.
// Each wavefront owns 64 features x 64 rows and takes ONE scalar branch per K-step on the type of the tile
// its 64 features lie in:
//   dense : 4 x v_mfma_f32_32x32x16_bf16   per 32x32 output block
//   2:4   : 2 x v_smfmac_f32_32x32x32_bf16 per 32x32 output block
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "epilogue.h"
#include "kernels.h"
#include "layout.h"
#include "prefill_parts.h"

namespace patch {

template <int TILE, int BM>
__global__ __launch_bounds__(256) void prefill_kernel_v0(const uint16_t* __restrict__ X, int64_t M, int64_t N, int64_t K,
                                                         const uint8_t* __restrict__ payload, const uint32_t* __restrict__ table,
                                                         int Tk, float* __restrict__ Y, int ybf16) {
    static_assert(BM == 128, "wave layout below assumes a 128 x 128 workgroup tile");
    constexpr int KPT = TILE / kStepCols;
    __shared__ __attribute__((aligned(16))) uint8_t As[2 * 4 * kDenseFragBytes];  // [half][strip][fragment]
    __shared__ __attribute__((aligned(16))) uint8_t Xs[BM * 128];

    const int tid = threadIdx.x, lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wn = w & 1, wm = w >> 1;  // wavefront's 64-feature half and 64-row half
    const int64_t n0 = (int64_t)blockIdx.x * 128, m0 = (int64_t)blockIdx.y * BM;
    const int i32 = lane & 31, q = lane >> 5;

    f32x16 acc[2][2];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.f;

    const int ksteps = (int)(K / kStepCols);
    for (int ks = 0; ks < ksteps; ++ks) {
        const int tk = ks / KPT, j = ks % KPT;
        __syncthreads();
        // ---- stage the weight fragments of both 64-feature halves
#pragma unroll
        for (int hn = 0; hn < 2; ++hn) {
            const int64_t nh = n0 + 64 * hn;
            if (nh >= N) continue;  // N is a multiple of 64 but not necessarily of 128
            const int tn = (int)(nh / TILE), s0 = (int)((nh % TILE) / kStripRows);
            const uint32_t e = table[(int64_t)tn * Tk + tk];
            const uint8_t* base = payload + entry_offset(e);
            if (entry_sparse(e)) {
                // 4 strips x 1024 B = 256 chunks: one per thread
                const int s = tid >> 6, c = tid & 63;
                const uint8_t* src = base + (size_t)((s0 + s) * KPT + j) * kSparseFragBytes + c * 16;
                *reinterpret_cast<u32x4*>(&As[(hn * 4 + s) * kDenseFragBytes + c * 16]) = *reinterpret_cast<const u32x4*>(src);
            } else {
#pragma unroll
                for (int it = 0; it < 2; ++it) {
                    const int cc = tid + 256 * it, s = cc >> 7, c = cc & 127;
                    const uint8_t* src = base + (size_t)((s0 + s) * KPT + j) * kDenseFragBytes + c * 16;
                    *reinterpret_cast<u32x4*>(&As[(hn * 4 + s) * kDenseFragBytes + c * 16]) = *reinterpret_cast<const u32x4*>(src);
                }
            }
        }
        // ---- stage the X tile (BM rows x 64 columns), rows beyond M are zero
#pragma unroll
        for (int it = 0; it < BM * 8 / 256; ++it) {
            const int cc = tid + 256 * it, m = cc >> 3, p = cc & 7;
            u32x4 v = {0u, 0u, 0u, 0u};
            if (m0 + m < M) v = *reinterpret_cast<const u32x4*>(X + (m0 + m) * K + (int64_t)ks * 64 + p * 8);
            *reinterpret_cast<u32x4*>(&Xs[xs_off(m, p)]) = v;
        }
        __syncthreads();

        // ---- X fragments of this wavefront: 2 row blocks of 32, chunks {q, 2+q, 4+q, 6+q}
        u32x4 xb[2][4];
#pragma unroll
        for (int b = 0; b < 2; ++b) {
            const int m = wm * 64 + b * 32 + i32;
#pragma unroll
            for (int c = 0; c < 4; ++c) xb[b][c] = *reinterpret_cast<const u32x4*>(&Xs[xs_off(m, 2 * c + q)]);
        }
        // ---- one uniform branch on the type of the tile this wavefront's 64 features lie in
        const int64_t nh = n0 + 64 * wn;
        if (nh >= N) continue;
        const int tn = (int)(nh / TILE), s0 = (int)((nh % TILE) / kStripRows);
        const uint32_t e = __builtin_amdgcn_readfirstlane(table[(int64_t)tn * Tk + tk]);
        const uint8_t* as = &As[wn * 4 * kDenseFragBytes];
        if (entry_sparse(e)) {
            const uint16_t* meta = reinterpret_cast<const uint16_t*>(payload + entry_offset(e) + sparse_vals_bytes(TILE));
#pragma unroll
            for (int a = 0; a < 2; ++a) {       // 32-feature block
                const int strip = 2 * a + (i32 >> 4);
#pragma unroll
                for (int u = 0; u < 2; ++u) {   // 32-column half of the K-step
                    const int fl = 16 * (2 * u + q) + (i32 & 15);
                    A8 av;
                    av.raw = *reinterpret_cast<const u32x4*>(as + strip * kDenseFragBytes + fl * 16);
                    const int idx = (int)meta[((s0 + strip) * 64 + fl) * KPT + j];
#pragma unroll
                    for (int b = 0; b < 2; ++b) {
                        B16 bv;
                        bv.raw[0] = xb[b][2 * u];
                        bv.raw[1] = xb[b][2 * u + 1];
                        acc[a][b] = __builtin_amdgcn_smfmac_f32_32x32x32_bf16(av.v, bv.v, acc[a][b], idx, 0, 0);
                    }
                }
            }
        } else {
#pragma unroll
            for (int a = 0; a < 2; ++a) {
                const int strip = 2 * a + (i32 >> 4);
#pragma unroll
                for (int c = 0; c < 4; ++c) {   // 16-column quarter of the K-step
                    const int h = c >> 1, qq = 2 * (c & 1) + q;
                    A8 av;
                    av.raw = *reinterpret_cast<const u32x4*>(as + strip * kDenseFragBytes + (h * 64 + 16 * qq + (i32 & 15)) * 16);
#pragma unroll
                    for (int b = 0; b < 2; ++b) {
                        A8 bv;
                        bv.raw = xb[b][c];
                        acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av.v, bv.v, acc[a][b], 0, 0, 0);
                    }
                }
            }
        }
    }

    // acc[a][b][r]: feature n0 + 64 wn + 32 a + 8 (r/4) + 4 q + r%4, row m0 + 64 wm + 32 b + i32
#pragma unroll
    for (int b = 0; b < 2; ++b) {
        const int64_t m = m0 + 64 * wm + 32 * b + i32;
        if (m >= M || n0 + 64 * wn >= N) continue;
#pragma unroll
        for (int a = 0; a < 2; ++a)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                f32x4 v = {acc[a][b][4 * g], acc[a][b][4 * g + 1], acc[a][b][4 * g + 2], acc[a][b][4 * g + 3]};
                store4(Y, m * N + n0 + 64 * wn + 32 * a + 8 * g + 4 * q, v, ybf16);
            }
    }
}

// ------------------------------------------------------------------------------------------------------
// LDS-staged prefill kernel (tile = 128 or 64): 256 features x 256 rows per workgroup, 8 wavefronts, 64-column
// K-steps, LDS double buffer filled by direct global->LDS loads.
//
//   wavefront w < 4 : features 0..127 of the block,   rows 64 w .. 64 w + 63
//   wavefront w >= 4: features 128..255 of the block, rows 64 (w-4) ..
// With tile 128 the two wavefronts that share a SIMD (w and w + 4) always own DIFFERENT tile rows, so every SIMD
// carries cost(tile row 0) + cost(tile row 1) matrix cycles per K-step whatever the tile types are: the
// dense/2:4 mix cannot unbalance the workgroup between two barriers.  With tile 64 a wavefront's 128 features
// are two tile rows (its 32-feature blocks 0-1 and 2-3), each with its own type, and every K-step is a new tile.
//
// LDS per stage: weight fragments [strip of the block][2048 B] (a 2:4 strip uses the first 1024 B), X tile
// 256 rows x 128 B with the XOR swizzle of xs_off(); plus the position words of the current 2:4 tiles
// (tile 128: 2 KB per tile row, kept for the tile's two K-steps in a buffer chosen by the tile's parity;
// tile 64: 512 B per tile row in a 1 KB slot, per stage).
// ------------------------------------------------------------------------------------------------------
constexpr int kPfBN = 256;
constexpr int kPfAStage = 2 * 8 * kDenseFragBytes;   // 32 KB
constexpr int kPfMetaBuf = 2 * 2048;                 // position words: two tile rows x 2 KB (tile 128), four x 1 KB (tile 64)
__host__ __device__ constexpr int pf_xstage(int bm) { return bm * 128; }   // X tile of a stage: 32 or 16 KB
__host__ __device__ constexpr int pf_lds_bytes(int bm) { return 2 * (kPfAStage + pf_xstage(bm)) + 2 * kPfMetaBuf; }   // 136 / 104 KB

// Table entries of the (up to four) tile rows of a block at one K-step.  Plain members, never indexed at run time: an
// array that is indexed by a wavefront-dependent value lives in scratch memory, and anything that makes the register
// allocator spill or copy around the matrix instructions of mma_step (which it cannot see) stores accumulators that
// are still being written.  tests/test_abi_host.py checks that the kernel uses no scratch memory at all.
struct PfEntries {
    uint32_t v0, v1, v2, v3;
};

// SPLIT: K cut into gridDim.y slices of whole tiles, one workgroup each; slice y writes its partial product (fp32) to
// Y + y M N - a workspace - and wr_reduce sums the slices in order.
template <int TILE, bool SPLIT, int BM>
__global__ __launch_bounds__(512) void prefill_kernel_lds(const uint16_t* __restrict__ X, int64_t M, int64_t N, int64_t K,
                                                          const uint8_t* __restrict__ payload, const uint32_t* __restrict__ table,
                                                          int Tk_all, int tiles_n, int tiles_m, float* __restrict__ Y, int ybf16) {
    constexpr int KPT = TILE / kStepCols;        // K-steps per tile: 2 or 1
    constexpr int SPT = TILE / kStripRows;       // strips per tile: 8 or 4
    constexpr int NR = kPfBN / TILE;             // tile rows per block: 2 or 4
    constexpr int NA = BM / 64;                  // 32-feature blocks per wavefront: 4 (128 features) or 2 (64)
    constexpr int WR = NA * 32 > TILE ? 2 : 1;   // tile rows per wavefront: 2 only for 128 features of tile 64
    constexpr int ESZ = 2 * KPT;                 // bytes of position bits per lane and strip
    constexpr int MROW = TILE == 128 ? 2048 : 1024;   // LDS bytes per tile row of position words
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
    constexpr int NS = 2, XSTAGE = pf_xstage(BM);
    uint8_t* const As = lds;                                      // [stage][strip of the block][2048]
    uint8_t* const Bs = lds + NS * kPfAStage;                     // [stage][BM rows][128 B] swizzled
    uint8_t* const Ms = lds + NS * kPfAStage + NS * XSTAGE;       // [buffer][tile row][MROW]

    const int tid = threadIdx.x, lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    // BM = 256: wavefront = 128-feature half of the block x one of four 64-row groups; BM = 128: 64-feature quarter x
    // one of two 64-row groups
    const int w4 = w >> 2;                                  // strip w of the block lies in its 128-feature half w4
    const int fo = BM == 256 ? 128 * (w >> 2) : 64 * (w >> 1);   // first feature of the wavefront inside the block
    const int wm = BM == 256 ? (w & 3) : (w & 1);

    // ---- block -> (n, m) tile of the output.  Consecutive blocks go to different XCDs (hardware round-robin),
    // each with its own L2, so every XCD gets a contiguous run of the tile order below, and that order walks
    // groups of 4 row blocks x all feature blocks: the ~32 workgroups an XCD runs at a time then cover about
    // 8 feature blocks x 4 row blocks and share both operands in L2 (2 x 16 measured 1 GB of L2 misses per
    // launch against 100 MB of operands).
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
        const int full = (tiles_m / GM) * GM * tiles_n;   // tiles in complete groups
        if (bid < full) {
            const int g = bid / (GM * tiles_n), rem = bid % (GM * tiles_n);
            bn = rem / GM;
            bm = g * GM + rem % GM;
        } else {                                          // last, narrower group
            const int gm = tiles_m % GM, rem = bid - full;
            bn = rem / gm;
            bm = (tiles_m / GM) * GM + rem % gm;
        }
    }
    const int64_t n0 = (int64_t)bn * kPfBN, m0 = (int64_t)bm * BM;
    // N is a multiple of the tile, not necessarily of 256: the last block has `live` tile rows.  Table rows of
    // the others alias the last live one (valid addresses); their weights are not copied and nothing of theirs is stored.
    const int live = (int)((N - n0) / TILE) < NR ? (int)((N - n0) / TILE) : NR;
    // this workgroup's K slice, in tiles: to the rest of the kernel it is a product with a shorter K
    const int t_begin = SPLIT ? (int)((int64_t)blockIdx.y * Tk_all / gridDim.y) : 0;
    const int Tk = SPLIT ? (int)((int64_t)(blockIdx.y + 1) * Tk_all / gridDim.y) - t_begin : Tk_all;
    const uint32_t* trow[NR];
#pragma unroll
    for (int i = 0; i < NR; ++i) trow[i] = table + ((int64_t)(n0 / TILE) + (i < live ? i : live - 1)) * Tk_all + t_begin;

    // ---- per-lane source pointers for the X tile copy: wavefront w copies 1 KB pieces w, w+8 (, w+16, w+24)
    constexpr int XP = BM / 64;
    const uint8_t* xsrc[XP];
#pragma unroll
    for (int i = 0; i < XP; ++i) {
        const int c = (w + 8 * i) * 64 + lane;       // physical 16-byte chunk of the tile
        const int m = c >> 3, pp = c & 7, pl = pp ^ ((m >> 1) & 7);
        int64_t row = m0 + m;
        if (row >= M) row = M - 1;                     // rows past M: any valid row, their outputs are not stored
        xsrc[i] = reinterpret_cast<const uint8_t*>(X + row * K + pl * 8 + (int64_t)t_begin * TILE);
    }

    // Fill one LDS stage with K-step ks; e[i] = table entry of tile row i of the block at that step.
    auto prefetch = [&](int ks, int stage, const PfEntries e) {
        const int tk = ks / KPT, j = ks % KPT;
        // weights: wavefront w copies strips w and w + 8 of the block's 16
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            // strip w + 8 h of the block: tile row h (tile 128) or w4 + 2 h (tile 64) - a choice between two entries at most
            const int sidx = w + 8 * h, tr = sidx / SPT, st = sidx % SPT;
            if (tr >= live) continue;
            const uint32_t ev = TILE == 128 ? (h ? e.v1 : e.v0) : (h ? (w4 ? e.v3 : e.v2) : (w4 ? e.v1 : e.v0));
            const uint8_t* tb = payload + entry_offset(ev);
            uint8_t* dst = As + stage * kPfAStage + sidx * kDenseFragBytes;
            if (entry_sparse(ev)) {
                g2l16(tb + (size_t)(st * KPT + j) * kSparseFragBytes + lane * 16, dst);
            } else {
                const uint8_t* f = tb + (size_t)(st * KPT + j) * kDenseFragBytes + lane * 16;
                g2l16(f, dst);
                g2l16(f + 1024, dst + 1024);
            }
        }
        // position words of the 2:4 tiles
        if constexpr (TILE == 128) {
            // 2 KB per tile, once per tile (its first K-step), by wavefronts 0 and 1
            if (j == 0 && w < 2) {
#pragma unroll
                for (int rr = 0; rr < NR; ++rr) {
                    const uint32_t ev = rr ? e.v1 : e.v0;
                    if (rr < live && entry_sparse(ev))
                        g2l16(payload + entry_offset(ev) + sparse_vals_bytes(TILE) + w * 1024 + lane * 16,
                              Ms + (tk & 1) * kPfMetaBuf + rr * MROW + w * 1024);
                }
            }
        } else {
            // 512 B per tile, every step, tile row w by wavefront w (the copy moves 1 KB: the second half is the
            // head of the next tile or the zeroed slack behind the payload, and lands in the unused half of the slot)
            if (w < NR && w < live) {
                const uint32_t ev01 = (w & 1) ? e.v1 : e.v0, ev23 = (w & 1) ? e.v3 : e.v2;
                const uint32_t ev = (w & 2) ? ev23 : ev01;
                if (entry_sparse(ev)) g2l16(payload + entry_offset(ev) + sparse_vals_bytes(TILE) + lane * 16, Ms + stage * kPfMetaBuf + w * MROW);
            }
        }
        // X tile
#pragma unroll
        for (int i = 0; i < XP; ++i) g2l16(xsrc[i] + (size_t)ks * 128, Bs + stage * XSTAGE + (w + 8 * i) * 1024);
    };

    f32x16 acc[NA][2];
#pragma unroll
    for (int a = 0; a < NA; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[a][b][i] = 0.f;

    const int i32 = lane & 31, q = lane >> 5;
    // LDS byte offsets of this lane inside a strip's fragment; a 32-feature block a covers strips 2a, 2a+1 of the
    // wavefront's eight (four)
    const int lane_frag = ((i32 >> 4) * kDenseFragBytes) + (16 * q + (i32 & 15)) * 16;
    const int lane_meta = ((i32 >> 4) * 64 + 16 * q + (i32 & 15)) * ESZ;
    // One K-step: wait for the stage, refill the other one, multiply.  e_mine[i]: table entry of this wavefront's
    // i-th tile row at step ks; (pf_ks, pf_e): the step to fetch into the idle stage and its entries.
    // (With blocks of 128 rows no single unit bounds the step - counters: LDS busy a third of the cycles, matrix pipes
    // a third; leaving out the matrix instructions, the global -> LDS loads or the LDS reads saves 18 %, 30 % or 12 %
    // of it.  The largest piece is the global -> LDS path: a compute unit fetches a step's 48 KB in 0.53 us when they
    // hit in L2 and in 0.76 us when they come from HBM (patch_probe_lds_fill), the same with one or two rounds in
    // flight - a rate, not a latency.  Accordingly a third stage fetched two steps ahead with counted waits, and a third
    // stage with the X fragments of the next step read between this step's matrix instructions, both measured 3 - 8 %
    // slower than this loop.)
    auto step = [&](int ks, uint32_t e_mine0, uint32_t e_mine1, int pf_ks, const PfEntries pf_e) {
        const int stage = ks & 1;
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        prefetch(pf_ks, stage ^ 1, pf_e);
        const int tk = ks / KPT, j = ks % KPT;
        const uint8_t* as = As + stage * kPfAStage + (fo / kStripRows) * kDenseFragBytes + lane_frag;
        const uint8_t* bs = Bs + stage * XSTAGE;
        // position words of block a (features fo + 32 a ..): tile row (fo + 32 a) / TILE of the block, in buffer
        // tk & 1 (tile 128) or this stage's (tile 64); strips ((fo + 32 a) % TILE) / 16, + 1 of the tile
        const uint8_t* ms = Ms + (TILE == 128 ? (tk & 1) : stage) * kPfMetaBuf + lane_meta;

        // X fragments as 8-register pairs: a 2:4 instruction takes a pair, a dense one either half
        B16 xb[2][2];
#pragma unroll
        for (int b = 0; b < 2; ++b) {
            const int m = wm * 64 + b * 32 + i32;
#pragma unroll
            for (int c = 0; c < 4; ++c) xb[b][c >> 1].raw[c & 1] = *reinterpret_cast<const u32x4*>(bs + xs_off(m, 2 * c + q));
        }
        // All LDS reads are unconditional: a 2:4 half-step reads one fragment it does not use, a dense one a
        // position word it does not use (LDS bandwidth has that slack, the register allocator has none).
        // The operands of a (block, half) are fetched two positions ahead of the matrix instructions that use
        // them: an LDS round trip is longer than the 64-128 matrix cycles of one position.
        A8 fa0[3], fa1[3];
        uint32_t fpw[3];
        auto fetch = [&](int pos, int buf) {
            const int a = pos >> 1, u = pos & 1;
            const int sp = (int)((WR == 1 || a < 2 ? e_mine0 : e_mine1) & 1u);
            // half-step u of a strip: 2:4 fragment half at u * 512, dense operand pair at u * 1024 and + 512
            const int ustride = sp ? 512 : 1024;
            fa0[buf].raw = *reinterpret_cast<const u32x4*>(as + a * 2 * kDenseFragBytes + u * ustride);
            fa1[buf].raw = *reinterpret_cast<const u32x4*>(as + a * 2 * kDenseFragBytes + u * ustride + 512);
            const int f = fo + 32 * a;
            const uint8_t* pw = ms + (f / TILE) * MROW + ((f % TILE) / kStripRows) * 64 * ESZ + u * 32 * ESZ;
            if constexpr (TILE == 128) fpw[buf] = *reinterpret_cast<const uint32_t*>(pw);
            else fpw[buf] = *reinterpret_cast<const uint16_t*>(pw);
        };
        fetch(0, 0);
        fetch(1, 1);
#pragma unroll
        for (int pos = 0; pos < 2 * NA; ++pos) {
            if (pos + 2 < 2 * NA) fetch(pos + 2, (pos + 2) % 3);
            const int a = pos >> 1, u = pos & 1, buf = pos % 3;
            const int sp = (int)((WR == 1 || a < 2 ? e_mine0 : e_mine1) & 1u);
            const int idx = TILE == 128 ? (int)(fpw[buf] >> (16 * j)) : (int)fpw[buf];
            mma_step(acc[a][0], acc[a][1], fa0[buf].v, fa1[buf].v, xb[0][u], xb[1][u], idx, sp);
        }
    };

    // Table entries are read one tile ahead of their first use, so no step starts by waiting for a scalar load.
    auto entries = [&](int tk) {
        PfEntries t;
        t.v0 = trow[0][tk];
        t.v1 = trow[1][tk];
        t.v2 = trow[NR > 2 ? 2 : 0][tk];
        t.v3 = trow[NR > 2 ? 3 : 0][tk];
        return t;
    };
    PfEntries e = entries(0);
    prefetch(0, 0, e);
    for (int tk = 0; tk < Tk; ++tk) {
        // (the very last step re-fetches itself into the idle stage: no branch around the loads; en = e there)
        const int more = tk + 1 < Tk ? 1 : 0;
        const PfEntries en = entries(tk + more);
        // this wavefront's tile rows.  128 features: w4 (tile 128), 2 w4 and 2 w4 + 1 (tile 64); 64 features: w4 (tile
        // 128), w / 2 (tile 64)
        uint32_t em0, em1;
        if constexpr (BM == 256) {
            em0 = WR == 1 ? (w4 ? e.v1 : e.v0) : (w4 ? e.v2 : e.v0);
            em1 = w4 ? e.v3 : e.v1;
        } else {
            const uint32_t lo = (w & 2) ? e.v1 : e.v0, hi = (w & 2) ? e.v3 : e.v2;
            em0 = TILE == 128 ? (w4 ? e.v1 : e.v0) : (w4 ? hi : lo);
            em1 = em0;
        }
        if constexpr (KPT == 2) {
            step(2 * tk, em0, em1, 2 * tk + 1, e);
            step(2 * tk + 1, em0, em1, 2 * tk + 1 + more, en);
        } else {
            step(tk, em0, em1, tk + more, en);
        }
        e = en;
    }

    // the idle-stage loads of the last step must land before this workgroup's LDS can be handed on
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    // the last matrix instructions may still be writing their accumulators: 16-pass results need up to 18 wait
    // states before another unit may read them
    asm volatile("s_nop 15\n\ts_nop 15\n\ts_nop 15" ::: "memory");
    // acc[a][b][i]: feature n0 + fo + 32 a + 8 (i/4) + 4 q + i%4, row m0 + 64 wm + 32 b + i32
    // (blocks of the last feature block past N computed on whatever was in LDS; nothing of theirs is stored)
#pragma unroll
    for (int b = 0; b < 2; ++b) {
        const int64_t m = m0 + 64 * wm + 32 * b + i32;
        if (m >= M) continue;
#pragma unroll
        for (int a = 0; a < NA; ++a) {
            if (n0 + fo + 32 * a >= N) continue;
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                f32x4 v = {acc[a][b][4 * g], acc[a][b][4 * g + 1], acc[a][b][4 * g + 2], acc[a][b][4 * g + 3]};
                // partial products stay fp32; their sum is rounded by the reduction
                store4(Y, (SPLIT ? (int64_t)blockIdx.y * M * N : 0) + m * N + n0 + fo + 32 * a + 8 * g + 4 * q, v, SPLIT ? 0 : ybf16);
            }
        }
    }
}

// ------------------------------------------------------------------------------------------------------
// Blocks of 256 features x BM rows with the weights straight into registers ("areg"): BM = 128 on both mask tiles (the
// 128-row kernel of the default choice), BM = 256 on mask tile 64 (its 256-row kernel; variant 6).
//
// The LDS-staged kernel is bound by what a compute unit can fetch per K-step, and the global -> LDS path is the
// slower way in (patch_probe_lds_fill).  Here only X goes that way (BM x 128 bytes per step, two LDS stages); a
// wavefront owns 32 features x ALL BM rows, so its weight fragments are its own: each lane loads its 16-byte pieces of
// the stored fragments (the gather the LDS kernel does with LDS reads) from global memory into registers one step
// ahead, by ordinary loads the compiler tracks, into two buffers that alternate (no copy).  No weight byte is fetched
// twice and none passes through LDS.  Mask tile 128: the two buffers are a tile's two K-steps, and the position dwords
// of a 2:4 tile (both K-steps in one dword) are loaded once per tile.  Mask tile 64: every step is a tile; steps go
// in pairs.
//   wavefront w : features 32 w .. 32 w + 31 of the block: tile row 32 w / TILE, two strips of that tile
//   a step      : BM / 32 positions (half-step u, pair of 32-row blocks) of mma_step, X fragments read from LDS two
//                 positions ahead
// ------------------------------------------------------------------------------------------------------
typedef const __attribute__((address_space(1))) u32x4* ar_g16_t;
typedef const __attribute__((address_space(1))) uint32_t* ar_g4_t;
typedef const __attribute__((address_space(1))) uint16_t* ar_g2_t;

// One step's weight operands of a wavefront.  Plain members, and the same member for the same use whatever the tile
// type (an array indexed by the type lands in scratch memory): half-step 0 multiplies (h0a, h0b), half-step 1
// (h1a, h1b); a 2:4 tile uses h0a and h1a only.
struct ArWeights {
    A8 h0a, h0b, h1a, h1b;
};

template <int TILE, int BM, bool SPLIT>
__global__ __launch_bounds__(512) void prefill_kernel_areg(const uint16_t* __restrict__ X, int64_t M, int64_t N, int64_t K,
                                                           const uint8_t* __restrict__ payload, const uint32_t* __restrict__ table,
                                                           int Tk_all, int tiles_n, int tiles_m, float* __restrict__ Y, int ybf16) {
    constexpr int KPT = TILE / kStepCols;  // K-steps per tile: 2 or 1
    constexpr int NB = BM / 32;            // 32-row blocks: 4 or 8
    constexpr int XP = BM / 64;            // 1 KB pieces of the X tile per wavefront
    constexpr int kArStage = BM * 128;     // 16 or 32 KB
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
    const int tid = threadIdx.x, lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int fo = 32 * w;                 // first feature of the wavefront inside the block
    const int w4 = fo / TILE;              // tile row of the block this wavefront's features lie in
    // block -> (n, m) as in prefill_kernel_lds: one contiguous run of the grouped order per XCD
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
    const int64_t n0 = (int64_t)bn * kPfBN, m0 = (int64_t)bm * BM;
    // N is a multiple of the tile, not necessarily of 256: a wavefront of a missing tile row works on the last live
    // one's weights (valid addresses) and stores nothing
    const int live = (int)((N - n0) / TILE) < kPfBN / TILE ? (int)((N - n0) / TILE) : kPfBN / TILE;
    const int t_begin = SPLIT ? (int)((int64_t)blockIdx.y * Tk_all / gridDim.y) : 0;
    const int Tk = SPLIT ? (int)((int64_t)(blockIdx.y + 1) * Tk_all / gridDim.y) - t_begin : Tk_all;
    const uint32_t* trow = table + ((int64_t)(n0 / TILE) + (w4 < live ? w4 : live - 1)) * Tk_all + t_begin;

    // X tile copy: wavefront w copies 1 KB pieces w, w + 8, ...
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
        for (int i = 0; i < XP; ++i) g2l16(xsrc[i] + (size_t)ks * 128, lds + stage * kArStage + (w + 8 * i) * 1024);
    };

    const int i32 = lane & 31, q = lane >> 5;
    // this lane's piece of a stored fragment: strip (32 w % TILE) / 16 + i32 / 16 of the tile, fragment lane 16 q + i32 % 16
    const int strip = (fo % TILE) / kStripRows + (i32 >> 4);
    const int flane = 16 * q + (i32 & 15);
    // one step's weights: tile entry e, K-step j of the tile
    auto load_w = [&](ArWeights& d, uint32_t e, int j) {
        const bool sp = entry_sparse(e);
        // the fragment of (strip, K-step j): 1 KB (2:4: halves of 512 B) or 2 KB (dense: two operands per half of 1 KB)
        const uint8_t* f = payload + entry_offset(e) + (size_t)(strip * KPT + j) * (sp ? kSparseFragBytes : kDenseFragBytes) + flane * 16;
        d.h0a.raw = *(ar_g16_t)(f);
        d.h1a.raw = *(ar_g16_t)(f + (sp ? 512 : 1024));
        if (!sp) {
            d.h0b.raw = *(ar_g16_t)(f + 512);
            d.h1b.raw = *(ar_g16_t)(f + 1536);
        }
    };
    // the position words of a 2:4 tile for half-steps 0 and 1 (fragment lanes flane and flane + 32): mask tile 128 a
    // dword holding both K-steps, mask tile 64 a 16-bit word
    auto load_pos = [&](uint32_t& d0, uint32_t& d1, uint32_t e) {
        if (entry_sparse(e)) {
            const uint8_t* pb = payload + entry_offset(e) + sparse_vals_bytes(TILE) + (size_t)(strip * 64 + flane) * (2 * KPT);
            if constexpr (KPT == 2) {
                d0 = *(ar_g4_t)(pb);
                d1 = *(ar_g4_t)(pb + 32 * 4);
            } else {
                d0 = *(ar_g2_t)(pb);
                d1 = *(ar_g2_t)(pb + 32 * 2);
            }
        }
    };

    f32x16 acc[NB];
#pragma unroll
    for (int b = 0; b < NB; ++b)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[b][i] = 0.f;

    // A K-step in two parts, with the next step's weight loads issued between them: (1) wait for the stage, refill the
    // other one; (2) multiply on the weights wc (tile type sp, position dwords p0 / p1, K-step j of the tile).
    auto step_begin = [&](int ks, int pf_ks) {
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        load_x(pf_ks, (ks & 1) ^ 1);
    };
    auto step_mma = [&](int ks, const ArWeights& wc, uint32_t p0, uint32_t p1, int sp, int j) {
        const uint8_t* bs = lds + (ks & 1) * kArStage;
        // position p = (half-step p / (NB / 2), row blocks 2 (p % (NB / 2)) and + 1); X fragments two positions ahead
        B16 xa[3], xb[3];
        auto fetch = [&](int p, int buf) {
            const int u = p / (NB / 2), b0 = 2 * (p % (NB / 2));
#pragma unroll
            for (int c = 0; c < 2; ++c) {
                xa[buf].raw[c] = *reinterpret_cast<const u32x4*>(bs + xs_off(32 * b0 + i32, 2 * (2 * u + c) + q));
                xb[buf].raw[c] = *reinterpret_cast<const u32x4*>(bs + xs_off(32 * (b0 + 1) + i32, 2 * (2 * u + c) + q));
            }
        };
        fetch(0, 0);
        fetch(1, 1);
#pragma unroll
        for (int p = 0; p < NB; ++p) {
            if (p + 2 < NB) fetch(p + 2, (p + 2) % 3);
            const int u = p / (NB / 2), b0 = 2 * (p % (NB / 2)), buf = p % 3;
            mma_step(acc[b0], acc[b0 + 1], u ? wc.h1a.v : wc.h0a.v, u ? wc.h1b.v : wc.h0b.v, xa[buf], xb[buf], (int)((u ? p1 : p0) >> (16 * j)), sp);
        }
    };

    if constexpr (KPT == 2) {
        ArWeights w0, w1;            // weights of the even / odd step of a tile
        uint32_t p0 = 0u, p1 = 0u, pn0 = 0u, pn1 = 0u;
        uint32_t e = trow[0];
        load_x(0, 0);
        load_w(w0, e, 0);
        load_pos(pn0, pn1, e);
        __builtin_assume(Tk > 0);        // every K slice holds at least one tile (prefill_lds_split)
        for (int tk = 0; tk < Tk; ++tk) {
            const int more = tk + 1 < Tk ? 1 : 0;
            const uint32_t en = trow[tk + more];
            const int sp = (int)(e & 1u);
            step_begin(2 * tk, 2 * tk + 1);
            // this tile's position dwords were loaded a step ago into (pn0, pn1) and have landed.  They are taken over here by
            // an opaque copy: a plain assignment becomes a copy on the loop's back edge, right behind the loads it then
            // has to wait for
            asm volatile("v_mov_b32 %0, %2\n\tv_mov_b32 %1, %3" : "=&v"(p0), "=&v"(p1) : "v"(pn0), "v"(pn1));
            load_w(w1, e, 1);
            step_mma(2 * tk, w0, p0, p1, sp, 0);
            // (the very last step fetches its own X again and the first step's weights of its own tile: no branch)
            step_begin(2 * tk + 1, 2 * tk + 1 + more);
            load_w(w0, en, 0);
            load_pos(pn0, pn1, en);
            step_mma(2 * tk + 1, w1, p0, p1, sp, 1);
            e = en;
        }
    } else {
        // Mask tile 64: every step is a tile of its own.  Steps go in pairs (the buffers w0 / w1 alternate without a
        // copy), table entries are read two steps ahead; past the end the last step is fetched again (no branch around
        // the loads), and the second step of the last pair is skipped when the count is odd.
        const int S = Tk;
        ArWeights w0, w1;
        uint32_t a0 = 0u, a1 = 0u, b0_ = 0u, b1_ = 0u;   // position words of w0 / w1
        uint32_t e0 = trow[0], e1 = trow[S > 1 ? 1 : 0];
        load_x(0, 0);
        load_w(w0, e0, 0);
        load_pos(a0, a1, e0);
        __builtin_assume(S > 0);
        for (int s_ = 0; s_ < S; s_ += 2) {
            const int s1 = s_ + 1 < S ? s_ + 1 : S - 1, s2 = s_ + 2 < S ? s_ + 2 : S - 1, s3 = s_ + 3 < S ? s_ + 3 : S - 1;
            const uint32_t e2 = trow[s2], e3 = trow[s3];
            step_begin(s_, s1);
            load_w(w1, e1, 0);
            load_pos(b0_, b1_, e1);
            step_mma(s_, w0, a0, a1, (int)(e0 & 1u), 0);
            if (s_ + 1 < S) {
                step_begin(s_ + 1, s2);
                load_w(w0, e2, 0);
                load_pos(a0, a1, e2);
                step_mma(s_ + 1, w1, b0_, b1_, (int)(e1 & 1u), 0);
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
                             M - (m0 + 32 * b), SPLIT ? 0 : ybf16);
    }
}

template <int TILE, int BM>
static void launch_prefill_areg(const GemmArgs& a, int split_k, hipStream_t stream) {
    constexpr int kLds = 2 * BM * 128;    // 32 or 64 KB
    const int tiles_n = (int)((a.N + kPfBN - 1) / kPfBN), tiles_m = (int)((a.M + BM - 1) / BM);
    const int nblk = tiles_n * tiles_m;
    const int grid = ((nblk + 7) / 8) * 8;
    const int split = prefill_lds_split(a, split_k, BM);
    if (split == 1) {
        hipLaunchKernelGGL((prefill_kernel_areg<TILE, BM, false>), dim3(grid), dim3(512), kLds, stream, a.X, a.M, a.N, a.K, a.payload, a.table,
                           a.Tk, tiles_n, tiles_m, a.Y, a.ybf16);
    } else {
        hipLaunchKernelGGL((prefill_kernel_areg<TILE, BM, true>), dim3(grid, split), dim3(512), kLds, stream, a.X, a.M, a.N, a.K, a.payload,
                           a.table, a.Tk, tiles_n, tiles_m, a.ws, 0);
        wr_reduce(a.ws, (size_t)a.M * (size_t)a.N / 4, split, a.Y, a.ybf16, stream);
    }
}

// K slices per output tile of the LDS-staged kernel: as prefill_wreg_split, each slice at least 512 columns long.
int prefill_lds_split(const GemmArgs& a, int requested, int bm) {
    const int tiles = (int)(((a.N + kPfBN - 1) / kPfBN) * ((a.M + bm - 1) / bm));
    const int min_tiles = 512 / a.tile;
    int s = requested;
    if (s <= 0) {
        s = 1;
        if (tiles < (a.n_cus * 2) / 3) {
            s = a.n_cus / tiles;
            if (s > a.Tk / min_tiles) s = a.Tk / min_tiles;
            if (s > 8) s = 8;
        }
    }
    if (s > a.Tk) s = a.Tk;
    const size_t per_slice = (size_t)a.M * (size_t)a.N * sizeof(float);
    const size_t fit = (a.ws && per_slice) ? a.ws_bytes / per_slice : 0;
    if ((size_t)s > fit) s = (int)fit;
    return s < 2 ? 1 : s;
}

// Blocks of 128 rows or of 256?  Few rows leave most of a 256-row block empty, and a weight of few feature blocks
// fills the chip only through a deep K split, whose partial products are written and read again.  Both sides are
// estimated from measured rates:
//     us = rounds x K-steps per workgroup x t_step + 3 + (split > 1 ? 3 + (2 split + 1) M N 4 B / 5.5 TB/s : 0)
// A step is slower the fuller the chip (shared L2 bandwidth, power): t_step = t0 + t1 x min(1, workgroups / compute
// units), with (t0, t1) = (0.90, 0.35) us for prefill_kernel_wreg, (1.26, 0.33) for the 256-row kernels of mask tile 64
// and of long K, and for prefill_kernel_areg with 128 rows (0.70, 0.24) on mask tile 128, (0.75, 0.22) on mask tile 64 (fitted
// to unsplit launches of 16 and of 256 workgroups at f = 0.6).  The 256-row side takes the
// split its launcher would take; the 128-row side its best split of at most 8 slices of at least 512 columns that the
// workspace holds.  Returns true, and the split, when 128 rows are estimated at least 3 % faster.
static double pf_estimate(const GemmArgs& a, int blocks, int split, double t0, double t1) {
    const int rounds = (blocks * split + a.n_cus - 1) / a.n_cus;
    const int steps = ((a.Tk + split - 1) / split) * (a.tile / kStepCols);
    const double fill = blocks * split < a.n_cus ? (double)(blocks * split) / a.n_cus : 1.0;
    double us = rounds * steps * (t0 + t1 * fill) + 3.0;
    if (split > 1) us += 3.0 + (2.0 * split + 1.0) * (double)a.M * (double)a.N * 4.0 / 5.5e6;
    return us;
}

bool prefill_prefers_128_rows(const GemmArgs& a, int* split) {
    const int tiles_n = (int)((a.N + kPfBN - 1) / kPfBN);
    const int b256 = tiles_n * (int)((a.M + 255) / 256), b128 = tiles_n * (int)((a.M + 127) / 128);
    const bool wreg = a.tile == 128 && prefill_wreg_supports(a);
    const double us256 = pf_estimate(a, b256, wreg ? prefill_wreg_split(a, 0) : prefill_lds_split(a, 0, 256), wreg ? 0.90 : 1.26,
                                     wreg ? 0.35 : 0.33);
    const size_t per_slice = (size_t)a.M * (size_t)a.N * sizeof(float);
    const int fit = a.ws ? (int)(a.ws_bytes / per_slice < 8 ? a.ws_bytes / per_slice : 8) : 1;
    const int longest = a.Tk * a.tile / 512;
    double best = 0.0;
    *split = 1;
    for (int sp = 1; sp <= 8 && (sp == 1 || (sp <= fit && sp <= longest)); ++sp) {
        const double us = pf_estimate(a, b128, sp, a.tile == 128 ? 0.70 : 0.75, a.tile == 128 ? 0.24 : 0.22);
        if (sp == 1 || us < best) { best = us; *split = sp; }
    }
    return best < 0.97 * us256;
}

// Kernel choice.  variant 0 (default): prefill_kernel_areg with blocks of 128 rows where prefill_prefers_128_rows says so
// (no split requested); else 256 rows: tile 128 -> prefill_kernel_wreg where its limits hold, else prefill_kernel_lds;
// tile 64 -> prefill_kernel_areg.  variant 1 forces prefill_kernel_v0, 2 prefill_kernel_lds (256 rows), 3
// prefill_kernel_wreg, 4 prefill_kernel_lds with 128 rows, 5 prefill_kernel_areg with 128 rows, 6 prefill_kernel_areg
// with 256 rows (mask tile 64 only); each falls back to the default choice where it does not apply.
template <int TILE, int BM>
static void launch_prefill_lds(const GemmArgs& a, int split_k, hipStream_t stream) {
    constexpr int kLds = pf_lds_bytes(BM);
    static const hipError_t granted0 = hipFuncSetAttribute(reinterpret_cast<const void*>(&prefill_kernel_lds<TILE, false, BM>),
                                                           hipFuncAttributeMaxDynamicSharedMemorySize, kLds);
    static const hipError_t granted1 = hipFuncSetAttribute(reinterpret_cast<const void*>(&prefill_kernel_lds<TILE, true, BM>),
                                                           hipFuncAttributeMaxDynamicSharedMemorySize, kLds);
    (void)granted0;
    (void)granted1;
    const int tiles_n = (int)((a.N + kPfBN - 1) / kPfBN), tiles_m = (int)((a.M + BM - 1) / BM);
    const int nblk = tiles_n * tiles_m;
    const int grid = ((nblk + 7) / 8) * 8;
    const int split = prefill_lds_split(a, split_k, BM);
    if (split == 1) {
        hipLaunchKernelGGL((prefill_kernel_lds<TILE, false, BM>), dim3(grid), dim3(512), kLds, stream, a.X, a.M, a.N, a.K, a.payload,
                           a.table, a.Tk, tiles_n, tiles_m, a.Y, a.ybf16);
    } else {
        hipLaunchKernelGGL((prefill_kernel_lds<TILE, true, BM>), dim3(grid, split), dim3(512), kLds, stream, a.X, a.M, a.N, a.K, a.payload,
                           a.table, a.Tk, tiles_n, tiles_m, a.ws, 0);
        wr_reduce(a.ws, (size_t)a.M * (size_t)a.N / 4, split, a.Y, a.ybf16, stream);
    }
}

void launch_prefill(const GemmArgs& a, int variant, int split_k, hipStream_t stream) {
    if (variant == 0 && split_k == 0) {
        int split128 = 1;
        if (prefill_prefers_128_rows(a, &split128)) {
            if (a.tile == 128) launch_prefill_areg<128, 128>(a, split128, stream);
            else launch_prefill_areg<64, 128>(a, split128, stream);
            return;
        }
    }
    if (a.tile == 128 && (variant == 0 || variant == 3) && prefill_wreg_supports(a)) { launch_prefill_wreg(a, split_k, stream); return; }
    if (variant == 5) {   // 128 rows, weights in registers
        if (a.tile == 128) launch_prefill_areg<128, 128>(a, split_k, stream);
        else launch_prefill_areg<64, 128>(a, split_k, stream);
        return;
    }
    if ((variant == 0 || variant == 6) && a.tile == 64) { launch_prefill_areg<64, 256>(a, split_k, stream); return; }   // 256 rows
    if (variant == 4) {   // the LDS-staged kernel with blocks of 128 rows
        if (a.tile == 128) launch_prefill_lds<128, 128>(a, split_k, stream);
        else launch_prefill_lds<64, 128>(a, split_k, stream);
        return;
    }
    if (variant != 1) {
        if (a.tile == 128) launch_prefill_lds<128, 256>(a, split_k, stream);
        else launch_prefill_lds<64, 256>(a, split_k, stream);
        return;
    }
    dim3 grid((unsigned)((a.N + 127) / 128), (unsigned)((a.M + 127) / 128)), block(256);
    if (a.tile == 128)
        hipLaunchKernelGGL((prefill_kernel_v0<128, 128>), grid, block, 0, stream, a.X, a.M, a.N, a.K, a.payload, a.table, a.Tk, a.Y, a.ybf16);
    else
        hipLaunchKernelGGL((prefill_kernel_v0<64, 128>), grid, block, 0, stream, a.X, a.M, a.N, a.K, a.payload, a.table, a.Tk, a.Y, a.ybf16);
}

}  // namespace patch
