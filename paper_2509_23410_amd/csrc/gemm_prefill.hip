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

#include "kernels.h"
#include "layout.h"

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

template <int TILE, int BM>
__global__ __launch_bounds__(256) void prefill_kernel_v0(const uint16_t* __restrict__ X, int64_t M, int64_t N, int64_t K,
                                                         const uint8_t* __restrict__ payload, const uint32_t* __restrict__ table,
                                                         int Tk, float* __restrict__ Y) {
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
                *reinterpret_cast<f32x4*>(Y + m * N + n0 + 64 * wn + 32 * a + 8 * g + 4 * q) = v;
            }
    }
}

void launch_prefill(const GemmArgs& a, int variant, hipStream_t stream) {
    (void)variant;
    dim3 grid((unsigned)((a.N + 127) / 128), (unsigned)((a.M + 127) / 128)), block(256);
    if (a.tile == 128)
        hipLaunchKernelGGL((prefill_kernel_v0<128, 128>), grid, block, 0, stream, a.X, a.M, a.N, a.K, a.payload, a.table, a.Tk, a.Y);
    else
        hipLaunchKernelGGL((prefill_kernel_v0<64, 128>), grid, block, 0, stream, a.X, a.M, a.N, a.K, a.payload, a.table, a.Tk, a.Y);
}

}  // namespace patch
