// Decode-shaped hybrid GEMM (at most 16 rows of X per launch), split-K with an in-kernel, fixed-order
// reduction.  This is the product Y = X * W_hat^T of Section 4 / Appendix A of the paper for the decoding
// input (batch x K), with "split-K" as the schedule Appendix A names.
//
// Mapping.  The weight is the A operand (the sparse operand of the gfx950 sparse matrix instruction is A),
// so the kernel computes Y^T = W_hat * X^T: a wavefront owns a strip of 16 output features and walks along
// K; the up-to-16 rows of X are the 16 columns of the instruction.  Weight fragments go HBM -> registers
// directly (every weight byte is used exactly once; layout.h gives the register-order storage); X is staged
// once per workgroup in LDS.  Per tile the wavefront takes ONE scalar branch on the tile type:
//   dense : 2 x v_mfma_f32_16x16x32_bf16 per 64 columns
//   2:4   : 1 x v_smfmac_f32_16x16x64_bf16 per 64 columns
// Workgroup = 4 wavefronts = 4 adjacent strips (64 output features) x one K slice.  Slices write fp32
// partials; the last-arriving workgroup of each 64-feature block sums them in slice order (deterministic)
// and resets the arrival counter.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "kernels.h"
#include "layout.h"

namespace patch {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr int kDecodeChunkK = 1024;  // columns of X staged in LDS at a time
constexpr int kXsStride = kDecodeChunkK + 8;

union AFrag { u32x4 raw; bf16x8 v; };
union BFrag { u32x4 raw[2]; bf16x8 h[2]; bf16x16 v; };

template <int TILE>
__global__ __launch_bounds__(256) void decode_kernel(const uint16_t* __restrict__ X, int64_t m0, int rows, int64_t K,
                                                     const uint8_t* __restrict__ payload, const uint32_t* __restrict__ table,
                                                     int Tk, int tiles_per_split, int S, float* __restrict__ ws,
                                                     unsigned* __restrict__ counters, float* __restrict__ Y, int64_t N) {
    constexpr int KPT = TILE / kStepCols, SPT = TILE / kStripRows, TC = kDecodeChunkK / TILE;
    __shared__ __attribute__((aligned(16))) uint16_t Xs[16 * kXsStride];
    __shared__ int s_is_last;

    const int tid = threadIdx.x, lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int strip = blockIdx.x * 4 + w;
    const int tn = strip / SPT, s = strip % SPT;
    const int split = blockIdx.y;
    const int tk0 = split * tiles_per_split;
    const int tk1 = (tk0 + tiles_per_split < Tk) ? tk0 + tiles_per_split : Tk;
    const int col = lane & 15, q = lane >> 4;

    f32x4 acc = {0.f, 0.f, 0.f, 0.f};

    for (int tkc = tk0; tkc < tk1; tkc += TC) {
        const int ntile = (tk1 - tkc < TC) ? tk1 - tkc : TC;
        const int klen = ntile * TILE;
        const int64_t kbase = (int64_t)tkc * TILE;
        __syncthreads();
        {
            const int cpr = klen / 8;  // 16-byte chunks per row
            for (int c = tid; c < 16 * cpr; c += 256) {
                const int r = c / cpr, kk = (c % cpr) * 8;
                u32x4 v = {0u, 0u, 0u, 0u};
                if (r < rows) v = *reinterpret_cast<const u32x4*>(X + (m0 + r) * K + kbase + kk);
                *reinterpret_cast<u32x4*>(&Xs[r * kXsStride + kk]) = v;
            }
        }
        __syncthreads();

        for (int ti = 0; ti < ntile; ++ti) {
            const uint32_t e = table[(int64_t)tn * Tk + tkc + ti];
            const uint8_t* base = payload + entry_offset(e);
            const uint16_t* xs = &Xs[col * kXsStride + ti * TILE + 8 * q];
            if (entry_sparse(e)) {
                const uint8_t* vals = base + (size_t)s * KPT * kSparseFragBytes + lane * 16;
                const uint16_t* meta = reinterpret_cast<const uint16_t*>(base + sparse_vals_bytes(TILE)) + (s * 64 + lane) * KPT;
                AFrag a[KPT];
                uint32_t idx;
#pragma unroll
                for (int j = 0; j < KPT; ++j) a[j].raw = *reinterpret_cast<const u32x4*>(vals + j * kSparseFragBytes);
                if constexpr (KPT == 2) idx = *reinterpret_cast<const uint32_t*>(meta);
                else idx = *meta;
#pragma unroll
                for (int j = 0; j < KPT; ++j) {
                    BFrag b;
                    b.raw[0] = *reinterpret_cast<const u32x4*>(xs + 64 * j);
                    b.raw[1] = *reinterpret_cast<const u32x4*>(xs + 64 * j + 32);
                    if (j == 0) acc = __builtin_amdgcn_smfmac_f32_16x16x64_bf16(a[j].v, b.v, acc, (int)idx, 0, 0);
                    else acc = __builtin_amdgcn_smfmac_f32_16x16x64_bf16(a[j].v, b.v, acc, (int)idx, 0, 1);
                }
            } else {
                const uint8_t* frag = base + (size_t)s * KPT * kDenseFragBytes + lane * 16;
                AFrag a[KPT * 2];
#pragma unroll
                for (int jh = 0; jh < KPT * 2; ++jh) a[jh].raw = *reinterpret_cast<const u32x4*>(frag + jh * 1024);
#pragma unroll
                for (int j = 0; j < KPT; ++j) {
                    BFrag b;
                    b.raw[0] = *reinterpret_cast<const u32x4*>(xs + 64 * j);
                    b.raw[1] = *reinterpret_cast<const u32x4*>(xs + 64 * j + 32);
                    acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[2 * j].v, b.h[0], acc, 0, 0, 0);
                    acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[2 * j + 1].v, b.h[1], acc, 0, 0, 0);
                }
            }
        }
    }

    // acc[r] = Y^T[strip*16 + 4 q + r][col]  ->  Y[m0 + col][strip*16 + 4 q + r]
    const int64_t n = (int64_t)strip * 16 + 4 * q;
    if (S == 1) {
        if (col < rows) *reinterpret_cast<f32x4*>(Y + (m0 + col) * N + n) = acc;
        return;
    }
    if (col < rows) *reinterpret_cast<f32x4*>(ws + ((int64_t)split * 16 + col) * N + n) = acc;
    __threadfence();
    __syncthreads();
    if (tid == 0) {
        const unsigned old = atomicAdd(&counters[blockIdx.x], 1u);
        s_is_last = (old == (unsigned)(S - 1));
    }
    __syncthreads();
    if (!s_is_last) return;
    __threadfence();
    {
        const int c = tid & 63;
        const int64_t nn = (int64_t)blockIdx.x * 64 + c;
        for (int r = tid >> 6; r < rows; r += 4) {
            float sum = 0.f;
            for (int sp = 0; sp < S; ++sp)
                sum += __hip_atomic_load(ws + ((int64_t)sp * 16 + r) * N + nn, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            Y[(m0 + r) * N + nn] = sum;
        }
    }
    if (tid == 0) atomicExch(&counters[blockIdx.x], 0u);
}

int decode_max_split(int64_t N, int Tk) {
    int64_t cap = 8192 / (N / 16);
    if (cap < 1) cap = 1;
    if (cap > 64) cap = 64;
    return (int)(cap < Tk ? cap : Tk);
}

int launch_decode(const GemmArgs& a, int64_t m0, int rows, int split_k, int variant, hipStream_t stream) {
    (void)variant;
    const int strips = (int)(a.N / 16);
    int S = split_k;
    if (S <= 0) {
        const int target_waves = a.n_cus * 16;
        S = (target_waves + strips / 2) / strips;
        if (S < 1) S = 1;
    }
    const int smax = decode_max_split(a.N, a.Tk);
    if (S > smax) S = smax;
    while (S > 1 && (size_t)S * 16 * (size_t)a.N > a.ws_floats) --S;
    int tps = (a.Tk + S - 1) / S;
    S = (a.Tk + tps - 1) / tps;
    dim3 grid((unsigned)(a.N / 64), (unsigned)S), block(256);
    if (a.tile == 128)
        hipLaunchKernelGGL(decode_kernel<128>, grid, block, 0, stream, a.X, m0, rows, a.K, a.payload, a.table, a.Tk, tps, S, a.ws,
                           a.counters, a.Y, a.N);
    else
        hipLaunchKernelGGL(decode_kernel<64>, grid, block, 0, stream, a.X, m0, rows, a.K, a.payload, a.table, a.Tk, tps, S, a.ws,
                           a.counters, a.Y, a.N);
    return S;
}

}  // namespace patch
