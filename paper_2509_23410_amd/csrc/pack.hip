// Mask merge, compression and decompression kernels (gfx950).
//
// Compression follows Appendix A of the paper (compress a mixed dense / 2:4 weight for a given tile size);
// the mask merge follows the last lines of Algorithm 1 / Eq. 4 with hard masks.  The byte layout written
// here is described in layout.h.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "kernels.h"
#include "layout.h"

namespace patch {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

// ------------------------------------------------------------------ mask merge
// One thread per 8 consecutive elements of a row (16 bytes of W, 8 bytes of mask).
// W_hat may be W itself (in place): neither is declared restrict.
__global__ __launch_bounds__(256) void apply_mask_kernel(const uint16_t* W, const uint8_t* __restrict__ mask24,
                                                         const uint8_t* __restrict__ tile_map, int64_t N, int64_t K, int tile,
                                                         uint16_t* W_hat) {
    const int64_t chunks_per_row = K / 8;
    const int64_t total = N * chunks_per_row;
    const int64_t Tk = K / tile;
    for (int64_t c = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; c < total; c += (int64_t)gridDim.x * blockDim.x) {
        const int64_t n = c / chunks_per_row, k = (c % chunks_per_row) * 8;
        const int m_tile = tile_map[(n / tile) * Tk + k / tile] ? 1 : 0;
        union { u32x4 v; uint16_t h[8]; } w;
        w.v = *reinterpret_cast<const u32x4*>(W + n * K + k);
        if (!m_tile) {
            union { uint2 v; uint8_t b[8]; } m;
            m.v = *reinterpret_cast<const uint2*>(mask24 + n * K + k);
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                // M* = M_tile + (1 - M_tile) * M_24 with M_tile = 0 here
                if (!m.b[e]) w.h[e] = 0;
            }
        }
        *reinterpret_cast<u32x4*>(W_hat + n * K + k) = w.v;
    }
}

void launch_apply_mask(const uint16_t* W, const uint8_t* mask24, const uint8_t* d_tile_map, int64_t N, int64_t K, int tile,
                       uint16_t* W_hat, hipStream_t stream) {
    const int64_t total = N * (K / 8);
    int blocks = (int)((total + 255) / 256);
    if (blocks > 256 * 32) blocks = 256 * 32;
    hipLaunchKernelGGL(apply_mask_kernel, dim3(blocks), dim3(256), 0, stream, W, mask24, d_tile_map, N, K, tile, W_hat);
}

// ------------------------------------------------------------------ hard 2:4 mask from the pattern logits
// One thread per group of four consecutive elements: the candidate with the largest of the six logits (first one on
// ties; a NaN never wins a comparison), written as four keep bytes.  Candidates in lexicographic order of the kept
// positions: (0,1) (0,2) (0,3) (1,2) (1,3) (2,3).
__global__ __launch_bounds__(256) void hard_mask24_kernel(const float* __restrict__ P24, int64_t G, uint32_t* __restrict__ mask24) {
    // keep bytes of candidate c, little endian: byte j = element j of the group
    constexpr uint32_t kPattern[6] = {0x00000101u, 0x00010001u, 0x01000001u, 0x00010100u, 0x01000100u, 0x01010000u};
    for (int64_t g = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; g < G; g += (int64_t)gridDim.x * blockDim.x) {
        float best = P24[g];
        uint32_t pat = kPattern[0];
#pragma unroll
        for (int c = 1; c < 6; ++c) {
            const float v = P24[(int64_t)c * G + g];
            const bool better = v > best;
            best = better ? v : best;
            pat = better ? kPattern[c] : pat;
        }
        mask24[g] = pat;
    }
}

void launch_hard_mask24(const float* P24, int64_t G, uint8_t* mask24, hipStream_t stream) {
    int blocks = (int)((G + 255) / 256);
    if (blocks > 256 * 32) blocks = 256 * 32;
    hipLaunchKernelGGL(hard_mask24_kernel, dim3(blocks), dim3(256), 0, stream, P24, G, reinterpret_cast<uint32_t*>(mask24));
}

// ------------------------------------------------------------------ compression
__device__ __forceinline__ bool bf16_nonzero(uint16_t h) { return (h & 0x7FFFu) != 0; }

// Compress 4 groups of 4 (16 consecutive elements of one row) into 8 kept values + 16 position bits.
// Returns false if some group holds more than two nonzeros.
__device__ __forceinline__ bool compress16(const uint16_t* in, uint16_t* out, uint32_t& idx) {
    bool ok = true;
    idx = 0;
#pragma unroll
    for (int g = 0; g < 4; ++g) {
        const uint16_t* grp = in + 4 * g;
        int nnz = 0;
        bool keep[4];
#pragma unroll
        for (int p = 0; p < 4; ++p) { keep[p] = bf16_nonzero(grp[p]); nnz += keep[p] ? 1 : 0; }
        if (nnz > 2) ok = false;
        // fewer than two nonzeros: also keep the lowest-index zeros
#pragma unroll
        for (int p = 0; p < 4; ++p)
            if (!keep[p] && nnz < 2) { keep[p] = true; ++nnz; }
        int p0 = -1, p1 = -1;
#pragma unroll
        for (int p = 0; p < 4; ++p)
            if (keep[p]) { if (p0 < 0) p0 = p; else if (p1 < 0) p1 = p; }
        if (p1 < 0) { p0 = 0; p1 = 1; }  // unreachable when ok; keeps indices in range otherwise
        out[2 * g] = grp[p0];
        out[2 * g + 1] = grp[p1];
        idx |= (uint32_t)(p0 | (p1 << 2)) << (4 * g);
    }
    return ok;
}

// One workgroup per tile.
__global__ __launch_bounds__(256) void pack_kernel(const uint16_t* __restrict__ W, int64_t K, const uint32_t* __restrict__ table,
                                                   int Tk, int tile, uint8_t* __restrict__ payload, int* __restrict__ err) {
    const int t = blockIdx.x;
    const int tn = t / Tk, tk = t % Tk;
    const uint32_t e = table[t];
    uint8_t* base = payload + entry_offset(e);
    const int64_t n0 = (int64_t)tn * tile, k0 = (int64_t)tk * tile;
    const int KPT = tile / kStepCols;
    if (!entry_sparse(e)) {
        const int nchunks = tile * tile / 8;
        for (int c = threadIdx.x; c < nchunks; c += blockDim.x) {
            const int lane = c & 63, h = (c >> 6) & 1, sj = c >> 7;
            const int j = sj % KPT, s = sj / KPT, i = lane & 15, q = lane >> 4;
            const uint16_t* src = W + (n0 + 16 * s + i) * K + k0 + 64 * j + 32 * h + 8 * q;
            *reinterpret_cast<u32x4*>(base + (size_t)c * 16) = *reinterpret_cast<const u32x4*>(src);
        }
    } else {
        const int nchunks = tile * tile / 16;
        uint16_t* meta = reinterpret_cast<uint16_t*>(base + sparse_vals_bytes(tile));
        bool ok = true;
        for (int c = threadIdx.x; c < nchunks; c += blockDim.x) {
            const int lane = c & 63, sj = c >> 6;
            const int j = sj % KPT, s = sj / KPT, i = lane & 15, qa = lane >> 4;
            const uint16_t* src = W + (n0 + 16 * s + i) * K + k0 + 64 * j + 16 * qa;
            union { u32x4 v[2]; uint16_t h[16]; } in;
            in.v[0] = *reinterpret_cast<const u32x4*>(src);
            in.v[1] = *reinterpret_cast<const u32x4*>(src + 8);
            union { u32x4 v; uint16_t h[8]; } out;
            uint32_t idx;
            ok = compress16(in.h, out.h, idx) && ok;
            *reinterpret_cast<u32x4*>(base + (size_t)c * 16) = out.v;
            meta[(s * 64 + lane) * KPT + j] = (uint16_t)idx;
        }
        if (!ok) atomicOr(err, 1);
    }
}

void launch_pack(const uint16_t* W, int64_t K, const uint32_t* d_table, int n_tiles, int Tk, int tile, uint8_t* payload, int* d_err,
                 hipStream_t stream) {
    hipLaunchKernelGGL(pack_kernel, dim3(n_tiles), dim3(256), 0, stream, W, K, d_table, Tk, tile, payload, d_err);
}

// ------------------------------------------------------------------ decompression
__global__ __launch_bounds__(256) void unpack_kernel(const uint8_t* __restrict__ payload, const uint32_t* __restrict__ table, int Tk,
                                                     int tile, int64_t K, uint16_t* __restrict__ W_out) {
    const int t = blockIdx.x;
    const int tn = t / Tk, tk = t % Tk;
    const uint32_t e = table[t];
    const uint8_t* base = payload + entry_offset(e);
    const int64_t n0 = (int64_t)tn * tile, k0 = (int64_t)tk * tile;
    const int KPT = tile / kStepCols;
    if (!entry_sparse(e)) {
        const int nchunks = tile * tile / 8;
        for (int c = threadIdx.x; c < nchunks; c += blockDim.x) {
            const int lane = c & 63, h = (c >> 6) & 1, sj = c >> 7;
            const int j = sj % KPT, s = sj / KPT, i = lane & 15, q = lane >> 4;
            uint16_t* dst = W_out + (n0 + 16 * s + i) * K + k0 + 64 * j + 32 * h + 8 * q;
            *reinterpret_cast<u32x4*>(dst) = *reinterpret_cast<const u32x4*>(base + (size_t)c * 16);
        }
    } else {
        const int nchunks = tile * tile / 16;
        const uint16_t* meta = reinterpret_cast<const uint16_t*>(base + sparse_vals_bytes(tile));
        for (int c = threadIdx.x; c < nchunks; c += blockDim.x) {
            const int lane = c & 63, sj = c >> 6;
            const int j = sj % KPT, s = sj / KPT, i = lane & 15, qa = lane >> 4;
            union { u32x4 v; uint16_t h[8]; } in;
            in.v = *reinterpret_cast<const u32x4*>(base + (size_t)c * 16);
            const uint32_t idx = meta[(s * 64 + lane) * KPT + j];
            union { u32x4 v[2]; uint16_t h[16]; } out;
            out.v[0] = u32x4{0, 0, 0, 0};
            out.v[1] = u32x4{0, 0, 0, 0};
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int p0 = (idx >> (4 * g)) & 3, p1 = (idx >> (4 * g + 2)) & 3;
#pragma unroll
                for (int p = 0; p < 4; ++p) {
                    uint16_t v = 0;
                    if (p == p0) v = in.h[2 * g];
                    if (p == p1) v = in.h[2 * g + 1];
                    out.h[4 * g + p] = v;
                }
            }
            uint16_t* dst = W_out + (n0 + 16 * s + i) * K + k0 + 64 * j + 16 * qa;
            *reinterpret_cast<u32x4*>(dst) = out.v[0];
            *reinterpret_cast<u32x4*>(dst + 8) = out.v[1];
        }
    }
}

void launch_unpack(const uint8_t* payload, const uint32_t* d_table, int n_tiles, int Tk, int tile, int64_t K, uint16_t* W_out,
                   hipStream_t stream) {
    hipLaunchKernelGGL(unpack_kernel, dim3(n_tiles), dim3(256), 0, stream, payload, d_table, Tk, tile, K, W_out);
}

}  // namespace patch
