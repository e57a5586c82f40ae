// Measured ceilings of the part, for the roofline figures the benchmark prints next to the product kernels:
//   matrix_rate_kernel  register-resident loops of the two matrix instructions the product kernels use
//                       (v_mfma_f32_16x16x32_bf16, v_smfmac_f32_16x16x64_bf16) and of their 32 x 32 shapes, no memory
//                       traffic inside the loop
//   stream_read_kernel  128-bit streaming read of a buffer (the HBM bound of the decode path)
//   store_tiles_kernel  the output stage of a prefill workgroup on its own, in two store patterns
//   lds_read_kernel     what four wavefronts of a compute unit read from LDS (the X fragments of the prefill kernels)
// They compute nothing of the method; the caller times them with events on the stream it passes.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/patch.h"

namespace patch {

typedef __bf16 cl_bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 cl_bf16x16 __attribute__((ext_vector_type(16)));
typedef float cl_f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int cl_u32x4 __attribute__((ext_vector_type(4)));

union ClA { cl_u32x4 raw; cl_bf16x8 v; };
union ClB { cl_u32x4 raw[2]; cl_bf16x8 h[2]; cl_bf16x16 v; };

// One workgroup of 4 wavefronts (one per SIMD) per launch slot.  Every lane takes 4 A and 4 B operands from
// `operands` (the caller fills it with random bf16 so that consecutive instructions see different data: the clock
// under matrix load depends on how many bits toggle) and runs `iters` rounds of 16 independent instructions.
// KIND 0: dense 16x16x32, 16384 flop per instruction; KIND 1: 2:4 16x16x64, 32768 dense-equivalent flop.
// KIND 2 / 3: the 32 x 32 shapes of the same two instructions (v_mfma_f32_32x32x16_bf16, 32768 flop, and
// v_smfmac_f32_32x32x32_bf16, 65536 dense-equivalent flop; 8 per round on four 16-register accumulators, two
// consecutive instructions sharing the B operand): half the operand registers read per flop - the product kernels do not
// use them (their layout is built on the 16 x 16 shapes); the figure says what that choice costs under the power limit.
template <int KIND>
__global__ __launch_bounds__(256) void matrix_rate_kernel(const cl_u32x4* __restrict__ operands, int iters, float* __restrict__ out) {
    const int tid = threadIdx.x;
    ClA a[4];
    ClB b[4];
    uint32_t idx[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        a[i].raw = operands[(size_t)(i * 256 + tid)];
        b[i].raw[0] = operands[(size_t)((4 + 2 * i) * 256 + tid)];
        b[i].raw[1] = operands[(size_t)((5 + 2 * i) * 256 + tid)];
        // position bits of a 2:4 operand: each pair of 2-bit fields must name two different positions, ascending
        const uint32_t r = a[i].raw[0];
        uint32_t w = 0;
#pragma unroll
        for (int g = 0; g < 8; ++g) {
            const uint32_t p0 = (r >> (4 * g)) & 1u, p1 = 2u + ((r >> (4 * g + 1)) & 1u);
            w |= (p0 | (p1 << 2)) << (4 * g);
        }
        idx[i] = w;
    }
    // The loop body is written out with named accumulation registers a[0:63]: left to the compiler the accumulators
    // travel through copies and wait states that the product kernels (which name their registers too) do not have.
#define PATCH_CL_CLOBBER                                                                                              \
    "a0", "a1", "a2", "a3", "a4", "a5", "a6", "a7", "a8", "a9", "a10", "a11", "a12", "a13", "a14", "a15", "a16", "a17", "a18", \
        "a19", "a20", "a21", "a22", "a23", "a24", "a25", "a26", "a27", "a28", "a29", "a30", "a31", "a32", "a33", "a34", "a35",  \
        "a36", "a37", "a38", "a39", "a40", "a41", "a42", "a43", "a44", "a45", "a46", "a47", "a48", "a49", "a50", "a51", "a52",  \
        "a53", "a54", "a55", "a56", "a57", "a58", "a59", "a60", "a61", "a62", "a63"
#define PATCH_CL_ZERO4(R) "v_accvgpr_write_b32 a[" #R "], 0\n\tv_accvgpr_write_b32 a[" #R "+1], 0\n\tv_accvgpr_write_b32 a[" #R "+2], 0\n\tv_accvgpr_write_b32 a[" #R "+3], 0\n\t"
    asm volatile(PATCH_CL_ZERO4(0) PATCH_CL_ZERO4(4) PATCH_CL_ZERO4(8) PATCH_CL_ZERO4(12) PATCH_CL_ZERO4(16) PATCH_CL_ZERO4(20)
                 PATCH_CL_ZERO4(24) PATCH_CL_ZERO4(28) PATCH_CL_ZERO4(32) PATCH_CL_ZERO4(36) PATCH_CL_ZERO4(40) PATCH_CL_ZERO4(44)
                 PATCH_CL_ZERO4(48) PATCH_CL_ZERO4(52) PATCH_CL_ZERO4(56) PATCH_CL_ZERO4(60) "s_nop 4" ::: PATCH_CL_CLOBBER);
// instruction J of a round: accumulator J, A operand J % 4; B operand: J / 4 - four consecutive instructions share it, as in the
// product kernels, where four strips meet one block of X (with a new B operand for every instruction the dense
// instruction issued at about 60 % of this rate)
#define PATCH_CL_D(J, A, BH) "v_mfma_f32_16x16x32_bf16 a[4*" #J ":4*" #J "+3], %[a" #A "], %[b" #BH "], a[4*" #J ":4*" #J "+3]\n\t"
#define PATCH_CL_S(J, A, B_) "v_smfmac_f32_16x16x64_bf16 a[4*" #J ":4*" #J "+3], %[a" #A "], %[b" #B_ "], %[i" #A "]\n\t"
#define PATCH_CL_D32(J, A, BH) "v_mfma_f32_32x32x16_bf16 a[16*" #J ":16*" #J "+15], %[a" #A "], %[b" #BH "], a[16*" #J ":16*" #J "+15]\n\t"
#define PATCH_CL_S32(J, A, B_) "v_smfmac_f32_32x32x32_bf16 a[16*" #J ":16*" #J "+15], %[a" #A "], %[b" #B_ "], %[i" #A "]\n\t"
    for (int it = 0; it < iters; ++it) {
        if (KIND == 2) {
            asm volatile(PATCH_CL_D32(0, 0, 00) PATCH_CL_D32(1, 1, 00) PATCH_CL_D32(2, 2, 11) PATCH_CL_D32(3, 3, 11)
                         PATCH_CL_D32(0, 0, 20) PATCH_CL_D32(1, 1, 20) PATCH_CL_D32(2, 2, 31) PATCH_CL_D32(3, 3, 31)
                         :
                         : [a0] "v"(a[0].v), [a1] "v"(a[1].v), [a2] "v"(a[2].v), [a3] "v"(a[3].v), [b00] "v"(b[0].h[0]),
                           [b11] "v"(b[1].h[1]), [b20] "v"(b[2].h[0]), [b31] "v"(b[3].h[1])
                         : PATCH_CL_CLOBBER);
        } else if (KIND == 3) {
            asm volatile(PATCH_CL_S32(0, 0, 0) PATCH_CL_S32(1, 1, 0) PATCH_CL_S32(2, 2, 1) PATCH_CL_S32(3, 3, 1)
                         PATCH_CL_S32(0, 0, 2) PATCH_CL_S32(1, 1, 2) PATCH_CL_S32(2, 2, 3) PATCH_CL_S32(3, 3, 3)
                         :
                         : [a0] "v"(a[0].v), [a1] "v"(a[1].v), [a2] "v"(a[2].v), [a3] "v"(a[3].v), [b0] "v"(b[0].v), [b1] "v"(b[1].v),
                           [b2] "v"(b[2].v), [b3] "v"(b[3].v), [i0] "v"(idx[0]), [i1] "v"(idx[1]), [i2] "v"(idx[2]), [i3] "v"(idx[3])
                         : PATCH_CL_CLOBBER);
        } else if (KIND == 0) {
            asm volatile(PATCH_CL_D(0, 0, 00) PATCH_CL_D(1, 1, 00) PATCH_CL_D(2, 2, 00) PATCH_CL_D(3, 3, 00)
                         PATCH_CL_D(4, 0, 11) PATCH_CL_D(5, 1, 11) PATCH_CL_D(6, 2, 11) PATCH_CL_D(7, 3, 11)
                         PATCH_CL_D(8, 0, 20) PATCH_CL_D(9, 1, 20) PATCH_CL_D(10, 2, 20) PATCH_CL_D(11, 3, 20)
                         PATCH_CL_D(12, 0, 31) PATCH_CL_D(13, 1, 31) PATCH_CL_D(14, 2, 31) PATCH_CL_D(15, 3, 31)
                         :
                         : [a0] "v"(a[0].v), [a1] "v"(a[1].v), [a2] "v"(a[2].v), [a3] "v"(a[3].v), [b00] "v"(b[0].h[0]),
                           [b01] "v"(b[0].h[1]), [b10] "v"(b[1].h[0]), [b11] "v"(b[1].h[1]), [b20] "v"(b[2].h[0]),
                           [b21] "v"(b[2].h[1]), [b30] "v"(b[3].h[0]), [b31] "v"(b[3].h[1])
                         : PATCH_CL_CLOBBER);
        } else {
            asm volatile(PATCH_CL_S(0, 0, 0) PATCH_CL_S(1, 1, 0) PATCH_CL_S(2, 2, 0) PATCH_CL_S(3, 3, 0)
                         PATCH_CL_S(4, 0, 1) PATCH_CL_S(5, 1, 1) PATCH_CL_S(6, 2, 1) PATCH_CL_S(7, 3, 1)
                         PATCH_CL_S(8, 0, 2) PATCH_CL_S(9, 1, 2) PATCH_CL_S(10, 2, 2) PATCH_CL_S(11, 3, 2)
                         PATCH_CL_S(12, 0, 3) PATCH_CL_S(13, 1, 3) PATCH_CL_S(14, 2, 3) PATCH_CL_S(15, 3, 3)
                         :
                         : [a0] "v"(a[0].v), [a1] "v"(a[1].v), [a2] "v"(a[2].v), [a3] "v"(a[3].v), [b0] "v"(b[0].v), [b1] "v"(b[1].v),
                           [b2] "v"(b[2].v), [b3] "v"(b[3].v), [i0] "v"(idx[0]), [i1] "v"(idx[1]), [i2] "v"(idx[2]), [i3] "v"(idx[3])
                         : PATCH_CL_CLOBBER);
        }
    }
    // one word per thread that depends on every accumulator
    float s = 0.f;
#define PATCH_CL_READ(R)                                                                           \
    {                                                                                              \
        float t_;                                                                                  \
        asm volatile("s_nop 7\n\ts_nop 7\n\tv_accvgpr_read_b32 %0, a[" #R "]" : "=v"(t_) : : PATCH_CL_CLOBBER); \
        s += t_;                                                                                   \
    }
    PATCH_CL_READ(0) PATCH_CL_READ(5) PATCH_CL_READ(10) PATCH_CL_READ(15) PATCH_CL_READ(16) PATCH_CL_READ(21) PATCH_CL_READ(26)
    PATCH_CL_READ(31) PATCH_CL_READ(32) PATCH_CL_READ(37) PATCH_CL_READ(42) PATCH_CL_READ(47) PATCH_CL_READ(48) PATCH_CL_READ(53)
    PATCH_CL_READ(58) PATCH_CL_READ(63)
    out[(size_t)blockIdx.x * 256 + tid] = s;
#undef PATCH_CL_READ
#undef PATCH_CL_D
#undef PATCH_CL_S
#undef PATCH_CL_D32
#undef PATCH_CL_S32
#undef PATCH_CL_ZERO4
#undef PATCH_CL_CLOBBER
}

// Every thread reads 16 bytes at a time, grid-stride, eight loads in flight, and folds what it read into one word
// (so that the reads cannot be dropped); one word per thread goes to `out`.
__global__ __launch_bounds__(1024) void stream_read_kernel(const cl_u32x4* __restrict__ src, size_t n16, uint32_t* __restrict__ out) {
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    uint32_t fold = 0;
    for (; i + 7 * stride < n16; i += 8 * stride) {
        cl_u32x4 v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = __builtin_nontemporal_load(src + i + u * stride);
#pragma unroll
        for (int u = 0; u < 8; ++u) fold ^= v[u][0] ^ v[u][1] ^ v[u][2] ^ v[u][3];
    }
    for (; i < n16; i += stride) {
        const cl_u32x4 v = __builtin_nontemporal_load(src + i);
        fold ^= v[0] ^ v[1] ^ v[2] ^ v[3];
    }
    out[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = fold;
}


// A workgroup of 8 wavefronts fetches 48 KB per round - what a K-step of the LDS-staged prefill kernel with blocks of
// 128 rows fetches - in six 1 KB pieces per wavefront, waits for them and meets at a barrier, `rounds` times over
// a window of `chunks` 48 KB chunks of src (chunk = (workgroup + round * workgroups) % chunks).
//   KIND 0: global -> LDS directly (global_load_lds, 16 bytes per lane)
//   KIND 1: global -> registers (128-bit loads) -> LDS (ds_write_b128)
//   KIND 2: global -> registers only, folded into one word
//   KIND 4: as 0 with rounds of half a chunk (three pieces per wavefront) into alternating halves of the buffer
//   KIND 3: as 4, but a round waits only for the round before it (two rounds in flight)
// One word per thread that depends on what was fetched goes to `out`.
template <int KIND>
__global__ __launch_bounds__(512) void lds_fill_kernel(const uint8_t* __restrict__ src, unsigned chunks, int rounds, uint32_t* __restrict__ out) {
    constexpr int kChunk = 48 * 1024;
    __shared__ __attribute__((aligned(16))) uint8_t buf[kChunk];
    const int tid = threadIdx.x, lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    uint32_t fold = 0;
    for (int r = 0; r < rounds; ++r) {
        const unsigned c = (unsigned)(((size_t)blockIdx.x + (size_t)r * gridDim.x) % chunks);
        const uint8_t* g = src + (size_t)c * kChunk + (size_t)(w * 6) * 1024 + lane * 16;
        if constexpr (KIND == 0) {
#pragma unroll
            for (int i = 0; i < 6; ++i)
                __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(g + i * 1024),
                                                 (__attribute__((address_space(3))) void*)(buf + (w * 6 + i) * 1024), 16, 0, 0);
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        } else if constexpr (KIND == 3 || KIND == 4) {
            // half a chunk per round into alternating halves of the buffer; KIND 3 waits for the round before this one
            // only (two rounds in flight), KIND 4 for this one
#pragma unroll
            for (int i = 0; i < 3; ++i)
                __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(g + i * 1024),
                                                 (__attribute__((address_space(3))) void*)(buf + ((r & 1) * 24 + w * 3 + i) * 1024), 16, 0, 0);
            if constexpr (KIND == 3) asm volatile("s_waitcnt vmcnt(3)" ::: "memory");
            else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        } else {
            cl_u32x4 v[6];
#pragma unroll
            for (int i = 0; i < 6; ++i) v[i] = *reinterpret_cast<const cl_u32x4*>(g + i * 1024);
#pragma unroll
            for (int i = 0; i < 6; ++i) {
                if constexpr (KIND == 1) *reinterpret_cast<cl_u32x4*>(buf + (w * 6 + i) * 1024 + lane * 16) = v[i];
                else fold ^= v[i][0] ^ v[i][1] ^ v[i][2] ^ v[i][3];
            }
        }
        __syncthreads();
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if constexpr (KIND != 2) fold = *reinterpret_cast<const uint32_t*>(buf + ((tid * 4 + 64) % kChunk));
    out[(size_t)blockIdx.x * 512 + tid] = fold;
}

// Stores only: workgroup t of 4 wavefronts writes output tile t (256 rows x 256 features of a row-major M x N matrix,
// tiles along N first) the way a prefill workgroup's output stage does, 64 store instructions per wavefront.
//   PAT 0: 16 rows x 16 bytes-per-lane quarters of 64 bytes - the accumulator layout of the 16 x 16 matrix instruction
//          stored as it lies (lane = row % 16 + 16 * (four features))
//   PAT 1: 4 rows x the wavefront's 64 features contiguous - the same data after a turn through LDS
// BF16: two bytes per element (8 bytes per lane) instead of four (16 bytes per lane).
typedef unsigned int cl_u32x2 __attribute__((ext_vector_type(2)));
template <int PAT, int BF16>
__global__ __launch_bounds__(256) void store_tiles_kernel(void* __restrict__ Y, long N, int tiles_n) {
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const long m0 = 256L * (blockIdx.x / tiles_n), n0 = 256L * (blockIdx.x % tiles_n);
    cl_f32x4 v = {(float)lane, (float)w, (float)blockIdx.x, 1.0f};
    for (int j = 0; j < 64; ++j) {
        long m, n;
        if (PAT == 0) { m = m0 + 16 * (j >> 2) + (lane & 15); n = n0 + 64 * w + 16 * (j & 3) + 4 * (lane >> 4); }
        else { m = m0 + 4 * j + (lane >> 4); n = n0 + 64 * w + 4 * (lane & 15); }
        v[3] += 1.0f;
        if (BF16) {
            const cl_u32x2 p = {(__float_as_uint(v[0]) >> 16) | (__float_as_uint(v[1]) & 0xffff0000u),
                                (__float_as_uint(v[2]) >> 16) | (__float_as_uint(v[3]) & 0xffff0000u)};
            *reinterpret_cast<cl_u32x2*>(static_cast<uint16_t*>(Y) + m * N + n) = p;
        } else {
            *reinterpret_cast<cl_f32x4*>(static_cast<float*>(Y) + m * N + n) = v;
        }
    }
}

// LDS reads only: a workgroup of 4 wavefronts (one per SIMD, as in the 256 x 256 prefill kernel), each reading its own
// 8 KB of a 32 KB buffer with ds_read_b128 - 64 lanes x 16 contiguous bytes, conflict-free - eight reads in flight,
// `iters` times.  Bytes per workgroup = iters * 8 * 1 KB * 4.
__global__ __launch_bounds__(256) void lds_read_kernel(int iters, float* __restrict__ out) {
    __shared__ __attribute__((aligned(16))) float buf[8192];
    const int tid = threadIdx.x;
    for (int i = tid; i < 8192; i += 256) buf[i] = (float)i;
    __syncthreads();
    const uint32_t a = (uint32_t)(size_t)((__attribute__((address_space(3))) void*)buf) + (tid & 63) * 16 + (tid >> 6) * 8192;
    float acc = 0.f;
    for (int it = 0; it < iters; ++it) {
        cl_f32x4 r0, r1, r2, r3, r4, r5, r6, r7;
        asm volatile(
            "ds_read_b128 %0, %8\n\tds_read_b128 %1, %8 offset:1024\n\tds_read_b128 %2, %8 offset:2048\n\tds_read_b128 %3, %8 offset:3072\n\t"
            "ds_read_b128 %4, %8 offset:4096\n\tds_read_b128 %5, %8 offset:5120\n\tds_read_b128 %6, %8 offset:6144\n\tds_read_b128 %7, %8 offset:7168\n\t"
            "s_waitcnt lgkmcnt(0)"
            : "=&v"(r0), "=&v"(r1), "=&v"(r2), "=&v"(r3), "=&v"(r4), "=&v"(r5), "=&v"(r6), "=&v"(r7)
            : "v"(a)
            : "memory");
        acc += r0[0] + r1[0] + r2[0] + r3[0] + r4[0] + r5[0] + r6[0] + r7[0];
    }
    out[(size_t)blockIdx.x * 256 + tid] = acc;
}

}  // namespace patch

extern "C" {

patch_status patch_probe_matrix_rate(int kind, const void* operands, size_t operand_bytes, int workgroups, int iters, void* out,
                                     size_t out_bytes, void* stream) {
    if (!operands || !out || workgroups < 1 || workgroups > 65536 || iters < 1 || kind < 0 || kind > 3) return PATCH_ERR_ARG;
    if ((reinterpret_cast<uintptr_t>(operands) & 15u) || (reinterpret_cast<uintptr_t>(out) & 3u)) return PATCH_ERR_ARG;
    if (operand_bytes < PATCH_PROBE_OPERAND_BYTES || out_bytes < (size_t)workgroups * 256 * sizeof(float)) return PATCH_ERR_SIZE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const patch::cl_u32x4* ops = static_cast<const patch::cl_u32x4*>(operands);
    float* o = static_cast<float*>(out);
    switch (kind) {
        case 0: hipLaunchKernelGGL(patch::matrix_rate_kernel<0>, dim3(workgroups), dim3(256), 0, s, ops, iters, o); break;
        case 1: hipLaunchKernelGGL(patch::matrix_rate_kernel<1>, dim3(workgroups), dim3(256), 0, s, ops, iters, o); break;
        case 2: hipLaunchKernelGGL(patch::matrix_rate_kernel<2>, dim3(workgroups), dim3(256), 0, s, ops, iters, o); break;
        default: hipLaunchKernelGGL(patch::matrix_rate_kernel<3>, dim3(workgroups), dim3(256), 0, s, ops, iters, o); break;
    }
    return hipGetLastError() == hipSuccess ? PATCH_OK : PATCH_ERR_HIP;
}

patch_status patch_probe_stream_read(const void* src, size_t bytes, int workgroups, int threads, void* out, size_t out_bytes, void* stream) {
    if (!src || !out || bytes < 16 || workgroups < 1 || workgroups > (1 << 20)) return PATCH_ERR_ARG;
    if (threads < 64 || threads > 1024 || threads % 64) return PATCH_ERR_ARG;
    if ((reinterpret_cast<uintptr_t>(src) & 15u) || (reinterpret_cast<uintptr_t>(out) & 3u)) return PATCH_ERR_ARG;
    if (out_bytes < (size_t)workgroups * threads * sizeof(uint32_t)) return PATCH_ERR_SIZE;
    hipLaunchKernelGGL(patch::stream_read_kernel, dim3(workgroups), dim3(threads), 0, static_cast<hipStream_t>(stream),
                       static_cast<const patch::cl_u32x4*>(src), bytes / 16, static_cast<uint32_t*>(out));
    return hipGetLastError() == hipSuccess ? PATCH_OK : PATCH_ERR_HIP;
}

patch_status patch_probe_lds_fill(int kind, const void* src, size_t bytes, int workgroups, int rounds, void* out, size_t out_bytes,
                                  void* stream) {
    if (!src || !out || kind < 0 || kind > 4 || workgroups < 1 || workgroups > 65536 || rounds < 1) return PATCH_ERR_ARG;
    if ((reinterpret_cast<uintptr_t>(src) & 15u) || (reinterpret_cast<uintptr_t>(out) & 3u)) return PATCH_ERR_ARG;
    const size_t chunks = bytes / (48 * 1024);
    if (chunks < 1 || chunks > 0xFFFFFFFFu) return PATCH_ERR_SIZE;
    if (out_bytes < (size_t)workgroups * 512 * sizeof(uint32_t)) return PATCH_ERR_SIZE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const uint8_t* p = static_cast<const uint8_t*>(src);
    uint32_t* o = static_cast<uint32_t*>(out);
    switch (kind) {
        case 0: hipLaunchKernelGGL(patch::lds_fill_kernel<0>, dim3(workgroups), dim3(512), 0, s, p, (unsigned)chunks, rounds, o); break;
        case 1: hipLaunchKernelGGL(patch::lds_fill_kernel<1>, dim3(workgroups), dim3(512), 0, s, p, (unsigned)chunks, rounds, o); break;
        case 2: hipLaunchKernelGGL(patch::lds_fill_kernel<2>, dim3(workgroups), dim3(512), 0, s, p, (unsigned)chunks, rounds, o); break;
        case 3: hipLaunchKernelGGL(patch::lds_fill_kernel<3>, dim3(workgroups), dim3(512), 0, s, p, (unsigned)chunks, rounds, o); break;
        default: hipLaunchKernelGGL(patch::lds_fill_kernel<4>, dim3(workgroups), dim3(512), 0, s, p, (unsigned)chunks, rounds, o); break;
    }
    return hipGetLastError() == hipSuccess ? PATCH_OK : PATCH_ERR_HIP;
}

patch_status patch_probe_store_tiles(int pattern, int bf16, void* Y, size_t y_bytes, int64_t M, int64_t N, void* stream) {
    if (!Y || pattern < 0 || pattern > 1 || M < 256 || N < 256 || M % 256 || N % 256) return PATCH_ERR_ARG;
    if (reinterpret_cast<uintptr_t>(Y) & 15u) return PATCH_ERR_ARG;
    const int64_t tiles = (M / 256) * (N / 256);
    if (tiles > (1 << 20)) return PATCH_ERR_ARG;
    if (y_bytes < (size_t)M * (size_t)N * (bf16 ? 2 : 4)) return PATCH_ERR_SIZE;   // every tile lies inside M x N
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int tn = (int)(N / 256);
    if (pattern == 0 && !bf16) hipLaunchKernelGGL((patch::store_tiles_kernel<0, 0>), dim3((unsigned)tiles), dim3(256), 0, s, Y, (long)N, tn);
    else if (pattern == 0) hipLaunchKernelGGL((patch::store_tiles_kernel<0, 1>), dim3((unsigned)tiles), dim3(256), 0, s, Y, (long)N, tn);
    else if (!bf16) hipLaunchKernelGGL((patch::store_tiles_kernel<1, 0>), dim3((unsigned)tiles), dim3(256), 0, s, Y, (long)N, tn);
    else hipLaunchKernelGGL((patch::store_tiles_kernel<1, 1>), dim3((unsigned)tiles), dim3(256), 0, s, Y, (long)N, tn);
    return hipGetLastError() == hipSuccess ? PATCH_OK : PATCH_ERR_HIP;
}

patch_status patch_probe_lds_read(int workgroups, int iters, void* out, size_t out_bytes, void* stream) {
    if (!out || workgroups < 1 || workgroups > 65536 || iters < 1) return PATCH_ERR_ARG;
    if (reinterpret_cast<uintptr_t>(out) & 3u) return PATCH_ERR_ARG;
    if (out_bytes < (size_t)workgroups * 256 * sizeof(float)) return PATCH_ERR_SIZE;
    hipLaunchKernelGGL(patch::lds_read_kernel, dim3(workgroups), dim3(256), 0, static_cast<hipStream_t>(stream), iters, static_cast<float*>(out));
    return hipGetLastError() == hipSuccess ? PATCH_OK : PATCH_ERR_HIP;
}

}  // extern "C"
