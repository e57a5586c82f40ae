// Internal launch interface between the C ABI (api.hip) and the kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace patch {

void launch_apply_mask(const uint16_t* W, const uint8_t* mask24, const uint8_t* d_tile_map, int64_t N, int64_t K, int tile,
                       uint16_t* W_hat, hipStream_t stream);
void launch_pack(const uint16_t* W, int64_t K, const uint32_t* d_table, int n_tiles, int Tk, int tile, uint8_t* payload, int* d_err,
                 hipStream_t stream);
void launch_unpack(const uint8_t* payload, const uint32_t* d_table, int n_tiles, int Tk, int tile, int64_t K, uint16_t* W_out,
                   hipStream_t stream);

// Operands shared by the GEMM launchers.
struct GemmArgs {
    const uint16_t* X;   // M x K bf16
    int64_t M, N, K;
    int tile, Tn, Tk;
    const uint8_t* payload;
    const uint32_t* table;  // Tn x Tk entries
    float* Y;               // M x N fp32
    int n_cus;
};

// M <= 16 rows of X starting at row m0 (decode shape).  split_k = K slices (wavefronts) per workgroup,
// 0 picks a default.  Returns the number used.
int launch_decode(const GemmArgs& a, int64_t m0, int rows, int split_k, int variant, hipStream_t stream);

// Any M (prefill shape).
void launch_prefill(const GemmArgs& a, int variant, hipStream_t stream);
bool prefill_wreg_supports(const GemmArgs& a);                  // tile 128, K <= 32768, M * K * 2 < 4 GB
void launch_prefill_wreg(const GemmArgs& a, hipStream_t stream);

}  // namespace patch
