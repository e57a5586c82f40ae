// Internal launch interface between the C ABI (api.hip) and the kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

// records the hipError_t that patch_last_hip_error reports (thread-local, in api.hip)
void patch_note_hip_error(int hip_error);

namespace patch {

void launch_apply_mask(const uint16_t* W, const uint8_t* mask24, const uint8_t* d_tile_map, int64_t N, int64_t K, int tile,
                       uint16_t* W_hat, hipStream_t stream);
// mask24 (N x K keep bytes, 4-byte aligned) from the 6 x G pattern logits, G = N K / 4 groups
void launch_hard_mask24(const float* P24, int64_t G, uint8_t* mask24, hipStream_t stream);
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
    float* ws = nullptr;    // caller's workspace for split-K partial products (prefill), may be null
    size_t ws_bytes = 0;
    int n_cus;
    int ybf16 = 0;          // nonzero: Y (and every Y of a set) is bf16, the accumulator rounded to nearest even
    int sparse_pct = 0;     // share of 2:4 tiles in the weight (all weights of a set), per cent: a hint for schedules
};

// Up to kMaxMany weights that share one X (same K, same tile), multiplied in one launch.  The launch numbers its
// units of features (decode: 16-feature strips; prefill: 256-feature blocks, each weight rounded up) across all
// weights; first[i] is the first unit of weight i.
constexpr int kMaxMany = 8;
struct WeightSet {
    const uint8_t* payload[kMaxMany];
    const uint32_t* table[kMaxMany];
    float* Y[kMaxMany];          // M x N[i] fp32
    int64_t N[kMaxMany];
    int first[kMaxMany];
    int count, units;            // weights, units in total
};
typedef WeightSet DecodeSet;
// A set of one, for the kernels' single-weight instantiations: 32 bytes of kernel arguments instead of 300.  Every
// wavefront reads its arguments before it can request anything else, the set's arrays in several dependent rounds
// (which weight? then that weight's pointers), and a decode launch is short enough for that to show.
struct WeightOne {
    const uint8_t* payload;
    const uint32_t* table;
    float* Y;
    int64_t N;
};

// Up to kDecodeRows rows of X starting at row m0 (decode shape; 16-row blocks, the weights streamed once per launch).
constexpr int kDecodeRows = 64;
//  split_k = K slices (wavefronts) per workgroup,
// 0 picks a default.  Returns the number used.
int launch_decode(const GemmArgs& a, int64_t m0, int rows, int split_k, int variant, hipStream_t stream);
// The same for a set of weights; a supplies X, K, tile, Tk, n_cus (its payload / table / Y / N are ignored).
int launch_decode_set(const GemmArgs& a, const DecodeSet& set, int64_t m0, int rows, int split_k, int variant, hipStream_t stream);

// Up to kDecodeRows rows of X starting at row m0 (batched decode): 64 features per wavefront, so X is read once per
// four strips.  set.units / first[] count 64-feature groups.  split > 1 (single weight only, a.ws must hold
// split x rows x N floats) cuts K into chunks over more workgroups; mid_split picks the count (1 without a.ws).
int mid_split(const GemmArgs& a, int rows, int requested);
void launch_mid_set(const GemmArgs& a, const WeightSet& set, int64_t m0, int rows, int split, hipStream_t stream);
// Y[i] = sum over the slices of ws[slice * n4 + i] (float4 units), slice 0 first
void wr_reduce(const float* ws, size_t n4, int slices, float* Y, int ybf16, hipStream_t stream);

// Any M (prefill shape).
void launch_prefill(const GemmArgs& a, int variant, int split_k, hipStream_t stream);
bool prefill_wreg_supports(const GemmArgs& a);                  // tile 128, K <= 32768, M * K * 2 < 4 GB
int prefill_wreg_split(const GemmArgs& a, int requested);       // K slices per output tile the launch will use
int prefill_lds_split(const GemmArgs& a, int requested, int bm = 256);   // the same for the LDS-staged kernel with blocks of bm rows
// whether the default choice (variant 0, no split requested) is the LDS-staged kernel with blocks of 128 rows, and its split
bool prefill_prefers_128_rows(const GemmArgs& a, int* split);
// K slices for the last *tail tiles of an unsplit launch with a part-filled last round (needs a.ws); 1 = none
int prefill_wreg_tail(const GemmArgs& a, int* tail);
int prefill_wreg_tail_of(int tiles, const GemmArgs& a, int* tail);   // the same for a given tile count (sets of weights)
void launch_prefill_wreg(const GemmArgs& a, int split_k, hipStream_t stream);
// The same for a set of weights; a supplies X, M, K, tile, Tk, n_cus and, optionally, ws / ws_bytes (then a
// part-filled last round is split as in launch_prefill_wreg).  All of the set must pass prefill_wreg_supports with
// these M, K.
void launch_prefill_wreg_set(const GemmArgs& a, const WeightSet& set, hipStream_t stream);

}  // namespace patch
