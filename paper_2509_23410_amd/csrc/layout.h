// Device layout of a compressed hybrid dense / 2:4 weight (product code; the CPU oracle has its own,
// unrelated, canonical format).
//
// The matrix W_hat (N x K, bf16) is cut into tile x tile blocks (tile = 64 or 128), stored one after the
// other in row-major tile order, each starting on a 256-byte granule.  Inside a tile the unit is a
// "fragment": 16 rows (a strip) x 64 columns (a K-step), stored in the exact register order of the
// gfx950 matrix instructions, so a wavefront loads lane * 16 bytes and feeds the instruction directly.
//
//   dense fragment, 2048 B = two operands of v_mfma_f32_16x16x32_bf16 (h = 0, 1):
//       byte ((h * 64 + lane) * 16 + 2 e) holds W[row0 + lane % 16][k0 + 32 h + 8 (lane / 16) + e], e < 8
//   2:4 fragment, 1024 B of values = one operand of v_smfmac_f32_16x16x64_bf16:
//       lane holds the 8 kept values of W[row0 + lane % 16][k0 + 16 (lane / 16) .. + 15] (4 groups of 4,
//       two kept values per group, ascending position), plus 16 bits of positions: bits [4g+1:4g] and
//       [4g+3:4g+2] are the in-group positions of the two kept values of group g.
//
//   dense tile  : fragments in (strip, K-step) order                                 -> 2 * tile^2 bytes
//   2:4 tile    : value fragments in (strip, K-step) order (tile^2 bytes), followed by the positions as
//                 uint16 [strip][lane][K-step] (tile^2 / 8 bytes).  For tile = 128 a lane's two K-steps
//                 form one dword whose halves are selected by the instruction's ABID field.
//
// The measured register layouts this relies on (one-hot probes on MI355X):
//   v_mfma_f32_16x16x32_bf16   A lane l: row l%16, k = 8 (l/16) + e;  B lane l: column l%16, same k;
//                              D lane l, reg r: row 4 (l/16) + r, column l%16.
//   v_mfma_f32_32x32x16_bf16   A lane l: row l%32, k = 8 (l/32) + e;  B alike;
//                              D lane l, reg r: row 8 (r/4) + 4 (l/32) + r%4, column l%32.
//   v_smfmac_f32_16x16x64_bf16 A lane l: row l%16, kept values of k in [16 (l/16), +16);
//                              B lane l: column l%16, e < 8: k = 8 (l/16) + e, e >= 8: k = 32 + 8 (l/16) + e - 8
//                              (i.e. the two dense B operands of the same 64 columns, concatenated);
//                              value c uses position bits [2c+1:2c] of the 16-bit half chosen by ABID.
//   v_smfmac_f32_32x32x32_bf16 A lane l: row l%32, kept values of k in [16 (l/32), +16);
//                              B lane l: column l%32, e < 8: k = 8 (l/32) + e, e >= 8: k = 16 + 8 (l/32) + e - 8.
#pragma once
#include <stdint.h>

namespace patch {

constexpr int kGranule = 256;        // tile start alignment / unit of the offset table
constexpr int kStripRows = 16;       // rows of a fragment
constexpr int kStepCols = 64;        // columns of a fragment
constexpr int kZeroPad = 1024;       // zeroed slack kept behind the payload
constexpr int kDenseFragBytes = 2048;
constexpr int kSparseFragBytes = 1024;

__host__ __device__ constexpr int dense_tile_bytes(int t) { return 2 * t * t; }
__host__ __device__ constexpr int sparse_vals_bytes(int t) { return t * t; }
__host__ __device__ constexpr int sparse_tile_bytes(int t) { return t * t + t * t / 8; }

// table entry: (offset in granules) << 1 | is_sparse
__host__ __device__ inline uint32_t make_entry(uint64_t byte_off, bool sparse) {
    return (uint32_t)((byte_off / kGranule) << 1) | (sparse ? 1u : 0u);
}
__host__ __device__ inline uint64_t entry_offset(uint32_t e) { return (uint64_t)(e >> 1) * kGranule; }
__host__ __device__ inline bool entry_sparse(uint32_t e) { return (e & 1u) != 0; }

}  // namespace patch
