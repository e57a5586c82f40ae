// A packed weight saved to host memory: header, tile map, then the device buffers as they lie in HBM (each part at a
// multiple of 64 bytes).  The payload's byte order is this library's stored register order (layout.h, quant4.hip);
// the header's layout number changes whenever that order does, and a buffer with another number is refused.
#pragma once
#include <stddef.h>
#include <stdint.h>
#include <string.h>

namespace patch {

struct SavedHeader {
    char magic[8];            // kSavedMagic16 (bf16 storage) or kSavedMagic4 (4-bit storage)
    uint32_t layout;          // kSavedLayout
    uint32_t tile;
    int64_t N, K;
    uint64_t map_bytes;       // (N / tile) (K / tile)
    uint64_t payload_bytes;
    uint64_t aux_bytes;       // 4-bit storage: the scales; else 0
    uint64_t checksum;        // FNV-1a (64 bit) over the tile map, the payload and the scales
};
static_assert(sizeof(SavedHeader) == 64, "saved header layout");

constexpr char kSavedMagic16[8] = {'P', 'A', 'T', 'C', 'H', 'P', 'K', 0};
constexpr char kSavedMagic4[8] = {'P', 'A', 'T', 'C', 'H', 'Q', '4', 0};
constexpr uint32_t kSavedLayout = 1;
constexpr size_t kSavedAlign = 64;
constexpr uint64_t kFnvBasis = 14695981039346656037ull;

inline size_t saved_round(size_t n) { return (n + kSavedAlign - 1) / kSavedAlign * kSavedAlign; }

inline uint64_t fnv1a(const uint8_t* p, size_t n, uint64_t h) {
    for (size_t i = 0; i < n; ++i) {
        h ^= p[i];
        h *= 1099511628211ull;
    }
    return h;
}

}  // namespace patch
