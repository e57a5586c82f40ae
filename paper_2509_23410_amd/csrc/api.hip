// C ABI of the library (see include/patch.h): argument checks, the patch_packed object, host-side table
// construction and kernel dispatch.  No device arithmetic here.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <string.h>

#include <algorithm>
#include <map>
#include <mutex>
#include <new>
#include <tuple>
#include <vector>

#include "../../include/patch.h"
#include "kernels.h"
#include "layout.h"
#include "saved.h"

using namespace patch;

struct patch_packed {
    int64_t N = 0, K = 0;
    int tile = 0;
    int Tn = 0, Tk = 0;
    int64_t n_sparse = 0;
    size_t payload_bytes = 0;   // sum of tile payloads (no alignment slack: tiles are granule multiples)
    uint8_t* d_payload = nullptr;
    uint32_t* d_table = nullptr;
    std::vector<uint8_t> tile_map;   // host copy, 1 = dense
    std::vector<uint32_t> table;     // host copy of the offset / type table
    std::vector<int32_t> pairs;      // tile rows two by two (see pair_tile_rows); behind the table on the device
    int device = 0;
    int n_cus = 256;
};

static thread_local int g_last_hip_error = 0;
void patch_note_hip_error(int hip_error) { g_last_hip_error = hip_error; }

#define HIP_TRY(expr)                                   \
    do {                                                \
        hipError_t e_ = (expr);                         \
        if (e_ != hipSuccess) {                         \
            g_last_hip_error = (int)e_;                 \
            return PATCH_ERR_HIP;                       \
        }                                               \
    } while (0)

static patch_status check_shape(int64_t N, int64_t K, int tile) {
    if (N <= 0 || K <= 0) return PATCH_ERR_ARG;
    if (tile != 64 && tile != 128) return PATCH_ERR_SHAPE;
    if (N % tile != 0 || K % tile != 0) return PATCH_ERR_SHAPE;
    if (N / tile > (1 << 20) || K / tile > (1 << 20)) return PATCH_ERR_SHAPE;
    return PATCH_OK;
}

// Which two tile rows share a prefill workgroup (tile-map-driven schedule; the paper leaves the schedule to the
// implementation).  The workgroup's wavefronts meet at a barrier every 64-column step, so a step in which one tile row
// is dense and the other 2:4 lasts as long as a dense one: a pair costs about Tk - 0.3 x (steps in which BOTH rows
// are 2:4).  Rows are therefore paired so that these common 2:4 steps are many: within windows of 256 rows, the free
// pair with the most of them first (ties: lowest row indices; counting agreeing steps of either type instead
// measured 1 - 3 % slower).  Returns 2 * ceil(Tn / 2) entries, pair p = rows out[2 p], out[2 p + 1]; -1 = no
// second row.
static std::vector<int32_t> pair_tile_rows(const std::vector<uint8_t>& tile_map, int Tn, int Tk) {
    std::vector<int32_t> out;
    out.reserve((size_t)Tn + 1);
    std::vector<int> carry;  // rows left single by earlier windows
    constexpr int kWindow = 256;
    struct Cand { int agree, a, b; };  // agree = steps in which both rows are 2:4
    for (int w0 = 0; w0 < Tn; w0 += kWindow) {
        std::vector<int> rows = carry;
        carry.clear();
        for (int r = w0; r < Tn && r < w0 + kWindow; ++r) rows.push_back(r);
        const int n = (int)rows.size();
        std::vector<Cand> cand;
        cand.reserve((size_t)n * (size_t)(n - 1) / 2);
        for (int i = 0; i < n; ++i)
            for (int j = i + 1; j < n; ++j) {
                const uint8_t* ra = &tile_map[(size_t)rows[i] * Tk];
                const uint8_t* rb = &tile_map[(size_t)rows[j] * Tk];
                int agree = 0;
                for (int k = 0; k < Tk; ++k) agree += ra[k] == 0 && rb[k] == 0;
                cand.push_back(Cand{agree, i, j});
            }
        std::stable_sort(cand.begin(), cand.end(), [](const Cand& x, const Cand& y) { return x.agree > y.agree; });
        std::vector<char> used((size_t)n, 0);
        for (const Cand& c : cand) {
            if (used[c.a] || used[c.b]) continue;
            used[c.a] = used[c.b] = 1;
            out.push_back(rows[c.a]);
            out.push_back(rows[c.b]);
        }
        for (int i = 0; i < n; ++i)
            if (!used[i]) carry.push_back(rows[i]);
    }
    for (size_t i = 0; i + 1 < carry.size(); i += 2) { out.push_back(carry[i]); out.push_back(carry[i + 1]); }
    if (carry.size() % 2) { out.push_back(carry.back()); out.push_back(-1); }
    // Order of the pairs = order of the feature blocks in the launch, of which every XCD runs a contiguous piece
    // (all, a half or a quarter of it, depending on M), its workgroups starting in that order as compute units
    // become free.  A pair costs about Tk - 0.3 x (steps in which both rows are 2:4).  The pairs are dealt by falling
    // cost into four piles, laid one after the other: every quarter of the order carries about the average cost, and
    // inside it the heaviest workgroups start first (alternating heaviest / lightest measured 0 - 4 % slower).
    const size_t np = out.size() / 2;
    std::vector<std::pair<int, size_t>> cost(np);
    for (size_t p = 0; p < np; ++p) {
        const int a = out[2 * p], b2 = out[2 * p + 1];
        int both = 0;
        for (int k = 0; k < Tk; ++k) both += tile_map[(size_t)a * Tk + k] == 0 && (b2 < 0 || tile_map[(size_t)b2 * Tk + k] == 0);
        cost[p] = {both, p};  // more common 2:4 steps = lighter
    }
    std::stable_sort(cost.begin(), cost.end(), [](const auto& x, const auto& y) { return x.first < y.first; });
    std::vector<int32_t> ordered;
    ordered.reserve(out.size());
    constexpr size_t kPiles = 4;
    for (size_t pile = 0; pile < kPiles; ++pile)
        for (size_t r = pile; r < np; r += kPiles) {
            const size_t h = cost[r].second;
            ordered.push_back(out[2 * h]); ordered.push_back(out[2 * h + 1]);
        }
    return ordered;
}

static bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Library-side scratch for patch_gemm_static (callers that cannot allocate): split-K partial products live here
// instead of a caller workspace.  One copy per GPU, held until the process ends.  In host code the array's name is
// only a handle for hipGetSymbolAddress; the device address is looked up once per device and kept.
constexpr size_t kStaticScratchBytes = PATCH_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
constexpr int kMaxDevices = 64;
static std::mutex g_scratch_mutex;
static void* g_scratch_ptr[kMaxDevices] = {};

// Device address of `scratch` on the current device (looked up on the first call per device).
static patch_status static_scratch(void** out) {
    int dev = 0;
    HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return PATCH_ERR_ARG;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p) { g_last_hip_error = (int)hipErrorInvalidSymbol; return PATCH_ERR_HIP; }
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return PATCH_OK;
}

extern "C" {

const char* patch_version(void) { return "patch-mi355x 0.1 (gfx950)"; }

int patch_last_hip_error(void) { return g_last_hip_error; }

const char* patch_strerror(patch_status s) {
    switch (s) {
        case PATCH_OK: return "ok";
        case PATCH_ERR_ARG: return "invalid argument (null or misaligned pointer, non-positive size, unknown option)";
        case PATCH_ERR_SHAPE: return "unsupported shape (tile must be 64 or 128 and divide N and K)";
        case PATCH_ERR_NOT_24: return "a group of four in a 2:4 tile holds more than two nonzeros";
        case PATCH_ERR_ALLOC: return "allocation failed";
        case PATCH_ERR_HIP: return "HIP runtime error";
        case PATCH_ERR_SIZE: return "caller buffer too small";
        case PATCH_ERR_NOT_FOUND: return "no tuned schedule stored for this key";
    }
    return "unknown status";
}

patch_status patch_apply_mask(const void* W, const void* mask24, const uint8_t* tile_map, int64_t N, int64_t K, int tile,
                              void* W_hat, void* stream) {
    if (!W || !mask24 || !tile_map || !W_hat) return PATCH_ERR_ARG;
    patch_status st = check_shape(N, K, tile);
    if (st != PATCH_OK) return st;
    if (!aligned16(W) || !aligned16(W_hat) || (reinterpret_cast<uintptr_t>(mask24) & 7u)) return PATCH_ERR_ARG;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const size_t T = (size_t)(N / tile) * (size_t)(K / tile);
    uint8_t* d_map = nullptr;
    if (hipMalloc(&d_map, T) != hipSuccess) { (void)hipGetLastError(); return PATCH_ERR_ALLOC; }
    hipError_t e = hipMemcpyAsync(d_map, tile_map, T, hipMemcpyHostToDevice, s);
    if (e == hipSuccess) {
        launch_apply_mask(static_cast<const uint16_t*>(W), static_cast<const uint8_t*>(mask24), d_map, N, K, tile,
                          static_cast<uint16_t*>(W_hat), s);
        e = hipGetLastError();
    }
    if (e == hipSuccess) e = hipStreamSynchronize(s);
    (void)hipFree(d_map);
    if (e != hipSuccess) { g_last_hip_error = (int)e; return PATCH_ERR_HIP; }
    return PATCH_OK;
}

patch_status patch_hard_masks(const float* P_tile, const void* P_24, int64_t N, int64_t K, int tile, uint8_t* tile_map,
                              void* mask24, void* stream) {
    if (!P_tile || !P_24 || !tile_map || !mask24) return PATCH_ERR_ARG;
    patch_status st = check_shape(N, K, tile);
    if (st != PATCH_OK) return st;
    if ((reinterpret_cast<uintptr_t>(P_24) & 3u) || (reinterpret_cast<uintptr_t>(mask24) & 7u)) return PATCH_ERR_ARG;
    const size_t T = (size_t)(N / tile) * (size_t)(K / tile);
    for (size_t i = 0; i < T; ++i) tile_map[i] = (P_tile[i] > 0.0f) ? 1 : 0;   // NaN and 0: the 2:4 class
    launch_hard_mask24(static_cast<const float*>(P_24), N * K / 4, static_cast<uint8_t*>(mask24), static_cast<hipStream_t>(stream));
    HIP_TRY(hipGetLastError());
    return PATCH_OK;
}

void patch_free(patch_packed* P) {
    if (!P) return;
    if (P->d_payload) (void)hipFree(P->d_payload);
    if (P->d_table) (void)hipFree(P->d_table);
    delete P;
}

// The host side of a packed weight (tile map, offset / type table, tile-row pairs) and its device buffers, the table
// uploaded on `s`, the payload not yet written.  Shared by patch_pack (which fills the payload from the matrix) and
// patch_deserialize (which copies a saved one).
static patch_status new_packed(int64_t N, int64_t K, const uint8_t* tile_map, int tile, hipStream_t s, patch_packed** out) {
    patch_packed* P = new (std::nothrow) patch_packed();
    if (!P) return PATCH_ERR_ALLOC;
    P->N = N; P->K = K; P->tile = tile;
    P->Tn = (int)(N / tile); P->Tk = (int)(K / tile);
    const size_t T = (size_t)P->Tn * (size_t)P->Tk;
    try {
        P->tile_map.resize(T);
        P->table.resize(T);
    } catch (...) { delete P; return PATCH_ERR_ALLOC; }
    uint64_t off = 0;
    for (size_t i = 0; i < T; ++i) {
        const bool sparse = tile_map[i] == 0;
        P->tile_map[i] = sparse ? 0 : 1;
        P->table[i] = make_entry(off, sparse);
        off += sparse ? sparse_tile_bytes(tile) : dense_tile_bytes(tile);
        if (sparse) ++P->n_sparse;
    }
    P->payload_bytes = off;
    if ((off / kGranule) >> 31) { delete P; return PATCH_ERR_SHAPE; }
    try {
        if (tile == 128) P->pairs = pair_tile_rows(P->tile_map, P->Tn, P->Tk);  // read by prefill_kernel_wreg only
    } catch (...) { delete P; return PATCH_ERR_ALLOC; }

    int dev = 0;
    hipDeviceProp_t prop;
    if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess) {
        g_last_hip_error = (int)hipGetLastError();
        delete P;
        return PATCH_ERR_HIP;
    }
    P->device = dev;
    P->n_cus = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;

    // a kilobyte of slack behind the payload keeps any over-read of the last tile inside the allocation
    const bool ok = hipMalloc(&P->d_payload, P->payload_bytes + kZeroPad) == hipSuccess &&
                    hipMalloc(&P->d_table, (T + P->pairs.size()) * sizeof(uint32_t)) == hipSuccess;
    if (!ok) {
        (void)hipGetLastError();
        patch_free(P);
        return PATCH_ERR_ALLOC;
    }
    hipError_t e = hipMemcpyAsync(P->d_table, P->table.data(), T * sizeof(uint32_t), hipMemcpyHostToDevice, s);
    if (e == hipSuccess)
        e = hipMemcpyAsync(P->d_table + T, P->pairs.data(), P->pairs.size() * sizeof(int32_t), hipMemcpyHostToDevice, s);
    if (e == hipSuccess) e = hipMemsetAsync(P->d_payload + P->payload_bytes, 0, kZeroPad, s);
    if (e != hipSuccess) {
        g_last_hip_error = (int)e;
        (void)hipStreamSynchronize(s);
        patch_free(P);
        return PATCH_ERR_HIP;
    }
    *out = P;
    return PATCH_OK;
}

patch_status patch_pack(const void* W_hat, int64_t N, int64_t K, const uint8_t* tile_map, int tile, void* stream,
                        patch_packed** out) {
    if (!W_hat || !tile_map || !out) return PATCH_ERR_ARG;
    patch_status st = check_shape(N, K, tile);
    if (st != PATCH_OK) return st;
    if (!aligned16(W_hat)) return PATCH_ERR_ARG;
    hipStream_t s = static_cast<hipStream_t>(stream);
    patch_packed* P = nullptr;
    st = new_packed(N, K, tile_map, tile, s, &P);
    if (st != PATCH_OK) return st;
    const size_t T = (size_t)P->Tn * (size_t)P->Tk;
    int* d_err = nullptr;
    if (hipMalloc(&d_err, sizeof(int)) != hipSuccess) {
        (void)hipGetLastError();
        (void)hipStreamSynchronize(s);
        patch_free(P);
        return PATCH_ERR_ALLOC;
    }
    hipError_t e = hipMemsetAsync(d_err, 0, sizeof(int), s);
    if (e == hipSuccess) {
        launch_pack(static_cast<const uint16_t*>(W_hat), K, P->d_table, (int)T, P->Tk, tile, P->d_payload, d_err, s);
        e = hipGetLastError();
    }
    int h_err = 0;
    if (e == hipSuccess) e = hipMemcpyAsync(&h_err, d_err, sizeof(int), hipMemcpyDeviceToHost, s);
    const hipError_t e_sync = hipStreamSynchronize(s);
    if (e == hipSuccess) e = e_sync;
    (void)hipFree(d_err);
    if (e != hipSuccess) {
        g_last_hip_error = (int)e;
        patch_free(P);
        return PATCH_ERR_HIP;
    }
    if (h_err) {
        patch_free(P);
        return PATCH_ERR_NOT_24;
    }
    *out = P;
    return PATCH_OK;
}

// ---- a packed weight saved to and loaded from host memory (saved.h)
size_t patch_serialized_bytes(const patch_packed* P) {
    if (!P) return 0;
    return saved_round(sizeof(SavedHeader)) + saved_round(P->tile_map.size()) + P->payload_bytes;
}

patch_status patch_serialize(const patch_packed* P, void* buf, size_t bytes, void* stream) {
    if (!P || !buf) return PATCH_ERR_ARG;
    if (bytes < patch_serialized_bytes(P)) return PATCH_ERR_SIZE;
    uint8_t* b = static_cast<uint8_t*>(buf);
    const size_t map_at = saved_round(sizeof(SavedHeader)), pay_at = map_at + saved_round(P->tile_map.size());
    memset(b, 0, pay_at);
    memcpy(b + map_at, P->tile_map.data(), P->tile_map.size());
    hipStream_t s = static_cast<hipStream_t>(stream);
    HIP_TRY(hipMemcpyAsync(b + pay_at, P->d_payload, P->payload_bytes, hipMemcpyDeviceToHost, s));
    HIP_TRY(hipStreamSynchronize(s));
    SavedHeader h = {};
    memcpy(h.magic, kSavedMagic16, 8);
    h.layout = kSavedLayout;
    h.tile = (uint32_t)P->tile;
    h.N = P->N;
    h.K = P->K;
    h.map_bytes = P->tile_map.size();
    h.payload_bytes = P->payload_bytes;
    h.checksum = fnv1a(b + pay_at, P->payload_bytes, fnv1a(b + map_at, P->tile_map.size(), kFnvBasis));
    memcpy(b, &h, sizeof(h));
    return PATCH_OK;
}

patch_status patch_deserialize(const void* buf, size_t bytes, void* stream, patch_packed** out) {
    if (!buf || !out) return PATCH_ERR_ARG;
    if (bytes < saved_round(sizeof(SavedHeader))) return PATCH_ERR_SIZE;
    const uint8_t* b = static_cast<const uint8_t*>(buf);
    SavedHeader h;
    memcpy(&h, b, sizeof(h));
    if (memcmp(h.magic, kSavedMagic16, 8) != 0 || h.layout != kSavedLayout) return PATCH_ERR_ARG;
    const patch_status shape = check_shape(h.N, h.K, (int)h.tile);
    if (shape != PATCH_OK) return shape;
    const uint64_t T = (uint64_t)(h.N / h.tile) * (uint64_t)(h.K / h.tile);
    if (h.map_bytes != T || h.aux_bytes != 0) return PATCH_ERR_ARG;
    const size_t map_at = saved_round(sizeof(SavedHeader)), pay_at = map_at + saved_round((size_t)T);
    if (bytes < pay_at || h.payload_bytes > bytes - pay_at) return PATCH_ERR_SIZE;
    for (uint64_t i = 0; i < T; ++i)
        if (b[map_at + i] > 1) return PATCH_ERR_ARG;
    if (fnv1a(b + pay_at, (size_t)h.payload_bytes, fnv1a(b + map_at, (size_t)T, kFnvBasis)) != h.checksum) return PATCH_ERR_ARG;
    hipStream_t s = static_cast<hipStream_t>(stream);
    patch_packed* P = nullptr;
    const patch_status st = new_packed(h.N, h.K, b + map_at, (int)h.tile, s, &P);
    if (st != PATCH_OK) return st;
    if (P->payload_bytes != h.payload_bytes) {   // the map decides the size: a header that disagrees is not ours
        (void)hipStreamSynchronize(s);
        patch_free(P);
        return PATCH_ERR_ARG;
    }
    hipError_t e = hipMemcpyAsync(P->d_payload, b + pay_at, P->payload_bytes, hipMemcpyHostToDevice, s);
    const hipError_t e_sync = hipStreamSynchronize(s);   // the caller's buffer is free to go when the call returns
    if (e == hipSuccess) e = e_sync;
    if (e != hipSuccess) {
        g_last_hip_error = (int)e;
        patch_free(P);
        return PATCH_ERR_HIP;
    }
    *out = P;
    return PATCH_OK;
}

// A pass on the decode path runs the 64-features-per-wavefront kernel (gemm_mid.hip) when asked for (variant 4) or,
// by default, when it can fill the chip and X is a large part of the traffic:
//   17 .. 64 rows: with K-chunks over a workspace, or with at least 72 groups of 64 features (measured at M = 32,
//     unsplit: 4096 x 4096, 64 groups, 19.6 us against 12.9 for the strip kernel; 5120 x 5120, 80 groups, 24.1
//     against 25.2; 13824 x 5120 25.7 against 46.3; at M = 64: 4864 x 896, 76 groups, 9.1 against 10.5);
//   12 .. 16 rows: with at least 160 groups (M = 16: 11008 x 4096 17.9 us against 19.9, 13824 x 5120 22.4 against
//     29.8; M = 8: 18.2 against 15.9 and 22.9 against 24.3; 4096 x 4096: the strip kernel at every M <= 16).
//     (a set of three 4096 x 4096 weights, 192 groups: from 8 rows, 20.0 us against 20.5; equal at M = 1)
static bool use_mid_kernel(int rows, int variant, int split_k, int mid_chunks, int64_t groups, bool set = false) {
    if (variant == 4) return true;
    if (variant != 0 || split_k != 0) return false;
    if (rows <= 16) return rows >= (set ? 8 : 12) && groups >= 160;
    return mid_chunks > 1 || groups >= 72;
}

// Measured crossovers between decode-path passes (up to 64 rows each; every pass streams the whole weight) and the
// 256 x 256-tile prefill kernel, f = 0.5, us at M = 32 / 64 / 128:
//   with a workspace (K split over otherwise idle compute units on either path):
//     4096 x 4096    passes 12.4 / 16.1 / 31.3    split prefill 21.1 / 21.7 / 24.4
//     5120 x 5120    passes 15.9 / 21.5 / 42.5    split prefill 23.4 / 25.2 / 28.2
//     13824 x 5120   passes 25.7 / 34.6 / 69.9    split prefill 35.2 / 39.6 / 42.9
//     5120 x 13824   passes 27.8 / 36.8 / 72.5    split prefill 42.1 / 43.0 / 45.9
//   without one the prefill grid is too small to fill the chip (66 - 93 us on these shapes) and the passes cost
//     4096 x 4096 12.9 / 20.7 / 41.2 (strip kernel), 5120 x 5120 24.1 / 32.9 / 66.1, 13824 x 5120 25.7 / 34.8 / 70.3.
// Without a workspace the choice is an estimate of both sides from the launch geometry (fitted to the same
// measurements; it reproduces the crossovers above - M = 192 at 4096 x 4096, 128 from 5120 features - and also holds
// for long-K weights of few features such as 4096 x 11008, where 16 output tiles run 172 steps each: 144 us, against
// 45 us for a 64-row pass):
//   unsplit prefill launch  rounds x 64-column steps x 1.0 us (tile 64 on the LDS-staged kernel: 1.45 us), or with
//                           blocks of 128 rows x 0.70 us (tile 64: 0.75), whichever is less (launch_prefill makes the
//                           same choice)
//   pass of up to 64 rows   steps x 0.3 us x (1 + 0.4 min(1, feature groups / 256)) x max(1, feature groups / 256)
// From 33 rows on the same estimate also decides a single pass against an unsplit prefill launch: only weights wider
// than the chip change side (65536 x 4096 at M = 64: 109 us in a pass, 90 us on the 128-row prefill kernel).
static int auto_path(int64_t M, const patch_packed* P, const patch_gemm_opts* opts, bool single = true) {
    const bool ws = opts && opts->workspace && opts->workspace_bytes >= 2 * (size_t)M * (size_t)P->N * sizeof(float);
    if (M <= 16) return PATCH_PATH_DECODE;
    // With a workspace, 33 .. 64 rows and a single weight of at least 160 feature groups (10240 features: the pass then
    // runs unsplit on the 64-features-per-wavefront kernel): the split prefill launch with 128-row blocks is ahead, e.g.
    // M = 33 / 64: 11008 x 4096 20.7 / 23.0 us against 21.2 / 26.6, 32000 x 4096 36.8 / 39.8 against 43.5 / 54.1 (8192 x
    // 4096 breaks even at 64 rows; 4096 features and fewer stay on the pass).
    if (ws && single && M > 32 && M <= kDecodeRows && P->N / 64 >= 160) return PATCH_PATH_PREFILL;
    if (ws) return M <= kDecodeRows ? PATCH_PATH_DECODE : PATCH_PATH_PREFILL;
    if (M <= 32 || (M <= kDecodeRows && !single)) return PATCH_PATH_DECODE;
    const double steps = (double)P->K / 64.0;
    const int64_t tiles = ((P->N + 255) / 256) * ((M + 255) / 256);
    const double rounds = (double)((tiles + P->n_cus - 1) / P->n_cus);
    const int64_t tiles128 = ((P->N + 255) / 256) * ((M + 127) / 128);   // blocks of 128 rows: 0.70 / 0.75 us per step
    const double us128 = (double)((tiles128 + P->n_cus - 1) / P->n_cus) * steps * (P->tile == 128 ? 0.70 : 0.75);
    const double us256 = rounds * steps * (P->tile == 128 ? 1.0 : 1.45);
    const double prefill_us = us128 < us256 ? us128 : us256;
    const double groups = (double)(P->N / 64);
    // (a weight of more feature groups than the chip takes at once - 65536 features - costs that many times more)
    const double pass_us = steps * 0.3 * (1.0 + 0.4 * (groups < 256.0 ? groups / 256.0 : 1.0)) * (groups > 256.0 ? groups / 256.0 : 1.0);
    // a last pass of r < 64 rows costs about (1 + r / 64) / 2 of a full one (11008 x 4096: 12.8 us for 1 row, 26.7 for 64)
    const int64_t full = M / kDecodeRows, rest = M % kDecodeRows;
    const double passes = (double)full + (rest ? 0.5 + 0.5 * (double)rest / kDecodeRows : 0.0);
    return passes * pass_us < prefill_us ? PATCH_PATH_DECODE : PATCH_PATH_PREFILL;
}

patch_status patch_gemm_ex(const void* X, int64_t M, const patch_packed* P, void* Y, void* stream, const patch_gemm_opts* opts) {
    if (!X || !P || !Y || M < 0) return PATCH_ERR_ARG;
    if (!aligned16(X) || !aligned16(Y)) return PATCH_ERR_ARG;
    int path = PATCH_PATH_AUTO, split_k = 0, variant = 0;
    if (opts) { path = opts->path; split_k = opts->split_k; variant = opts->variant; }
    if (path < PATCH_PATH_AUTO || path > PATCH_PATH_PREFILL || split_k < 0 || split_k > 16 || variant < 0) return PATCH_ERR_ARG;
    if (opts && opts->workspace && !aligned16(opts->workspace)) return PATCH_ERR_ARG;
    if (M == 0) return PATCH_OK;  // an empty batch: nothing to launch, Y has no rows
    if (path == PATCH_PATH_AUTO) path = auto_path(M, P, opts);
    hipStream_t s = static_cast<hipStream_t>(stream);
    GemmArgs a;
    a.X = static_cast<const uint16_t*>(X);
    a.M = M; a.N = P->N; a.K = P->K;
    a.tile = P->tile; a.Tn = P->Tn; a.Tk = P->Tk;
    a.payload = P->d_payload; a.table = P->d_table;
    a.Y = static_cast<float*>(Y);
    a.n_cus = P->n_cus;
    a.sparse_pct = (int)(100 * P->n_sparse / ((int64_t)P->Tn * P->Tk));
    if (opts && opts->workspace) { a.ws = static_cast<float*>(opts->workspace); a.ws_bytes = opts->workspace_bytes; }
    a.ybf16 = (opts && opts->y_bf16) ? 1 : 0;
    if (path == PATCH_PATH_DECODE) {
        WeightSet one = {};
        one.payload[0] = a.payload; one.table[0] = a.table; one.Y[0] = a.Y; one.N[0] = a.N;
        one.count = 1;
        one.units = (int)(a.N / 64);
        for (int64_t m0 = 0; m0 < M; m0 += kDecodeRows) {
            const int rows = (int)((M - m0 < kDecodeRows) ? M - m0 : kDecodeRows);
            const int chunks = (rows > 16 || variant == 4) ? mid_split(a, rows, variant == 4 ? split_k : 0) : 1;
            if (use_mid_kernel(rows, variant, split_k, chunks, a.N / 64)) launch_mid_set(a, one, m0, rows, chunks, s);
            else launch_decode(a, m0, rows, split_k, variant, s);
        }
    } else {
        launch_prefill(a, variant, split_k, s);
    }
    HIP_TRY(hipGetLastError());
    return PATCH_OK;
}

patch_status patch_tune_all(const void* X, int64_t M, const patch_packed* P, void* Y, void* workspace, size_t workspace_bytes,
                            void* stream, int reps, patch_tune_result* results, size_t cap, size_t* count) {
    if (!X || !P || !Y || !results || !count || M <= 0 || reps < 1) return PATCH_ERR_ARG;
    if (!aligned16(X) || !aligned16(Y) || (workspace && !aligned16(workspace))) return PATCH_ERR_ARG;
    hipStream_t s = static_cast<hipStream_t>(stream);
    std::vector<patch_gemm_opts> cand;
    auto add = [&](int path, int split_k, int variant, bool ws) {
        cand.push_back(patch_gemm_opts{path, split_k, variant, ws ? workspace : nullptr, ws ? workspace_bytes : 0, 0});
    };
    const int steps = P->Tk * (P->tile / kStepCols);
    if (M <= 256) {  // every pass of 64 rows streams the whole weight again: no contender beyond that
        add(PATCH_PATH_DECODE, 0, 0, false);
        add(PATCH_PATH_DECODE, 0, 2, false);   // 8 K-steps per wavefront
        add(PATCH_PATH_DECODE, 0, 3, false);   // 4 K-steps per wavefront
        if (M <= 8) {                          // X loads: two per step / one for several steps
            add(PATCH_PATH_DECODE, 0, 5, false);
            add(PATCH_PATH_DECODE, 0, 6, false);
        }
        for (int kw : {2, 4, 8, 16})           // wavefronts per workgroup
            for (int v : {2, 3})
                if (kw * (v == 2 ? 8 : 4) <= 2 * steps && (kw <= 8 || v == 3)) add(PATCH_PATH_DECODE, kw, v, false);
        if (M >= 12) {  // the 64-features-per-wavefront kernel, unsplit and with K-chunks over the workspace
            add(PATCH_PATH_DECODE, 0, 4, false);
            const size_t per_slice = (size_t)(M < kDecodeRows ? M : kDecodeRows) * (size_t)P->N * sizeof(float);
            if (workspace)
                for (int sk : {2, 3, 4, 6, 8})
                    if ((size_t)sk * per_slice <= workspace_bytes && sk <= P->Tk) add(PATCH_PATH_DECODE, sk, 4, true);
        }
    }
    const size_t per_slice = (size_t)M * (size_t)P->N * sizeof(float);
    const int tiles_per_slice = 512 / P->tile;   // K slices of at least 512 columns
    if (P->tile == 128) {
        add(PATCH_PATH_PREFILL, 1, 0, false);   // 256 x 256, one wavefront per SIMD
        add(PATCH_PATH_PREFILL, 1, 2, false);   // 256 x 256, two wavefronts per SIMD
        add(PATCH_PATH_PREFILL, 1, 1, false);   // 128 x 128: the small execution tile
        if (workspace) add(PATCH_PATH_PREFILL, 0, 0, true);   // automatic: may split a part-filled last round only
        if (workspace)
            for (int sk : {2, 3, 4, 6, 8, 12, 16})
                if ((size_t)sk * per_slice <= workspace_bytes && sk * 2 <= P->Tk) add(PATCH_PATH_PREFILL, sk, 0, true);
    } else {
        add(PATCH_PATH_PREFILL, 1, 0, false);   // 256 x 256 with the weights in registers (the tile-64 default)
        add(PATCH_PATH_PREFILL, 1, 2, false);   // 256 x 256 LDS-staged
        add(PATCH_PATH_PREFILL, 1, 1, false);   // 128 x 128: the small execution tile
        if (workspace) add(PATCH_PATH_PREFILL, 0, 0, true);   // automatic
        if (workspace)
            for (int sk : {2, 3, 4, 6, 8})
                if ((size_t)sk * per_slice <= workspace_bytes && sk * 4 <= P->Tk) add(PATCH_PATH_PREFILL, sk, 0, true);
    }
    if (M <= 4096) {   // 256 features x 128 rows per workgroup: beyond a few thousand rows never ahead
        for (int v : {4, 5}) {   // LDS-staged; weights in registers
            add(PATCH_PATH_PREFILL, 1, v, false);
            if (workspace)
                for (int sk : {2, 3, 4, 6, 8})
                    if ((size_t)sk * per_slice <= workspace_bytes && sk * tiles_per_slice <= P->Tk) add(PATCH_PATH_PREFILL, sk, v, true);
        }
    }
    hipEvent_t e0, e1;
    HIP_TRY(hipEventCreate(&e0));
    if (hipError_t e = hipEventCreate(&e1); e != hipSuccess) { (void)hipEventDestroy(e0); g_last_hip_error = (int)e; return PATCH_ERR_HIP; }
    patch_status st = PATCH_OK;
    for (size_t i = 0; i < cand.size() && st == PATCH_OK; ++i) {
        for (int r = 0; r < 2 && st == PATCH_OK; ++r) st = patch_gemm_ex(X, M, P, Y, stream, &cand[i]);
        if (st != PATCH_OK) break;
        hipError_t e = hipEventRecord(e0, s);
        for (int r = 0; r < reps && st == PATCH_OK; ++r) st = patch_gemm_ex(X, M, P, Y, stream, &cand[i]);
        if (e == hipSuccess) e = hipEventRecord(e1, s);
        if (e == hipSuccess) e = hipEventSynchronize(e1);
        float ms = 0.f;
        if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
        if (e != hipSuccess) { g_last_hip_error = (int)e; st = PATCH_ERR_HIP; break; }
        if (i < cap) results[i] = patch_tune_result{cand[i], ms * 1000.f / (float)reps};
    }
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (st != PATCH_OK) return st;
    *count = cand.size();
    return PATCH_OK;
}

patch_status patch_tune(const void* X, int64_t M, const patch_packed* P, void* Y, void* workspace, size_t workspace_bytes,
                        void* stream, int reps, patch_gemm_opts* best, float* best_us) {
    if (!best) return PATCH_ERR_ARG;
    constexpr size_t kCap = 64;
    patch_tune_result res[kCap];
    size_t n = 0;
    const patch_status st = patch_tune_all(X, M, P, Y, workspace, workspace_bytes, stream, reps, res, kCap, &n);
    if (st != PATCH_OK) return st;
    if (n > kCap) n = kCap;
    size_t bi = 0;
    for (size_t i = 1; i < n; ++i)
        if (res[i].us < res[bi].us) bi = i;
    *best = res[bi].opts;
    if (best_us) *best_us = res[bi].us;
    // leave the product of the chosen schedule in Y
    return patch_gemm_ex(X, M, P, Y, stream, best);
}

// ---- table of tuned schedules
struct TuneKey {
    int64_t bucket, N, K, n_sparse;
    int tile;
    bool operator<(const TuneKey& o) const {
        return std::tie(bucket, N, K, n_sparse, tile) < std::tie(o.bucket, o.N, o.K, o.n_sparse, o.tile);
    }
};
struct TuneEntry { int path, split_k, variant, y_bf16; bool uses_ws; };
struct patch_tune_table {
    mutable std::mutex mu;
    std::map<TuneKey, TuneEntry> entries;
};

int64_t patch_tune_bucket(int64_t M) {
    if (M <= 1) return 1;
    int64_t b = 1;
    while (b < M && b < ((int64_t)1 << 62)) b <<= 1;
    return b;
}

patch_status patch_tune_table_create(patch_tune_table** out) {
    if (!out) return PATCH_ERR_ARG;
    patch_tune_table* t = new (std::nothrow) patch_tune_table();
    if (!t) return PATCH_ERR_ALLOC;
    *out = t;
    return PATCH_OK;
}

void patch_tune_table_destroy(patch_tune_table* t) { delete t; }

size_t patch_tune_table_size(const patch_tune_table* t) {
    if (!t) return 0;
    std::lock_guard<std::mutex> lock(t->mu);
    return t->entries.size();
}

static bool tune_key_ok(int64_t M, int64_t N, int64_t K, int tile, int64_t ns) {
    return M >= 1 && ns >= 0 && check_shape(N, K, tile) == PATCH_OK && ns <= (N / tile) * (K / tile);
}

patch_status patch_tune_table_put(patch_tune_table* t, int64_t M, int64_t N, int64_t K, int tile, int64_t n_sparse_tiles,
                                  const patch_gemm_opts* opts) {
    if (!t || !opts || !tune_key_ok(M, N, K, tile, n_sparse_tiles)) return PATCH_ERR_ARG;
    if (opts->path < PATCH_PATH_AUTO || opts->path > PATCH_PATH_PREFILL || opts->split_k < 0 || opts->split_k > 16 || opts->variant < 0)
        return PATCH_ERR_ARG;
    const TuneKey k{patch_tune_bucket(M), N, K, n_sparse_tiles, tile};
    const TuneEntry e{opts->path, opts->split_k, opts->variant, opts->y_bf16 ? 1 : 0, opts->workspace != nullptr};
    std::lock_guard<std::mutex> lock(t->mu);
    try { t->entries[k] = e; } catch (...) { return PATCH_ERR_ALLOC; }
    return PATCH_OK;
}

patch_status patch_tune_table_get(const patch_tune_table* t, int64_t M, int64_t N, int64_t K, int tile, int64_t n_sparse_tiles,
                                  void* workspace, size_t workspace_bytes, patch_gemm_opts* out) {
    if (!t || !out || !tune_key_ok(M, N, K, tile, n_sparse_tiles)) return PATCH_ERR_ARG;
    const TuneKey k{patch_tune_bucket(M), N, K, n_sparse_tiles, tile};
    std::lock_guard<std::mutex> lock(t->mu);
    const auto it = t->entries.find(k);
    if (it == t->entries.end()) return PATCH_ERR_NOT_FOUND;
    const TuneEntry& e = it->second;
    if (e.uses_ws && !workspace) return PATCH_ERR_NOT_FOUND;
    *out = patch_gemm_opts{e.path, e.split_k, e.variant, e.uses_ws ? workspace : nullptr, e.uses_ws ? workspace_bytes : 0, e.y_bf16};
    return PATCH_OK;
}

patch_status patch_tune_table_export(const patch_tune_table* t, patch_tune_entry* entries, size_t cap, size_t* count) {
    if (!t || !count || (!entries && cap)) return PATCH_ERR_ARG;
    std::lock_guard<std::mutex> lock(t->mu);
    *count = t->entries.size();
    if (!entries) return PATCH_OK;          // a size query
    if (cap < t->entries.size()) return PATCH_ERR_SIZE;
    size_t i = 0;
    for (const auto& kv : t->entries) {
        const TuneKey& k = kv.first;
        const TuneEntry& e = kv.second;
        entries[i++] = patch_tune_entry{k.bucket, k.N, k.K, k.n_sparse, k.tile, e.path, e.split_k, e.variant, e.y_bf16, e.uses_ws ? 1 : 0};
    }
    return PATCH_OK;
}

patch_status patch_tune_table_import(patch_tune_table* t, const patch_tune_entry* entries, size_t count) {
    if (!t || (!entries && count)) return PATCH_ERR_ARG;
    // all or nothing: every entry is checked before the first is stored
    for (size_t i = 0; i < count; ++i) {
        const patch_tune_entry& e = entries[i];
        if (!tune_key_ok(e.m_bucket, e.N, e.K, e.tile, e.n_sparse_tiles) || patch_tune_bucket(e.m_bucket) != e.m_bucket) return PATCH_ERR_ARG;
        if (e.path < PATCH_PATH_AUTO || e.path > PATCH_PATH_PREFILL || e.split_k < 0 || e.split_k > 16 || e.variant < 0) return PATCH_ERR_ARG;
    }
    std::lock_guard<std::mutex> lock(t->mu);
    try {
        for (size_t i = 0; i < count; ++i) {
            const patch_tune_entry& e = entries[i];
            t->entries[TuneKey{e.m_bucket, e.N, e.K, e.n_sparse_tiles, e.tile}] =
                TuneEntry{e.path, e.split_k, e.variant, e.y_bf16 ? 1 : 0, e.uses_workspace != 0};
        }
    } catch (...) { return PATCH_ERR_ALLOC; }
    return PATCH_OK;
}

patch_status patch_tune_layer(patch_tune_table* t, const void* X_decode, int64_t M_decode, const void* X_prefill, int64_t M_prefill,
                              const patch_packed* P, void* Y, void* workspace, size_t workspace_bytes, void* stream, int reps) {
    if (!t || !P || !X_decode || !X_prefill || M_decode < 1 || M_prefill < 1) return PATCH_ERR_ARG;
    // the decode input first, then the prefill input, both from the one packed weight
    const void* xs[2] = {X_decode, X_prefill};
    const int64_t ms[2] = {M_decode, M_prefill};
    for (int i = 0; i < 2; ++i) {
        patch_gemm_opts best;
        patch_status st = patch_tune(xs[i], ms[i], P, Y, workspace, workspace_bytes, stream, reps, &best, nullptr);
        if (st != PATCH_OK) return st;
        st = patch_tune_table_put(t, ms[i], P->N, P->K, P->tile, P->n_sparse, &best);
        if (st != PATCH_OK) return st;
    }
    return PATCH_OK;
}

size_t patch_gemm_workspace_bytes(int64_t M, const patch_packed* P, const patch_gemm_opts* opts) {
    if (!P || M <= 0) return 0;
    int path = PATCH_PATH_AUTO, split_k = 0, variant = 0;
    if (opts) { path = opts->path; split_k = opts->split_k; variant = opts->variant; }
    patch_gemm_opts enough = {path, split_k, variant, reinterpret_cast<void*>(16), ~(size_t)0, 0};  // the choice given enough
    if (path == PATCH_PATH_AUTO) path = auto_path(M, P, &enough);
    GemmArgs a;
    a.X = nullptr; a.M = M; a.N = P->N; a.K = P->K;
    a.tile = P->tile; a.Tn = P->Tn; a.Tk = P->Tk;
    a.payload = nullptr; a.table = nullptr; a.Y = nullptr;
    a.n_cus = P->n_cus;
    a.ws = reinterpret_cast<float*>(16);  // "enough": ask for the unconstrained choice
    a.ws_bytes = ~(size_t)0;
    if (path == PATCH_PATH_DECODE) {
        // passes of 17 .. 64 rows may cut K into chunks over the workspace (the largest pass decides)
        const int rows = (int)(M < kDecodeRows ? M : kDecodeRows);
        if (rows <= 16 && variant != 4) return 0;
        const int chunks = mid_split(a, rows, variant == 4 ? split_k : 0);
        if (!use_mid_kernel(rows, variant, split_k, chunks, a.N / 64) || chunks < 2) return 0;
        return (size_t)chunks * (size_t)rows * (size_t)P->N * sizeof(float);
    }
    if (variant == 1) return 0;
    if (variant == 0 && split_k == 0) {
        int split128 = 1;
        if (prefill_prefers_128_rows(a, &split128)) return split128 > 1 ? (size_t)split128 * (size_t)M * (size_t)P->N * sizeof(float) : 0;
    }
    if (variant == 2 || variant == 4 || variant == 5 || (variant == 6 && a.tile == 64) || !prefill_wreg_supports(a)) {   // whole-launch K split only (same for both 256-row kernels)
        const int sl = prefill_lds_split(a, split_k, variant == 4 || variant == 5 ? 128 : 256);
        return sl > 1 ? (size_t)sl * (size_t)M * (size_t)P->N * sizeof(float) : 0;
    }
    const int s = prefill_wreg_split(a, split_k);
    if (s > 1) return (size_t)s * (size_t)M * (size_t)P->N * sizeof(float);
    if (split_k != 0) return 0;
    int tail = 0;
    const int ts = prefill_wreg_tail(a, &tail);   // K slices for the part-filled last round only
    return ts > 1 ? (size_t)ts * (size_t)tail * 256 * 256 * sizeof(float) : 0;
}

patch_status patch_gemm_many(const void* X, int64_t M, const patch_packed* const* P, void* const* Y, int count, void* stream,
                             const patch_gemm_opts* opts) {
    if (!X || !P || !Y || M < 0 || count < 1 || count > PATCH_MAX_MANY) return PATCH_ERR_ARG;
    static_assert(PATCH_MAX_MANY == kMaxMany, "header and kernels disagree");
    if (!aligned16(X)) return PATCH_ERR_ARG;
    for (int i = 0; i < count; ++i) {
        if (!P[i] || !Y[i] || !aligned16(Y[i])) return PATCH_ERR_ARG;
        if (P[i]->K != P[0]->K || P[i]->tile != P[0]->tile) return PATCH_ERR_SHAPE;
    }
    int path = PATCH_PATH_AUTO, split_k = 0, variant = 0;
    if (opts) { path = opts->path; split_k = opts->split_k; variant = opts->variant; }
    if (path < PATCH_PATH_AUTO || path > PATCH_PATH_PREFILL || split_k < 0 || split_k > 16 || variant < 0) return PATCH_ERR_ARG;
    if (M == 0) return PATCH_OK;
    if (path == PATCH_PATH_AUTO) path = auto_path(M, P[0], opts, count == 1);
    hipStream_t s = static_cast<hipStream_t>(stream);
    GemmArgs a = {};
    a.X = static_cast<const uint16_t*>(X);
    a.M = M; a.K = P[0]->K; a.N = P[0]->N;
    a.tile = P[0]->tile; a.Tk = P[0]->Tk;
    a.n_cus = P[0]->n_cus;
    {
        int64_t sparse = 0, tiles = 0;
        for (int i = 0; i < count; ++i) {
            if (!P[i]) return PATCH_ERR_ARG;
            sparse += P[i]->n_sparse;
            tiles += (int64_t)P[i]->Tn * P[i]->Tk;
        }
        a.sparse_pct = (int)(100 * sparse / tiles);
    }
    a.ybf16 = (opts && opts->y_bf16) ? 1 : 0;
    if (opts && opts->workspace && !aligned16(opts->workspace)) return PATCH_ERR_ARG;
    if (opts && opts->workspace && split_k == 0) { a.ws = static_cast<float*>(opts->workspace); a.ws_bytes = opts->workspace_bytes; }
    if (path == PATCH_PATH_PREFILL && count > 1 && (variant == 0 || variant == 3) && split_k <= 1 && prefill_wreg_supports(a)) {
        // one launch over the feature blocks of all weights (with a workspace and few blocks: K in slices over the
        // whole set, see launch_prefill_wreg_set)
        int blocks = 0;
        WeightSet set = {};
        for (int i = 0; i < count; ++i) {
            set.payload[i] = P[i]->d_payload;
            set.table[i] = P[i]->d_table;
            set.Y[i] = static_cast<float*>(Y[i]);
            set.N[i] = P[i]->N;
            set.first[i] = blocks;
            blocks += (int)((P[i]->N + 255) / 256);
        }
        set.count = count;
        set.units = blocks;
        launch_prefill_wreg_set(a, set, s);
        HIP_TRY(hipGetLastError());
        return PATCH_OK;
    }
    if (path == PATCH_PATH_PREFILL || count == 1) {
        patch_gemm_opts o = {path, split_k, variant, opts ? opts->workspace : nullptr, opts ? opts->workspace_bytes : 0, a.ybf16};
        for (int i = 0; i < count; ++i) {
            const patch_status st = patch_gemm_ex(X, M, P[i], Y[i], stream, &o);
            if (st != PATCH_OK) return st;
        }
        return PATCH_OK;
    }
    DecodeSet set = {};
    int strips = 0;
    for (int i = 0; i < count; ++i) {
        set.payload[i] = P[i]->d_payload;
        set.table[i] = P[i]->d_table;
        set.Y[i] = static_cast<float*>(Y[i]);
        set.N[i] = P[i]->N;
        set.first[i] = strips;
        strips += (int)(P[i]->N / 16);
    }
    set.count = count;
    set.units = strips;
    // the same set in units of 64-feature groups, for passes of more than 16 rows
    WeightSet wide = set;
    int groups = 0;
    for (int i = 0; i < count; ++i) {
        wide.first[i] = groups;
        groups += (int)(P[i]->N / 64);
    }
    wide.units = groups;
    for (int64_t m0 = 0; m0 < M; m0 += kDecodeRows) {
        const int rows = (int)((M - m0 < kDecodeRows) ? M - m0 : kDecodeRows);
        if (use_mid_kernel(rows, variant, split_k, 1, groups, true)) launch_mid_set(a, wide, m0, rows, 1, s);
        else launch_decode_set(a, set, m0, rows, split_k, variant, s);
    }
    HIP_TRY(hipGetLastError());
    return PATCH_OK;
}

patch_status patch_gemm(const void* X, int64_t M, const patch_packed* P, void* Y, void* stream) {
    return patch_gemm_ex(X, M, P, Y, stream, nullptr);
}

patch_status patch_gemm_static(const void* X, int64_t M, const patch_packed* P, void* Y, void* stream) {
    if (!X || !P || !Y || M < 0) return PATCH_ERR_ARG;
    // what the automatic schedule would use given any amount of workspace: beyond the static array, refuse
    const size_t need = patch_gemm_workspace_bytes(M, P, nullptr);
    if (need > kStaticScratchBytes) return PATCH_ERR_SIZE;
    void* ws = nullptr;
    const patch_status st = static_scratch(&ws);
    if (st != PATCH_OK) return st;
    const patch_gemm_opts o = {PATCH_PATH_AUTO, 0, 0, ws, kStaticScratchBytes, 0};
    return patch_gemm_ex(X, M, P, Y, stream, &o);
}

patch_status patch_unpack(const patch_packed* P, void* W_out, void* stream) {
    if (!P || !W_out || !aligned16(W_out)) return PATCH_ERR_ARG;
    launch_unpack(P->d_payload, P->d_table, P->Tn * P->Tk, P->Tk, P->tile, P->K, static_cast<uint16_t*>(W_out),
                  static_cast<hipStream_t>(stream));
    HIP_TRY(hipGetLastError());
    return PATCH_OK;
}

size_t patch_packed_bytes(const patch_packed* P) { return P ? P->payload_bytes : 0; }
size_t patch_table_bytes(const patch_packed* P) { return P ? (P->table.size() + P->pairs.size()) * sizeof(uint32_t) : 0; }

patch_status patch_packed_dims(const patch_packed* P, int64_t* N, int64_t* K, int* tile, int64_t* n_sparse_tiles) {
    if (!P) return PATCH_ERR_ARG;
    if (N) *N = P->N;
    if (K) *K = P->K;
    if (tile) *tile = P->tile;
    if (n_sparse_tiles) *n_sparse_tiles = P->n_sparse;
    return PATCH_OK;
}

patch_status patch_packed_tile_map(const patch_packed* P, uint8_t* tile_map, size_t bytes) {
    if (!P || !tile_map) return PATCH_ERR_ARG;
    if (bytes < P->tile_map.size()) return PATCH_ERR_SIZE;
    memcpy(tile_map, P->tile_map.data(), P->tile_map.size());
    return PATCH_OK;
}

patch_status patch_packed_row_order(const patch_packed* P, int32_t* order, size_t cap, size_t* count) {
    if (!P || !order || !count) return PATCH_ERR_ARG;
    if (cap < P->pairs.size()) return PATCH_ERR_SIZE;
    if (!P->pairs.empty()) memcpy(order, P->pairs.data(), P->pairs.size() * sizeof(int32_t));
    *count = P->pairs.size();
    return PATCH_OK;
}

patch_status patch_canonical_sizes(const patch_packed* P, size_t* vals_bytes, size_t* meta_bytes) {
    if (!P) return PATCH_ERR_ARG;
    const size_t t2 = (size_t)P->tile * P->tile;
    const size_t n_dense = P->tile_map.size() - (size_t)P->n_sparse;
    if (vals_bytes) *vals_bytes = 2 * (n_dense * t2 + (size_t)P->n_sparse * t2 / 2);
    if (meta_bytes) *meta_bytes = (size_t)P->n_sparse * t2 / 8;
    return PATCH_OK;
}

// Host-side re-ordering of the device layout into the canonical order (test hook; not a hot path).
patch_status patch_export_canonical(const patch_packed* P, void* vals, size_t vals_bytes, void* meta, size_t meta_bytes) {
    if (!P || !vals || (!meta && P->n_sparse)) return PATCH_ERR_ARG;
    size_t need_v = 0, need_m = 0;
    patch_canonical_sizes(P, &need_v, &need_m);
    if (vals_bytes < need_v || meta_bytes < need_m) return PATCH_ERR_SIZE;
    std::vector<uint8_t> host;
    try { host.resize(P->payload_bytes); } catch (...) { return PATCH_ERR_ALLOC; }
    HIP_TRY(hipDeviceSynchronize());
    HIP_TRY(hipMemcpy(host.data(), P->d_payload, P->payload_bytes, hipMemcpyDeviceToHost));
    const int t = P->tile, KPT = t / kStepCols;
    uint16_t* v = static_cast<uint16_t*>(vals);
    uint8_t* mt = static_cast<uint8_t*>(meta);
    if (need_m) memset(mt, 0, need_m);
    size_t vi = 0, nib = 0;
    for (size_t ti = 0; ti < P->table.size(); ++ti) {
        const uint32_t e = P->table[ti];
        const uint8_t* base = host.data() + entry_offset(e);
        for (int r = 0; r < t; ++r) {
            const int s = r / 16, i = r % 16;
            if (!entry_sparse(e)) {
                for (int c = 0; c < t; ++c) {
                    const int j = c / 64, h = (c % 64) / 32, q = (c % 32) / 8, el = c % 8;
                    const size_t byte = (size_t)(((s * KPT + j) * 2 + h) * 64 + (16 * q + i)) * 16 + 2 * el;
                    uint16_t x;
                    memcpy(&x, base + byte, 2);
                    v[vi++] = x;
                }
            } else {
                for (int g = 0; g < t / 4; ++g) {
                    const int c = 4 * g, j = c / 64, qa = (c % 64) / 16, gl = (c % 16) / 4;
                    const int lane = 16 * qa + i;
                    const size_t byte = (size_t)((s * KPT + j) * 64 + lane) * 16 + 4 * gl;
                    uint16_t x[2];
                    memcpy(x, base + byte, 4);
                    v[vi++] = x[0];
                    v[vi++] = x[1];
                    uint16_t idx;
                    memcpy(&idx, base + sparse_vals_bytes(t) + (size_t)((s * 64 + lane) * KPT + j) * 2, 2);
                    const uint8_t nibble = (uint8_t)((idx >> (4 * gl)) & 0xF);
                    mt[nib >> 1] |= (uint8_t)(nibble << (4 * (nib & 1)));
                    ++nib;
                }
            }
        }
    }
    return PATCH_OK;
}

}  // extern "C"
