/*
 * Sanitizer driver for the CPU oracle (test infrastructure): compiled together with patch_oracle.c under
 * -fsanitize=address,undefined and run by tests/test_oracle_pins.py.  It walks every oracle routine over small
 * seeded inputs - ragged tile counts, all-dense and all-2:4 maps, groups with zero, one and two nonzeros, the
 * rejection path - so that an out-of-bounds access, a use of uninitialised heap or undefined arithmetic in the
 * oracle aborts the run.  It checks no numbers beyond round trips; the pins do that.
 */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

int patch_oracle_apply_mask(const uint16_t*, const uint8_t*, const uint8_t*, int64_t, int64_t, int, uint16_t*);
int patch_oracle_hard_masks(const float*, const float*, int64_t, int64_t, int, uint8_t*, uint8_t*);
int patch_oracle_packed_sizes(int64_t, int64_t, int, const uint8_t*, int64_t*, int64_t*);
int patch_oracle_pack(const uint16_t*, int64_t, int64_t, const uint8_t*, int, uint16_t*, uint8_t*, int64_t*);
int patch_oracle_unpack(const uint16_t*, const uint8_t*, int64_t, int64_t, const uint8_t*, int, uint16_t*);
int patch_oracle_gemm(const uint16_t*, int64_t, const uint16_t*, const uint8_t*, int64_t, int64_t, const uint8_t*, int, double*);
int patch_oracle_gemm_points(const uint16_t*, int64_t, const uint16_t*, int64_t, int64_t, const int64_t*, int64_t, double*);
int patch_oracle_round_bf16(const double*, int64_t, uint16_t*);
int patch_oracle_quantize4(const uint16_t*, int64_t, int64_t, int, int8_t*, uint16_t*);
int patch_oracle_dequantize4(const int8_t*, const uint16_t*, int64_t, int64_t, int, uint16_t*);
int patch_oracle_packed4_sizes(int64_t, int64_t, int, const uint8_t*, int64_t*, int64_t*, int64_t*);

static uint64_t state = 0x9E3779B97F4A7C15ull;
static uint32_t rnd(void) {
    state ^= state << 13; state ^= state >> 7; state ^= state << 17;
    return (uint32_t)(state >> 32);
}

#define REQUIRE(c) do { if (!(c)) { fprintf(stderr, "sanitize_check: %s failed at line %d\n", #c, __LINE__); return 1; } } while (0)

static int one_case(int64_t N, int64_t K, int t, int64_t M, int map_kind) {
    const int64_t Tn = N / t, Tk = K / t, T = Tn * Tk;
    uint16_t* W = malloc((size_t)(N * K) * 2);
    uint16_t* W_hat = malloc((size_t)(N * K) * 2);
    uint16_t* W_back = malloc((size_t)(N * K) * 2);
    uint8_t* m24 = malloc((size_t)(N * K));
    uint8_t* tm = malloc((size_t)T);
    uint16_t* X = malloc((size_t)(M * K) * 2);
    double* Y = malloc((size_t)(M * N) * sizeof(double));
    REQUIRE(W && W_hat && W_back && m24 && tm && X && Y);
    for (int64_t i = 0; i < N * K; ++i) {
        const uint32_t r = rnd();
        /* small normal numbers, some exact zeros, negative zeros and a denormal */
        W[i] = (r % 11 == 0) ? 0x0000 : (r % 13 == 0) ? 0x8000 : (r % 97 == 0) ? 0x0001 : (uint16_t)(0x3C00 + (r & 0x83FF));
    }
    for (int64_t g = 0; g < N * K / 4; ++g) {   /* keep-mask: two, sometimes one or zero, of every four */
        const uint32_t r = rnd();
        uint8_t* m = m24 + 4 * g;
        memset(m, 0, 4);
        m[r & 3] = 1;
        if (r % 7) m[(r >> 2) & 3] = 1;
        if (r % 29 == 0) memset(m, 0, 4);
    }
    for (int64_t i = 0; i < T; ++i) tm[i] = map_kind == 0 ? 1 : map_kind == 1 ? 0 : (uint8_t)(rnd() & 1);
    for (int64_t i = 0; i < M * K; ++i) X[i] = (uint16_t)(0x3F00 + (rnd() & 0x80FF));
    REQUIRE(patch_oracle_apply_mask(W, tm, m24, N, K, t, W_hat) == 0);
    int64_t nv = 0, nm = 0, bad[2] = {0, 0};
    REQUIRE(patch_oracle_packed_sizes(N, K, t, tm, &nv, &nm) == 0);
    uint16_t* vals = malloc((size_t)(nv > 0 ? nv : 1) * 2);
    uint8_t* meta = calloc((size_t)(nm > 0 ? nm : 1), 1);
    REQUIRE(vals && meta);
    REQUIRE(patch_oracle_pack(W_hat, N, K, tm, t, vals, meta, bad) == 0);
    REQUIRE(patch_oracle_unpack(vals, meta, N, K, tm, t, W_back) == 0);
    for (int64_t i = 0; i < N * K; ++i) REQUIRE((W_back[i] & 0x7FFF) == (W_hat[i] & 0x7FFF));
    REQUIRE(patch_oracle_gemm(X, M, vals, meta, N, K, tm, t, Y) == 0);
    int64_t pts[6] = {0, 0, M - 1, N - 1, M / 2, N / 2};
    double yp[3];
    REQUIRE(patch_oracle_gemm_points(X, M, W_hat, N, K, pts, 3, yp) == 0);
    REQUIRE(yp[0] == Y[0] && yp[1] == Y[(M - 1) * N + N - 1]);
    uint16_t* yb = malloc((size_t)(M * N) * 2);
    REQUIRE(yb && patch_oracle_round_bf16(Y, M * N, yb) == 0);
    {   /* 4-bit storage of the pruned matrix */
        int8_t* codes = malloc((size_t)(N * K));
        uint16_t* scales = malloc((size_t)(N * (K / t)) * 2);
        int64_t cb, mb, sb;
        REQUIRE(codes && scales);
        REQUIRE(patch_oracle_quantize4(W_hat, N, K, t, codes, scales) == 0);
        REQUIRE(patch_oracle_dequantize4(codes, scales, N, K, t, W_back) == 0);
        REQUIRE(patch_oracle_packed4_sizes(N, K, t, tm, &cb, &mb, &sb) == 0 && cb > 0 && sb == N * (K / t) * 2);
        for (int64_t i = 0; i < N * K; ++i) REQUIRE(codes[i] >= -7 && codes[i] <= 7 && ((W_hat[i] & 0x7FFF) != 0 || codes[i] == 0));
        free(codes); free(scales);
    }
    if (map_kind != 0) {   /* an unmasked matrix under a map with 2:4 tiles must be rejected, without stray writes */
        int dense_enough = 0;
        for (int64_t i = 0; i < N * K && !dense_enough; i += 4)
            dense_enough = (W[i] & 0x7FFF) && (W[i + 1] & 0x7FFF) && (W[i + 2] & 0x7FFF) && tm[(i / K / t) * Tk + (i % K) / t] == 0;
        const int rc = patch_oracle_pack(W, N, K, tm, t, vals, meta, bad);
        REQUIRE(dense_enough ? rc == 3 : (rc == 0 || rc == 3));
    }
    /* hard masks from logits */
    float* pt = malloc((size_t)T * sizeof(float));
    float* p24 = malloc((size_t)(6 * N * K / 4) * sizeof(float));
    REQUIRE(pt && p24);
    for (int64_t i = 0; i < T; ++i) pt[i] = (float)((int)(rnd() % 21) - 10);
    for (int64_t i = 0; i < 6 * N * K / 4; ++i) p24[i] = (float)((int)(rnd() % 9) - 4);
    REQUIRE(patch_oracle_hard_masks(pt, p24, N, K, t, tm, m24) == 0);
    REQUIRE(patch_oracle_apply_mask(W, tm, m24, N, K, t, W_hat) == 0);
    REQUIRE(patch_oracle_packed_sizes(N, K, t, tm, &nv, &nm) == 0);
    free(vals); free(meta);
    vals = malloc((size_t)(nv > 0 ? nv : 1) * 2);
    meta = calloc((size_t)(nm > 0 ? nm : 1), 1);
    REQUIRE(vals && meta && patch_oracle_pack(W_hat, N, K, tm, t, vals, meta, bad) == 0);
    free(W); free(W_hat); free(W_back); free(m24); free(tm); free(X); free(Y); free(vals); free(meta); free(yb); free(pt); free(p24);
    return 0;
}

int main(void) {
    const struct { int64_t N, K; int t; int64_t M; } shapes[] = {
        {8, 8, 8, 3}, {64, 64, 64, 1}, {128, 192, 64, 5}, {256, 128, 128, 17}, {384, 640, 128, 2}, {24, 40, 8, 7}};
    for (unsigned s = 0; s < sizeof shapes / sizeof shapes[0]; ++s)
        for (int kind = 0; kind < 3; ++kind)
            if (one_case(shapes[s].N, shapes[s].K, shapes[s].t, shapes[s].M, kind)) return 1;
    /* argument errors must be refused without touching memory */
    if (patch_oracle_packed_sizes(8, 8, 3, NULL, NULL, NULL) == 0) return 1;
    if (patch_oracle_round_bf16(NULL, 4, NULL) == 0) return 1;
    double edge[6] = {0.0, -0.0, 1e300, -1e300, 1e-300, 3.0e38};
    uint16_t eb[6];
    if (patch_oracle_round_bf16(edge, 6, eb) != 0) return 1;
    printf("sanitize_check ok\n");
    return 0;
}
