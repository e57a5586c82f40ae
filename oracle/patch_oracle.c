/*
 * CPU oracle for the tile-level hybrid dense / 2:4 linear layer of PATCH (arXiv 2509.23410).
 *
 * THIS IS TEST INFRASTRUCTURE, NOT PRODUCT CODE.  It is a plain, slow, obviously-correct statement of
 * what the GPU library must compute.  Only the tests, the smoke check and the benchmark's cpu_baseline
 * leg may build or call it.  It shares no code, table or helper with the HIP path.
 *
 * What it follows (paper passages, restated):
 *   - Hard masks (Algorithm 1, final four lines; Eq. 3 and Eq. 4 with hard instead of soft masks):
 *       M*_tile  is constant over each b1 x b2 tile, 1 = tile stays dense, 0 = tile is 2:4 sparse;
 *       M*       = M*_tile + (1 - M*_tile) (.) M*_2:4 ;   W_hat = W (.) M* .
 *   - 2:4 pattern (Section 1 and Section 2, "Learnable 2:4 Mask"): in every group of four consecutive
 *     elements at most two are kept.  Groups run along d2, the input-feature (reduction) dimension.
 *   - Inference product (Section 4, Appendix A): the linear layer Y = X * W_hat^T with W_hat of shape
 *     d1 x d2 = N x K (out x in features), X of shape M x K.
 *   - Compression (Appendix A): a 2:4 tile is stored as its kept values plus per-value 2-bit positions.
 *     The paper does not print a storage format; the canonical one defined here is this project's:
 *       values : tiles in row-major tile order; a dense tile contributes its t*t elements row-major,
 *                a sparse tile contributes, row by row and group by group along K, the two kept
 *                elements in ascending position;
 *       meta   : sparse tiles only, same order; one nibble per group = pos0 | pos1 << 2 with
 *                pos0 < pos1, two nibbles per byte, the earlier group in the low nibble.
 *     Kept set of a group with fewer than two nonzeros: its nonzero positions plus the lowest-index
 *     zero positions, sorted.  "Nonzero" is decided on the bit pattern: (bits & 0x7FFF) != 0.
 *
 * All bf16 data are passed as uint16_t bit patterns.  The product is evaluated in IEEE double with
 * k ascending, one independent dot product per output element (no blocking, no reordering).
 *
 * Output in bf16 (an option of this project's library; the paper fixes no output type): the exact product,
 * here the double, rounded ONCE to the nearest bf16 value, ties to the even significand
 * (patch_oracle_round_bf16).  The library rounds its fp32 accumulator instead, so the two may differ by one
 * unit in the last place; the tests allow exactly that.
 *
 * 4-bit weight-only storage (Section 5.2, "Quantization", and the table of 4-bit results there: the pruned weights are
 * stored in 4 bits; the table's compression ratios are 16 / (4 (1 - f) + 3 f) for a fraction f of 2:4 tiles, i.e. 4 bits
 * per element of a dense tile and 2 x 4 + 4 bits per group of four of a 2:4 tile, scales not counted).  The paper
 * names no quantizer; the reading taken (patch_oracle_quantize4): symmetric, 15 levels, one scale per row of a tile:
 *     s = bf16( max|w| / 7 )  (float division, rounded to nearest even),   q = clamp( rint( w / s ), -7, 7 )  (float
 *     division, ties to even),   s = 0 (an all-zero row) gives q = 0;
 *     the weight the product then uses is  bf16( q s )  (exact product, one rounding): patch_oracle_dequantize4.
 * A pruned weight is 0 and keeps code 0, so a 2:4 tile stays 2:4; its kept positions are those of the unquantized
 * matrix.  Both decisions (s and q) are taken in float, the precision the library takes them in.
 *
 * Parity pins (see tests/test_oracle_*.py): hand-worked packed example, closed-form sizes, round trip,
 * naive dense GEMM (bit-equal), library dense GEMM, direct 2:4 GEMM on (values, positions), exact
 * rational brute force over all six patterns, linearity and tile-map invariance.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define PO_OK 0
#define PO_ERR_ARG 1
#define PO_ERR_SHAPE 2
#define PO_ERR_NOT_24 3
#define PO_ERR_ALLOC 4
#define PO_ERR_META 5

static double bf16_to_double(uint16_t h) {
    uint32_t u = (uint32_t)h << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f; /* exact */
}

static int is_nonzero(uint16_t h) { return (h & 0x7FFFu) != 0; }

static int check_shape(int64_t N, int64_t K, int t) {
    if (N <= 0 || K <= 0 || t <= 0) return PO_ERR_ARG;
    if (t % 4 != 0) return PO_ERR_SHAPE;
    if (N % t != 0 || K % t != 0) return PO_ERR_SHAPE;
    return PO_OK;
}

/* W_hat = W (.) M*, M* = M_tile + (1 - M_tile) (.) M_24  (Algorithm 1, last three lines; Eq. 4).
 * tile_map: (N/t) x (K/t), 1 = dense tile.  mask24: N x K bytes, 1 = keep.  Pruned entries become +0. */
int patch_oracle_apply_mask(const uint16_t* W, const uint8_t* tile_map, const uint8_t* mask24,
                            int64_t N, int64_t K, int t, uint16_t* W_hat) {
    int rc = check_shape(N, K, t);
    if (rc) return rc;
    int64_t Tk = K / t;
    for (int64_t n = 0; n < N; ++n)
        for (int64_t k = 0; k < K; ++k) {
            int m_tile = tile_map[(n / t) * Tk + (k / t)] ? 1 : 0;
            int m_24 = mask24[n * K + k] ? 1 : 0;
            int m_star = m_tile + (1 - m_tile) * m_24;
            W_hat[n * K + k] = m_star ? W[n * K + k] : (uint16_t)0;
        }
    return PO_OK;
}

/* Hard masks from the learned logits (Algorithm 1, first two lines after the training loop; Section 3,
 * "Inference"; Section 2, "Learnable 2:4 Mask"):
 *   tile_map[i] = 1[P_tile[i] > 0]            (a positive logit keeps the tile dense; the sparse class is the
 *                                              concatenated zero logit, so 0 and NaN mean "2:4")
 *   mask24      = for every group of four consecutive elements (row-major, along K) the candidate pattern with
 *                 the largest of its six logits.  P_24 is 6 x (N K / 4), row c = logits of candidate c for all
 *                 groups; the candidates are the rows of S: all 4-vectors with two ones, here in lexicographic
 *                 order of the kept positions (0,1) (0,2) (0,3) (1,2) (1,3) (2,3).  Ties: the first candidate.
 */
int patch_oracle_hard_masks(const float* P_tile, const float* P_24, int64_t N, int64_t K, int t,
                            uint8_t* tile_map, uint8_t* mask24) {
    static const uint8_t S[6][4] = {{1, 1, 0, 0}, {1, 0, 1, 0}, {1, 0, 0, 1}, {0, 1, 1, 0}, {0, 1, 0, 1}, {0, 0, 1, 1}};
    int rc = check_shape(N, K, t);
    if (rc) return rc;
    int64_t T = (N / t) * (K / t), G = N * K / 4;
    for (int64_t i = 0; i < T; ++i) tile_map[i] = (P_tile[i] > 0.0f) ? 1 : 0;
    for (int64_t g = 0; g < G; ++g) {
        int best = 0;
        for (int c = 1; c < 6; ++c)
            if (P_24[c * G + g] > P_24[best * G + g]) best = c;
        for (int j = 0; j < 4; ++j) mask24[4 * g + j] = S[best][j];
    }
    return PO_OK;
}

/* Element counts of the canonical arrays: values (uint16) and meta (bytes). */
int patch_oracle_packed_sizes(int64_t N, int64_t K, int t, const uint8_t* tile_map,
                              int64_t* n_vals, int64_t* n_meta) {
    int rc = check_shape(N, K, t);
    if (rc) return rc;
    if (t % 8 != 0) return PO_ERR_SHAPE; /* a tile row must hold an even number of groups (whole meta bytes) */
    int64_t T = (N / t) * (K / t), vals = 0, meta = 0;
    for (int64_t i = 0; i < T; ++i) {
        if (tile_map[i]) vals += (int64_t)t * t;
        else { vals += (int64_t)t * t / 2; meta += (int64_t)t * t / 8; }
    }
    *n_vals = vals;
    *n_meta = meta;
    return PO_OK;
}

/* Compress.  Returns PO_ERR_NOT_24 (and the row / column of the offending group in bad_nk) if a group of
 * a 2:4 tile holds more than two nonzeros; vals/meta contents are then unspecified. */
int patch_oracle_pack(const uint16_t* W_hat, int64_t N, int64_t K, const uint8_t* tile_map, int t,
                      uint16_t* vals, uint8_t* meta, int64_t* bad_nk) {
    int64_t nv, nm;
    int rc = patch_oracle_packed_sizes(N, K, t, tile_map, &nv, &nm);
    if (rc) return rc;
    int64_t Tn = N / t, Tk = K / t, vi = 0, nib = 0;
    if (nm) memset(meta, 0, (size_t)nm);
    for (int64_t tn = 0; tn < Tn; ++tn)
        for (int64_t tk = 0; tk < Tk; ++tk) {
            int dense = tile_map[tn * Tk + tk] != 0;
            for (int r = 0; r < t; ++r) {
                const uint16_t* row = W_hat + (tn * t + r) * K + tk * t;
                if (dense) {
                    for (int c = 0; c < t; ++c) vals[vi++] = row[c];
                    continue;
                }
                for (int g = 0; g < t / 4; ++g) {
                    const uint16_t* grp = row + 4 * g;
                    int keep[4] = {0, 0, 0, 0}, nnz = 0;
                    for (int p = 0; p < 4; ++p)
                        if (is_nonzero(grp[p])) { keep[p] = 1; ++nnz; }
                    if (nnz > 2) {
                        if (bad_nk) { bad_nk[0] = tn * t + r; bad_nk[1] = tk * t + 4 * g; }
                        return PO_ERR_NOT_24;
                    }
                    for (int p = 0; p < 4 && nnz < 2; ++p) /* pad with lowest-index zero positions */
                        if (!keep[p]) { keep[p] = 1; ++nnz; }
                    int pos[2], j = 0;
                    for (int p = 0; p < 4; ++p)
                        if (keep[p]) pos[j++] = p;
                    vals[vi++] = grp[pos[0]];
                    vals[vi++] = grp[pos[1]];
                    uint8_t nibble = (uint8_t)(pos[0] | (pos[1] << 2));
                    meta[nib >> 1] |= (uint8_t)(nibble << (4 * (nib & 1)));
                    ++nib;
                }
            }
        }
    return PO_OK;
}

/* Decompress the canonical form into a row-major N x K matrix.  Dropped positions become +0.
 * Returns PO_ERR_META if a nibble does not satisfy pos0 < pos1. */
int patch_oracle_unpack(const uint16_t* vals, const uint8_t* meta, int64_t N, int64_t K,
                        const uint8_t* tile_map, int t, uint16_t* W_out) {
    int64_t nv, nm;
    int rc = patch_oracle_packed_sizes(N, K, t, tile_map, &nv, &nm);
    if (rc) return rc;
    int64_t Tn = N / t, Tk = K / t, vi = 0, nib = 0;
    for (int64_t tn = 0; tn < Tn; ++tn)
        for (int64_t tk = 0; tk < Tk; ++tk) {
            int dense = tile_map[tn * Tk + tk] != 0;
            for (int r = 0; r < t; ++r) {
                uint16_t* row = W_out + (tn * t + r) * K + tk * t;
                if (dense) {
                    for (int c = 0; c < t; ++c) row[c] = vals[vi++];
                    continue;
                }
                for (int g = 0; g < t / 4; ++g) {
                    uint8_t nibble = (uint8_t)((meta[nib >> 1] >> (4 * (nib & 1))) & 0xF);
                    ++nib;
                    int p0 = nibble & 3, p1 = (nibble >> 2) & 3;
                    if (p0 >= p1) return PO_ERR_META;
                    row[4 * g + 0] = row[4 * g + 1] = row[4 * g + 2] = row[4 * g + 3] = 0;
                    row[4 * g + p0] = vals[vi++];
                    row[4 * g + p1] = vals[vi++];
                }
            }
        }
    return PO_OK;
}

/* Y = X * W_hat^T in double, from the compressed form: decompress first, verify the 2:4 property of
 * every group of every sparse tile, then one dot product per output, k ascending.
 * X: M x K bf16 bits, Y: M x N doubles.  OpenMP splits the independent outputs only. */
int patch_oracle_gemm(const uint16_t* X, int64_t M, const uint16_t* vals, const uint8_t* meta,
                      int64_t N, int64_t K, const uint8_t* tile_map, int t, double* Y) {
    if (M <= 0) return PO_ERR_ARG;
    uint16_t* W_hat = (uint16_t*)malloc((size_t)N * (size_t)K * sizeof(uint16_t));
    if (!W_hat) return PO_ERR_ALLOC;
    int rc = patch_oracle_unpack(vals, meta, N, K, tile_map, t, W_hat);
    if (rc) { free(W_hat); return rc; }
    int64_t Tk = K / t;
    for (int64_t n = 0; n < N && !rc; ++n)
        for (int64_t g = 0; g < K / 4; ++g) {
            if (tile_map[(n / t) * Tk + (4 * g) / t]) continue;
            int nnz = 0;
            for (int p = 0; p < 4; ++p) nnz += is_nonzero(W_hat[n * K + 4 * g + p]);
            if (nnz > 2) { rc = PO_ERR_NOT_24; break; }
        }
    if (rc) { free(W_hat); return rc; }
    double* Wd = (double*)malloc((size_t)N * (size_t)K * sizeof(double));
    double* Xd = (double*)malloc((size_t)M * (size_t)K * sizeof(double));
    if (!Wd || !Xd) { free(W_hat); free(Wd); free(Xd); return PO_ERR_ALLOC; }
    for (int64_t i = 0; i < N * K; ++i) Wd[i] = bf16_to_double(W_hat[i]);
    for (int64_t i = 0; i < M * K; ++i) Xd[i] = bf16_to_double(X[i]);
    free(W_hat);
#pragma omp parallel for collapse(2) schedule(static)
    for (int64_t m = 0; m < M; ++m)
        for (int64_t n = 0; n < N; ++n) {
            double acc = 0.0;
            for (int64_t k = 0; k < K; ++k) acc += Xd[m * K + k] * Wd[n * K + k];
            Y[m * N + n] = acc;
        }
    free(Wd);
    free(Xd);
    return PO_OK;
}

/* Same product for a list of (m, n) output coordinates only (for spot checks at sizes where the full
 * product is too slow on a CPU).  W_hat_dense: an already decompressed N x K matrix. */
int patch_oracle_gemm_points(const uint16_t* X, int64_t M, const uint16_t* W_hat_dense, int64_t N, int64_t K,
                             const int64_t* mn, int64_t n_points, double* out) {
    for (int64_t i = 0; i < n_points; ++i) {
        int64_t m = mn[2 * i], n = mn[2 * i + 1];
        if (m < 0 || m >= M || n < 0 || n >= N) return PO_ERR_ARG;
    }
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n_points; ++i) {
        int64_t m = mn[2 * i], n = mn[2 * i + 1];
        double acc = 0.0;
        for (int64_t k = 0; k < K; ++k) acc += bf16_to_double(X[m * K + k]) * bf16_to_double(W_hat_dense[n * K + k]);
        out[i] = acc;
    }
    return PO_OK;
}

/* y[i] (double) -> nearest bf16 value (8 significand bits, exponent range of binary32), ties to even, as a
 * bit pattern.  Written on the value, with frexp / nearbyint in the default rounding mode, not on bit patterns:
 *   |y| = m 2^e, 0.5 <= m < 1  ->  quantum q = 2^(e - 8) (2^-133 below the normal range), result = rint(|y| / q) q.
 * Overflow past the largest finite bf16 gives infinity; NaN gives a quiet NaN. */
#include <math.h>
int patch_oracle_round_bf16(const double* y, int64_t n, uint16_t* out) {
    if (!y || !out || n < 0) return PO_ERR_ARG;
    for (int64_t i = 0; i < n; ++i) {
        const double v = y[i];
        uint16_t sign = signbit(v) ? 0x8000u : 0u;
        if (isnan(v)) { out[i] = (uint16_t)(sign | 0x7FC0u); continue; }
        const double a = fabs(v);
        if (isinf(a)) { out[i] = (uint16_t)(sign | 0x7F80u); continue; }
        if (a == 0.0) { out[i] = sign; continue; }
        int e;
        (void)frexp(a, &e);                 /* a = m 2^e with 0.5 <= m < 1: the leading bit has weight 2^(e-1) */
        int qe = e - 8;                     /* 8 significand bits: the last one has weight 2^(e-8) */
        if (qe < -133) qe = -133;           /* subnormal range: fixed quantum 2^-133 */
        const double r = nearbyint(ldexp(a, -qe));   /* an integer <= 256, ties to even */
        const double rounded = ldexp(r, qe);
        if (rounded > 3.3895313892515355e38) { out[i] = (uint16_t)(sign | 0x7F80u); continue; }  /* > max finite bf16 */
        const float f = (float)rounded;     /* exact: 8 significant bits within the binary32 range */
        uint32_t u;
        memcpy(&u, &f, sizeof u);
        out[i] = (uint16_t)(sign | (uint16_t)(u >> 16));
    }
    return PO_OK;
}

static uint16_t float_to_bf16_rne(float f) {
    uint32_t u;
    memcpy(&u, &f, sizeof u);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (uint16_t)((u >> 16) | 0x40u);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

/* codes[n][k] in [-7, 7] (0 where W_hat is zero), scales[n][k / t] as bf16 bit patterns: see the header. */
int patch_oracle_quantize4(const uint16_t* W_hat, int64_t N, int64_t K, int t, int8_t* codes, uint16_t* scales) {
    if (!W_hat || !codes || !scales) return PO_ERR_ARG;
    int rc = check_shape(N, K, t);
    if (rc) return rc;
    const int64_t Tk = K / t;
    for (int64_t n = 0; n < N; ++n)
        for (int64_t g = 0; g < Tk; ++g) {
            const uint16_t* w = W_hat + n * K + g * t;
            float amax = 0.0f;
            for (int k = 0; k < t; ++k) {
                const float a = fabsf((float)bf16_to_double(w[k]));
                if (a > amax) amax = a;
            }
            const uint16_t sb = float_to_bf16_rne(amax / 7.0f);
            const float s = (float)bf16_to_double(sb);
            scales[n * Tk + g] = sb;
            for (int k = 0; k < t; ++k) {
                int q = 0;
                if (s > 0.0f) {
                    float r = rintf((float)bf16_to_double(w[k]) / s);
                    if (r > 7.0f) r = 7.0f;
                    if (r < -7.0f) r = -7.0f;
                    q = (int)r;
                }
                codes[n * K + g * t + k] = (int8_t)q;
            }
        }
    return PO_OK;
}

/* W_deq[n][k] = bf16( codes[n][k] * scales[n][k / t] ), the exact product rounded once. */
int patch_oracle_dequantize4(const int8_t* codes, const uint16_t* scales, int64_t N, int64_t K, int t, uint16_t* W_deq) {
    if (!codes || !scales || !W_deq) return PO_ERR_ARG;
    int rc = check_shape(N, K, t);
    if (rc) return rc;
    const int64_t Tk = K / t;
    for (int64_t n = 0; n < N; ++n)
        for (int64_t k = 0; k < K; ++k) {
            const double v = (double)codes[n * K + k] * bf16_to_double(scales[n * Tk + k / t]);
            rc = patch_oracle_round_bf16(&v, 1, &W_deq[n * K + k]);
            if (rc) return rc;
        }
    return PO_OK;
}

/* Bytes of the 4-bit storage: codes (4 bits per element of a dense tile, per kept element of a 2:4 tile), positions
 * (2 bits per kept element) and scales (one bf16 per row of a tile). */
int patch_oracle_packed4_sizes(int64_t N, int64_t K, int t, const uint8_t* tile_map, int64_t* code_bytes, int64_t* meta_bytes,
                               int64_t* scale_bytes) {
    int rc = check_shape(N, K, t);
    if (rc) return rc;
    if (!tile_map || !code_bytes || !meta_bytes || !scale_bytes) return PO_ERR_ARG;
    int64_t T = (N / t) * (K / t), c = 0, m = 0;
    for (int64_t i = 0; i < T; ++i) {
        if (tile_map[i]) c += (int64_t)t * t / 2;
        else { c += (int64_t)t * t / 4; m += (int64_t)t * t / 8; }
    }
    *code_bytes = c;
    *meta_bytes = m;
    *scale_bytes = T * t * 2;
    return PO_OK;
}

int patch_oracle_num_threads(void) {
    int n = 1;
#ifdef _OPENMP
#pragma omp parallel
    {
#pragma omp single
        n = omp_get_num_threads();
    }
#endif
    return n;
}
