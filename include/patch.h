/*
 * patch.h -- C ABI of the MI355X (gfx950) library for the inference linear layer of PATCH
 * (arXiv 2509.23410): Y = X * W_hat^T where W_hat (N x K = d1 x d2, out x in features) is cut into
 * tile x tile blocks and every block is either dense or 2:4 sparse along K.
 *
 * Conventions
 *   - All matrices are row-major.  bf16 = IEEE bfloat16 (upper 16 bits of binary32).
 *   - "DEVICE" pointers are HIP device memory of the current device; "HOST" pointers are ordinary host
 *     memory.  The caller owns every buffer it passes in; the library owns a patch_packed until
 *     patch_free.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *   - No exception crosses this boundary: every failure is a patch_status.  Argument and shape errors
 *     are detected on the host before any device work.
 *   - tile_map is HOST memory, row-major (N/tile) x (K/tile) bytes: nonzero = the tile is dense,
 *     0 = the tile is 2:4 sparse.  This is the hard tile mask 1[P_tile > 0] of Algorithm 1 (first
 *     line after the training loop); a positive logit means "dense" (Section 3, "Inference").
 *   - 2:4: in every group of four consecutive elements along K (the input-feature dimension) at most
 *     two are nonzero (Section 1; Section 2, "Learnable 2:4 Mask").  An element is "zero" when its
 *     bit pattern & 0x7FFF is 0.
 */
#ifndef PATCH_H_
#define PATCH_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct patch_packed patch_packed; /* opaque: compressed weight + per-tile tables */

typedef enum {
    PATCH_OK = 0,
    PATCH_ERR_ARG = 1,    /* null pointer, non-positive size, unknown option                         */
    PATCH_ERR_SHAPE = 2,  /* tile not in {64, 128}, or N / K not a multiple of tile                  */
    PATCH_ERR_NOT_24 = 3, /* a group of four in a tile flagged 2:4 holds more than two nonzeros      */
    PATCH_ERR_ALLOC = 4,  /* device or host allocation failed                                        */
    PATCH_ERR_HIP = 5,    /* a HIP runtime call failed (patch_last_hip_error gives the code)         */
    PATCH_ERR_SIZE = 6,   /* a caller-provided host buffer is too small                              */
    PATCH_ERR_NOT_FOUND = 7 /* patch_tune_table_get: no schedule stored for this key                       */
} patch_status;

/* Which kernel family patch_gemm_ex uses.  DECODE handles M in passes of up to 64 rows (the weight is streamed
 * once per pass: 16-feature strips per workgroup for few rows, 64 features per wavefront for more rows where that
 * fills the chip), PREFILL in blocks of 256 rows (128 where an estimate of both says so: few rows, or a weight of
 * few feature blocks that would otherwise need a deep K split).  AUTO (measured crossovers): decode up to M = 64 (with a
 * workspace, a single weight of at least 10240 features goes to prefill from M = 33); beyond, with a
 * workspace for at least two slices (see patch_gemm_opts) prefill, whose K split then fills the chip; without one
 * the cheaper of repeated passes and one unsplit prefill launch by an estimate from the launch geometry (passes up to
 * M = 192 at 4096 x 4096, up to M = 128 from 5120 features, further for long-K weights of few features). */
typedef enum { PATCH_PATH_AUTO = 0, PATCH_PATH_DECODE = 1, PATCH_PATH_PREFILL = 2 } patch_path;

/* Schedule options (the knobs the paper's Appendix A leaves to an autotuner: tile shape and
 * schedule, e.g. split-K).  A zero field means "library default". */
typedef struct {
    int path;    /* patch_path                                                                      */
    int split_k; /* decode: K slices (one wavefront each) per workgroup whose fp32 partials are     */
                 /* reduced in slice order; rounded down to a power of two in 1..16, 0 = auto.       */
                 /* prefill: K slices per output tile, one workgroup each, whose partial             */
                 /* products go to `workspace` and are summed in slice order by a second launch;     */
                 /* 0 = auto (1 unless the tile grid would leave a third of the chip idle; with a    */
                 /* workspace a part-filled last round of at most half the chip is split on its own - */
                 /* tile 128 only),                                                                   */
                 /* 1 = no split.  Never more slices than the workspace holds: without one, no split. */
    int variant; /* kernel variant within the path, 0 = default.  Prefill: 1 = simple 128 x 128 kernel, */
                 /* 2 = 256 x 256 LDS-staged kernel (tile 128 beyond the limits of 3), 3 = 256 x 256 weights-in- */
                 /* registers kernel (the default for tile 128 where K <= 32768 and M K 2 < 4 GB), 4 = the  */
                 /* LDS-staged kernel with blocks of 256 features x 128 rows, 5 = blocks of 128 rows with  */
                 /* the weights loaded straight into registers, 6 = the same with 256 rows (tile 64 only:  */
                 /* its 256-row default).                                                                  */
                 /* Blocks of 128 rows (5) are the default, with no split requested, where estimated       */
                 /* faster (up to a few hundred rows).  Decode: 2 / 3 = 8 / 4                              */
                 /* K-steps per wavefront of the 16-feature-strip kernel; 4 = the kernel with 64         */
                 /* features per wavefront (its split_k = K chunks over `workspace`, 0 = auto; the       */
                 /* default for passes of 17 .. 64 rows when a workspace allows chunks or N >= 4608, and */
                 /* for 12 .. 16 rows when N >= 10240); 5 / 6 = the strip kernel with two X loads per    */
                 /* step / with one X load for several steps (up to 8 rows; the default picks 6 where at */
                 /* least a quarter of the tiles are 2:4).  A variant that does not apply falls back to  */
                 /* the default.                                                                         */
    void* workspace;        /* DEVICE, 16-byte aligned, caller-owned scratch for launches that split K   */
                            /* over workgroups (prefill; decode passes of 17 .. 64 rows), or NULL.  The  */
                            /* library never allocates in a product call.  Launches that may run         */
                            /* concurrently need distinct workspaces.                                    */
    size_t workspace_bytes; /* its size; patch_gemm_workspace_bytes says what a launch would use         */
    int y_bf16;             /* nonzero: Y (every Y of patch_gemm_many) is M x N bf16 instead of fp32: the fp32  */
                            /* accumulator - after the sum over K slices, where K is split - rounded to nearest, */
                            /* ties to even.  The paper fixes no output type; half-precision inference feeds the */
                            /* product to the next layer in 16 bits.  Same alignment (16 bytes) as the fp32 Y.   */
} patch_gemm_opts;

/*
 * Hard masks from the learned logits (Algorithm 1, the two lines after the training loop; Section 3, "Inference";
 * Section 2, "Learnable 2:4 Mask"):
 *   tile_map[i] = 1[P_tile[i] > 0]   a positive logit keeps the tile dense; 0 and NaN give the 2:4 class
 *   mask24      for every group of four consecutive elements (row-major, along K) the candidate pattern with the
 *               largest of its six logits; ties: the first.  Candidates = the six 4-vectors with two ones, in
 *               lexicographic order of the kept positions (0,1) (0,2) (0,3) (1,2) (1,3) (2,3).
 *   P_tile   HOST, (N/tile) x (K/tile) fp32, row-major        tile_map  HOST out, same shape, bytes (for patch_pack)
 *   P_24     DEVICE, 6 x (N K / 4) fp32, row c = logits of candidate c for all groups, 4-byte aligned
 *   mask24   DEVICE out, N x K bytes, 1 = keep, 8-byte aligned (the input of patch_apply_mask, which reads it in
 *            8-byte pieces)
 * tile_map is complete on return; mask24 is written asynchronously on `stream`.  Errors: PATCH_ERR_ARG,
 * PATCH_ERR_SHAPE (as patch_apply_mask), PATCH_ERR_HIP.
 */
patch_status patch_hard_masks(const float* P_tile, const void* P_24, int64_t N, int64_t K, int tile, uint8_t* tile_map,
                              void* mask24, void* stream);

/*
 * Merge of the hard masks and pruning of the weights (Algorithm 1, last three lines; Eq. 4 with hard
 * masks):  M* = M_tile + (1 - M_tile) (.) M_24,  W_hat = W (.) M*.
 *   W      DEVICE, N x K bf16, 16-byte aligned
 *   mask24 DEVICE, N x K bytes, nonzero = keep (used only inside tiles whose tile_map entry is 0), 8-byte aligned
 *   W_hat  DEVICE, N x K bf16, 16-byte aligned; either W itself (in place) or a buffer that does not overlap W;
 *          pruned entries are written as +0
 * Misaligned pointers: PATCH_ERR_ARG.
 * Synchronous: uploads the tile map, runs on `stream` and waits for it (a one-off conversion step).
 */
patch_status patch_apply_mask(const void* W, const void* mask24, const uint8_t* tile_map, int64_t N,
                              int64_t K, int tile, void* W_hat, void* stream);

/*
 * Compression (Appendix A: the compressed values and the position metadata depend on the tile size, which is
 * therefore fixed at pack time): 2:4 tiles become kept values + 2-bit positions laid out for the gfx950 sparse
 * matrix instructions; dense tiles are re-ordered into matrix-instruction operand order.
 *   W_hat  DEVICE, N x K bf16, already pruned.
 *   tile   64 or 128; N and K must be multiples of it.
 *   *out   receives a new patch_packed on success, untouched otherwise.
 * Kept positions of a group with fewer than two nonzeros: its nonzeros plus the lowest-index zeros.
 * Synchronises `stream` once (to learn whether the 2:4 check failed).  Returns PATCH_ERR_NOT_24 if it did.
 */
patch_status patch_pack(const void* W_hat, int64_t N, int64_t K, const uint8_t* tile_map, int tile,
                        void* stream, patch_packed** out);

/*
 * The product (Section 4; Appendix A decode input BS x K and prefill input BS*SL x K):
 *   Y[m, n] = sum_k X[m, k] * W_hat[n, k],   bf16 x bf16 products accumulated in fp32.
 *   X  DEVICE, M x K bf16;  Y  DEVICE, M x N fp32;  M >= 0 arbitrary (M = 0: PATCH_OK, nothing is launched;
 *   the pointers must still be non-null and aligned).
 * Asynchronous on `stream`; allocates nothing and never synchronises.  A patch_packed is read-only for
 * patch_gemm, so concurrent calls on different streams are allowed as long as their Y buffers differ.
 * Results are bit-reproducible from call to call (fixed reduction order, no atomics).
 */
patch_status patch_gemm(const void* X, int64_t M, const patch_packed* P, void* Y, void* stream);
patch_status patch_gemm_ex(const void* X, int64_t M, const patch_packed* P, void* Y, void* stream,
                           const patch_gemm_opts* opts);

/*
 * The same product for callers that cannot allocate device memory or pass a workspace (code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc): patch_gemm_ex with the automatic schedule and,
 * in place of patch_gemm_opts.workspace, a scratch array of PATCH_STATIC_SCRATCH_BYTES that is part of the
 * library's device image (one copy per GPU, held until the process ends).  Calls no hipMalloc / hipFree and no
 * allocating routine; the first call on a device looks the array's address up (hipGetSymbolAddress).
 *   X, M, P, Y, stream   as for patch_gemm
 * The schedule is the one patch_gemm_ex picks when given a workspace of that size, so results are bit-equal to
 * patch_gemm_ex with such a caller workspace.  Returns PATCH_ERR_SIZE - nothing is launched - when that schedule
 * would want more scratch than the array holds (patch_gemm_workspace_bytes(M, P, NULL) > PATCH_STATIC_SCRATCH_BYTES;
 * e.g. split launches of large M x N); use patch_gemm_ex with a workspace of your own then.  Every partial sum the
 * kernels read from the scratch is written by the same call first, so nothing needs clearing between calls, but
 * all calls on one GPU share the one array: calls that overlap in time on the same GPU (different streams or
 * threads) race on it.  Errors otherwise as patch_gemm_ex.
 */
#define PATCH_STATIC_SCRATCH_BYTES ((size_t)32 << 20)
patch_status patch_gemm_static(const void* X, int64_t M, const patch_packed* P, void* Y, void* stream);

/*
 * Schedule autotuner (Appendix A leaves the execution tile and the schedule - e.g. split-K - to an autotuner that is
 * run per layer and input shape, on the decode input first).  patch_tune_all times every candidate schedule of
 * patch_gemm_ex for this M and P on the device, on real operands; patch_tune returns the fastest.  Candidates:
 *   decode path (M <= 256): 16-feature-strip kernel with 8 or 4 K-steps per wavefront (variants 2 / 3) and 2 .. 16
 *     wavefronts per workgroup (split_k: the wavefronts-per-compute-unit dimension), up to 8 rows both ways of loading
 *     X (variants 5 / 6), the 64-features-per-wavefront kernel (variant 4) unsplit and with K chunks over the workspace;
 *   prefill path, tile 128: the execution tiles 256 x 256 with one wavefront per SIMD (default), 256 x 256 with two
 *     (variant 2) and the small 128 x 128 tile (variant 1; Appendix O reports that small execution tiles under-use
 *     the matrix units - it is timed so that the report shows it), and the K-split counts the workspace allows;
 *   prefill path, tile 64: 256 x 256 with the weights in registers (default), LDS-staged (variant 2), the small
 *     128 x 128 tile, K-split counts;
 *   prefill path, M <= 4096: blocks of 256 features x 128 rows (variants 4 and 5), unsplit and split.
 *   X, Y       as for patch_gemm (Y is overwritten several times; after patch_tune it holds the product)
 *   workspace  DEVICE scratch for split launches or NULL (then only unsplit candidates), caller-owned
 *   reps       timed launches per candidate after two warm-up launches (HIP events on `stream`); >= 1
 *   results    HOST array of `cap` entries; receives min(*count, cap) candidates in candidate order, each with its
 *              average time per launch; *count = number of candidates timed
 *   best       OUT: the options to pass to patch_gemm_ex / patch_gemm_many (workspace fields included: NULL when the
 *              winner was timed without one - then run it without one)
 *   best_us    OUT, may be NULL: its average time per launch in microseconds
 * Not hot-path calls: they create and destroy two HIP events and synchronise `stream` after every candidate.
 * Errors as patch_gemm_ex, plus PATCH_ERR_ARG for reps < 1 or a NULL `best` / `results` / `count`.
 */
typedef struct {
    patch_gemm_opts opts;
    float us;
} patch_tune_result;
patch_status patch_tune_all(const void* X, int64_t M, const patch_packed* P, void* Y, void* workspace, size_t workspace_bytes,
                            void* stream, int reps, patch_tune_result* results, size_t cap, size_t* count);
patch_status patch_tune(const void* X, int64_t M, const patch_packed* P, void* Y, void* workspace, size_t workspace_bytes,
                        void* stream, int reps, patch_gemm_opts* best, float* best_us);

/*
 * Table of tuned schedules (host memory; Appendix A: the tuner's choice is kept per layer shape and input shape and
 * reused).  Key = (M bucket, N, K, tile, number of 2:4 tiles); the M bucket is the smallest power of two >= M
 * (patch_tune_bucket).  A stored schedule remembers whether it was timed with a workspace, not the pointer.
 *   patch_tune_table_put  stores / replaces; opts->workspace != NULL marks "uses a workspace"
 *   patch_tune_table_get  PATCH_OK and *out filled (its workspace fields = the arguments when the schedule uses a
 *                         workspace, else NULL / 0); PATCH_ERR_NOT_FOUND if no entry, or if the entry uses a
 *                         workspace and none is given
 *   patch_tune_layer      the paper's order for one layer: tunes the decode input first, then the prefill input, and
 *                         stores both.  What the decode choice pins for prefill in the paper - the mask tile and with
 *                         it the compressed layout - is fixed when P is packed here, and both inputs run from the one
 *                         P; the kernels' execution tiles are independent of the layout, so the second search is not
 *                         narrowed by the first.  Y must hold max(M_decode, M_prefill) x N floats.
 *   patch_tune_table_export  the entries as plain records, for the caller to keep between processes (a tuned table
 *                         holds for the GPU model it was timed on): *count = entries in the table; entries == NULL
 *                         with cap 0 only asks for that number; PATCH_ERR_SIZE if cap is too small
 *   patch_tune_table_import  stores / replaces `count` records; every record is checked first (shape, bucket a power
 *                         of two, path, split, variant) and nothing is stored if one is bad (PATCH_ERR_ARG)
 * The table is internally locked; entries are plain values.  Errors: PATCH_ERR_ARG, PATCH_ERR_ALLOC, and those of
 * patch_tune.
 */
typedef struct patch_tune_table patch_tune_table;
typedef struct {
    int64_t m_bucket, N, K, n_sparse_tiles;
    int tile;
    int path, split_k, variant, y_bf16;
    int uses_workspace;   /* the schedule was timed with a workspace and needs one */
} patch_tune_entry;
int64_t patch_tune_bucket(int64_t M);
patch_status patch_tune_table_create(patch_tune_table** out);
void patch_tune_table_destroy(patch_tune_table* t);
size_t patch_tune_table_size(const patch_tune_table* t);
patch_status patch_tune_table_put(patch_tune_table* t, int64_t M, int64_t N, int64_t K, int tile, int64_t n_sparse_tiles,
                                  const patch_gemm_opts* opts);
patch_status patch_tune_table_get(const patch_tune_table* t, int64_t M, int64_t N, int64_t K, int tile, int64_t n_sparse_tiles,
                                  void* workspace, size_t workspace_bytes, patch_gemm_opts* out);
patch_status patch_tune_table_export(const patch_tune_table* t, patch_tune_entry* entries, size_t cap, size_t* count);
patch_status patch_tune_table_import(patch_tune_table* t, const patch_tune_entry* entries, size_t count);
patch_status patch_tune_layer(patch_tune_table* t, const void* X_decode, int64_t M_decode, const void* X_prefill, int64_t M_prefill,
                              const patch_packed* P, void* Y, void* workspace, size_t workspace_bytes, void* stream, int reps);

/* Bytes of patch_gemm_opts.workspace the product with these M, P and opts (path, split_k; NULL = defaults) would
 * use if it were given enough: slices x M x N x 4 for a split prefill launch, slices x tiles x 256 KB when only the
 * part-filled last round of a prefill launch is split, chunks x min(M, 64) x N x 4 for decode passes of 17 .. 64
 * rows, else 0. */
size_t patch_gemm_workspace_bytes(int64_t M, const patch_packed* P, const patch_gemm_opts* opts);

/*
 * The same product for several weights that share one input: Y[i] = X * W_hat[i]^T, i < count (the q / k / v
 * projections of an attention block, the gate / up projections of an MLP; Appendix A times the layer's products
 * for one decode input and one prefill input).  On the decode path all weights run in ONE launch per pass of up
 * to 64 rows of X, which amortises launch and ramp-up over all their bytes; on the prefill path (tile 128) one launch covers the
 * output tiles of all weights - one tail instead of one per weight - unless they are so few that splitting K pays
 * (a workspace is given, split_k = 0), or opts ask for a kernel variant or split: then one launch per weight.
 *   P      HOST array of count handles; all with the same K and the same tile, N may differ
 *   Y      HOST array of count DEVICE pointers, Y[i] is M x N[i] fp32 row-major, 16-byte aligned, distinct
 *   count  1 .. PATCH_MAX_MANY
 *   opts   as for patch_gemm_ex, NULL = defaults
 * Errors: PATCH_ERR_ARG (null, count out of range, misaligned), PATCH_ERR_SHAPE (K or tile differ).  Same
 * asynchrony, ownership and reproducibility as patch_gemm; both arrays are read before the call returns.
 */
#define PATCH_MAX_MANY 8
patch_status patch_gemm_many(const void* X, int64_t M, const patch_packed* const* P, void* const* Y, int count,
                             void* stream, const patch_gemm_opts* opts);

/* Decompression back to a row-major N x K bf16 matrix (DEVICE, 16-byte aligned).  Dropped positions become +0.
 * This project's hook for round-trip tests (the inverse of the Appendix A compression step); the paper defines no
 * such call. */
patch_status patch_unpack(const patch_packed* P, void* W_out, void* stream);

/*
 * Test hook (this project's; no passage of the paper): the compressed matrix in the layout-independent canonical order.
 *   vals (HOST, uint16): tiles in row-major tile order; dense tile = its tile*tile elements row-major;
 *                        2:4 tile = per row, per group along K, the two kept elements, ascending position.
 *   meta (HOST, bytes) : 2:4 tiles only, same order; per group one nibble pos0 | pos1 << 2 (pos0 < pos1),
 *                        two nibbles per byte, earlier group in the low nibble.
 * Sizes come from patch_canonical_sizes; smaller buffers give PATCH_ERR_SIZE.  Synchronous.
 */
patch_status patch_canonical_sizes(const patch_packed* P, size_t* vals_bytes, size_t* meta_bytes);
patch_status patch_export_canonical(const patch_packed* P, void* vals, size_t vals_bytes, void* meta,
                                    size_t meta_bytes);

/* Getters, lifetime and diagnostics below are this project's (no passage of the paper).
 * Compressed weight bytes (values + positions; tables excluded): 2NK (1 - 7/16 * n_sparse / T). */
size_t patch_packed_bytes(const patch_packed* P);
/* Bytes of the per-tile tables the kernels read in addition (offset / type table, row order of the prefill launch). */
size_t patch_table_bytes(const patch_packed* P);
patch_status patch_packed_dims(const patch_packed* P, int64_t* N, int64_t* K, int* tile,
                               int64_t* n_sparse_tiles);
/* HOST copy of the tile map held by P (N/tile * K/tile bytes). */
patch_status patch_packed_tile_map(const patch_packed* P, uint8_t* tile_map, size_t bytes);
/* The prefill launch order chosen from the tile map (tile 128; the schedule is left to the implementation by
 * Appendix A): `order` (HOST) receives 2 * ceil(N / 256) tile-row indices, two per workgroup of 256 features, in
 * launch order; -1 marks a missing second row.  *count = entries written (0 for tile 64); `cap` = entries `order`
 * can hold, PATCH_ERR_SIZE if too few. */
patch_status patch_packed_row_order(const patch_packed* P, int32_t* order, size_t cap, size_t* count);

/*
 * A packed weight saved to and loaded from HOST memory (this project's; no passage of the paper - Appendix A compresses
 * once per weight and tile size, these calls keep the result): header (magic, layout number, tile, N, K, sizes,
 * checksum), the tile map, then the payload exactly as it lies in device memory.  The byte order of the payload is the
 * library's own; the layout number changes with it and patch_deserialize refuses any other number.
 *   patch_serialized_bytes  size of the buffer patch_serialize fills (0 for NULL)
 *   patch_serialize    buf: HOST, at least that many bytes (else PATCH_ERR_SIZE); copies on `stream` and waits for it
 *   patch_deserialize  buf: HOST, as written by patch_serialize; checks magic, layout number, shape, sizes against the
 *                      tile map, map entries (0 / 1) and the checksum (FNV-1a over map and payload: about a second per
 *                      GB) before any device work - PATCH_ERR_ARG / PATCH_ERR_SHAPE / PATCH_ERR_SIZE (buffer shorter
 *                      than its header says); rebuilds the tables and the launch order from the tile map as patch_pack
 *                      does, allocates, copies the payload on `stream` and waits for it.  *out: caller frees with
 *                      patch_free; it multiplies bit-identically to the handle that was saved.
 * patch_serialized4_bytes / patch_serialize4 / patch_deserialize4: the same for the 4-bit storage below (payload, then
 * the scales; its own magic).
 */
size_t patch_serialized_bytes(const patch_packed* P);
patch_status patch_serialize(const patch_packed* P, void* buf, size_t bytes, void* stream);
patch_status patch_deserialize(const void* buf, size_t bytes, void* stream, patch_packed** out);

/*
 * 4-bit weight-only storage of the pruned weight and its decode-shaped product (Section 5.2, "Quantization": the
 * hybrid-sparse model composed with 4-bit weight-only quantization; its table counts 4 bits per element of a dense tile
 * and 2 x 4 + 4 bits per group of four of a 2:4 tile).  The paper names no quantizer; this library's is symmetric with
 * 15 levels and one scale per row of a tile:  s = bf16(max|w| / 7),  q = clamp(rint(w / s), -7, 7)  (fp32, ties to
 * even; an all-zero row: s = 0, q = 0); the weight the product uses is bf16(q s).  A pruned weight keeps code 0, so a 2:4
 * tile stays 2:4 (its kept positions are those of W_hat).
 *   patch_pack4    W_hat, N, K, tile_map, tile, stream, *out as for patch_pack; synchronises `stream` once; returns
 *                  PATCH_ERR_NOT_24 like patch_pack
 *   patch_gemm4    Y[m, n] = sum_k X[m, k] * bf16(q s)[n, k]: X DEVICE M x K bf16, Y DEVICE M x N fp32, both 16-byte
 *                  aligned; asynchronous, allocates nothing, bit-reproducible.  Decode-shaped: the weight is streamed
 *                  once per 64 rows of X; for prefill shapes dequantize once (patch_unpack4) and patch_pack the result
 *   patch_gemm4_ex  the same product with an optional caller workspace (DEVICE, 16-byte aligned, or NULL; used when it
 *                  holds at least two slices of M x N fp32).  A prefill-shaped kernel reads the 4-bit weight once per
 *                  128 rows of X and dequantizes in registers (no bf16 copy of the weight); with a workspace it splits K
 *                  over workgroups (partial sums in the workspace, summed in slice order).  It is taken where an
 *                  estimate of both sides puts it ahead of passes of up to 64 rows (with a workspace from about 65
 *                  rows, from 48 on wide weights; without one from a few hundred rows, from 129 on wide weights);
 *                  otherwise passes as patch_gemm4 (= patch_gemm4_ex without a workspace).  Launches that may run
 *                  concurrently need distinct workspaces
 *   patch_gemm4_many  up to PATCH_MAX_MANY weights with the same K and tile against one X in one launch per 64 rows
 *                  (q / k / v, gate / up): Y[i] is M x N_i fp32; bit-reproducible, and equal to the single calls up to
 *                  the order of the fp32 partial sums (the split of K over wavefronts depends on the number of
 *                  workgroups); PATCH_ERR_SHAPE when K or tile differ
 *   patch_unpack4  any of: W_deq (DEVICE, N x K bf16, 16-byte aligned) = bf16(q s), 0 at pruned positions; codes
 *                  (DEVICE, N x K int8, 0 at pruned positions); scales (DEVICE, N x (K / tile) bf16); NULL = not wanted
 *   patch_pack_from4  the dequantized weight bf16(q s) packed for patch_gemm (the prefill path of a 4-bit model:
 *                  dequantize once, then every prefill kernel runs unchanged): patch_unpack4 into a temporary N x K
 *                  bf16 buffer, patch_pack with the tile map P4 was built with; synchronises `stream`; *out is the
 *                  caller's to free (patch_free); PATCH_ERR_ALLOC when the temporary does not fit
 *   patch_packed4_bytes  codes + positions + scales, without alignment padding
 * Errors as for their bf16 counterparts.
 */
typedef struct patch_packed4 patch_packed4;
patch_status patch_pack4(const void* W_hat, int64_t N, int64_t K, const uint8_t* tile_map, int tile, void* stream,
                         patch_packed4** out);
patch_status patch_gemm4(const void* X, int64_t M, const patch_packed4* P, void* Y, void* stream);
patch_status patch_gemm4_ex(const void* X, int64_t M, const patch_packed4* P, void* Y, void* workspace, size_t workspace_bytes,
                            void* stream);
patch_status patch_gemm4_many(const void* X, int64_t M, const patch_packed4* const* P, void* const* Y, int count, void* stream);
patch_status patch_unpack4(const patch_packed4* P, void* W_deq, void* codes, void* scales, void* stream);
patch_status patch_pack_from4(const patch_packed4* P4, void* stream, patch_packed** out);
size_t patch_packed4_bytes(const patch_packed4* P);
patch_status patch_packed4_dims(const patch_packed4* P, int64_t* N, int64_t* K, int* tile, int64_t* n_sparse_tiles);
void patch_free4(patch_packed4* P);
size_t patch_serialized4_bytes(const patch_packed4* P);
patch_status patch_serialize4(const patch_packed4* P, void* buf, size_t bytes, void* stream);
patch_status patch_deserialize4(const void* buf, size_t bytes, void* stream, patch_packed4** out);

/*
 * Measurement probes (this project's; no passage of the paper): kernels that run nothing of the method, for the
 * measured ceilings the benchmark prints beside the product kernels.  All are asynchronous on `stream` and
 * allocate nothing; the caller times them with events.
 *   patch_probe_matrix_rate  `workgroups` workgroups of 4 wavefronts each run `iters` rounds of 16 independent matrix
 *                            instructions on register operands: kind 0 = v_mfma_f32_16x16x32_bf16 (16384 flop each),
 *                            kind 1 = v_smfmac_f32_16x16x64_bf16 (32768 dense-equivalent flop each).  Total instructions
 *                            = workgroups * 4 * iters * 16.  kind 2 = v_mfma_f32_32x32x16_bf16 (32768 flop) and kind 3 =
 *                            v_smfmac_f32_32x32x32_bf16 (65536 dense-equivalent flop), the 32 x 32 shapes the product
 *                            kernels do not use: rounds of 8, i.e. the same flops per round.  operands: DEVICE, 16-byte aligned, at least
 *                            PATCH_PROBE_OPERAND_BYTES of bf16 data (random data gives the rate under realistic
 *                            switching activity; zeros give the clock-unconstrained rate); out: DEVICE,
 *                            workgroups * 256 floats (keeps the results alive).
 *   patch_probe_stream_read  reads `bytes` (16-byte aligned, multiple of 16) at src with 128-bit loads, grid-stride
 *                            over workgroups x threads (threads a multiple of 64, at most 1024); out: DEVICE,
 *                            workgroups * threads 32-bit words.
 *   patch_probe_lds_fill     `workgroups` workgroups of 8 wavefronts each fetch 48 KB per round (six 1 KB pieces per
 *                            wavefront, then a wait and a barrier: the fetch pattern of a K-step of the LDS-staged
 *                            prefill kernel) for `rounds` rounds, walking over the floor(bytes / 48 KB) chunks of src
 *                            (16-byte aligned): kind 0 = global -> LDS directly, kind 1 = global -> registers -> LDS,
 *                            kind 2 = global -> registers only; kind 4 = as 0 with rounds of 24 KB (three pieces per
 *                            wavefront) into alternating halves of the buffer, kind 3 = as 4 but waiting only for the
 *                            round before the one just issued (two rounds in flight).  out: DEVICE, workgroups * 512
 *                            32-bit words.
 *   patch_probe_store_tiles  stores only: one workgroup of 4 wavefronts per 256 x 256 tile of a row-major M x N
 *                            matrix Y (DEVICE, 16-byte aligned, y_bytes >= M * N * 4, or * 2 with bf16; M and N multiples
 *                            of 256), 64 store instructions per wavefront as in the output stage of the prefill kernel:
 *                            pattern 0 = 16 rows x 64 bytes per instruction (the accumulator layout stored as it lies),
 *                            pattern 1 = 4 rows x 256 contiguous bytes (after a turn through LDS); with bf16 half the
 *                            bytes per lane.  The values written are arbitrary.
 *   patch_probe_lds_read     LDS reads only: `workgroups` workgroups of 4 wavefronts, each wavefront reading its own
 *                            8 KB of LDS with conflict-free 128-bit reads, 8 in flight, `iters` times (bytes per
 *                            workgroup = iters * 32 KB).  out: DEVICE, workgroups * 256 floats.
 * Errors: PATCH_ERR_ARG, PATCH_ERR_SIZE (a buffer too small), PATCH_ERR_HIP.
 */
#define PATCH_PROBE_OPERAND_BYTES ((size_t)12 * 256 * 16)
patch_status patch_probe_matrix_rate(int kind, const void* operands, size_t operand_bytes, int workgroups, int iters, void* out,
                                     size_t out_bytes, void* stream);
patch_status patch_probe_stream_read(const void* src, size_t bytes, int workgroups, int threads, void* out, size_t out_bytes,
                                     void* stream);
patch_status patch_probe_lds_fill(int kind, const void* src, size_t bytes, int workgroups, int rounds, void* out, size_t out_bytes,
                                  void* stream);
patch_status patch_probe_store_tiles(int pattern, int bf16, void* Y, size_t y_bytes, int64_t M, int64_t N, void* stream);
patch_status patch_probe_lds_read(int workgroups, int iters, void* out, size_t out_bytes, void* stream);

void patch_free(patch_packed* P);
const char* patch_strerror(patch_status s);
int patch_last_hip_error(void); /* hipError_t of the most recent PATCH_ERR_HIP on this thread */
const char* patch_version(void);

#ifdef __cplusplus
}
#endif
#endif /* PATCH_H_ */
