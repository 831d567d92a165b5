/*
 * libqamw -- QAM-W per-weight-matrix codec for AMD MI355X (gfx950).
 *
 * The codec of arxiv 2605.26339, Sec. 3: a weight matrix W (d_out x d_in) is coded row by row.
 *   encode: W D_s (Sec. B.2) -> row norm r, u = w/r (Sec. 3.1 step 1) -> y = F S u, the sign-masked
 *           block-Hadamard rotation (Defs 1-3, Lemma 1) -> adjacent coordinates paired (step 3)
 *           -> each pair divided by sigma_k (step 4, Eq. 1) -> nearest entry of one 2^B-point 2-D
 *           codebook (Sec. 3.5) -> B-bit indices bit-packed per row (step 6).
 *   decode: unpack -> centroid lookup -> times sigma_k -> u~ = S F y^ -> times r -> D_s^-1 -> bf16
 *           (Sec. 3.2, Sec. B.2; the pipeline dequantises to BF16 before the matmul, Sec. 1).
 *
 * Conventions
 *   - C ABI, every function returns an int status (QAMW_OK = 0).  No exception crosses the boundary.
 *   - "host" pointers are ordinary CPU memory, "device" pointers are HIP device memory of the
 *     current device.  The caller owns every buffer, scratch included; the library allocates no
 *     device memory and keeps no state between calls (qamw_set_kernel_path is the one switch).
 *   - Device entry points validate their arguments on the host, synchronously, BEFORE any launch
 *     and return an error code without touching the outputs; otherwise they enqueue their kernels
 *     on `stream` (a hipStream_t passed as void*, NULL = the default stream) and return without
 *     waiting.  A launch failure is reported as QAMW_ERR_DEVICE.  Outputs are unspecified after
 *     an error.  Behaviour on non-finite input values is unspecified.
 *   - Matrices are row-major with an explicit leading dimension in ELEMENTS.
 *   - Packed buffers (packed, packed_out) are 4-byte aligned: the stream is read and written in 32-bit words;
 *     a misaligned one is an INVALID_ARG.
 *   - P = d_in/2 pairs per row, K = 2^bits codewords.  Pair k of a row is columns (2k, 2k+1).
 *
 * Packed layout (the paper leaves it open; this is the library's definition): per row, pair k
 * occupies bits [k*bits, (k+1)*bits) of the row's bit stream, least significant bit first; stream
 * bit n is bit (n mod 8) of byte floor(n/8); unused bits are zero; the row stride in bytes is
 * qamw_packed_row_bytes() = ceil(P*bits/8) rounded up to a multiple of 4.
 *
 * Arithmetic (fp32 unless noted), in this order, each result rounded once:
 *   ws = W*s;  r = fp32(sqrt(sum_j ws^2 accumulated in fp64));  u = ws / r (IEEE division; r = 0: u = 0);
 *   v = sign*u;  per block of `block` columns, butterflies with stride 1, 2, 4, ..., block/2:
 *   (a, b) <- (a+b, a-b);  y = t * fp32(block^-1/2);  x_k = (y_2k, y_2k+1) * g_k with
 *   g_k = 1/sigma_k (IEEE division), or fp32(sqrt(d_in)) when no sigma is given.
 *   Nearest codeword: exact fp32 squared distances decide; lowest index wins exact ties.
 *   decode: y^ = sigma_k * c[idx];  same butterflies;  times fp32(block^-1/2);  times sign;
 *   times r;  times fp32(1/s_j);  bf16 round-to-nearest-even.
 */
#ifndef QAMW_H
#define QAMW_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    QAMW_OK = 0,
    QAMW_ERR_INVALID_ARG = 1, /* NULL required pointer, value out of range                */
    QAMW_ERR_SHAPE = 2,       /* d_in odd, block not a power of two / not dividing d_in,  */
                              /* leading dimension smaller than the row                   */
    QAMW_ERR_UNSUPPORTED = 3, /* a valid request this build has no kernel for             */
    QAMW_ERR_DEVICE = 4       /* HIP reported an error at launch                          */
};

enum { QAMW_DTYPE_F32 = 0, QAMW_DTYPE_BF16 = 1 };

enum { QAMW_MAX_BITS = 12, QAMW_MAX_BLOCK = 1024 };

enum { QAMW_MAX_BATCH = 32 };   /* matrices per qamw_calibrate_sigma_batch / qamw_encode_batch / qamw_decode_batch call */

/* Text for a status code (static storage, never NULL). */
const char *qamw_status_string(int status);

/* ---------------------------------------------------------------------------------------------
 * Host helpers (no GPU involved)
 * ------------------------------------------------------------------------------------------ */

/* Row stride of the packed stream in bytes: ceil((d_in/2)*bits/8) rounded up to 4 (Sec. 3.1 step 6;
 * Sec. 3.6 mentions row-level packing and alignment without fixing them).
 * Errors: d_in <= 0 or odd -> SHAPE; bits outside [1,12] or out NULL -> INVALID_ARG. */
int qamw_packed_row_bytes(int d_in, int bits, size_t *out);

/* Block-size rule of Sec. 3.3: the largest power of two dividing d_in, capped at 1024
 * (worked examples there: 2048 -> 1024, 5632 -> 512). */
int qamw_paper_block_size(int d_in, int *block_out);

/* Eq. 3: bpw = bits/2 + 16/d_in; with_f16_scales adds the per-input-channel scale metadata of
 * Sec. 3.7, 16 bits per column, i.e. 16/d_out per weight. */
int qamw_bpw(int d_in, int d_out, int bits, int with_f16_scales, double *out);

/* Def. 3: the +-1 sign mask from a 64-bit seed.  Generator (the paper names none): word n of the
 * stream is the SplitMix64 output function applied to seed + (n+1)*0x9E3779B97F4A7C15; element j
 * takes bit (j mod 64) of word floor(j/64); 0 -> +1, 1 -> -1.  signs_out: host, d_in int8. */
int qamw_sign_mask(uint64_t seed, int d_in, int8_t *signs_out);

/* Sec. B.2: s_j proportional to act_rms_j^alpha, geometric mean normalised to one, then clamped to
 * [1/16, 16] (no renormalisation after the clamp).  act_rms below 1e-30 is floored.  Host arrays
 * of d_in floats.  alpha outside [0, 1] -> INVALID_ARG. */
int qamw_channel_scales(const float *act_rms, int d_in, float alpha, float *s_out);

/* Sec. 3.5, Eq. 2: Lloyd iterations for a 2^bits-point codebook on n_samples draws of the unit
 * circular Gaussian (CPU, off the hot path; multi-threaded, result independent of thread count).
 * Samples: draw i uses words 2i and 2i+1 of the SplitMix64 stream above as uniforms (top 53 bits;
 * u1 in (0,1], u2 in [0,1)) and the Box-Muller map.  Initial points: golden-angle spiral with
 * radii at the (i+0.5)/K quantiles of a circular Gaussian of variance 2 per axis.  Each iteration
 * assigns every sample to its nearest point (fp64, lowest index on ties) and, unless it is the
 * last, moves every point to the mean of its cell (an empty cell moves onto the sample with the
 * largest error).  Stops when the relative change of the mean squared error drops below tol, or
 * after max_iters assignments.
 * codebook_out: host, 2^bits x 2 floats (x, y).  mse_out / iters_out: nullable.
 * Errors: bits outside [1,12], n_samples < 2^bits, max_iters < 1, tol < 0, NULL output. */
int qamw_train_codebook(int bits, uint64_t n_samples, uint64_t seed, int max_iters, double tol,
                        float *codebook_out, double *mse_out, int *iters_out);

/* ---------------------------------------------------------------------------------------------
 * Device entry points.  Common arguments:
 *   dtype       QAMW_DTYPE_F32 or QAMW_DTYPE_BF16: element type of W (bf16 is widened exactly)
 *   d_out,d_in  matrix shape; d_in even
 *   ldw         leading dimension of W in elements, >= d_in
 *   chan_scale  device, d_in floats s_j > 0, or NULL (= all ones)          [Sec. B.2]
 *   signs       device, d_in int8 in {+1,-1}, or NULL (= all +1)           [Def. 3]
 *   pair_sigma  device, P floats sigma_k > 0, or NULL (= 1/sqrt(d_in))     [Eq. 1]
 *   codebook    device, K x 2 floats                                       [Sec. 3.5]
 *   bits        1..12;  hadamard_block: power of two, 2..1024, dividing d_in
 *   stream      hipStream_t as void*
 * Errors common to all: NULL required pointer, d_out/d_in <= 0, bits out of range -> INVALID_ARG;
 * odd d_in, bad block, ldw < d_in -> SHAPE.
 * ------------------------------------------------------------------------------------------ */

/* Eq. 1: sigma_k = mean over the first n = min(d_out, max_rows) rows of |z_k| / sqrt(pi/2), where
 * z_k are the pairs of the unit-normalised, rotated rows (encoder steps 1-3); amplitudes and the
 * mean in fp64; an estimate that is not positive is replaced by 1/sqrt(d_in).
 * workspace: device scratch of at least qamw_calibrate_workspace_bytes() bytes, 16-byte aligned,
 * owned by the caller (holds those rows' norms and per-row-group partial sums; contents are
 * unspecified afterwards).  sigma_out: device, P floats.
 * Errors: max_rows < 1, workspace NULL / too small / misaligned -> INVALID_ARG. */
int qamw_calibrate_workspace_bytes(int d_in, int d_out, int max_rows, size_t *bytes_out);
int qamw_calibrate_sigma(const void *W, int dtype, int d_out, int d_in, int64_t ldw,
                         const float *chan_scale, const int8_t *signs, int hadamard_block,
                         int max_rows, void *workspace, size_t workspace_bytes, float *sigma_out,
                         void *stream);

/* qamw_calibrate_sigma for several matrices that share the element type and hadamard_block, in one pair of launches
 * (the calibration of one matrix is tens of microseconds of work on a fraction of the chip).  items: HOST array, read
 * during the call only; every pointer in it is a device pointer with the meaning it has in qamw_calibrate_sigma.
 * workspace: at least the sum over the items of qamw_calibrate_workspace_bytes() each rounded up to a multiple of 256,
 * 16-byte aligned.  Results are identical, bit for bit, to n_items calls of qamw_calibrate_sigma.  Items the fast
 * kernels cannot take make the whole call fall back to one call per item.
 * Errors: items NULL, n_items outside [1, QAMW_MAX_BATCH], workspace NULL / misaligned / too small, any item invalid
 * as for qamw_calibrate_sigma. */
typedef struct qamw_calibrate_item {
    const void *W;               /* d_out rows of d_in elements of the batch's dtype, leading dimension ldw */
    int64_t ldw;
    const float *chan_scale;     /* d_in floats or NULL                                                   */
    const int8_t *signs;         /* d_in int8 or NULL                                                     */
    float *sigma_out;            /* d_in/2 floats                                                         */
    int32_t d_out, d_in;
} qamw_calibrate_item;
int qamw_calibrate_sigma_batch(const qamw_calibrate_item *items, int n_items, int dtype, int hadamard_block,
                               int max_rows, void *workspace, size_t workspace_bytes, void *stream);

/* qamw_calibrate_sigma for callers that cannot allocate device memory or pass a workspace: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments without the workspace,
 * same kernels, same result bit for bit; the scratch is a static device array of QAMW_STATIC_SCRATCH_BYTES
 * inside the library (every GPU the library runs on holds it until the process ends).  The call allocates
 * and frees nothing.  The first call on a device looks up the array's address on that device (no allocation,
 * but make that first call outside a capture).
 * Limit: qamw_calibrate_workspace_bytes(d_in, d_out, max_rows) <= QAMW_STATIC_SCRATCH_BYTES, i.e. d_in up to
 * 16384 at max_rows = 1024; anything larger -> QAMW_ERR_UNSUPPORTED, nothing launched.
 * All calls on one GPU share the one array: calls that overlap on the same GPU (different streams, or
 * threads) race and give wrong pair scales; order them on one stream or use qamw_calibrate_sigma with
 * separate workspaces.  Nothing in the array has to be cleared between calls. */
enum { QAMW_STATIC_SCRATCH_BYTES = 8 * 1024 * 1024 + 4096 };
int qamw_calibrate_sigma_static(const void *W, int dtype, int d_out, int d_in, int64_t ldw,
                                const float *chan_scale, const int8_t *signs, int hadamard_block,
                                int max_rows, float *sigma_out, void *stream);

/* Encoder of Sec. 3.1 with the channel scaling of Sec. B.2.
 * packed_out: device, d_out * qamw_packed_row_bytes(d_in, bits) bytes, fully overwritten.
 * row_norms_out: device, d_out floats (norm of the SCALED row W D_s). */
int qamw_encode(const void *W, int dtype, int d_out, int d_in, int64_t ldw, const float *chan_scale,
                const int8_t *signs, const float *pair_sigma, const float *codebook, int bits,
                int hadamard_block, uint8_t *packed_out, float *row_norms_out, void *stream);

/* qamw_encode that also counts how the indices were decided.  The fast encoders shortlist with approximate
 * scores and decide every index by exact fp32 squared distances, inside the best chunk of codewords when the
 * shortlist separates it provably from the rest, otherwise by an exact scan of the whole codebook.
 * full_scans: device, one 64-bit counter; the number of pairs that took the whole-codebook scan is ADDED to
 * it (the caller zeroes it); the general kernels, which scan everything for every pair, do not count.
 * The packed output is identical to qamw_encode's. */
int qamw_encode_stats(const void *W, int dtype, int d_out, int d_in, int64_t ldw, const float *chan_scale,
                      const int8_t *signs, const float *pair_sigma, const float *codebook, int bits,
                      int hadamard_block, uint8_t *packed_out, float *row_norms_out,
                      unsigned long long *full_scans, void *stream);

/* Several matrices that share codebook, bits, hadamard_block and element type encoded in ONE launch (Sec. 3.1; a
 * TinyLlama-sized projection is a fraction of a millisecond of work, so per-launch ramp-up and tail are a large part
 * of qamw_encode for small matrices; a batch, e.g. a layer's seven projections, amortises them).
 * items: HOST array of n_items descriptors (read during the call, not retained); every pointer inside is a device
 * pointer with the meaning it has in qamw_encode.  1 <= n_items <= QAMW_MAX_BATCH.
 * Results are identical, bit for bit, to n_items calls of qamw_encode.  Items the batched kernel cannot take
 * (shape, alignment, codebooks of fewer than 64 or more than 2048 points) make the whole call fall back to one
 * qamw_encode per item.  Errors: items NULL, n_items out of range, any item invalid as for qamw_encode. */
typedef struct qamw_encode_item {
    const void *W;               /* d_out rows of d_in elements of the batch's dtype, leading dimension ldw */
    int64_t ldw;
    const float *chan_scale;     /* d_in floats or NULL                                                   */
    const int8_t *signs;         /* d_in int8 or NULL                                                     */
    const float *pair_sigma;     /* d_in/2 floats or NULL                                                 */
    uint8_t *packed_out;         /* d_out * qamw_packed_row_bytes(d_in, bits) bytes                       */
    float *row_norms_out;        /* d_out floats                                                          */
    int32_t d_out, d_in;
} qamw_encode_item;
int qamw_encode_batch(const qamw_encode_item *items, int n_items, int dtype, const float *codebook, int bits,
                      int hadamard_block, void *stream);

/* Codebook training on the device (Sec. 3.5; a codebook fitted to a checkpoint's own pairs is the follow-up
 * named in the paper's discussion).
 *
 * qamw_normalised_pairs: the points the encoder quantises -- encoder steps 1-4 (channel scale, row norm,
 * rotation, division by sigma_k) written out instead of searched: pairs_out[i][2k], [2k+1] = pair k of row i,
 * bit for bit what qamw_encode sees.  pairs_out: device, d_out * d_in floats, 16-byte aligned.
 * row_norms_out: device, d_out floats.  Shapes as qamw_encode_polar; otherwise QAMW_ERR_UNSUPPORTED.
 *
 * qamw_lloyd_device: Lloyd iterations over n_samples 2-D points in device memory (8-byte aligned, x then y).
 * codebook: device, 2^bits x 2 floats: the initial points on entry, the trained points on return.  Each
 * iteration assigns every sample to its nearest point by exact fp32 squared distances over the whole
 * codebook (lowest index on ties) and moves every point to the mean of its cell; the cell sums are kept in
 * 64-bit fixed point (2^-30; coordinates beyond +-256 enter the sums clamped), so the result is the same on
 * every run.  An empty cell keeps its point (the CPU trainer re-seeds it).  Stops as qamw_train_codebook
 * does: relative change of the mean squared error below tol, or max_iters assignments; the points are not
 * moved after the last assignment, so the codebook and *mse_out belong together.
 * The call BLOCKS: it synchronises the stream once per iteration to read the error.
 * workspace: device, qamw_lloyd_workspace_bytes() bytes, 16-byte aligned, owned by the caller.
 * mse_out / iters_out: host, nullable.
 * Errors: bits outside [1,12], n_samples < 2^bits or > 2^24, max_iters < 1, tol < 0, NULL or misaligned
 * buffers, workspace too small -> INVALID_ARG. */
int qamw_normalised_pairs(const void *W, int dtype, int d_out, int d_in, int64_t ldw, const float *chan_scale,
                          const int8_t *signs, const float *pair_sigma, int hadamard_block, float *pairs_out,
                          float *row_norms_out, void *stream);
int qamw_lloyd_workspace_bytes(int bits, size_t *bytes_out);
int qamw_lloyd_device(const float *samples, uint64_t n_samples, int bits, float *codebook, int max_iters,
                      double tol, void *workspace, size_t workspace_bytes, double *mse_out, int *iters_out,
                      void *stream);

/* Pruned nearest-codeword search (the search step of Sec. 3.1 with fewer distance evaluations; the index is
 * the one the whole-codebook search of qamw_encode returns, bit for bit).
 *
 * qamw_search_grid_size (host): the grid has G x G cells, G = 2^floor((bits + 6) / 2); the table takes
 * 32 + 16 G^2 bytes.  Either output may be NULL.
 *
 * qamw_search_grid_build (host): codebook: host, 2^bits x 2 finite floats.  grid_out: host, grid_bytes >=
 * the size above.  Layout: eight 32-bit words {0x44524751, bits, G, 8, fp32 cells per unit length
 * inv_h = G / 2R, fp32 R, 0, 0}, R = 1.25 max |coordinate| of the codebook (1 if that is 0); then G x G
 * records, record iy * G + ix for the cell {x : floor(x0 inv_h + G/2) = ix, floor(x1 inv_h + G/2) = iy},
 * each eight 16-bit codeword indices in ascending order: every codeword that can be nearest to a point of
 * the cell (a codeword is left out only if its smallest distance to the cell, widened by the rounding of
 * the cell lookup, exceeds by more than 1e-5 relative the smallest over the codebook of the largest
 * distance to the cell).  A shorter list is padded with its first entry; a cell with more than eight
 * candidates holds the first seven and 0xFFFF, and its points get the whole-codebook scan.
 * max_candidates_out / overflow_cells_out (nullable): the longest list, the number of such cells.
 * Errors: bits outside [1,12], NULL codebook or grid_out, non-finite codeword, grid_bytes too small.
 *
 * qamw_encode_pruned (device): qamw_encode with the search restricted to the pair's cell record; pairs
 * outside [-R, R)^2 or in an overflowing cell are decided by the whole-codebook scan and, if full_scans
 * (device, one 64-bit counter, nullable) is given, ADDED to it.  grid: device, the table as built, 16-byte
 * aligned; it must have been built from `codebook` with the same bits -- a table of another codebook gives
 * wrong indices (never an out-of-range access: the grid size is taken from bits, indices are reduced mod K).
 * Shapes: as qamw_encode_polar; anything else -> QAMW_ERR_UNSUPPORTED. */
int qamw_search_grid_size(int bits, int *cells_per_side_out, size_t *bytes_out);
int qamw_search_grid_build(const float *codebook, int bits, void *grid_out, size_t grid_bytes,
                           int *max_candidates_out, uint64_t *overflow_cells_out);
int qamw_encode_pruned(const void *W, int dtype, int d_out, int d_in, int64_t ldw, const float *chan_scale,
                       const int8_t *signs, const float *pair_sigma, const float *codebook, int bits,
                       int hadamard_block, const void *grid, uint8_t *packed_out, float *row_norms_out,
                       unsigned long long *full_scans, void *stream);

/* Polar baseline of Sec. 3 ("Polar Baseline"; distortion: the polar pair theorem and the
 * Rayleigh-Lloyd corollary).
 *
 * qamw_polar_codebook (host): the 2^bits_a Lloyd-Max levels of the unit Rayleigh density
 * f(r) = r exp(-r^2/2), by numerical integration up to the cutoff 8 (the remark after the corollary).
 * levels_out: host, 2^bits_a floats, increasing.  table_out: host, 2^(bits_a+bits_p) x 2 floats or NULL:
 * entry ia * 2^bits_p + ip = level ia at phase (2 ip + 1) pi / 2^bits_p (the bin centres of the corollary);
 * with this table as `codebook`, qamw_decode / qamw_decode_batch decode a polar code.  c_lm_out (nullable):
 * the levels' distortion E (U - Q(U))^2.
 * Errors: bits_a outside [0, QAMW_MAX_POLAR_AMPLITUDE_BITS], bits_p outside [0,12], bits_a + bits_p outside
 * [1,12], NULL levels_out.
 *
 * qamw_encode_polar (device): the encoder's front half unchanged, then per pair the nearest amplitude
 * level (decided on squared amplitudes against squared midpoints; the lower level on a tie) and the
 * phase bin [2k pi/Np, 2(k+1) pi/Np) containing atan2(x1, x0) in [0, 2 pi) (the origin: bin 0).
 * Index = amplitude index * 2^bits_p + phase index, packed with bits_a + bits_p bits per pair as
 * qamw_encode packs.  levels: device, 2^bits_a floats.
 * Shapes: d_in a multiple of max(hadamard_block, 16), hadamard_block >= 64, W and the optional vectors
 * 16-byte aligned, ldw a multiple of 4 (fp32) or 8 (bf16); anything else -> QAMW_ERR_UNSUPPORTED. */
enum { QAMW_MAX_POLAR_AMPLITUDE_BITS = 6 };
int qamw_polar_codebook(int bits_a, int bits_p, float *levels_out, float *table_out, double *c_lm_out);
int qamw_encode_polar(const void *W, int dtype, int d_out, int d_in, int64_t ldw, const float *chan_scale,
                      const int8_t *signs, const float *pair_sigma, const float *levels, int bits_a,
                      int bits_p, int hadamard_block, uint8_t *packed_out, float *row_norms_out,
                      void *stream);

/* Decoder of Sec. 3.2 with D_s^-1 of Sec. B.2, bf16 output (uint16 bit patterns).
 * W_out: device, d_out rows of d_in bf16 with leading dimension ldo >= d_in (elements). */
int qamw_decode(const uint8_t *packed, const float *row_norms, int d_out, int d_in,
                const float *chan_scale, const int8_t *signs, const float *pair_sigma,
                const float *codebook, int bits, int hadamard_block, uint16_t *W_out, int64_t ldo,
                void *stream);

/* Same decoder, writing the fp32 value before the bf16 cast (for accuracy checks). */
int qamw_decode_f32(const uint8_t *packed, const float *row_norms, int d_out, int d_in,
                    const float *chan_scale, const int8_t *signs, const float *pair_sigma,
                    const float *codebook, int bits, int hadamard_block, float *W_out, int64_t ldo,
                    void *stream);

/* Several matrices that share codebook, bits and hadamard_block decoded to bf16 in ONE launch (the
 * decoder of Sec. 3.2 is bandwidth bound and a single LLM projection matrix is only microseconds of
 * HBM time, so per-launch ramp-up and tail are a large part of qamw_decode; a batch amortises them).
 * items: HOST array of n_items descriptors (read during the call, not retained); every pointer
 * inside is a device pointer with the meaning it has in qamw_decode.  1 <= n_items <= QAMW_MAX_BATCH.
 * Results are identical to n_items calls of qamw_decode.  Items the fast kernel cannot take
 * (shape, alignment) make the whole call fall back to one general launch per item.
 * Errors: items NULL, n_items out of range, any item invalid as for qamw_decode. */
typedef struct qamw_decode_item {
    const uint8_t *packed;       /* d_out * qamw_packed_row_bytes(d_in, bits) bytes            */
    const float *row_norms;      /* d_out floats                                               */
    const float *chan_scale;     /* d_in floats or NULL                                        */
    const int8_t *signs;         /* d_in int8 or NULL                                          */
    const float *pair_sigma;     /* d_in/2 floats or NULL                                      */
    uint16_t *W_out;             /* d_out rows of d_in bf16, leading dimension ldo             */
    int64_t ldo;
    int32_t d_out, d_in;
} qamw_decode_item;
int qamw_decode_batch(const qamw_decode_item *items, int n_items, const float *codebook, int bits,
                      int hadamard_block, void *stream);

/* Measurement aid for the decoder of Sec. 3.2: the launch of qamw_decode_batch for these items with every load and
 * store it issues (same addresses, widths, order and launch shape) and none of the arithmetic in between.  The time of
 * this launch is what the memory system allows the decoder's access pattern, i.e. the ceiling its bandwidth figure is
 * to be read against.  W_out of every item is OVERWRITTEN WITH MEANINGLESS VALUES.  Only for shapes the fast decoder
 * takes (bits in {7, 8, 11}, hadamard_block >= 64, d_in a multiple of max(hadamard_block, 16), 16-byte aligned outputs
 * and side vectors, 4-byte aligned packed rows); anything else -> QAMW_ERR_UNSUPPORTED, nothing launched.
 * Errors otherwise as qamw_decode_batch. */
int qamw_decode_traffic_probe(const qamw_decode_item *items, int n_items, const float *codebook, int bits,
                              int hadamard_block, void *stream);

/* Fused dequantise-and-multiply (the follow-up the paper's Limitations paragraph on inference kernels names):
 * Y = X W^T for m <= QAMW_MATMUL_MAX_ROWS activation rows, W = the matrix
 * that qamw_decode_f32 would produce from (packed, row_norms, ...), without materialising W.
 * By the linearity of the decoder (Sec. 3.2, Sec. B.2) and the symmetry of F (Lemma 1),
 *     <w_i, x> = r_i * sum_k < c[idx_ik], z_k >,   z = the pairs of sigma (.) F S (x / s):
 * the activations are rotated once, then every packed index costs one lookup and two multiply-adds per
 * activation row; the matrix is read once, packed.
 * X: device, m rows of d_in elements (fp32 or bf16), leading dimension ldx.  Y: device, m rows of d_out
 * floats, leading dimension ldy.  workspace: device, at least qamw_matmul_workspace_bytes() bytes, 16-byte
 * aligned, owned by the caller (the rotated activations; contents unspecified afterwards).
 * Accumulation is fp32 in a fixed order that depends on the matrix's shape and m only: deterministic, and the
 * same bits whether a product is computed alone or inside a batch.
 * m <= QAMW_MATMUL_VECTOR_ROWS: all arithmetic in fp32 on the vector ALU (error about 1e-8 ||x|| ||w_i||).
 * m > QAMW_MATMUL_VECTOR_ROWS: the products run on the bf16 matrix cores -- z and the codewords are rounded to
 * bf16 (round to nearest even), products are exact, accumulation is fp32: what the paper's pipeline
 * (dequantise to bf16, then a bf16 matmul) does to its operands, in the rotated domain; the error is about
 * 2^-9 per operand.  This path also needs d_in a multiple of 256 and 8-byte aligned packed rows.
 * m > QAMW_MATMUL_TILE_ROWS: the activation rows are processed in ceil(m / QAMW_MATMUL_TILE_ROWS) tiles of equal size
 * (at most QAMW_MATMUL_TILE_ROWS rows), one rotation + product launch per tile on the stream, the packed matrix read
 * once per tile; the workspace is that of one tile.  Row t of Y is the same whatever m is above the vector range.
 * Errors: m outside [1, QAMW_MATMUL_MAX_ROWS], NULL pointers, workspace too small or misaligned ->
 * INVALID_ARG; ldx < d_in, ldy < d_out -> SHAPE.  Shapes: bits in {7, 8, 11}, hadamard_block >= 64, d_in a
 * multiple of max(hadamard_block, 16), packed 4-byte aligned; anything else -> QAMW_ERR_UNSUPPORTED. */
enum { QAMW_MATMUL_MAX_ROWS = 4096, QAMW_MATMUL_TILE_ROWS = 64, QAMW_MATMUL_VECTOR_ROWS = 8, QAMW_MATMUL_MAX_BATCH = 16 };
int qamw_matmul_workspace_bytes(int d_in, int d_out, int m, size_t *bytes_out);
int qamw_matmul(const void *X, int x_dtype, int m, int64_t ldx, const uint8_t *packed, const float *row_norms,
                int d_out, int d_in, const float *chan_scale, const int8_t *signs, const float *pair_sigma,
                const float *codebook, int bits, int hadamard_block, void *workspace, size_t workspace_bytes,
                float *Y, int64_t ldy, void *stream);

/* The same for up to QAMW_MATMUL_MAX_BATCH independent products Y_i = X_i W_i^T that share the codebook, bits,
 * hadamard_block, m and the element type of X (for instance the projections of one layer applied to their
 * inputs): two launches in all (rotation, products) instead of two per matrix.  items: host array, read during the call only;
 * every pointer in it is a device pointer.  workspace: at least the sum of qamw_matmul_workspace_bytes() over
 * the items, 16-byte aligned.  Errors as qamw_matmul, per item; nothing is launched if any item is rejected. */
typedef struct qamw_matmul_item {
    const void *X;               /* m rows of d_in elements, leading dimension ldx                */
    int64_t ldx;
    const uint8_t *packed;       /* d_out rows of qamw_packed_row_bytes(d_in, bits) bytes        */
    const float *row_norms;      /* d_out floats                                                */
    const float *chan_scale;     /* d_in floats or NULL                                         */
    const int8_t *signs;         /* d_in int8 or NULL                                           */
    const float *pair_sigma;     /* d_in/2 floats or NULL                                       */
    float *Y;                    /* m rows of d_out floats, leading dimension ldy               */
    int64_t ldy;
    int32_t d_out, d_in;
} qamw_matmul_item;
int qamw_matmul_batch(const qamw_matmul_item *items, int n_items, int x_dtype, int m, const float *codebook,
                      int bits, int hadamard_block, void *workspace, size_t workspace_bytes, void *stream);

/* Which implementation the device entry points use: 0 = automatic (fast kernels when the shape
 * allows, otherwise the general ones), 1 = always the general kernels, 2 = as 0 but the encoder's
 * shortlist runs on the vector ALU instead of the matrix cores.  All three give the same indices.
 * qamw_encode_pruned: 0 = chosen by the amount of work, 1 = every cell record read from global memory,
 * 2 = the central cells in LDS whatever the size.  qamw_matmul / qamw_matmul_batch with one or two
 * activation rows: 0 = chosen by the size of the launch, 1 = activations rotated by a launch of their
 * own, 2 = rotated inside the product kernel; the results are the same, bit for bit.
 * This is the library's ONE piece of process-wide state: an atomic integer, safe to set from any thread, but it
 * affects every call of every thread made afterwards -- a switch for tests and measurements, not for production code
 * (all settings give the same results).  Returns the previous value (also for a value out of range, which changes
 * nothing). */
int qamw_set_kernel_path(int path);

#ifdef __cplusplus
}
#endif
#endif /* QAMW_H */
