/*
 * QAM-W codec oracle -- TEST INFRASTRUCTURE, NOT THE PRODUCT.
 *
 * A plain, slow, single-threaded CPU statement of what the QAM-W per-matrix codec
 * computes, written from the paper (arxiv 2605.26339) step by step.  It shares no
 * code with the HIP library.  Only tests, the smoke check and the CPU-baseline leg
 * of the benchmark may call it.
 *
 * Two modes, one structure:
 *   mode 0 "truth": every floating-point step in fp64; the rotation is a product
 *                   with the explicit Walsh-Hadamard matrix of Def. 1.
 *   mode 1 "spec" : the same steps in fp32, each one rounded once, in the order
 *                   written below, so that the integer decisions (the codeword
 *                   indices) are taken on exactly the numbers a fp32 device
 *                   kernel sees.  The argmin itself is always evaluated in fp64.
 *
 * Parity pins (tests/test_oracle_*.py): Hadamard orthogonality and symmetry in
 * integers, rotation isometry, brute-force argmin, hand-computed packed bytes,
 * printed bits-per-weight values, Rayleigh mean closed form, Lloyd fixed-point
 * conditions, library bf16 cast; for the polar baseline: centroid conditions and
 * C_LM by numerical quadrature, the one-level textbook values, brute-force
 * amplitude/phase decisions, the pair distortion identity and the corollary's
 * closed form on samples.  What cannot be pinned: agreement with the
 * authors' own bytes (their sign generator, packing layout and codebook are not
 * published) -- parity unpinned for that, by necessity.
 *
 * Build: gcc -O2 -ffp-contract=off -fPIC -shared (no fast-math, no FMA fusion).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifndef M_PI
#define M_PI 3.14159265358979323846
#endif

#define ORC_OK 0
#define ORC_ERR 1

/* ------------------------------------------------------------------------- */
/* Def. 1: unnormalised Walsh-Hadamard matrix, Sylvester recursion.           */
/* H_1 = [1];  H_2n = [[H_n, H_n], [H_n, -H_n]].  H is b x b, row-major.       */
/* ------------------------------------------------------------------------- */
void orc_hadamard(int b, int8_t *H)
{
    H[0] = 1;
    for (int n = 1; n < b; n *= 2) {
        for (int i = 0; i < n; ++i) {
            for (int j = 0; j < n; ++j) {
                int8_t h = H[(size_t)i * b + j];
                H[(size_t)i * b + (j + n)] = h;
                H[(size_t)(i + n) * b + j] = h;
                H[(size_t)(i + n) * b + (j + n)] = (int8_t)-h;
            }
        }
    }
}

/* Rotation-choice rule of Sec. 3.3: largest power of two dividing d_in, capped at 1024. */
int orc_paper_block_size(int d_in)
{
    int b = 1;
    while (b < 1024 && d_in % (2 * b) == 0)
        b *= 2;
    return b;
}

/* Eq. 3: bpw = B/2 + 16/d_in.  Optional f16 per-input-channel scales add 16 bits per
 * column of a d_out x d_in matrix, i.e. 16/d_out per weight (Sec. 3.7). */
double orc_bpw(int d_in, int d_out, int bits, int with_f16_scales)
{
    double v = (double)bits / 2.0 + 16.0 / (double)d_in;
    if (with_f16_scales)
        v += 16.0 / (double)d_out;
    return v;
}

/* ------------------------------------------------------------------------- */
/* Counter-based generator shared by definition (not by code) with the       */
/* library: output n of stream `seed` is the SplitMix64 finaliser applied to */
/* seed + (n+1)*0x9E3779B97F4A7C15.                                           */
/* ------------------------------------------------------------------------- */
static uint64_t mix64(uint64_t seed, uint64_t n)
{
    uint64_t z = seed + (n + 1u) * 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

/* Def. 3: the sign mask.  Element j takes bit (j mod 64) of output floor(j/64);
 * bit 0 -> +1, bit 1 -> -1. */
void orc_sign_mask(uint64_t seed, int d_in, int8_t *signs)
{
    for (int j = 0; j < d_in; ++j) {
        uint64_t w = mix64(seed, (uint64_t)(j / 64));
        signs[j] = ((w >> (j % 64)) & 1u) ? -1 : 1;
    }
}

/* Samples of the unit circular Gaussian of Eq. 2: sample i uses outputs 2i, 2i+1 as
 * uniforms u1 in (0,1], u2 in [0,1) (top 53 bits) and the Box-Muller map. */
void orc_gauss_samples(uint64_t seed, int64_t n, double *xy)
{
    const double two_pi = 6.283185307179586476925286766559;
    for (int64_t i = 0; i < n; ++i) {
        uint64_t a = mix64(seed, (uint64_t)(2 * i));
        uint64_t b = mix64(seed, (uint64_t)(2 * i + 1));
        double u1 = ((double)(a >> 11) + 1.0) * (1.0 / 9007199254740992.0);
        double u2 = (double)(b >> 11) * (1.0 / 9007199254740992.0);
        double rad = sqrt(-2.0 * log(u1));
        xy[2 * i] = rad * cos(two_pi * u2);
        xy[2 * i + 1] = rad * sin(two_pi * u2);
    }
}

/* ------------------------------------------------------------------------- */
/* Sec. B.2: s_j proportional to r_j^alpha, geometric mean normalised to 1,   */
/* then clamped to [1/16, 16].  r_j below 1e-30 is floored before the log.    */
/* ------------------------------------------------------------------------- */
void orc_channel_scales(const float *act_rms, int d_in, double alpha, float *s_out)
{
    double mean_log = 0.0;
    for (int j = 0; j < d_in; ++j) {
        double r = (double)act_rms[j];
        if (r < 1e-30)
            r = 1e-30;
        mean_log += alpha * log(r);
    }
    mean_log /= (double)d_in;
    for (int j = 0; j < d_in; ++j) {
        double r = (double)act_rms[j];
        if (r < 1e-30)
            r = 1e-30;
        double p = exp(alpha * log(r) - mean_log);
        if (p > 16.0)
            p = 16.0;
        if (p < 1.0 / 16.0)
            p = 1.0 / 16.0;
        s_out[j] = (float)p;
    }
}

/* bf16 round-to-nearest-even of a finite fp32 value (the cast PyTorch performs). */
uint16_t orc_bf16_rne(float f)
{
    uint32_t u;
    memcpy(&u, &f, 4);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u)
        return (uint16_t)((u >> 16) | 0x40u); /* quiet NaN */
    uint32_t lsb = (u >> 16) & 1u;
    u += 0x7FFFu + lsb;
    return (uint16_t)(u >> 16);
}

/* ------------------------------------------------------------------------- */
/* Rotation, forward: y = F S v (Lemma 1: R_fwd = F S), one row of d_in.      */
/* ------------------------------------------------------------------------- */

/* truth: explicit matrix, fp64 */
static void rotate_fwd_truth(const double *v, int d_in, int b, const int8_t *signs,
                             const int8_t *H, double *y)
{
    double inv_sqrt_b = 1.0 / sqrt((double)b);
    for (int blk = 0; blk < d_in / b; ++blk) {
        const double *vb = v + (size_t)blk * b;
        for (int i = 0; i < b; ++i) {
            double acc = 0.0;
            for (int j = 0; j < b; ++j) {
                double sj = signs ? (double)signs[blk * b + j] : 1.0;
                acc += (double)H[(size_t)i * b + j] * (sj * vb[j]);
            }
            y[(size_t)blk * b + i] = acc * inv_sqrt_b;
        }
    }
}

/* truth: u = S F yhat (R_inv = S F) */
static void rotate_inv_truth(const double *yh, int d_in, int b, const int8_t *signs,
                             const int8_t *H, double *u)
{
    double inv_sqrt_b = 1.0 / sqrt((double)b);
    for (int blk = 0; blk < d_in / b; ++blk) {
        const double *yb = yh + (size_t)blk * b;
        for (int j = 0; j < b; ++j) {
            double acc = 0.0;
            for (int i = 0; i < b; ++i)
                acc += (double)H[(size_t)j * b + i] * yb[i];
            double sj = signs ? (double)signs[blk * b + j] : 1.0;
            u[(size_t)blk * b + j] = sj * (acc * inv_sqrt_b);
        }
    }
}

/* spec: in-place butterflies, stride h = 1, 2, 4, ..., b/2 in that order; every
 * sum and difference rounded to fp32 once.  Unnormalised (the caller scales). */
void orc_fwht_spec(float *t, int b)
{
    for (int h = 1; h < b; h *= 2) {
        for (int i = 0; i < b; ++i) {
            if ((i & h) == 0) {
                volatile float lo = t[i], hi = t[i + h];
                volatile float sum = lo + hi;
                volatile float dif = lo - hi;
                t[i] = sum;
                t[i + h] = dif;
            }
        }
    }
}

/* Exported wrappers so tests can drive the rotation alone. */
void orc_rotate_fwd_truth(const double *v, int d_in, int b, const int8_t *signs, double *y)
{
    int8_t *H = (int8_t *)malloc((size_t)b * b);
    orc_hadamard(b, H);
    rotate_fwd_truth(v, d_in, b, signs, H, y);
    free(H);
}

void orc_rotate_inv_truth(const double *yh, int d_in, int b, const int8_t *signs, double *u)
{
    int8_t *H = (int8_t *)malloc((size_t)b * b);
    orc_hadamard(b, H);
    rotate_inv_truth(yh, d_in, b, signs, H, u);
    free(H);
}

/* spec-mode forward rotation of one row: y = fl32(FWHT(sign*u) * fl32(b^-1/2)) */
static void rotate_fwd_spec(const float *u, int d_in, int b, const int8_t *signs, float *y)
{
    volatile float cb = (float)(1.0 / sqrt((double)b));
    for (int j = 0; j < d_in; ++j)
        y[j] = (signs && signs[j] < 0) ? -u[j] : u[j];
    for (int blk = 0; blk < d_in / b; ++blk)
        orc_fwht_spec(y + (size_t)blk * b, b);
    for (int j = 0; j < d_in; ++j) {
        volatile float p = y[j] * cb;
        y[j] = p;
    }
}

void orc_rotate_fwd_spec(const float *u, int d_in, int b, const int8_t *signs, float *y)
{
    rotate_fwd_spec(u, d_in, b, signs, y);
}

/* ------------------------------------------------------------------------- */
/* Encoder front half, Sec. 3.1 steps 1-4 on one row: channel scale (Sec.    */
/* B.2), row norm, normalise, rotate, pair-normalise.  Produces the P        */
/* normalised pairs x_k = z_k / sigma_k and the row norm.                     */
/* ------------------------------------------------------------------------- */
static void front_truth(const float *w, int d_in, const float *chan_scale, const int8_t *signs,
                        const float *pair_sigma, int b, const int8_t *H, double *x /*2P*/,
                        double *y /*d_in, rotated unit row*/, double *norm_out)
{
    double *ws = (double *)malloc(sizeof(double) * (size_t)d_in);
    double s2 = 0.0;
    for (int j = 0; j < d_in; ++j) {
        ws[j] = (double)w[j] * (chan_scale ? (double)chan_scale[j] : 1.0);
        s2 += ws[j] * ws[j];
    }
    double r = sqrt(s2);
    for (int j = 0; j < d_in; ++j)
        ws[j] = (r > 0.0) ? ws[j] / r : 0.0;
    rotate_fwd_truth(ws, d_in, b, signs, H, y);
    for (int k = 0; k < d_in / 2; ++k) {
        double sig = pair_sigma ? (double)pair_sigma[k] : 1.0 / sqrt((double)d_in);
        x[2 * k] = y[2 * k] / sig;
        x[2 * k + 1] = y[2 * k + 1] / sig;
    }
    *norm_out = r;
    free(ws);
}

static void front_spec(const float *w, int d_in, const float *chan_scale, const int8_t *signs,
                       const float *pair_sigma, int b, float *x /*2P*/, float *y /*d_in*/,
                       float *norm_out)
{
    float *u = (float *)malloc(sizeof(float) * (size_t)d_in);
    double s2 = 0.0;
    for (int j = 0; j < d_in; ++j) {
        volatile float p = chan_scale ? w[j] * chan_scale[j] : w[j]; /* fl32(W*s) */
        u[j] = p;
        s2 += (double)p * (double)p; /* exact products, fp64 running sum */
    }
    volatile float r = (float)sqrt(s2);
    for (int j = 0; j < d_in; ++j) {
        volatile float q = (r > 0.0f) ? u[j] / r : 0.0f; /* IEEE fp32 division */
        u[j] = q;
    }
    rotate_fwd_spec(u, d_in, b, signs, y);
    volatile float g_default = (float)sqrt((double)d_in);
    for (int k = 0; k < d_in / 2; ++k) {
        volatile float g = g_default;
        if (pair_sigma)
            g = 1.0f / pair_sigma[k]; /* fl32(1/sigma_k) */
        volatile float x0 = y[2 * k] * g;
        volatile float x1 = y[2 * k + 1] * g;
        x[2 * k] = x0;
        x[2 * k + 1] = x1;
    }
    *norm_out = r;
    free(u);
}

/* Sec. 3.5: nearest codebook entry by Euclidean distance, all K evaluated in fp64,
 * lowest index wins exact ties.  Also returns the two smallest squared distances. */
static int32_t nearest(double x0, double x1, const float *codebook, int K, double *d1_out,
                       double *d2_out)
{
    int32_t best = 0;
    double d1 = INFINITY, d2 = INFINITY;
    for (int c = 0; c < K; ++c) {
        double e0 = x0 - (double)codebook[2 * c];
        double e1 = x1 - (double)codebook[2 * c + 1];
        double d = e0 * e0 + e1 * e1;
        if (d < d1) {
            d2 = d1;
            d1 = d;
            best = c;
        } else if (d < d2) {
            d2 = d;
        }
    }
    *d1_out = d1;
    *d2_out = d2;
    return best;
}

/*
 * Encode rows [row0,row1) of a row-major fp32 matrix (leading dimension ldw).
 * Outputs are indexed by absolute row: idx[i*P + k], norms[i], d1/d2[i*P + k] (nullable),
 * x_out[(i*P + k)*2 + e] (nullable; the normalised pairs the argmin saw).
 */
int orc_encode_rows(const float *W, int64_t ldw, int row0, int row1, int d_in,
                    const float *chan_scale, const int8_t *signs, const float *pair_sigma,
                    const float *codebook, int bits, int block, int mode, int32_t *idx,
                    double *norms, double *d1, double *d2, double *x_out)
{
    if (d_in <= 0 || (d_in & 1) || block < 2 || (block & (block - 1)) || d_in % block ||
        bits < 1 || bits > 12)
        return ORC_ERR;
    int P = d_in / 2, K = 1 << bits;
    int8_t *H = NULL;
    if (mode == 0) {
        H = (int8_t *)malloc((size_t)block * block);
        orc_hadamard(block, H);
    }
    double *xd = (double *)malloc(sizeof(double) * (size_t)d_in);
    double *yd = (double *)malloc(sizeof(double) * (size_t)d_in);
    float *xf = (float *)malloc(sizeof(float) * (size_t)d_in);
    float *yf = (float *)malloc(sizeof(float) * (size_t)d_in);
    for (int i = row0; i < row1; ++i) {
        const float *w = W + (size_t)i * (size_t)ldw;
        if (mode == 0) {
            front_truth(w, d_in, chan_scale, signs, pair_sigma, block, H, xd, yd, &norms[i]);
        } else {
            float r;
            front_spec(w, d_in, chan_scale, signs, pair_sigma, block, xf, yf, &r);
            norms[i] = (double)r;
            for (int j = 0; j < d_in; ++j)
                xd[j] = (double)xf[j];
        }
        for (int k = 0; k < P; ++k) {
            double a, b2;
            idx[(size_t)i * P + k] = nearest(xd[2 * k], xd[2 * k + 1], codebook, K, &a, &b2);
            if (d1)
                d1[(size_t)i * P + k] = a;
            if (d2)
                d2[(size_t)i * P + k] = b2;
            if (x_out) {
                x_out[((size_t)i * P + k) * 2] = xd[2 * k];
                x_out[((size_t)i * P + k) * 2 + 1] = xd[2 * k + 1];
            }
        }
    }
    free(xd);
    free(yd);
    free(xf);
    free(yf);
    free(H);
    return ORC_OK;
}

/* ------------------------------------------------------------------------- */
/* Sec. 3.1 step 6 / Sec. 3.2: the bit-packed byte stream of one row.  Pair k */
/* occupies stream bits [k*B, (k+1)*B), least significant bit first; stream   */
/* bit n is bit (n mod 8) of byte floor(n/8); unused bits are zero.           */
/* ------------------------------------------------------------------------- */
int64_t orc_packed_row_bytes(int d_in, int bits)
{
    int64_t nbits = (int64_t)(d_in / 2) * bits;
    int64_t bytes = (nbits + 7) / 8;
    return (bytes + 3) / 4 * 4; /* row stride rounded up to 4 bytes */
}

void orc_pack_row(const int32_t *idx, int P, int bits, uint8_t *row, int64_t row_bytes)
{
    memset(row, 0, (size_t)row_bytes);
    for (int k = 0; k < P; ++k)
        for (int t = 0; t < bits; ++t)
            if ((idx[k] >> t) & 1) {
                int64_t n = (int64_t)k * bits + t;
                row[n / 8] |= (uint8_t)(1u << (n % 8));
            }
}

void orc_unpack_row(const uint8_t *row, int P, int bits, int32_t *idx)
{
    for (int k = 0; k < P; ++k) {
        int32_t v = 0;
        for (int t = 0; t < bits; ++t) {
            int64_t n = (int64_t)k * bits + t;
            if ((row[n / 8] >> (n % 8)) & 1)
                v |= (1 << t);
        }
        idx[k] = v;
    }
}

/* ------------------------------------------------------------------------- */
/* Decoder, Sec. 3.2 + Sec. B.2: centroid lookup, times sigma_k, inverse      */
/* rotation R_inv = S F, times the stored row norm, times 1/s_j; bf16 output. */
/* w_pre (nullable) receives the value before the bf16 cast, w_bf16 (nullable, */
/* spec mode only) the cast.  Both [rows][d_in], indexed by absolute row.      */
/* yhat_out (nullable) receives the reconstructed rotated unit row.            */
/* ------------------------------------------------------------------------- */
int orc_decode_rows(const int32_t *idx, int row0, int row1, int d_in, const float *norms,
                    const float *chan_scale, const int8_t *signs, const float *pair_sigma,
                    const float *codebook, int bits, int block, int mode, double *w_pre,
                    uint16_t *w_bf16, double *yhat_out)
{
    if (d_in <= 0 || (d_in & 1) || block < 2 || (block & (block - 1)) || d_in % block ||
        bits < 1 || bits > 12)
        return ORC_ERR;
    int P = d_in / 2;
    int8_t *H = NULL;
    if (mode == 0) {
        H = (int8_t *)malloc((size_t)block * block);
        orc_hadamard(block, H);
    }
    double *yd = (double *)malloc(sizeof(double) * (size_t)d_in);
    double *ud = (double *)malloc(sizeof(double) * (size_t)d_in);
    float *tf = (float *)malloc(sizeof(float) * (size_t)d_in);
    for (int i = row0; i < row1; ++i) {
        const int32_t *ix = idx + (size_t)i * P;
        if (mode == 0) {
            for (int k = 0; k < P; ++k) {
                double sig = pair_sigma ? (double)pair_sigma[k] : 1.0 / sqrt((double)d_in);
                yd[2 * k] = sig * (double)codebook[2 * ix[k]];
                yd[2 * k + 1] = sig * (double)codebook[2 * ix[k] + 1];
            }
            rotate_inv_truth(yd, d_in, block, signs, H, ud);
            for (int j = 0; j < d_in; ++j) {
                double v = (double)norms[i] * ud[j];
                if (chan_scale)
                    v = v / (double)chan_scale[j];
                if (w_pre)
                    w_pre[(size_t)i * d_in + j] = v;
                if (yhat_out)
                    yhat_out[(size_t)i * d_in + j] = yd[j];
            }
        } else {
            volatile float sig_default = (float)(1.0 / sqrt((double)d_in));
            volatile float cb = (float)(1.0 / sqrt((double)block));
            for (int k = 0; k < P; ++k) {
                volatile float sig = pair_sigma ? pair_sigma[k] : sig_default;
                volatile float y0 = sig * codebook[2 * ix[k]];
                volatile float y1 = sig * codebook[2 * ix[k] + 1];
                tf[2 * k] = y0;
                tf[2 * k + 1] = y1;
                if (yhat_out) {
                    yhat_out[(size_t)i * d_in + 2 * k] = (double)y0;
                    yhat_out[(size_t)i * d_in + 2 * k + 1] = (double)y1;
                }
            }
            for (int blk = 0; blk < d_in / block; ++blk)
                orc_fwht_spec(tf + (size_t)blk * block, block);
            for (int j = 0; j < d_in; ++j) {
                volatile float z = tf[j] * cb;           /* fl32(t * fl32(b^-1/2)) */
                if (signs && signs[j] < 0)
                    z = -z;                              /* S: exact */
                volatile float ws = norms[i] * z;        /* fl32(r * u) */
                volatile float w = ws;
                if (chan_scale) {
                    volatile float q = 1.0f / chan_scale[j]; /* fl32(1/s_j) */
                    w = ws * q;                          /* D_s^-1 as a multiply */
                }
                if (w_pre)
                    w_pre[(size_t)i * d_in + j] = (double)w;
                if (w_bf16)
                    w_bf16[(size_t)i * d_in + j] = orc_bf16_rne(w);
            }
        }
    }
    free(yd);
    free(ud);
    free(tf);
    free(H);
    return ORC_OK;
}

/* ------------------------------------------------------------------------- */
/* Eq. 1: sigma_k = mean_rows(|z_k|) / sqrt(pi/2) over the first              */
/* n = min(d_out, max_rows) unit-normalised, rotated rows.  A zero estimate   */
/* falls back to 1/sqrt(d_in).  Amplitudes and the mean in fp64.              */
/* ------------------------------------------------------------------------- */
int orc_calibrate_sigma(const float *W, int64_t ldw, int d_out, int d_in, const float *chan_scale,
                        const int8_t *signs, int block, int max_rows, int mode, float *sigma_out)
{
    if (d_in <= 0 || (d_in & 1) || block < 2 || (block & (block - 1)) || d_in % block)
        return ORC_ERR;
    int P = d_in / 2;
    int n = d_out < max_rows ? d_out : max_rows;
    int8_t *H = NULL;
    if (mode == 0) {
        H = (int8_t *)malloc((size_t)block * block);
        orc_hadamard(block, H);
    }
    float *unit_sigma = (float *)malloc(sizeof(float) * (size_t)P);
    for (int k = 0; k < P; ++k)
        unit_sigma[k] = 1.0f;
    double *acc = (double *)calloc((size_t)P, sizeof(double));
    double *xd = (double *)malloc(sizeof(double) * (size_t)d_in);
    double *yd = (double *)malloc(sizeof(double) * (size_t)d_in);
    float *xf = (float *)malloc(sizeof(float) * (size_t)d_in);
    float *yf = (float *)malloc(sizeof(float) * (size_t)d_in);
    for (int i = 0; i < n; ++i) {
        const float *w = W + (size_t)i * (size_t)ldw;
        if (mode == 0) {
            double r;
            front_truth(w, d_in, chan_scale, signs, unit_sigma, block, H, xd, yd, &r);
        } else {
            float r;
            front_spec(w, d_in, chan_scale, signs, unit_sigma, block, xf, yf, &r);
            for (int j = 0; j < d_in; ++j)
                yd[j] = (double)yf[j];
        }
        for (int k = 0; k < P; ++k)
            acc[k] += sqrt(yd[2 * k] * yd[2 * k] + yd[2 * k + 1] * yd[2 * k + 1]);
    }
    const double sqrt_half_pi = 1.2533141373155002512078826424055;
    for (int k = 0; k < P; ++k) {
        double s = (acc[k] / (double)n) / sqrt_half_pi;
        float sf = (float)s;
        if (!(sf > 0.0f))
            sf = (float)(1.0 / sqrt((double)d_in));
        sigma_out[k] = sf;
    }
    free(unit_sigma);
    free(acc);
    free(xd);
    free(yd);
    free(xf);
    free(yf);
    free(H);
    return ORC_OK;
}

/* ------------------------------------------------------------------------- */
/* Sec. 3.5: Lloyd iterations for a K-point codebook on samples of the unit   */
/* circular Gaussian.  codebook holds the initial points on entry and the     */
/* trained points on return (fp64, K x 2).                                    */
/*   repeat: assign every sample to its nearest point (lowest index on ties); */
/*           D = mean squared error of that assignment;                       */
/*           stop if iteration > 0 and |D_prev - D| < tol * D_prev;           */
/*           move every point to the mean of its samples; an empty cell is    */
/*           moved onto the sample with the largest current error.            */
/* The points are not moved after the last assignment (convergence or         */
/* max_iters), so the returned points and mse_out belong together.            */
/* ------------------------------------------------------------------------- */
void orc_codebook_init(int K, double *codebook)
{
    /* Golden-angle spiral; radius of point i is the (i+0.5)/K quantile of the
     * radial law of a circular Gaussian of variance 2 per axis (the high-rate
     * optimal point density for this source is proportional to sqrt(f)). */
    const double golden = 2.3999632297286533222315555066336; /* pi*(3-sqrt(5)) */
    for (int i = 0; i < K; ++i) {
        double q = ((double)i + 0.5) / (double)K;
        double rad = sqrt(-4.0 * log(1.0 - q));
        double th = golden * (double)i;
        codebook[2 * i] = rad * cos(th);
        codebook[2 * i + 1] = rad * sin(th);
    }
}

int orc_lloyd(const double *samples, int64_t n, int K, double *codebook, int max_iters,
              double tol, double *mse_out, int *iters_out)
{
    int32_t *assign = (int32_t *)malloc(sizeof(int32_t) * (size_t)n);
    double *err = (double *)malloc(sizeof(double) * (size_t)n);
    double *sum = (double *)malloc(sizeof(double) * 2 * (size_t)K);
    int64_t *cnt = (int64_t *)malloc(sizeof(int64_t) * (size_t)K);
    double prev = INFINITY, D = INFINITY;
    int it = 0;
    for (it = 0; it < max_iters; ++it) {
        double tot = 0.0;
        for (int64_t s = 0; s < n; ++s) {
            double best = INFINITY;
            int32_t bi = 0;
            for (int c = 0; c < K; ++c) {
                double e0 = samples[2 * s] - codebook[2 * c];
                double e1 = samples[2 * s + 1] - codebook[2 * c + 1];
                double d = e0 * e0 + e1 * e1;
                if (d < best) {
                    best = d;
                    bi = c;
                }
            }
            assign[s] = bi;
            err[s] = best;
            tot += best;
        }
        D = tot / (double)n;
        if ((it > 0 && fabs(prev - D) < tol * prev) || it == max_iters - 1) {
            ++it;
            break; /* the points are not moved after the last assignment */
        }
        prev = D;
        memset(sum, 0, sizeof(double) * 2 * (size_t)K);
        memset(cnt, 0, sizeof(int64_t) * (size_t)K);
        for (int64_t s = 0; s < n; ++s) {
            sum[2 * assign[s]] += samples[2 * s];
            sum[2 * assign[s] + 1] += samples[2 * s + 1];
            cnt[assign[s]]++;
        }
        for (int c = 0; c < K; ++c) {
            if (cnt[c] > 0) {
                codebook[2 * c] = sum[2 * c] / (double)cnt[c];
                codebook[2 * c + 1] = sum[2 * c + 1] / (double)cnt[c];
            } else {
                int64_t worst = 0;
                for (int64_t s = 1; s < n; ++s)
                    if (err[s] > err[worst])
                        worst = s;
                codebook[2 * c] = samples[2 * worst];
                codebook[2 * c + 1] = samples[2 * worst + 1];
                err[worst] = 0.0;
            }
        }
    }
    *mse_out = D;
    *iters_out = it;
    free(assign);
    free(err);
    free(sum);
    free(cnt);
    return ORC_OK;
}

/* One nearest-neighbour pass over samples (fp64): assignment, squared error per
 * sample.  Used to check the Lloyd conditions of any codebook on fresh samples. */
void orc_assign(const double *samples, int64_t n, const double *codebook, int K, int32_t *assign,
                double *err)
{
    for (int64_t s = 0; s < n; ++s) {
        double best = INFINITY;
        int32_t bi = 0;
        for (int c = 0; c < K; ++c) {
            double e0 = samples[2 * s] - codebook[2 * c];
            double e1 = samples[2 * s + 1] - codebook[2 * c + 1];
            double d = e0 * e0 + e1 * e1;
            if (d < best) {
                best = d;
                bi = c;
            }
        }
        assign[s] = bi;
        err[s] = best;
    }
}

/* ------------------------------------------------------------------------- */
/* Polar baseline (Sec. 3 "Polar Baseline"; Thm. "Polar QAM pair distortion   */
/* decomposition"; Cor. "Rayleigh-Lloyd polar distortion bound" and the       */
/* remark after it).                                                          */
/*                                                                            */
/* Amplitude: an Na-level Lloyd-Max quantiser for the unit Rayleigh density   */
/* f(r) = r exp(-r^2/2), integrated up to the cutoff rmax (the remark: 8).    */
/* Lloyd-Max fixed point: thresholds at the midpoints of neighbouring levels, */
/* levels at the centroids of their cells.  The three integrals needed have   */
/* closed forms:                                                              */
/*   int f      = -exp(-r^2/2)                                                */
/*   int r f    = -r exp(-r^2/2) + sqrt(pi/2) erf(r/sqrt 2)                   */
/*   int r^2 f  = -(r^2 + 2) exp(-r^2/2)                                      */
/* Start: level i at the (i+0.5)/Na quantile, sqrt(-2 ln(1 - q)).             */
/* Returns the number of iterations; c_lm_out = E (U - Q(U))^2 of the final   */
/* levels for the untruncated Rayleigh law (last cell runs to infinity).      */
/* ------------------------------------------------------------------------- */
static double ray_i0(double r) { return -exp(-0.5 * r * r); }
static double ray_i1(double r) { return -r * exp(-0.5 * r * r) + sqrt(M_PI / 2.0) * erf(r / sqrt(2.0)); }
static double ray_i2(double r) { return -(r * r + 2.0) * exp(-0.5 * r * r); }

double orc_rayleigh_distortion(const double *levels, int Na)
{
    double D = 0.0;
    for (int i = 0; i < Na; ++i) {
        double lo = (i == 0) ? 0.0 : 0.5 * (levels[i - 1] + levels[i]);
        double a = levels[i];
        double m0, m1, m2;
        if (i == Na - 1) { /* to infinity: i0 -> 0, i1 -> sqrt(pi/2), i2 -> 0 */
            m0 = 0.0 - ray_i0(lo);
            m1 = sqrt(M_PI / 2.0) - ray_i1(lo);
            m2 = 0.0 - ray_i2(lo);
        } else {
            double hi = 0.5 * (levels[i] + levels[i + 1]);
            m0 = ray_i0(hi) - ray_i0(lo);
            m1 = ray_i1(hi) - ray_i1(lo);
            m2 = ray_i2(hi) - ray_i2(lo);
        }
        D += m2 - 2.0 * a * m1 + a * a * m0;
    }
    return D;
}

int orc_rayleigh_lloyd_max(int Na, double rmax, int max_iters, double tol, double *levels,
                           double *c_lm_out)
{
    for (int i = 0; i < Na; ++i)
        levels[i] = sqrt(-2.0 * log(1.0 - ((double)i + 0.5) / (double)Na));
    double *next = (double *)malloc(sizeof(double) * (size_t)Na);
    int it;
    for (it = 0; it < max_iters; ++it) {
        double move = 0.0;
        for (int i = 0; i < Na; ++i) {
            double lo = (i == 0) ? 0.0 : 0.5 * (levels[i - 1] + levels[i]);
            double hi = (i == Na - 1) ? rmax : 0.5 * (levels[i] + levels[i + 1]);
            double mass = ray_i0(hi) - ray_i0(lo);
            next[i] = (mass > 0.0) ? (ray_i1(hi) - ray_i1(lo)) / mass : levels[i];
            if (fabs(next[i] - levels[i]) > move)
                move = fabs(next[i] - levels[i]);
        }
        memcpy(levels, next, sizeof(double) * (size_t)Na);
        if (move < tol)
            break;
    }
    free(next);
    if (c_lm_out)
        *c_lm_out = orc_rayleigh_distortion(levels, Na);
    return it;
}

/* The 2^B-entry table that makes the polar code a plain lookup: entry ia*Np + ip is the point with  */
/* amplitude levels[ia] and phase (2 ip + 1) h, h = pi / Np (bin centres of Cor. 1).  The           */
/* amplitude-major index order is this implementation's choice (the paper fixes none).              */
void orc_polar_table(const float *levels, int Na, int Np, float *table)
{
    double h = M_PI / (double)Np;
    for (int ia = 0; ia < Na; ++ia)
        for (int ip = 0; ip < Np; ++ip) {
            double ph = (2.0 * (double)ip + 1.0) * h;
            table[2 * ((size_t)ia * Np + ip)] = (float)((double)levels[ia] * cos(ph));
            table[2 * ((size_t)ia * Np + ip) + 1] = (float)((double)levels[ia] * sin(ph));
        }
}

/* Polar quantisation of n points (x0, x1): amplitude |x| to the nearest level (lowest index on a    */
/* tie), phase atan2(x1, x0), taken in [0, 2 pi), to the bin [2 k h, 2 (k+1) h) whose centre          */
/* (2k+1) h is the nearest phase level.  The origin has phase 0.  Also returned, for the             */
/* acceptance test of a lower-precision implementation: how close each decision was --               */
/* amp_margin = |a - nearest threshold| / a (infinity with one level or a = 0),                      */
/* phase_margin = angular distance to the nearest bin boundary in radians.                           */
void orc_polar_quantize(const double *x, int64_t n, const float *levels, int Na, int Np,
                        int32_t *idx, double *amp_margin, double *phase_margin)
{
    double two_h = 2.0 * M_PI / (double)Np;
    for (int64_t s = 0; s < n; ++s) {
        double x0 = x[2 * s], x1 = x[2 * s + 1];
        double a = sqrt(x0 * x0 + x1 * x1);
        int ia = 0;
        double best = INFINITY;
        for (int i = 0; i < Na; ++i) {
            double d = fabs(a - (double)levels[i]);
            if (d < best) {
                best = d;
                ia = i;
            }
        }
        double am = INFINITY;
        for (int i = 1; i < Na; ++i) {
            double t = 0.5 * ((double)levels[i - 1] + (double)levels[i]);
            double m = fabs(a - t);
            if (m < am)
                am = m;
        }
        double th = (a > 0.0) ? atan2(x1, x0) : 0.0;
        if (th < 0.0)
            th += 2.0 * M_PI;
        int ip = (int)floor(th / two_h);
        if (ip >= Np)
            ip = Np - 1; /* th rounded up to 2 pi */
        double off = th - (double)ip * two_h;
        double pm = off < two_h - off ? off : two_h - off;
        idx[s] = ia * Np + ip;
        if (amp_margin)
            amp_margin[s] = (a > 0.0) ? am / a : INFINITY;
        if (phase_margin)
            phase_margin[s] = (a > 0.0) ? pm : INFINITY;
    }
}
