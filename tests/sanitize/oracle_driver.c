/* Runs every exported function of the CPU oracle on small inputs with exactly sized heap buffers, so that a build
 * with -fsanitize=address,undefined reports any access outside them and any undefined arithmetic.  Values are
 * only sanity-checked here (the pins live in the Python tests); the exit status is what the test reads. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

void orc_hadamard(int b, int8_t *H);
int orc_paper_block_size(int d_in);
double orc_bpw(int d_in, int d_out, int bits, int with_f16_scales);
void orc_sign_mask(uint64_t seed, int d_in, int8_t *signs);
void orc_gauss_samples(uint64_t seed, int64_t n, double *xy);
void orc_channel_scales(const float *act_rms, int d_in, double alpha, float *s_out);
void orc_fwht_spec(float *t, int b);
void orc_rotate_fwd_truth(const double *v, int d_in, int b, const int8_t *signs, double *y);
void orc_rotate_inv_truth(const double *yh, int d_in, int b, const int8_t *signs, double *u);
void orc_rotate_fwd_spec(const float *u, int d_in, int b, const int8_t *signs, float *y);
int orc_encode_rows(const float *W, int64_t ldw, int row0, int row1, int d_in, const float *chan_scale, const int8_t *signs,
                    const float *pair_sigma, const float *codebook, int bits, int block, int mode, int32_t *idx, double *norms,
                    double *d1, double *d2, double *x_out);
int64_t orc_packed_row_bytes(int d_in, int bits);
void orc_pack_row(const int32_t *idx, int P, int bits, uint8_t *row, int64_t row_bytes);
void orc_unpack_row(const uint8_t *row, int P, int bits, int32_t *idx);
int orc_decode_rows(const int32_t *idx, int row0, int row1, int d_in, const float *norms, const float *chan_scale,
                    const int8_t *signs, const float *pair_sigma, const float *codebook, int bits, int block, int mode,
                    double *w_pre, uint16_t *w_bf16, double *yhat_out);
int orc_calibrate_sigma(const float *W, int64_t ldw, int d_out, int d_in, const float *chan_scale, const int8_t *signs, int block,
                        int max_rows, int mode, float *sigma_out);
void orc_codebook_init(int K, double *codebook);
int orc_lloyd(const double *samples, int64_t n, int K, double *codebook, int max_iters, double tol, double *mse_out, int *iters_out);
void orc_assign(const double *samples, int64_t n, const double *codebook, int K, int32_t *assign, double *err);
uint16_t orc_bf16_rne(float x);
double orc_rayleigh_distortion(const double *levels, int Na);
int orc_rayleigh_lloyd_max(int Na, double rmax, int max_iters, double tol, double *levels, double *c_lm_out);
void orc_polar_table(const float *levels, int Na, int Np, float *table);
void orc_polar_quantize(const double *x, int64_t n, const float *levels, int Na, int Np, int32_t *idx, double *amp_margin,
                        double *phase_margin);

#define NEW(T, n) ((T *)malloc(sizeof(T) * (size_t)(n)))
static int fails = 0;
#define EXPECT(c) do { if (!(c)) { printf("FAILED: %s (line %d)\n", #c, __LINE__); ++fails; } } while (0)

static void codec(int d_out, int d_in, int bits, int block, int mode, int with_side)
{
    const int P = d_in / 2, K = 1 << bits;
    float *W = NEW(float, d_out * d_in), *s = NEW(float, d_in), *rms = NEW(float, d_in), *sigma = NEW(float, P), *cb = NEW(float, 2 * K);
    int8_t *sg = NEW(int8_t, d_in);
    double *xy = NEW(double, 2 * (d_out * d_in / 2 + K + d_in));
    orc_gauss_samples(7 + (uint64_t)d_in, d_out * d_in / 2 + K + d_in, xy);
    for (int i = 0; i < d_out * d_in; ++i) W[i] = (float)xy[i];
    for (int i = 0; i < 2 * K; ++i) cb[i] = (float)xy[d_out * d_in + i];
    for (int j = 0; j < d_in; ++j) rms[j] = (float)exp(xy[d_out * d_in + 2 * K + j]);
    if (d_out > 2) memset(W + (size_t)2 * d_in, 0, sizeof(float) * (size_t)d_in);       /* a zero row */
    orc_channel_scales(rms, d_in, 0.3, s);
    orc_sign_mask(3, d_in, sg);
    EXPECT(orc_calibrate_sigma(W, d_in, d_out, d_in, with_side ? s : NULL, with_side ? sg : NULL, block, 1024, mode, sigma) == 0);
    int32_t *idx = NEW(int32_t, d_out * P), *back = NEW(int32_t, P);
    double *norms = NEW(double, d_out), *d1 = NEW(double, d_out * P), *d2 = NEW(double, d_out * P), *x = NEW(double, d_out * d_in);
    EXPECT(orc_encode_rows(W, d_in, 0, d_out, d_in, with_side ? s : NULL, with_side ? sg : NULL, with_side ? sigma : NULL, cb, bits,
                           block, mode, idx, norms, d1, d2, x) == 0);
    const int64_t rb = orc_packed_row_bytes(d_in, bits);
    uint8_t *row = NEW(uint8_t, rb);
    for (int i = 0; i < d_out; ++i) {
        orc_pack_row(idx + (size_t)i * P, P, bits, row, rb);
        orc_unpack_row(row, P, bits, back);
        EXPECT(memcmp(back, idx + (size_t)i * P, sizeof(int32_t) * (size_t)P) == 0);
    }
    float *nf = NEW(float, d_out);
    for (int i = 0; i < d_out; ++i) nf[i] = (float)norms[i];
    double *w = NEW(double, d_out * d_in), *yh = NEW(double, d_out * d_in);
    uint16_t *bf = NEW(uint16_t, d_out * d_in);
    EXPECT(orc_decode_rows(idx, 0, d_out, d_in, nf, with_side ? s : NULL, with_side ? sg : NULL, with_side ? sigma : NULL, cb, bits,
                           block, mode, w, mode == 1 ? bf : NULL, yh) == 0);
    for (int i = 0; i < d_out * d_in; ++i) EXPECT(isfinite(w[i]));
    free(W); free(s); free(rms); free(sigma); free(cb); free(sg); free(xy); free(idx); free(back); free(norms); free(d1); free(d2);
    free(x); free(row); free(nf); free(w); free(yh); free(bf);
}

int main(void)
{
    for (int b = 2; b <= 64; b <<= 1) {
        int8_t *H = NEW(int8_t, b * b);
        orc_hadamard(b, H);
        long dot = 0;
        for (int j = 0; j < b; ++j) dot += H[j] * H[b + j];
        EXPECT(dot == 0);
        free(H);
    }
    EXPECT(orc_paper_block_size(5632) == 512 && orc_paper_block_size(2048) == 1024 && orc_paper_block_size(6) == 2);
    EXPECT(fabs(orc_bpw(2048, 2048, 11, 0) - 5.5078125) < 1e-12 && orc_bpw(2048, 5632, 7, 1) > 3.5);
    for (int d = 1; d <= 130; d += 43) {
        int8_t *sg = NEW(int8_t, d);
        orc_sign_mask(0x9E3779B97F4A7C15ull, d, sg);
        for (int j = 0; j < d; ++j) EXPECT(sg[j] == 1 || sg[j] == -1);
        free(sg);
    }
    {
        float t[32];
        double v[48], y[48], u[48];
        float uf[48], yf[48];
        int8_t sg[48];
        orc_sign_mask(5, 48, sg);
        for (int i = 0; i < 32; ++i) t[i] = (float)(i % 7) - 3.0f;
        orc_fwht_spec(t, 32);
        for (int i = 0; i < 48; ++i) { v[i] = sin(i + 1.0); uf[i] = (float)v[i]; }
        orc_rotate_fwd_truth(v, 48, 16, sg, y);
        orc_rotate_inv_truth(y, 48, 16, sg, u);
        for (int i = 0; i < 48; ++i) EXPECT(fabs(u[i] - v[i]) < 1e-12);
        orc_rotate_fwd_spec(uf, 48, 16, NULL, yf);
    }
    codec(5, 24, 3, 8, 0, 1);
    codec(5, 24, 3, 8, 1, 1);
    codec(3, 2, 1, 2, 1, 0);
    codec(4, 256, 5, 128, 1, 1);
    codec(7, 96, 12, 32, 0, 0);
    codec(2, 2048, 7, 1024, 1, 1);
    {
        const int n = 4096, K = 16;
        double *xy = NEW(double, 2 * n), *cb = NEW(double, 2 * K), *err = NEW(double, n), mse = 0.0;
        int32_t *as = NEW(int32_t, n);
        int iters = 0;
        orc_gauss_samples(11, n, xy);
        orc_codebook_init(K, cb);
        EXPECT(orc_lloyd(xy, n, K, cb, 25, 1e-6, &mse, &iters) == 0 && mse > 0.0 && iters >= 1);
        orc_assign(xy, n, cb, K, as, err);
        for (int i = 0; i < n; ++i) EXPECT(as[i] >= 0 && as[i] < K);
        free(xy); free(cb); free(err); free(as);
    }
    EXPECT(orc_bf16_rne(1.0f) == 0x3F80 && orc_bf16_rne(-2.0f) == 0xC000 && orc_bf16_rne(INFINITY) == 0x7F80);
    (void)orc_bf16_rne(NAN);
    (void)orc_bf16_rne(3.4e38f);
    {
        const int Na = 8, Np = 16, n = 64;
        double *lv = NEW(double, Na), c_lm = 0.0, *x = NEW(double, 2 * n), *am = NEW(double, n), *pm = NEW(double, n);
        float *lf = NEW(float, Na), *table = NEW(float, 2 * Na * Np);
        int32_t *idx = NEW(int32_t, n);
        EXPECT(orc_rayleigh_lloyd_max(Na, 8.0, 20000, 1e-12, lv, &c_lm) > 0 && c_lm > 0.0);
        EXPECT(fabs(orc_rayleigh_distortion(lv, Na) - c_lm) < 1e-6);
        for (int i = 0; i < Na; ++i) lf[i] = (float)lv[i];
        orc_polar_table(lf, Na, Np, table);
        orc_gauss_samples(13, n, x);
        x[0] = x[1] = 0.0;                                                           /* the origin */
        orc_polar_quantize(x, n, lf, Na, Np, idx, am, pm);
        for (int i = 0; i < n; ++i) EXPECT(idx[i] >= 0 && idx[i] < Na * Np);
        free(lv); free(x); free(am); free(pm); free(lf); free(table); free(idx);
    }
    printf(fails ? "oracle driver: %d failed checks\n" : "oracle driver ok\n", fails);
    return fails ? 1 : 0;
}
