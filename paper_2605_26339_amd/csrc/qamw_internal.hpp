// Internal launch interface between libqamw's entry points and its kernel files.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace qamw {

// Everything a codec kernel needs to know about one matrix.  Host-computed constants are passed
// in so that host and device agree on them bit for bit.
struct Problem {
    int d_out = 0, d_in = 0;
    int bits = 0, K = 0, block = 0;
    const float *chan_scale = nullptr;   // device, d_in, nullable
    const int8_t *signs = nullptr;       // device, d_in, nullable
    const float *pair_sigma = nullptr;   // device, d_in/2, nullable
    const float *codebook = nullptr;     // device, K x 2
    float inv_sqrt_block = 0.f;          // fp32(block^-1/2)
    float g_default = 0.f;               // fp32(sqrt(d_in)): pair gain when no sigma is given
    float sigma_default = 0.f;           // fp32(d_in^-1/2)
    int64_t row_bytes = 0;               // packed row stride
    unsigned long long *full_scans = nullptr;   // device counter of pairs decided by the exact whole-codebook scan, nullable
    hipStream_t stream = nullptr;
};

// General kernels: any even d_in, any power-of-two block <= 1024 dividing d_in.
hipError_t launch_row_norms(const void *W, int dtype, int64_t ldw, int n_rows, const Problem &p, float *norms);
hipError_t launch_encode_general(const void *W, int dtype, int64_t ldw, const Problem &p, const float *norms,
                                 uint8_t *packed);
hipError_t launch_decode_general(const uint8_t *packed, const float *norms, const Problem &p, void *out,
                                 int64_t ldo, bool out_bf16);
hipError_t launch_calibrate_general(const void *W, int dtype, int64_t ldw, int n_rows, const Problem &p,
                                    const float *norms, float *sigma_out);

// Vectorised row norms: returns false (nothing launched) when alignment rules it out.
bool launch_row_norms_fast(const void *W, int dtype, int64_t ldw, int n_rows, const Problem &p, float *norms,
                           hipError_t *err);
// Two-step calibration through caller-provided partial sums (calibrate_partial_bytes() of them).
size_t calibrate_partial_bytes(int d_in, int n_rows);
bool fast_calibrate_supported(const void *W, int dtype, int64_t ldw, const Problem &p);
hipError_t launch_calibrate_fast(const void *W, int dtype, int64_t ldw, int n_rows, const Problem &p, double *partial,
                                 float *sigma_out);
// Several matrices in one pair of launches (every item checked with fast_calibrate_supported() by the caller).
constexpr int CAL_MAX_BATCH = 32;
struct CalItem {
    const void *W;
    int64_t ldw;
    const float *chan_scale;
    const int8_t *signs;
    double *partial;                      // calibrate_partial_bytes(d_in, n_rows) bytes
    float *sigma_out;
    int n_rows, d_in;                     // n_rows: the head rows used
};
hipError_t launch_calibrate_batch_fast(const CalItem *items, int n, int dtype, int block, hipStream_t stream);

// One matrix of a decode batch (host-side description).
constexpr int QAMW_DECODE_MAX_BATCH = 32;
struct DecodeItem {
    const uint8_t *packed;
    const float *norms;
    const float *chan_scale;
    const int8_t *signs;
    const float *pair_sigma;
    void *out;
    int64_t ldo;
    int d_out, d_in;
};
// Several matrices sharing codebook, bits and block in ONE launch; hipErrorNotSupported = nothing launched.
// traffic_only: the loads and stores of the bf16 decoder without its arithmetic (a measurement of the memory system).
hipError_t launch_decode_batch_fast(const DecodeItem *items, int n, const Problem &p, bool out_bf16, bool traffic_only = false);

// Fast kernels: return hipErrorNotSupported when the shape is outside what they cover.
bool fast_decode_supported(const Problem &p);
hipError_t launch_decode_fast(const uint8_t *packed, const float *norms, const Problem &p, void *out,
                              int64_t ldo, bool out_bf16);
bool fast_encode_supported(const Problem &p);
// norms_ready = false: the kernel computes the row norms itself (one read of W) and writes them to `norms`.
hipError_t launch_encode_fast(const void *W, int dtype, int64_t ldw, const Problem &p, float *norms, bool norms_ready,
                              uint8_t *packed);
bool fused_norms_supported(const Problem &p);   // rows short enough for the kernels to compute their own norms
bool polar_encode_launchable(const void *W, int dtype, int64_t ldw, const Problem &p, int bits_a, int bits_p);
hipError_t launch_encode_polar(const void *W, int dtype, int64_t ldw, const Problem &p, const float *levels, int bits_a,
                               int bits_p, float *norms, bool norms_ready, uint8_t *packed);
bool matmul_supported(const Problem &p, int m);
size_t matmul_workspace_bytes(int d_in, int d_out, int m);
constexpr int QAMW_MATMUL_MAX_BATCH = 16;
struct MatmulItem {
    const void *X;
    int64_t ldx;
    const uint8_t *packed;
    const float *norms, *chan_scale;
    const int8_t *signs;
    const float *pair_sigma;
    float *Y;
    int64_t ldy;
    int d_out, d_in;
};
hipError_t launch_matmul_batch(const MatmulItem *items, int n, int xdtype, int m, const Problem &p, void *workspace, int variant);
size_t lloyd_workspace_bytes(int K);
hipError_t run_lloyd(const float *samples, long long n, int K, float *codebook, int max_iters, double tol, void *workspace,
                     double *mse_out, int *iters_out, hipStream_t stream);
bool pairs_launchable(const void *W, int dtype, int64_t ldw, const Problem &p, const float *pairs);
hipError_t launch_pairs(const void *W, int dtype, int64_t ldw, const Problem &p, float *norms, bool norms_ready, float *pairs);
// The pruned-search table in device memory (layout: qamw_search_grid_build) and its grid size, which follows from bits.
struct SearchGridView {
    const void *table;
    int G;
    int variant = 0;   // 0: chosen by size; 1: every record from global memory; 2: central cells in LDS whatever the size
};
bool grid_encode_launchable(const void *W, int dtype, int64_t ldw, const Problem &p, const SearchGridView &g);
hipError_t launch_encode_grid(const void *W, int dtype, int64_t ldw, const Problem &p, const SearchGridView &g,
                              const float *norms, uint8_t *packed);
bool mfma_encode_supported(const Problem &p);
hipError_t launch_encode_mfma(const void *W, int dtype, int64_t ldw, const Problem &p, float *norms, bool norms_ready,
                              uint8_t *packed);
// One matrix of an encode batch (host-side description) and the batch launch of the matrix-core encoder.
constexpr int QAMW_ENCODE_MAX_BATCH = 32;
struct EncodeItem {
    const void *W;
    int64_t ldw;
    const float *chan_scale;
    const int8_t *signs;
    const float *pair_sigma;
    float *norms;
    uint8_t *packed;
    int d_out, d_in;
};
hipError_t launch_encode_batch_mfma(const EncodeItem *items, int n, int dtype, const Problem &p, bool norms_ready);

}  // namespace qamw
