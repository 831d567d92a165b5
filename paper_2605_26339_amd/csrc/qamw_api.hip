// libqamw device entry points: argument validation on the host, then kernel dispatch.
#include <atomic>
#include <cmath>
#include <mutex>

#include "qamw.h"
#include "qamw_internal.hpp"

namespace {

std::atomic<int> g_kernel_path{0};

// The packed stream is read and written in 32-bit words (its rows are multiples of 4 bytes).
bool misaligned4(const void *q) { return (reinterpret_cast<uintptr_t>(q) & 3) != 0; }

int check_common(int d_out, int d_in, int bits, int block) {
    if (d_out <= 0 || d_in <= 0 || bits < 1 || bits > QAMW_MAX_BITS) return QAMW_ERR_INVALID_ARG;
    if (d_in & 1) return QAMW_ERR_SHAPE;
    if (block < 2 || block > QAMW_MAX_BLOCK || (block & (block - 1)) || d_in % block) return QAMW_ERR_SHAPE;
    return QAMW_OK;
}

qamw::Problem make_problem(int d_out, int d_in, const float *chan_scale, const int8_t *signs, const float *pair_sigma,
                           const float *codebook, int bits, int block, void *stream) {
    qamw::Problem p;
    p.d_out = d_out;
    p.d_in = d_in;
    p.bits = bits;
    p.K = 1 << bits;
    p.block = block;
    p.chan_scale = chan_scale;
    p.signs = signs;
    p.pair_sigma = pair_sigma;
    p.codebook = codebook;
    p.inv_sqrt_block = (float)(1.0 / std::sqrt((double)block));
    p.g_default = (float)std::sqrt((double)d_in);
    p.sigma_default = (float)(1.0 / std::sqrt((double)d_in));
    size_t rb = 0;
    qamw_packed_row_bytes(d_in, bits, &rb);
    p.row_bytes = (int64_t)rb;
    p.stream = (hipStream_t)stream;
    return p;
}

hipError_t launch_norms(const void *W, int dtype, int64_t ldw, int n_rows, const qamw::Problem &p, float *norms) {
    hipError_t e = hipSuccess;
    if (g_kernel_path.load() != 1 && qamw::launch_row_norms_fast(W, dtype, ldw, n_rows, p, norms, &e)) return e;
    return qamw::launch_row_norms(W, dtype, ldw, n_rows, p, norms);
}

int decode_any(const uint8_t *packed, const float *row_norms, int d_out, int d_in, const float *chan_scale,
               const int8_t *signs, const float *pair_sigma, const float *codebook, int bits, int block, void *out,
               int64_t ldo, void *stream, bool bf16) {
    if (!packed || !row_norms || !codebook || !out || misaligned4(packed)) return QAMW_ERR_INVALID_ARG;
    int rc = check_common(d_out, d_in, bits, block);
    if (rc != QAMW_OK) return rc;
    if (ldo < d_in) return QAMW_ERR_SHAPE;
    qamw::Problem p = make_problem(d_out, d_in, chan_scale, signs, pair_sigma, codebook, bits, block, stream);
    hipError_t e;
    if (g_kernel_path.load() != 1 && qamw::fast_decode_supported(p))
        e = qamw::launch_decode_fast(packed, row_norms, p, out, ldo, bf16);
    else
        e = qamw::launch_decode_general(packed, row_norms, p, out, ldo, bf16);
    return e == hipSuccess ? QAMW_OK : QAMW_ERR_DEVICE;
}

}  // namespace

extern "C" {

int qamw_set_kernel_path(int path) {
    if (path < 0 || path > 2) return g_kernel_path.load();
    return g_kernel_path.exchange(path);
}

static size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

int qamw_calibrate_workspace_bytes(int d_in, int d_out, int max_rows, size_t *bytes_out) {
    if (!bytes_out || max_rows < 1 || d_out <= 0) return QAMW_ERR_INVALID_ARG;
    if (d_in <= 0 || (d_in & 1)) return QAMW_ERR_SHAPE;
    const int n = d_out < max_rows ? d_out : max_rows;
    *bytes_out = align_up((size_t)n * sizeof(float), 256) + qamw::calibrate_partial_bytes(d_in, n);
    return QAMW_OK;
}

static int calibrate_impl(const void *W, int dtype, int d_out, int d_in, int64_t ldw, const float *chan_scale,
                          const int8_t *signs, int hadamard_block, int max_rows, void *workspace, float *sigma_out,
                          void *stream) {
    qamw::Problem p = make_problem(d_out, d_in, chan_scale, signs, nullptr, nullptr, 1, hadamard_block, stream);
    const int n = d_out < max_rows ? d_out : max_rows;
    float *row_norms = static_cast<float *>(workspace);
    double *partial = reinterpret_cast<double *>(static_cast<char *>(workspace) + align_up((size_t)n * sizeof(float), 256));
    hipError_t e;
    if (g_kernel_path.load() != 1 && qamw::fast_calibrate_supported(W, dtype, ldw, p)) {
        e = qamw::launch_calibrate_fast(W, dtype, ldw, n, p, partial, sigma_out);      // computes the rows' norms itself
    } else {
        if (launch_norms(W, dtype, ldw, n, p, row_norms) != hipSuccess) return QAMW_ERR_DEVICE;
        e = qamw::launch_calibrate_general(W, dtype, ldw, n, p, row_norms, sigma_out);
    }
    return e == hipSuccess ? QAMW_OK : QAMW_ERR_DEVICE;
}

static int calibrate_check(const void *W, int dtype, int d_out, int d_in, int64_t ldw, int hadamard_block, int max_rows,
                           const float *sigma_out) {
    if (!W || !sigma_out || max_rows < 1) return QAMW_ERR_INVALID_ARG;
    if (dtype != QAMW_DTYPE_F32 && dtype != QAMW_DTYPE_BF16) return QAMW_ERR_INVALID_ARG;
    int rc = check_common(d_out, d_in, 1, hadamard_block);
    if (rc != QAMW_OK) return rc;
    return ldw < d_in ? QAMW_ERR_SHAPE : QAMW_OK;
}

int qamw_calibrate_sigma(const void *W, int dtype, int d_out, int d_in, int64_t ldw, const float *chan_scale,
                         const int8_t *signs, int hadamard_block, int max_rows, void *workspace,
                         size_t workspace_bytes, float *sigma_out, void *stream) {
    if (!workspace) return QAMW_ERR_INVALID_ARG;
    int rc = calibrate_check(W, dtype, d_out, d_in, ldw, hadamard_block, max_rows, sigma_out);
    if (rc != QAMW_OK) return rc;
    size_t need = 0;
    qamw_calibrate_workspace_bytes(d_in, d_out, max_rows, &need);
    if (workspace_bytes < need || (reinterpret_cast<uintptr_t>(workspace) & 15)) return QAMW_ERR_INVALID_ARG;
    return calibrate_impl(W, dtype, d_out, d_in, ldw, chan_scale, signs, hadamard_block, max_rows, workspace, sigma_out, stream);
}

int qamw_calibrate_sigma_batch(const qamw_calibrate_item *items, int n_items, int dtype, int hadamard_block, int max_rows,
                               void *workspace, size_t workspace_bytes, void *stream) {
    static_assert(QAMW_MAX_BATCH == qamw::CAL_MAX_BATCH, "batch limits differ");
    if (!items || !workspace || n_items < 1 || n_items > QAMW_MAX_BATCH) return QAMW_ERR_INVALID_ARG;
    if (reinterpret_cast<uintptr_t>(workspace) & 15) return QAMW_ERR_INVALID_ARG;
    qamw::CalItem its[QAMW_MAX_BATCH];
    char *ws = static_cast<char *>(workspace);
    size_t used = 0;
    bool fast = g_kernel_path.load() != 1;
    for (int i = 0; i < n_items; ++i) {
        const qamw_calibrate_item &q = items[i];
        int rc = calibrate_check(q.W, dtype, q.d_out, q.d_in, q.ldw, hadamard_block, max_rows, q.sigma_out);
        if (rc != QAMW_OK) return rc;
        size_t need = 0;
        qamw_calibrate_workspace_bytes(q.d_in, q.d_out, max_rows, &need);
        need = align_up(need, 256);
        if (used + need > workspace_bytes) return QAMW_ERR_INVALID_ARG;
        const int n = q.d_out < max_rows ? q.d_out : max_rows;
        double *partial = reinterpret_cast<double *>(ws + used + align_up((size_t)n * sizeof(float), 256));
        its[i] = qamw::CalItem{q.W, q.ldw, q.chan_scale, q.signs, partial, q.sigma_out, n, q.d_in};
        qamw::Problem pi = make_problem(q.d_out, q.d_in, q.chan_scale, q.signs, nullptr, nullptr, 1, hadamard_block, stream);
        fast = fast && qamw::fast_calibrate_supported(q.W, dtype, q.ldw, pi);
        used += need;
    }
    if (fast) {
        hipError_t e = qamw::launch_calibrate_batch_fast(its, n_items, dtype, hadamard_block, (hipStream_t)stream);
        if (e == hipSuccess) return QAMW_OK;
        if (e != hipErrorNotSupported) return QAMW_ERR_DEVICE;
    }
    used = 0;
    for (int i = 0; i < n_items; ++i) {                         // nothing was launched: one call per item, each in its own piece
        const qamw_calibrate_item &q = items[i];
        size_t need = 0;
        qamw_calibrate_workspace_bytes(q.d_in, q.d_out, max_rows, &need);
        int rc = calibrate_impl(q.W, dtype, q.d_out, q.d_in, q.ldw, q.chan_scale, q.signs, hadamard_block, max_rows, ws + used,
                                q.sigma_out, stream);
        if (rc != QAMW_OK) return rc;
        used += align_up(need, 256);
    }
    return QAMW_OK;
}

// ---------------------------------------------------------------------------------------------
// The calibration for callers that cannot allocate: its scratch is this file-scope device array.
// Every device the library runs on holds its own copy at its own address; the name below is only
// the host-side handle of the symbol, the address kernels get is the one hipGetSymbolAddress
// returns for the current device, looked up once per device and kept.
// ---------------------------------------------------------------------------------------------
static __device__ __align__(256) unsigned char scratch[QAMW_STATIC_SCRATCH_BYTES];

namespace {
constexpr int MAX_DEVICES = 64;
std::mutex g_scratch_mutex;
void *g_scratch_ptr[MAX_DEVICES] = {};

// Device address of `scratch` on the current device (nullptr + *err on failure).
void *static_scratch(hipError_t *err) {
    int dev = -1;
    *err = hipGetDevice(&dev);
    if (*err != hipSuccess) return nullptr;
    if (dev < 0 || dev >= MAX_DEVICES) {
        *err = hipErrorInvalidDevice;
        return nullptr;
    }
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *ptr = nullptr;
        *err = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (*err != hipSuccess || !ptr) {
            if (*err == hipSuccess) *err = hipErrorInvalidSymbol;
            return nullptr;
        }
        g_scratch_ptr[dev] = ptr;
    }
    return g_scratch_ptr[dev];
}
}  // namespace

int qamw_calibrate_sigma_static(const void *W, int dtype, int d_out, int d_in, int64_t ldw, const float *chan_scale,
                                const int8_t *signs, int hadamard_block, int max_rows, float *sigma_out, void *stream) {
    int rc = calibrate_check(W, dtype, d_out, d_in, ldw, hadamard_block, max_rows, sigma_out);
    if (rc != QAMW_OK) return rc;
    size_t need = 0;
    qamw_calibrate_workspace_bytes(d_in, d_out, max_rows, &need);
    if (need > (size_t)QAMW_STATIC_SCRATCH_BYTES) return QAMW_ERR_UNSUPPORTED;   // beyond the library's own scratch
    hipError_t e = hipSuccess;
    void *ws = static_scratch(&e);
    if (!ws) {
        (void)hipGetLastError();
        return QAMW_ERR_DEVICE;
    }
    // Nothing in the scratch has to start at zero: the row norms and every partial sum the finishing kernel
    // reads are written by this call's own kernels before they are read.
    return calibrate_impl(W, dtype, d_out, d_in, ldw, chan_scale, signs, hadamard_block, max_rows, ws, sigma_out, stream);
}

static int encode_impl(const void *W, int dtype, int d_out, int d_in, int64_t ldw, const float *chan_scale,
                       const int8_t *signs, const float *pair_sigma, const float *codebook, int bits, int hadamard_block,
                       uint8_t *packed_out, float *row_norms_out, unsigned long long *full_scans, void *stream) {
    if (!W || !codebook || !packed_out || !row_norms_out || misaligned4(packed_out)) return QAMW_ERR_INVALID_ARG;
    if (dtype != QAMW_DTYPE_F32 && dtype != QAMW_DTYPE_BF16) return QAMW_ERR_INVALID_ARG;
    int rc = check_common(d_out, d_in, bits, hadamard_block);
    if (rc != QAMW_OK) return rc;
    if (ldw < d_in) return QAMW_ERR_SHAPE;
    qamw::Problem p = make_problem(d_out, d_in, chan_scale, signs, pair_sigma, codebook, bits, hadamard_block, stream);
    p.full_scans = full_scans;
    // The fast kernels compute the row norms themselves (W is fetched once); rows too long for that, and the general
    // kernels, get them from a launch of their own first.
    const int path = g_kernel_path.load();
    const bool fused = path != 1 && qamw::fused_norms_supported(p);
    if (!fused && launch_norms(W, dtype, ldw, d_out, p, row_norms_out) != hipSuccess) return QAMW_ERR_DEVICE;
    hipError_t e = hipErrorNotSupported;                        // "not supported" = nothing launched yet
    if (path == 0) e = qamw::launch_encode_mfma(W, dtype, ldw, p, row_norms_out, !fused, packed_out);
    if (e == hipErrorNotSupported && path != 1) e = qamw::launch_encode_fast(W, dtype, ldw, p, row_norms_out, !fused, packed_out);
    if (e == hipErrorNotSupported) {
        if (fused && launch_norms(W, dtype, ldw, d_out, p, row_norms_out) != hipSuccess) return QAMW_ERR_DEVICE;
        e = qamw::launch_encode_general(W, dtype, ldw, p, row_norms_out, packed_out);
    }
    return e == hipSuccess ? QAMW_OK : QAMW_ERR_DEVICE;
}

int qamw_encode(const void *W, int dtype, int d_out, int d_in, int64_t ldw, const float *chan_scale,
                const int8_t *signs, const float *pair_sigma, const float *codebook, int bits, int hadamard_block,
                uint8_t *packed_out, float *row_norms_out, void *stream) {
    return encode_impl(W, dtype, d_out, d_in, ldw, chan_scale, signs, pair_sigma, codebook, bits, hadamard_block, packed_out,
                       row_norms_out, nullptr, stream);
}

int qamw_encode_stats(const void *W, int dtype, int d_out, int d_in, int64_t ldw, const float *chan_scale,
                      const int8_t *signs, const float *pair_sigma, const float *codebook, int bits, int hadamard_block,
                      uint8_t *packed_out, float *row_norms_out, unsigned long long *full_scans, void *stream) {
    if (!full_scans) return QAMW_ERR_INVALID_ARG;
    return encode_impl(W, dtype, d_out, d_in, ldw, chan_scale, signs, pair_sigma, codebook, bits, hadamard_block, packed_out,
                       row_norms_out, full_scans, stream);
}

int qamw_encode_batch(const qamw_encode_item *items, int n_items, int dtype, const float *codebook, int bits,
                      int hadamard_block, void *stream) {
    static_assert(QAMW_MAX_BATCH == qamw::QAMW_ENCODE_MAX_BATCH, "batch limits differ");
    if (!items || !codebook || n_items < 1 || n_items > QAMW_MAX_BATCH) return QAMW_ERR_INVALID_ARG;
    if (dtype != QAMW_DTYPE_F32 && dtype != QAMW_DTYPE_BF16) return QAMW_ERR_INVALID_ARG;
    qamw::EncodeItem its[QAMW_MAX_BATCH];
    bool fused = true;
    for (int i = 0; i < n_items; ++i) {
        const qamw_encode_item &q = items[i];
        if (!q.W || !q.packed_out || !q.row_norms_out || misaligned4(q.packed_out)) return QAMW_ERR_INVALID_ARG;
        int rc = check_common(q.d_out, q.d_in, bits, hadamard_block);
        if (rc != QAMW_OK) return rc;
        if (q.ldw < q.d_in) return QAMW_ERR_SHAPE;
        its[i] = qamw::EncodeItem{q.W, q.ldw, q.chan_scale, q.signs, q.pair_sigma, q.row_norms_out, q.packed_out, q.d_out, q.d_in};
        qamw::Problem pi = make_problem(q.d_out, q.d_in, nullptr, nullptr, nullptr, codebook, bits, hadamard_block, stream);
        fused = fused && qamw::fused_norms_supported(pi);
    }
    if (g_kernel_path.load() == 0 && fused) {
        qamw::Problem shared = make_problem(items[0].d_out, items[0].d_in, nullptr, nullptr, nullptr, codebook, bits,
                                            hadamard_block, stream);
        hipError_t e = qamw::launch_encode_batch_mfma(its, n_items, dtype, shared, false);
        if (e == hipSuccess) return QAMW_OK;
        if (e != hipErrorNotSupported) return QAMW_ERR_DEVICE;
    }
    for (int i = 0; i < n_items; ++i) {                         // nothing was launched: one call per item
        const qamw_encode_item &q = items[i];
        int rc = encode_impl(q.W, dtype, q.d_out, q.d_in, q.ldw, q.chan_scale, q.signs, q.pair_sigma, codebook, bits,
                             hadamard_block, q.packed_out, q.row_norms_out, nullptr, stream);
        if (rc != QAMW_OK) return rc;
    }
    return QAMW_OK;
}

int qamw_normalised_pairs(const void *W, int dtype, int d_out, int d_in, int64_t ldw, const float *chan_scale,
                          const int8_t *signs, const float *pair_sigma, int hadamard_block, float *pairs_out,
                          float *row_norms_out, void *stream) {
    if (!W || !pairs_out || !row_norms_out) return QAMW_ERR_INVALID_ARG;
    if (dtype != QAMW_DTYPE_F32 && dtype != QAMW_DTYPE_BF16) return QAMW_ERR_INVALID_ARG;
    int rc = check_common(d_out, d_in, 1, hadamard_block);
    if (rc != QAMW_OK) return rc;
    if (ldw < d_in) return QAMW_ERR_SHAPE;
    qamw::Problem p = make_problem(d_out, d_in, chan_scale, signs, pair_sigma, nullptr, 1, hadamard_block, stream);
    if (!qamw::pairs_launchable(W, dtype, ldw, p, pairs_out)) return QAMW_ERR_UNSUPPORTED;
    const bool fused = qamw::fused_norms_supported(p);
    if (!fused && launch_norms(W, dtype, ldw, d_out, p, row_norms_out) != hipSuccess) return QAMW_ERR_DEVICE;
    return qamw::launch_pairs(W, dtype, ldw, p, row_norms_out, !fused, pairs_out) == hipSuccess ? QAMW_OK : QAMW_ERR_DEVICE;
}

int qamw_lloyd_workspace_bytes(int bits, size_t *bytes_out) {
    if (!bytes_out || bits < 1 || bits > QAMW_MAX_BITS) return QAMW_ERR_INVALID_ARG;
    *bytes_out = qamw::lloyd_workspace_bytes(1 << bits);
    return QAMW_OK;
}

int qamw_lloyd_device(const float *samples, uint64_t n_samples, int bits, float *codebook, int max_iters, double tol,
                      void *workspace, size_t workspace_bytes, double *mse_out, int *iters_out, void *stream) {
    if (!samples || !codebook || !workspace || bits < 1 || bits > QAMW_MAX_BITS || max_iters < 1 || !(tol >= 0.0))
        return QAMW_ERR_INVALID_ARG;
    const int K = 1 << bits;
    if (n_samples < (uint64_t)K || n_samples > (1ull << 24)) return QAMW_ERR_INVALID_ARG;
    if (workspace_bytes < qamw::lloyd_workspace_bytes(K) || (reinterpret_cast<uintptr_t>(workspace) & 15) ||
        (reinterpret_cast<uintptr_t>(samples) & 7) || (reinterpret_cast<uintptr_t>(codebook) & 7))
        return QAMW_ERR_INVALID_ARG;
    hipError_t e = qamw::run_lloyd(samples, (long long)n_samples, K, codebook, max_iters, tol, workspace, mse_out, iters_out,
                                   (hipStream_t)stream);
    return e == hipSuccess ? QAMW_OK : QAMW_ERR_DEVICE;
}

int qamw_encode_polar(const void *W, int dtype, int d_out, int d_in, int64_t ldw, const float *chan_scale,
                      const int8_t *signs, const float *pair_sigma, const float *levels, int bits_a, int bits_p,
                      int hadamard_block, uint8_t *packed_out, float *row_norms_out, void *stream) {
    if (!W || !levels || !packed_out || !row_norms_out || misaligned4(packed_out)) return QAMW_ERR_INVALID_ARG;
    if (dtype != QAMW_DTYPE_F32 && dtype != QAMW_DTYPE_BF16) return QAMW_ERR_INVALID_ARG;
    if (bits_a < 0 || bits_a > QAMW_MAX_POLAR_AMPLITUDE_BITS || bits_p < 0 || bits_p > 12) return QAMW_ERR_INVALID_ARG;
    int rc = check_common(d_out, d_in, bits_a + bits_p, hadamard_block);
    if (rc != QAMW_OK) return rc;
    if (ldw < d_in) return QAMW_ERR_SHAPE;
    qamw::Problem p = make_problem(d_out, d_in, chan_scale, signs, pair_sigma, nullptr, bits_a + bits_p, hadamard_block,
                                   stream);
    // nothing is launched for a shape outside the kernel's range
    if (!qamw::polar_encode_launchable(W, dtype, ldw, p, bits_a, bits_p)) return QAMW_ERR_UNSUPPORTED;
    const bool fused = qamw::fused_norms_supported(p);
    if (!fused && launch_norms(W, dtype, ldw, d_out, p, row_norms_out) != hipSuccess) return QAMW_ERR_DEVICE;
    hipError_t e = qamw::launch_encode_polar(W, dtype, ldw, p, levels, bits_a, bits_p, row_norms_out, !fused, packed_out);
    return e == hipSuccess ? QAMW_OK : QAMW_ERR_DEVICE;
}

int qamw_encode_pruned(const void *W, int dtype, int d_out, int d_in, int64_t ldw, const float *chan_scale,
                       const int8_t *signs, const float *pair_sigma, const float *codebook, int bits, int hadamard_block,
                       const void *grid, uint8_t *packed_out, float *row_norms_out, unsigned long long *full_scans,
                       void *stream) {
    if (!W || !codebook || !grid || !packed_out || !row_norms_out || misaligned4(packed_out)) return QAMW_ERR_INVALID_ARG;
    if (dtype != QAMW_DTYPE_F32 && dtype != QAMW_DTYPE_BF16) return QAMW_ERR_INVALID_ARG;
    int rc = check_common(d_out, d_in, bits, hadamard_block);
    if (rc != QAMW_OK) return rc;
    if (ldw < d_in) return QAMW_ERR_SHAPE;
    if (reinterpret_cast<uintptr_t>(grid) & 15) return QAMW_ERR_INVALID_ARG;
    qamw::Problem p = make_problem(d_out, d_in, chan_scale, signs, pair_sigma, codebook, bits, hadamard_block, stream);
    p.full_scans = full_scans;
    qamw::SearchGridView g;
    g.table = grid;
    g.variant = g_kernel_path.load();
    if (qamw_search_grid_size(bits, &g.G, nullptr) != QAMW_OK) return QAMW_ERR_INVALID_ARG;
    // nothing is launched for a shape outside the kernel's range
    if (!qamw::grid_encode_launchable(W, dtype, ldw, p, g)) return QAMW_ERR_UNSUPPORTED;
    if (launch_norms(W, dtype, ldw, d_out, p, row_norms_out) != hipSuccess) return QAMW_ERR_DEVICE;
    hipError_t e = qamw::launch_encode_grid(W, dtype, ldw, p, g, row_norms_out, packed_out);
    return e == hipSuccess ? QAMW_OK : QAMW_ERR_DEVICE;
}

int qamw_decode(const uint8_t *packed, const float *row_norms, int d_out, int d_in, const float *chan_scale,
                const int8_t *signs, const float *pair_sigma, const float *codebook, int bits, int hadamard_block,
                uint16_t *W_out, int64_t ldo, void *stream) {
    return decode_any(packed, row_norms, d_out, d_in, chan_scale, signs, pair_sigma, codebook, bits, hadamard_block,
                      W_out, ldo, stream, true);
}

static int decode_batch_impl(const qamw_decode_item *items, int n_items, const float *codebook, int bits, int hadamard_block,
                             void *stream, bool traffic_only) {
    static_assert(QAMW_MAX_BATCH == qamw::QAMW_DECODE_MAX_BATCH, "batch limits differ");
    if (!items || !codebook || n_items < 1 || n_items > QAMW_MAX_BATCH) return QAMW_ERR_INVALID_ARG;
    qamw::DecodeItem its[QAMW_MAX_BATCH];
    for (int i = 0; i < n_items; ++i) {
        const qamw_decode_item &q = items[i];
        if (!q.packed || !q.row_norms || !q.W_out || misaligned4(q.packed)) return QAMW_ERR_INVALID_ARG;
        int rc = check_common(q.d_out, q.d_in, bits, hadamard_block);
        if (rc != QAMW_OK) return rc;
        if (q.ldo < q.d_in) return QAMW_ERR_SHAPE;
        its[i] = qamw::DecodeItem{q.packed, q.row_norms, q.chan_scale, q.signs, q.pair_sigma, q.W_out, q.ldo, q.d_out, q.d_in};
    }
    qamw::Problem shared = make_problem(items[0].d_out, items[0].d_in, nullptr, nullptr, nullptr, codebook, bits,
                                        hadamard_block, stream);
    if (g_kernel_path.load() != 1 || traffic_only) {
        hipError_t e = qamw::launch_decode_batch_fast(its, n_items, shared, true, traffic_only);
        if (e == hipSuccess) return QAMW_OK;
        if (e != hipErrorNotSupported) return QAMW_ERR_DEVICE;
    }
    if (traffic_only) return QAMW_ERR_UNSUPPORTED;              // only the fast kernel has this mode
    for (int i = 0; i < n_items; ++i) {                         // nothing was launched: one general launch per item
        const qamw_decode_item &q = items[i];
        int rc = decode_any(q.packed, q.row_norms, q.d_out, q.d_in, q.chan_scale, q.signs, q.pair_sigma, codebook, bits,
                            hadamard_block, q.W_out, q.ldo, stream, true);
        if (rc != QAMW_OK) return rc;
    }
    return QAMW_OK;
}

int qamw_decode_batch(const qamw_decode_item *items, int n_items, const float *codebook, int bits, int hadamard_block,
                      void *stream) {
    return decode_batch_impl(items, n_items, codebook, bits, hadamard_block, stream, false);
}

int qamw_decode_traffic_probe(const qamw_decode_item *items, int n_items, const float *codebook, int bits,
                              int hadamard_block, void *stream) {
    return decode_batch_impl(items, n_items, codebook, bits, hadamard_block, stream, true);
}

// More than QAMW_MATMUL_TILE_ROWS activation rows are processed in tiles of equal size (all above the vector kernel's
// range, so every row of a product is computed by the same kernel): rows per tile.
static int matmul_tile_rows(int m) {
    if (m <= QAMW_MATMUL_TILE_ROWS) return m;
    const int tiles = (m + QAMW_MATMUL_TILE_ROWS - 1) / QAMW_MATMUL_TILE_ROWS;
    return (m + tiles - 1) / tiles;
}

int qamw_matmul_workspace_bytes(int d_in, int d_out, int m, size_t *bytes_out) {
    if (!bytes_out || d_out <= 0 || m < 1 || m > QAMW_MATMUL_MAX_ROWS) return QAMW_ERR_INVALID_ARG;
    if (d_in <= 0 || (d_in & 1)) return QAMW_ERR_SHAPE;
    *bytes_out = qamw::matmul_workspace_bytes(d_in, d_out, matmul_tile_rows(m));
    return QAMW_OK;
}

static int matmul_batch_impl(const qamw_matmul_item *items, int n_items, int x_dtype, int m, const float *codebook, int bits,
                             int hadamard_block, void *workspace, size_t workspace_bytes, void *stream) {
    static_assert(QAMW_MATMUL_MAX_BATCH == qamw::QAMW_MATMUL_MAX_BATCH, "batch limits differ");
    if (!items || !codebook || !workspace || n_items < 1 || n_items > QAMW_MATMUL_MAX_BATCH) return QAMW_ERR_INVALID_ARG;
    if (x_dtype != QAMW_DTYPE_F32 && x_dtype != QAMW_DTYPE_BF16) return QAMW_ERR_INVALID_ARG;
    if (m < 1 || m > QAMW_MATMUL_MAX_ROWS) return QAMW_ERR_INVALID_ARG;
    const int tile = matmul_tile_rows(m);
    qamw::MatmulItem its[QAMW_MATMUL_MAX_BATCH];
    size_t need = 0;
    bool supported = true;
    for (int i = 0; i < n_items; ++i) {
        const qamw_matmul_item &q = items[i];
        if (!q.X || !q.packed || !q.row_norms || !q.Y) return QAMW_ERR_INVALID_ARG;
        int rc = check_common(q.d_out, q.d_in, bits, hadamard_block);
        if (rc != QAMW_OK) return rc;
        if (q.ldx < q.d_in || q.ldy < q.d_out) return QAMW_ERR_SHAPE;
        qamw::Problem pi = make_problem(q.d_out, q.d_in, nullptr, nullptr, nullptr, codebook, bits, hadamard_block, stream);
        if (!qamw::matmul_supported(pi, tile) || (reinterpret_cast<uintptr_t>(q.packed) & 3)) supported = false;
        need += qamw::matmul_workspace_bytes(q.d_in, q.d_out, tile);
        its[i] = qamw::MatmulItem{q.X, q.ldx, q.packed, q.row_norms, q.chan_scale, q.signs, q.pair_sigma, q.Y, q.ldy, q.d_out, q.d_in};
    }
    if (workspace_bytes < need || (reinterpret_cast<uintptr_t>(workspace) & 15)) return QAMW_ERR_INVALID_ARG;
    if (!supported) return QAMW_ERR_UNSUPPORTED;
    qamw::Problem p = make_problem(items[0].d_out, items[0].d_in, nullptr, nullptr, nullptr, codebook, bits, hadamard_block, stream);
    const size_t x_elem = x_dtype == QAMW_DTYPE_F32 ? sizeof(float) : sizeof(uint16_t);
    // one launch pair per tile of activation rows; the tiles follow one another on the stream and share the workspace
    for (int t0 = 0; t0 < m; t0 += tile) {
        const int rows = m - t0 < tile ? m - t0 : tile;
        if (t0 > 0) {
            for (int i = 0; i < n_items; ++i) {
                its[i].X = static_cast<const char *>(items[i].X) + (size_t)t0 * (size_t)items[i].ldx * x_elem;
                its[i].Y = items[i].Y + (size_t)t0 * (size_t)items[i].ldy;
            }
        }
        hipError_t e = qamw::launch_matmul_batch(its, n_items, x_dtype, rows, p, workspace, g_kernel_path.load());
        if (e == hipErrorNotSupported) return QAMW_ERR_UNSUPPORTED;
        if (e != hipSuccess) return QAMW_ERR_DEVICE;
    }
    return QAMW_OK;
}

int qamw_matmul_batch(const qamw_matmul_item *items, int n_items, int x_dtype, int m, const float *codebook, int bits,
                      int hadamard_block, void *workspace, size_t workspace_bytes, void *stream) {
    return matmul_batch_impl(items, n_items, x_dtype, m, codebook, bits, hadamard_block, workspace, workspace_bytes, stream);
}

int qamw_matmul(const void *X, int x_dtype, int m, int64_t ldx, const uint8_t *packed, const float *row_norms, int d_out,
                int d_in, const float *chan_scale, const int8_t *signs, const float *pair_sigma, const float *codebook,
                int bits, int hadamard_block, void *workspace, size_t workspace_bytes, float *Y, int64_t ldy,
                void *stream) {
    qamw_matmul_item it;
    it.X = X;
    it.ldx = ldx;
    it.packed = packed;
    it.row_norms = row_norms;
    it.chan_scale = chan_scale;
    it.signs = signs;
    it.pair_sigma = pair_sigma;
    it.Y = Y;
    it.ldy = ldy;
    it.d_out = d_out;
    it.d_in = d_in;
    return matmul_batch_impl(&it, 1, x_dtype, m, codebook, bits, hadamard_block, workspace, workspace_bytes, stream);
}

int qamw_decode_f32(const uint8_t *packed, const float *row_norms, int d_out, int d_in, const float *chan_scale,
                    const int8_t *signs, const float *pair_sigma, const float *codebook, int bits,
                    int hadamard_block, float *W_out, int64_t ldo, void *stream) {
    return decode_any(packed, row_norms, d_out, d_in, chan_scale, signs, pair_sigma, codebook, bits, hadamard_block,
                      W_out, ldo, stream, false);
}

}  // extern "C"
