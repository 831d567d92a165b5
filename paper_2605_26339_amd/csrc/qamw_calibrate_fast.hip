// Vectorised row norms and the shape-specialised pair-scale calibration (Eq. 1).
#include "qamw_front.hpp"

namespace qamw {

constexpr int CF_THREADS = 256;
constexpr int CF_WAVES = CF_THREADS / WAVE;
constexpr int CSLAB = 1024;
constexpr int CAL_ROWS = 8;     // calibration rows a wave accumulates before writing a partial sum

// ---------------------------------------------------------------------------------------------
// Row norms, one wave per row, 16-byte loads.  Squares are exact in fp64; the lane-strided sums
// are combined with the fixed butterfly of wave_sum().
// ---------------------------------------------------------------------------------------------
template <int DTYPE>
__global__ __launch_bounds__(CF_THREADS) void k_row_norms_vec(const void *__restrict__ W, int64_t ldw, int n_rows, int d_in,
                                                             const float *__restrict__ s, float *__restrict__ norms) {
    const int lane = threadIdx.x & (WAVE - 1);
    const int row = __builtin_amdgcn_readfirstlane(blockIdx.x * CF_WAVES + (threadIdx.x >> 6));
    if (row >= n_rows) return;
    constexpr int V = DTYPE == 0 ? 4 : 8;                       // elements per 16-byte load
    double acc = 0.0;
    for (int j = lane * V; j < d_in; j += WAVE * V) {
        float w[V];
        if (DTYPE == 0) {
            float4 v = *reinterpret_cast<const float4 *>(reinterpret_cast<const float *>(W) + (int64_t)row * ldw + j);
            w[0] = v.x; w[1] = v.y; w[2] = v.z; w[3] = v.w;
        } else {
            uint4 v = *reinterpret_cast<const uint4 *>(reinterpret_cast<const uint16_t *>(W) + (int64_t)row * ldw + j);
            const uint32_t u[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                w[2 * q] = __uint_as_float(u[q] << 16);
                w[2 * q + 1] = __uint_as_float(u[q] & 0xFFFF0000u);
            }
        }
        if (s) {
#pragma unroll
            for (int t = 0; t < V; t += 4) {
                float4 sv = *reinterpret_cast<const float4 *>(s + j + t);
                w[t] *= sv.x; w[t + 1] *= sv.y; w[t + 2] *= sv.z; w[t + 3] *= sv.w;
            }
        }
#pragma unroll
        for (int t = 0; t < V; ++t) acc += (double)w[t] * (double)w[t];
    }
    acc = wave_sum(acc);
    if (lane == 0) norms[row] = (float)sqrt(acc);
}

bool launch_row_norms_fast(const void *W, int dtype, int64_t ldw, int n_rows, const Problem &p, float *norms,
                           hipError_t *err) {
    const int v = dtype == 0 ? 4 : 8;
    if (p.d_in % v || ldw % v || (reinterpret_cast<uintptr_t>(W) & 15) || (reinterpret_cast<uintptr_t>(p.chan_scale) & 15))
        return false;
    dim3 grid((n_rows + CF_WAVES - 1) / CF_WAVES);
    if (dtype == 0)
        hipLaunchKernelGGL(k_row_norms_vec<0>, grid, dim3(CF_THREADS), 0, p.stream, W, ldw, n_rows, p.d_in, p.chan_scale, norms);
    else
        hipLaunchKernelGGL(k_row_norms_vec<1>, grid, dim3(CF_THREADS), 0, p.stream, W, ldw, n_rows, p.d_in, p.chan_scale, norms);
    *err = hipGetLastError();
    return true;
}

// ---------------------------------------------------------------------------------------------
// Calibration, step 1: one workgroup per chunk of CAL_ROWS consecutive rows.  It first computes the norms of its rows
// (slab sums in LDS, as the encoders do: the head rows are fetched from memory once), then wave w takes the slabs
// w, w + CF_WAVES, ... and sums |z_k| over the chunk's rows, row by row, in fp64, and writes one partial sum per pair.
// ---------------------------------------------------------------------------------------------
template <int DTYPE, int B>
__global__ __launch_bounds__(CF_THREADS) void k_calibrate_partial(const void *__restrict__ W, int64_t ldw, int n_rows,
                                                                  Problem p, double *__restrict__ partial, int n_slabs) {
    __shared__ double norm_part[CAL_ROWS * FUSED_NORM_MAX_SLABS];
    const int lane = threadIdx.x & (WAVE - 1);
    const int wid = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int chunk = blockIdx.x;
    const int row0 = chunk * CAL_ROWS, row1 = min(n_rows, row0 + CAL_ROWS);
    const int tasks = (row1 - row0) * n_slabs;
    for (int t = wid; t < tasks; t += CF_WAVES) {
        const int dr = t / n_slabs, slab = t - dr * n_slabs;
        const double s2 = slab_sum_of_squares<DTYPE>(W, (int64_t)(row0 + dr) * ldw, slab, p, lane);
        if (lane == 0) norm_part[t] = s2;
    }
    __syncthreads();
    float rn[CAL_ROWS];
#pragma unroll
    for (int dr = 0; dr < CAL_ROWS; ++dr) {
        double s2 = 0.0;
        if (row0 + dr < row1)
            for (int s = 0; s < n_slabs; ++s) s2 += norm_part[dr * n_slabs + s];
        rn[dr] = (float)sqrt(s2);
    }
    const LaneSigns<B> ls(lane);
    for (int slab = wid; slab < n_slabs; slab += CF_WAVES) {
        const int col0 = slab * CSLAB + 16 * slab_pos(lane);
        const bool active = col0 < p.d_in;
        const int c = active ? col0 : 0;
        double acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
        for (int dr = 0; dr < CAL_ROWS; ++dr) {
            if (row0 + dr < row1) {
                float y[16];
                rotated_unit_row<DTYPE, B>(y, W, (int64_t)(row0 + dr) * ldw, c, rn[dr], p, ls);
#pragma unroll
                for (int k = 0; k < 8; ++k)
                    acc[k] += sqrt((double)y[2 * k] * (double)y[2 * k] + (double)y[2 * k + 1] * (double)y[2 * k + 1]);
            }
        }
        if (active) {
            double *dst = partial + (int64_t)chunk * (p.d_in >> 1) + (c >> 1);
#pragma unroll
            for (int k = 0; k < 8; ++k) dst[k] = acc[k];
        }
    }
}

// Step 2: per pair, add the partial sums in chunk order and apply Eq. 1.
__global__ __launch_bounds__(CF_THREADS) void k_calibrate_finish(const double *__restrict__ partial, int n_chunks, int n_rows,
                                                                 int n_pairs, float sigma_default,
                                                                 float *__restrict__ sigma_out) {
    const int k = blockIdx.x * CF_THREADS + threadIdx.x;
    if (k >= n_pairs) return;
    double acc = 0.0;
    int q = 0;
    for (; q + 16 <= n_chunks; q += 16) {                       // 16 loads in flight, added in chunk order
        double v[16];
#pragma unroll
        for (int t = 0; t < 16; ++t) v[t] = partial[(int64_t)(q + t) * n_pairs + k];
#pragma unroll
        for (int t = 0; t < 16; ++t) acc += v[t];
    }
    for (; q < n_chunks; ++q) acc += partial[(int64_t)q * n_pairs + k];
    const double sqrt_half_pi = 1.2533141373155002512078826424055;
    const float s = (float)((acc / (double)n_rows) / sqrt_half_pi);
    sigma_out[k] = (s > 0.0f) ? s : sigma_default;
}

bool fused_norms_supported(const Problem &p) { return (p.d_in + 1023) / 1024 <= FUSED_NORM_MAX_SLABS; }

size_t calibrate_partial_bytes(int d_in, int n_rows) {
    const size_t n_chunks = (size_t)(n_rows + CAL_ROWS - 1) / CAL_ROWS;
    return n_chunks * (size_t)(d_in / 2) * sizeof(double);
}

template <int DTYPE, int B>
static hipError_t launch_cal(const void *W, int64_t ldw, int n_rows, const Problem &p, double *partial, float *sigma_out) {
    const int n_slabs = (p.d_in + CSLAB - 1) / CSLAB;
    const int n_chunks = (n_rows + CAL_ROWS - 1) / CAL_ROWS;
    hipLaunchKernelGGL((k_calibrate_partial<DTYPE, B>), dim3(n_chunks), dim3(CF_THREADS), 0, p.stream, W, ldw, n_rows, p,
                       partial, n_slabs);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const int n_pairs = p.d_in / 2;
    hipLaunchKernelGGL(k_calibrate_finish, dim3((n_pairs + CF_THREADS - 1) / CF_THREADS), dim3(CF_THREADS), 0, p.stream,
                       partial, n_chunks, n_rows, n_pairs, p.sigma_default, sigma_out);
    return hipGetLastError();
}

template <int DTYPE>
static hipError_t launch_cal_d(const void *W, int64_t ldw, int n_rows, const Problem &p, double *partial, float *sigma_out) {
    switch (p.block) {
        case 64: return launch_cal<DTYPE, 64>(W, ldw, n_rows, p, partial, sigma_out);
        case 128: return launch_cal<DTYPE, 128>(W, ldw, n_rows, p, partial, sigma_out);
        case 256: return launch_cal<DTYPE, 256>(W, ldw, n_rows, p, partial, sigma_out);
        case 512: return launch_cal<DTYPE, 512>(W, ldw, n_rows, p, partial, sigma_out);
        case 1024: return launch_cal<DTYPE, 1024>(W, ldw, n_rows, p, partial, sigma_out);
        default: return hipErrorNotSupported;
    }
}

bool fast_calibrate_supported(const void *W, int dtype, int64_t ldw, const Problem &p) {
    const int unit = p.block > 16 ? p.block : 16;
    return p.d_in % unit == 0 && p.block >= 64 && fused_norms_supported(p) && front_alignment_ok(W, dtype, ldw, p);
}

// Two launches; the kernels compute the head rows' norms themselves.
hipError_t launch_calibrate_fast(const void *W, int dtype, int64_t ldw, int n_rows, const Problem &p, double *partial,
                                 float *sigma_out) {
    return dtype == 0 ? launch_cal_d<0>(W, ldw, n_rows, p, partial, sigma_out)
                      : launch_cal_d<1>(W, ldw, n_rows, p, partial, sigma_out);
}

}  // namespace qamw
