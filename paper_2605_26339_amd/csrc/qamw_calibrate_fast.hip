// Vectorised row norms and the shape-specialised pair-scale calibration (Eq. 1).
#include <cmath>

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
    constexpr int U = 4;                                        // loads requested together: a wave alone on its row has
                                                                // nothing else to hide the memory round trip behind
    const char *base = reinterpret_cast<const char *>(W) + (int64_t)row * ldw * (DTYPE == 0 ? 4 : 2);
    double acc = 0.0;
    for (int j0 = lane * V; j0 < d_in; j0 += U * WAVE * V) {
        uint4 raw[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int j = j0 + u * WAVE * V;
            raw[u] = make_uint4(0, 0, 0, 0);
            if (j < d_in) raw[u] = *reinterpret_cast<const uint4 *>(base + (int64_t)j * (DTYPE == 0 ? 4 : 2));
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int j = j0 + u * WAVE * V;
            if (j >= d_in) break;
            float w[V];
            const uint32_t q4[4] = {raw[u].x, raw[u].y, raw[u].z, raw[u].w};
            if (DTYPE == 0) {
#pragma unroll
                for (int q = 0; q < 4; ++q) w[q] = __uint_as_float(q4[q]);
            } else {
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    w[2 * q] = __uint_as_float(q4[q] << 16);
                    w[2 * q + 1] = __uint_as_float(q4[q] & 0xFFFF0000u);
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
// Calibration of up to CAL_MAX_BATCH matrices in one pair of launches.
// Step 1: one workgroup per chunk of CAL_ROWS consecutive rows of one matrix.  It first computes the norms of its
// rows (slab sums in LDS, as the encoders do: the head rows are fetched from memory once), then wave w takes the slabs
// w, w + CF_WAVES, ... and sums |z_k| over the chunk's rows, row by row, in fp64, and writes one partial sum per pair.
// Step 2: per pair, the partial sums added in chunk order, then Eq. 1.
// ---------------------------------------------------------------------------------------------
struct CalMat {
    const void *W;
    int64_t ldw;
    const float *chan_scale;
    const int8_t *signs;
    double *partial;                      // n_chunks x (d_in / 2) partial sums
    float *sigma_out;
    int n_rows, d_in, n_slabs, n_chunks;
    float sigma_default;
};
struct CalBatch {
    CalMat m[CAL_MAX_BATCH];
    int chunk_begin[CAL_MAX_BATCH + 1];   // first step-1 workgroup of each matrix
    int fin_begin[CAL_MAX_BATCH + 1];     // first step-2 workgroup of each matrix
    int n;
    float inv_sqrt_block;
};

template <int DTYPE, int B>
__global__ __launch_bounds__(CF_THREADS) void k_calibrate_partial(CalBatch bt) {
    __shared__ double norm_part[CAL_ROWS * FUSED_NORM_MAX_SLABS];
    const int lane = threadIdx.x & (WAVE - 1);
    const int wid = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    int mi = 0;
    while (mi + 1 < bt.n && (int)blockIdx.x >= bt.chunk_begin[mi + 1]) ++mi;
    const CalMat &M = bt.m[mi];
    Problem p;
    p.d_in = M.d_in;
    p.chan_scale = M.chan_scale;
    p.signs = M.signs;
    p.inv_sqrt_block = bt.inv_sqrt_block;
    const void *__restrict__ W = M.W;
    const int64_t ldw = M.ldw;
    const int n_rows = M.n_rows, n_slabs = M.n_slabs;
    double *__restrict__ partial = M.partial;
    const int chunk = (int)blockIdx.x - bt.chunk_begin[mi];
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

__global__ __launch_bounds__(CF_THREADS) void k_calibrate_finish(CalBatch bt) {
    int mi = 0;
    while (mi + 1 < bt.n && (int)blockIdx.x >= bt.fin_begin[mi + 1]) ++mi;
    const CalMat &M = bt.m[mi];
    const int n_pairs = M.d_in >> 1, n_chunks = M.n_chunks;
    const double *__restrict__ partial = M.partial;
    const int k = ((int)blockIdx.x - bt.fin_begin[mi]) * CF_THREADS + threadIdx.x;
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
    const float s = (float)((acc / (double)M.n_rows) / sqrt_half_pi);
    M.sigma_out[k] = (s > 0.0f) ? s : M.sigma_default;
}

bool fused_norms_supported(const Problem &p) { return (p.d_in + 1023) / 1024 <= FUSED_NORM_MAX_SLABS; }

size_t calibrate_partial_bytes(int d_in, int n_rows) {
    const size_t n_chunks = (size_t)(n_rows + CAL_ROWS - 1) / CAL_ROWS;
    return n_chunks * (size_t)(d_in / 2) * sizeof(double);
}

template <int DTYPE, int B> static hipError_t launch_cal(const CalBatch &bt, hipStream_t stream) {
    hipLaunchKernelGGL((k_calibrate_partial<DTYPE, B>), dim3(bt.chunk_begin[bt.n]), dim3(CF_THREADS), 0, stream, bt);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(k_calibrate_finish, dim3(bt.fin_begin[bt.n]), dim3(CF_THREADS), 0, stream, bt);
    return hipGetLastError();
}

template <int DTYPE> static hipError_t launch_cal_d(const CalBatch &bt, int block, hipStream_t stream) {
    switch (block) {
        case 64: return launch_cal<DTYPE, 64>(bt, stream);
        case 128: return launch_cal<DTYPE, 128>(bt, stream);
        case 256: return launch_cal<DTYPE, 256>(bt, stream);
        case 512: return launch_cal<DTYPE, 512>(bt, stream);
        case 1024: return launch_cal<DTYPE, 1024>(bt, stream);
        default: return hipErrorNotSupported;
    }
}

bool fast_calibrate_supported(const void *W, int dtype, int64_t ldw, const Problem &p) {
    const int unit = p.block > 16 ? p.block : 16;
    return p.d_in % unit == 0 && p.block >= 64 && fused_norms_supported(p) && front_alignment_ok(W, dtype, ldw, p);
}

// n <= CAL_MAX_BATCH matrices, two launches in all; the kernels compute the head rows' norms themselves.  The caller
// has checked every item with fast_calibrate_supported().
hipError_t launch_calibrate_batch_fast(const CalItem *items, int n, int dtype, int block, hipStream_t stream) {
    if (n < 1 || n > CAL_MAX_BATCH) return hipErrorNotSupported;
    CalBatch bt;
    int64_t chunks = 0, fin = 0;
    for (int i = 0; i < n; ++i) {
        CalMat &M = bt.m[i];
        M.W = items[i].W;
        M.ldw = items[i].ldw;
        M.chan_scale = items[i].chan_scale;
        M.signs = items[i].signs;
        M.partial = items[i].partial;
        M.sigma_out = items[i].sigma_out;
        M.n_rows = items[i].n_rows;
        M.d_in = items[i].d_in;
        M.n_slabs = (items[i].d_in + CSLAB - 1) / CSLAB;
        M.n_chunks = (items[i].n_rows + CAL_ROWS - 1) / CAL_ROWS;
        M.sigma_default = (float)(1.0 / std::sqrt((double)items[i].d_in));
        bt.chunk_begin[i] = (int)chunks;
        bt.fin_begin[i] = (int)fin;
        chunks += M.n_chunks;
        fin += (items[i].d_in / 2 + CF_THREADS - 1) / CF_THREADS;
        if (chunks > 0x3fffffff || fin > 0x3fffffff) return hipErrorNotSupported;
    }
    for (int i = n; i <= CAL_MAX_BATCH; ++i) {
        bt.chunk_begin[i] = (int)chunks;
        bt.fin_begin[i] = (int)fin;
    }
    for (int i = n; i < CAL_MAX_BATCH; ++i) bt.m[i] = bt.m[0];
    bt.n = n;
    bt.inv_sqrt_block = (float)(1.0 / std::sqrt((double)block));
    return dtype == 0 ? launch_cal_d<0>(bt, block, stream) : launch_cal_d<1>(bt, block, stream);
}

hipError_t launch_calibrate_fast(const void *W, int dtype, int64_t ldw, int n_rows, const Problem &p, double *partial,
                                 float *sigma_out) {
    const CalItem it{W, ldw, p.chan_scale, p.signs, partial, sigma_out, n_rows, p.d_in};
    return launch_calibrate_batch_fast(&it, 1, dtype, p.block, p.stream);
}

}  // namespace qamw
