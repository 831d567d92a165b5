// Codebook training on the device (Sec. 3.5: Lloyd iterations; a codebook fitted to a checkpoint's own
// pair distribution is the follow-up the paper names) and the samples for it: the normalised pairs the
// encoder quantises.
//
// k_pairs: the encoder's front half (channel scale, row norm, rotation, pair gain), written out instead
// of quantised: bit for bit the points whose nearest codeword qamw_encode stores.
// k_lloyd_assign: every sample to its nearest point by exact fp32 squared distances over the whole
// codebook (lowest index on ties), sums of each cell accumulated in 64-bit fixed point (2^-30), so the
// result does not depend on the order the atomics land in.
// k_lloyd_update: every point to the mean of its cell (an empty cell keeps its point).
#include <cmath>

#include "qamw_front.hpp"

namespace qamw {

constexpr int LL_THREADS = 256;
constexpr double LL_SCALE = 1073741824.0;          // 2^30
constexpr float LL_CLAMP = 256.0f;                 // coordinates beyond +-256 enter the sums clamped (2^38 * n < 2^63 for n <= 2^24)

// Accumulators of one assignment pass (in the caller's workspace, after the fp64 codebook).
struct LloydAcc {
    double *cb;                     // K x 2, the points in fp64
    long long *sx, *sy;             // K fixed-point sums
    unsigned long long *cnt;        // K counts
    unsigned long long *err;        // 1: fixed-point sum of squared distances
};

// LDS_SUMS: the cell sums are first accumulated per workgroup in LDS (small codebooks, where thousands of
// samples land on every cell and global atomics on the same address would serialise).
template <bool LDS_SUMS>
__global__ __launch_bounds__(LL_THREADS) void k_lloyd_assign(const float2 *__restrict__ samples, long long n, int K,
                                                             LloydAcc acc) {
    extern __shared__ __align__(16) float2 ll_cb[];
    unsigned long long *lsum = reinterpret_cast<unsigned long long *>(ll_cb + K);   // [3][K]: sx, sy, count (LDS_SUMS only)
    for (int i = threadIdx.x; i < K; i += LL_THREADS) {
        ll_cb[i] = make_float2((float)acc.cb[2 * i], (float)acc.cb[2 * i + 1]);
        if (LDS_SUMS) {
            lsum[i] = 0;
            lsum[K + i] = 0;
            lsum[2 * K + i] = 0;
        }
    }
    __syncthreads();
    double err = 0.0;
    for (long long i = (long long)blockIdx.x * LL_THREADS + threadIdx.x; i < n; i += (long long)gridDim.x * LL_THREADS) {
        const float2 x = samples[i];
        float bd = 3.0e38f;
        int bi = 0;
        for (int k = 0; k < K; ++k) {                           // uniform address: an LDS broadcast
            const float2 c = ll_cb[k];
            const float e0 = x.x - c.x, e1 = x.y - c.y;
            const float d = __builtin_fmaf(e1, e1, e0 * e0);
            if (d < bd) {
                bd = d;
                bi = k;
            }
        }
        const float cx = fminf(fmaxf(x.x, -LL_CLAMP), LL_CLAMP), cy = fminf(fmaxf(x.y, -LL_CLAMP), LL_CLAMP);
        const unsigned long long fx = (unsigned long long)__double2ll_rn((double)cx * LL_SCALE);
        const unsigned long long fy = (unsigned long long)__double2ll_rn((double)cy * LL_SCALE);
        if (LDS_SUMS) {
            atomicAdd(lsum + bi, fx);
            atomicAdd(lsum + K + bi, fy);
            atomicAdd(lsum + 2 * K + bi, 1ull);
        } else {
            atomicAdd(reinterpret_cast<unsigned long long *>(acc.sx + bi), fx);
            atomicAdd(reinterpret_cast<unsigned long long *>(acc.sy + bi), fy);
            atomicAdd(acc.cnt + bi, 1ull);
        }
        err += (double)fminf(bd, 2.0f * LL_CLAMP * LL_CLAMP);
    }
    if (LDS_SUMS) {
        __syncthreads();
        for (int i = threadIdx.x; i < K; i += LL_THREADS) {
            if (lsum[2 * K + i]) {
                atomicAdd(reinterpret_cast<unsigned long long *>(acc.sx + i), lsum[i]);
                atomicAdd(reinterpret_cast<unsigned long long *>(acc.sy + i), lsum[K + i]);
                atomicAdd(acc.cnt + i, lsum[2 * K + i]);
            }
        }
    }
    // one atomic per wave for the error sum
#pragma unroll
    for (int s = 1; s < WAVE; s <<= 1) err += __shfl_xor(err, s, WAVE);
    if ((threadIdx.x & (WAVE - 1)) == 0) atomicAdd(acc.err, (unsigned long long)__double2ll_rn(err * LL_SCALE));
}

// report[0] = mean squared error of the assignment pass just done
__global__ void k_lloyd_report(long long n, LloydAcc acc, double *report) { report[0] = (double)(*acc.err) / LL_SCALE / (double)n; }

// Either move the points to the means of their cells (move != 0; an empty cell keeps its point) or leave them;
// write the fp32 codebook; clear the sums for the next pass.
__global__ __launch_bounds__(LL_THREADS) void k_lloyd_update(int K, LloydAcc acc, int move, float *codebook_f32) {
    const int i = blockIdx.x * LL_THREADS + threadIdx.x;
    if (i == 0) *acc.err = 0;
    if (i < K) {
        const unsigned long long c = acc.cnt[i];
        if (move && c > 0) {
            acc.cb[2 * i] = (double)acc.sx[i] / LL_SCALE / (double)c;
            acc.cb[2 * i + 1] = (double)acc.sy[i] / LL_SCALE / (double)c;
        }
        codebook_f32[2 * i] = (float)acc.cb[2 * i];
        codebook_f32[2 * i + 1] = (float)acc.cb[2 * i + 1];
        acc.sx[i] = 0;
        acc.sy[i] = 0;
        acc.cnt[i] = 0;
    }
}

__global__ __launch_bounds__(LL_THREADS) void k_lloyd_init(int K, LloydAcc acc, const float *codebook_f32) {
    const int i = blockIdx.x * LL_THREADS + threadIdx.x;
    if (i == 0) *acc.err = 0;
    if (i < K) {
        acc.cb[2 * i] = (double)codebook_f32[2 * i];
        acc.cb[2 * i + 1] = (double)codebook_f32[2 * i + 1];
        acc.sx[i] = 0;
        acc.sy[i] = 0;
        acc.cnt[i] = 0;
    }
}

size_t lloyd_workspace_bytes(int K) { return (size_t)K * (2 * sizeof(double) + 3 * sizeof(long long)) + 64; }

static LloydAcc lloyd_layout(void *workspace, int K) {
    LloydAcc a;
    char *p = static_cast<char *>(workspace);
    a.cb = reinterpret_cast<double *>(p);
    p += (size_t)K * 2 * sizeof(double);
    a.sx = reinterpret_cast<long long *>(p);
    p += (size_t)K * sizeof(long long);
    a.sy = reinterpret_cast<long long *>(p);
    p += (size_t)K * sizeof(long long);
    a.cnt = reinterpret_cast<unsigned long long *>(p);
    p += (size_t)K * sizeof(long long);
    a.err = reinterpret_cast<unsigned long long *>(p);
    return a;
}

// Lloyd iterations with the stopping rule of the CPU trainer: after each assignment the mean squared error D is
// read back; stop when |D_prev - D| < tol * D_prev (from the second assignment on) or after max_iters assignments;
// the points are not moved after the last assignment.  Blocks the host on the stream once per iteration.
hipError_t run_lloyd(const float *samples, long long n, int K, float *codebook, int max_iters, double tol, void *workspace,
                     double *mse_out, int *iters_out, hipStream_t stream) {
    const LloydAcc acc = lloyd_layout(workspace, K);
    double *report = reinterpret_cast<double *>(reinterpret_cast<char *>(acc.err) + 16);
    const unsigned kb = (unsigned)((K + LL_THREADS - 1) / LL_THREADS);
    const bool lds_sums = K <= 1024;
    const long long want = (n + LL_THREADS - 1) / LL_THREADS, cap = lds_sums ? 1024 : 4096;
    const unsigned blocks = (unsigned)(want < cap ? (want < 1 ? 1 : want) : cap);
    hipLaunchKernelGGL(k_lloyd_init, dim3(kb), dim3(LL_THREADS), 0, stream, K, acc, codebook);
    double prev = 0.0, D = 0.0;
    int it = 0;
    for (;; ++it) {
        if (lds_sums)
            hipLaunchKernelGGL(k_lloyd_assign<true>, dim3(blocks), dim3(LL_THREADS), (size_t)K * (sizeof(float2) + 24), stream,
                               reinterpret_cast<const float2 *>(samples), n, K, acc);
        else
            hipLaunchKernelGGL(k_lloyd_assign<false>, dim3(blocks), dim3(LL_THREADS), (size_t)K * sizeof(float2), stream,
                               reinterpret_cast<const float2 *>(samples), n, K, acc);
        // the decision to move needs D on the host: read it with the sums still in place, then move or not
        hipLaunchKernelGGL(k_lloyd_report, dim3(1), dim3(1), 0, stream, n, acc, report);
        hipError_t e = hipMemcpyAsync(&D, report, sizeof(double), hipMemcpyDeviceToHost, stream);
        if (e != hipSuccess) return e;
        e = hipStreamSynchronize(stream);
        if (e != hipSuccess) return e;
        const bool stop = (it > 0 && std::fabs(prev - D) < tol * prev) || it + 1 >= max_iters;
        hipLaunchKernelGGL(k_lloyd_update, dim3(kb), dim3(LL_THREADS), 0, stream, K, acc, stop ? 0 : 1, codebook);
        prev = D;
        if (stop) break;
    }
    if (mse_out) *mse_out = D;
    if (iters_out) *iters_out = it + 1;
    hipError_t e = hipStreamSynchronize(stream);
    return e != hipSuccess ? e : hipGetLastError();
}

// ---------------------------------------------------------------------------------------------- pairs
template <int DTYPE, int B>
__global__ __launch_bounds__(LL_THREADS) void k_pairs(const void *__restrict__ W, int64_t ldw, Problem p,
                                                      const float *__restrict__ norms_in, float *__restrict__ norms_out,
                                                      float *__restrict__ pairs, int n_slabs, int n_items, int n_blocks) {
    constexpr int NW = LL_THREADS / WAVE;
    __shared__ double norm_part[2 * FUSED_NORM_MAX_SLABS];
    const int lane = threadIdx.x & (WAVE - 1);
    const int wid = threadIdx.x >> 6;
    // norms_in == NULL: the workgroup computes the norms of the rows its items touch (and writes them out)
    const bool fused = norms_in == nullptr;
    const int item0 = (fused ? fused_norm_block(blockIdx.x, n_blocks) : (int)blockIdx.x) * NW;
    if (fused) {
        if (item0 < n_items) block_slab_sums<DTYPE, NW>(norm_part, W, ldw, p, item0, n_items, n_slabs, lane, wid);
        __syncthreads();
    }
    const int item = __builtin_amdgcn_readfirstlane(item0 + wid);
    if (item >= n_items) return;
    const int row = item / n_slabs, slab = item - row * n_slabs;
    float rnorm;
    if (fused) {
        rnorm = row_norm_from_slab_sums(norm_part, row, item0, n_slabs);
        if (slab == 0 && lane == 0) norms_out[row] = rnorm;
    } else {
        rnorm = norms_in[row];
    }
    const LaneSigns<B> ls(lane);
    const int pos = slab_pos(lane);
    const int col0 = slab * 1024 + 16 * pos;
    const bool active = col0 < p.d_in;
    const int c = active ? col0 : 0;
    float x[16];
    rotated_unit_row<DTYPE, B>(x, W, (int64_t)row * ldw, c, rnorm, p, ls);
    float g[8];
    if (p.pair_sigma) {
        const float4 *g4 = reinterpret_cast<const float4 *>(p.pair_sigma + (c >> 1));
        float4 a = g4[0], b = g4[1];
        const float sg8[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
#pragma unroll
        for (int k = 0; k < 8; ++k) g[k] = 1.0f / sg8[k];                         // IEEE division
    } else {
#pragma unroll
        for (int k = 0; k < 8; ++k) g[k] = p.g_default;
    }
    if (active) {
        float4 *dst = reinterpret_cast<float4 *>(pairs + (int64_t)row * p.d_in + c);
#pragma unroll
        for (int t = 0; t < 4; ++t)
            dst[t] = make_float4(x[4 * t] * g[2 * t], x[4 * t + 1] * g[2 * t], x[4 * t + 2] * g[2 * t + 1], x[4 * t + 3] * g[2 * t + 1]);
    }
}

bool pairs_launchable(const void *W, int dtype, int64_t ldw, const Problem &p, const float *pairs) {
    const int unit = p.block > 16 ? p.block : 16;
    return p.d_in % unit == 0 && p.block >= 64 && front_alignment_ok(W, dtype, ldw, p) &&
           (reinterpret_cast<uintptr_t>(pairs) & 15) == 0;
}

template <int DTYPE>
static hipError_t launch_pairs_d(const void *W, int64_t ldw, const Problem &p, float *norms, bool norms_ready, float *pairs) {
    const int n_slabs = (p.d_in + 1023) / 1024;
    const int64_t n_items = (int64_t)p.d_out * n_slabs;
    if (n_items > 0x7fffffff) return hipErrorNotSupported;
    if (!norms_ready && n_slabs > FUSED_NORM_MAX_SLABS) return hipErrorNotSupported;
    static_assert(LL_THREADS / WAVE == 4, "four items per workgroup");
    const int n_blocks = (int)((n_items + 3) / 4);
    const unsigned blocks = (unsigned)(norms_ready ? n_blocks : fused_norm_grid(n_blocks));
    const float *norms_in = norms_ready ? norms : nullptr;
#define QAMW_PAIRS(BB) \
    case BB: hipLaunchKernelGGL((k_pairs<DTYPE, BB>), dim3(blocks), dim3(LL_THREADS), 0, p.stream, W, ldw, p, norms_in, norms, pairs, n_slabs, (int)n_items, n_blocks); break;
    switch (p.block) {
        QAMW_PAIRS(64) QAMW_PAIRS(128) QAMW_PAIRS(256) QAMW_PAIRS(512) QAMW_PAIRS(1024)
        default: return hipErrorNotSupported;
    }
#undef QAMW_PAIRS
    return hipGetLastError();
}

hipError_t launch_pairs(const void *W, int dtype, int64_t ldw, const Problem &p, float *norms, bool norms_ready, float *pairs) {
    if (!pairs_launchable(W, dtype, ldw, p, pairs)) return hipErrorNotSupported;
    return dtype == 0 ? launch_pairs_d<0>(W, ldw, p, norms, norms_ready, pairs) : launch_pairs_d<1>(W, ldw, p, norms, norms_ready, pairs);
}

}  // namespace qamw
