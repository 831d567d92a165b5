// General QAM-W kernels: one workgroup per row, the row staged through LDS in chunks.  They cover
// every shape the library accepts (any even d_in, any power-of-two Hadamard block up to 1024) and
// are the fallback of the shape-specialised kernels.
#include "qamw_common.hpp"
#include "qamw_internal.hpp"

namespace qamw {

constexpr int GEN_THREADS = 256;
constexpr int GEN_CHUNK = 8192;   // columns staged at once: a multiple of every block size and of 64

// ---------------------------------------------------------------------------------------------
// Row norms of the channel-scaled matrix (Sec. 3.1 step 1 applied to W D_s of Sec. B.2).
// Squares are exact in fp64; lanes accumulate a strided subset, then a fixed reduction tree.
// ---------------------------------------------------------------------------------------------
template <int DTYPE>
__global__ __launch_bounds__(GEN_THREADS) void k_row_norms(const void *__restrict__ W, int64_t ldw, int d_in,
                                                           const float *__restrict__ s, float *__restrict__ norms) {
    const int row = blockIdx.x;
    const int64_t base = (int64_t)row * ldw;
    double acc = 0.0;
    for (int j = threadIdx.x; j < d_in; j += GEN_THREADS) {
        float w = Elem<DTYPE>::load(W, base + j);
        float ws = s ? w * s[j] : w;
        acc += (double)ws * (double)ws;
    }
    acc = wave_sum(acc);
    __shared__ double part[GEN_THREADS / WAVE];
    if ((threadIdx.x & (WAVE - 1)) == 0) part[threadIdx.x / WAVE] = acc;
    __syncthreads();
    if (threadIdx.x == 0) {
        double t = ((part[0] + part[1]) + part[2]) + part[3];
        norms[row] = (float)sqrt(t);
    }
}

// In-LDS butterflies of the unnormalised block Walsh-Hadamard transform over a staged chunk whose
// length n is a multiple of `block`: stride 1, 2, ..., block/2, one barrier per stage.
__device__ __forceinline__ void lds_fwht(float *buf, int n, int block) {
    for (int h = 1; h < block; h <<= 1) {
        for (int t = threadIdx.x; t < n / 2; t += GEN_THREADS) {
            int i = ((t & ~(h - 1)) << 1) | (t & (h - 1));
            float a = buf[i], b = buf[i + h];
            buf[i] = a + b;
            buf[i + h] = a - b;
        }
        __syncthreads();
    }
}

// Load one chunk of a row as v = sign * (W*s / r) (encoder steps 1-2 up to the sign mask).
template <int DTYPE>
__device__ __forceinline__ void stage_unit_row(float *buf, const void *W, int64_t base, int c0, int n, float r,
                                               const float *s, const int8_t *signs) {
    for (int j = threadIdx.x; j < n; j += GEN_THREADS) {
        float w = Elem<DTYPE>::load(W, base + c0 + j);
        float ws = s ? w * s[c0 + j] : w;
        float u = (r > 0.0f) ? ws / r : 0.0f;
        if (signs && signs[c0 + j] < 0) u = -u;
        buf[j] = u;
    }
    __syncthreads();
}

// ---------------------------------------------------------------------------------------------
// Encoder (Sec. 3.1): exact fp32 squared distances to all K codewords, lowest index on ties.
// ---------------------------------------------------------------------------------------------
template <int DTYPE>
__global__ __launch_bounds__(GEN_THREADS) void k_encode_general(const void *__restrict__ W, int64_t ldw, Problem p,
                                                                const float *__restrict__ norms,
                                                                uint8_t *__restrict__ packed) {
    __shared__ float buf[GEN_CHUNK];
    int *ibuf = reinterpret_cast<int *>(buf);
    const int row = blockIdx.x;
    const float r = norms[row];
    const int64_t base = (int64_t)row * ldw;
    uint32_t *prow = reinterpret_cast<uint32_t *>(packed + (int64_t)row * p.row_bytes);
    const float2 *cbk = reinterpret_cast<const float2 *>(p.codebook);

    for (int c0 = 0; c0 < p.d_in; c0 += GEN_CHUNK) {
        const int n = min(GEN_CHUNK, p.d_in - c0);
        stage_unit_row<DTYPE>(buf, W, base, c0, n, r, p.chan_scale, p.signs);
        lds_fwht(buf, n, p.block);
        for (int k = threadIdx.x; k < n / 2; k += GEN_THREADS) {
            float y0 = buf[2 * k] * p.inv_sqrt_block;
            float y1 = buf[2 * k + 1] * p.inv_sqrt_block;
            float g = p.pair_sigma ? 1.0f / p.pair_sigma[c0 / 2 + k] : p.g_default;
            float x0 = y0 * g, x1 = y1 * g;
            float best = INFINITY;
            int bi = 0;
            for (int c = 0; c < p.K; ++c) {
                float2 cw = cbk[c];
                float e0 = x0 - cw.x, e1 = x1 - cw.y;
                float d = __fmaf_rn(e1, e1, e0 * e0);
                if (d < best) {
                    best = d;
                    bi = c;
                }
            }
            ibuf[2 * k] = bi;
        }
        __syncthreads();
        // bit-pack this chunk: its first pair starts on a dword boundary (4096*bits is a multiple of 32)
        const int n_pairs = n / 2;
        const int n_dw = (n_pairs * p.bits + 31) / 32;
        const int dw0 = (int)(((int64_t)(c0 / 2) * p.bits) / 32);
        for (int w = threadIdx.x; w < n_dw; w += GEN_THREADS) {
            const int lo = 32 * w;
            uint32_t out = 0;
            for (int k = lo / p.bits; k < n_pairs && k * p.bits < lo + 32; ++k) {
                uint32_t v = (uint32_t)ibuf[2 * k];
                int sh = k * p.bits - lo;
                out |= (sh >= 0) ? (v << sh) : (v >> (-sh));
            }
            prow[dw0 + w] = out;
        }
        __syncthreads();
    }
}

// ---------------------------------------------------------------------------------------------
// Decoder (Sec. 3.2 + Sec. B.2).
// ---------------------------------------------------------------------------------------------
template <bool OUT_BF16>
__global__ __launch_bounds__(GEN_THREADS) void k_decode_general(const uint8_t *__restrict__ packed,
                                                                const float *__restrict__ norms, Problem p,
                                                                void *__restrict__ out, int64_t ldo) {
    __shared__ float buf[GEN_CHUNK];
    const int row = blockIdx.x;
    const float r = norms[row];
    const uint32_t *prow = reinterpret_cast<const uint32_t *>(packed + (int64_t)row * p.row_bytes);
    const int row_dwords = (int)(p.row_bytes / 4);
    const float2 *cbk = reinterpret_cast<const float2 *>(p.codebook);

    for (int c0 = 0; c0 < p.d_in; c0 += GEN_CHUNK) {
        const int n = min(GEN_CHUNK, p.d_in - c0);
        for (int k = threadIdx.x; k < n / 2; k += GEN_THREADS) {
            uint32_t idx = unpack_field(prow, row_dwords, c0 / 2 + k, p.bits);
            float2 cw = cbk[idx];
            float sig = p.pair_sigma ? p.pair_sigma[c0 / 2 + k] : p.sigma_default;
            buf[2 * k] = sig * cw.x;
            buf[2 * k + 1] = sig * cw.y;
        }
        __syncthreads();
        lds_fwht(buf, n, p.block);
        for (int j = threadIdx.x; j < n; j += GEN_THREADS) {
            float z = buf[j] * p.inv_sqrt_block;
            if (p.signs && p.signs[c0 + j] < 0) z = -z;
            float w = r * z;
            if (p.chan_scale) w = w * (1.0f / p.chan_scale[c0 + j]);
            if (OUT_BF16)
                reinterpret_cast<uint16_t *>(out)[(int64_t)row * ldo + c0 + j] = (uint16_t)bf16_rne_bits(w);
            else
                reinterpret_cast<float *>(out)[(int64_t)row * ldo + c0 + j] = w;
        }
        __syncthreads();
    }
}

// ---------------------------------------------------------------------------------------------
// Pair-scale calibration (Eq. 1).  One workgroup per Hadamard block column-slab; it walks the
// calibration rows in order so that every pair's fp64 sum is accumulated row by row.
// ---------------------------------------------------------------------------------------------
constexpr int CAL_TILE = 1024;   // elements staged per step: max(block, 512)

template <int DTYPE>
__global__ __launch_bounds__(GEN_THREADS) void k_calibrate_general(const void *__restrict__ W, int64_t ldw, int n_rows,
                                                                   Problem p, const float *__restrict__ norms,
                                                                   float *__restrict__ sigma_out) {
    __shared__ float tile[CAL_TILE];
    __shared__ double amp[CAL_TILE / 2];
    const int b = p.block;
    const int col0 = blockIdx.x * b;
    const int rows_per_step = (b >= 512) ? 1 : 512 / b;       // rows staged together
    const int half = b / 2;                                    // pairs per row in this slab
    double acc0 = 0.0, acc1 = 0.0;                             // thread t owns pairs t and t+256 of the slab
    for (int r0 = 0; r0 < n_rows; r0 += rows_per_step) {
        const int nr = min(rows_per_step, n_rows - r0);
        const int n = nr * b;
        for (int e = threadIdx.x; e < n; e += GEN_THREADS) {
            int rr = e / b, j = e - rr * b;
            int row = r0 + rr;
            float rn = norms[row];
            float w = Elem<DTYPE>::load(W, (int64_t)row * ldw + col0 + j);
            float ws = p.chan_scale ? w * p.chan_scale[col0 + j] : w;
            float u = (rn > 0.0f) ? ws / rn : 0.0f;
            if (p.signs && p.signs[col0 + j] < 0) u = -u;
            tile[e] = u;
        }
        __syncthreads();
        lds_fwht(tile, n, b);
        for (int q = threadIdx.x; q < n / 2; q += GEN_THREADS) {
            float y0 = tile[2 * q] * p.inv_sqrt_block;
            float y1 = tile[2 * q + 1] * p.inv_sqrt_block;
            amp[q] = sqrt((double)y0 * (double)y0 + (double)y1 * (double)y1);
        }
        __syncthreads();
        if ((int)threadIdx.x < half)
            for (int rr = 0; rr < nr; ++rr) acc0 += amp[rr * half + threadIdx.x];
        if ((int)threadIdx.x + GEN_THREADS < half)
            for (int rr = 0; rr < nr; ++rr) acc1 += amp[rr * half + threadIdx.x + GEN_THREADS];
        __syncthreads();
    }
    const double sqrt_half_pi = 1.2533141373155002512078826424055;
    if ((int)threadIdx.x < half) {
        float s = (float)((acc0 / (double)n_rows) / sqrt_half_pi);
        sigma_out[col0 / 2 + threadIdx.x] = (s > 0.0f) ? s : p.sigma_default;
    }
    if ((int)threadIdx.x + GEN_THREADS < half) {
        float s = (float)((acc1 / (double)n_rows) / sqrt_half_pi);
        sigma_out[col0 / 2 + threadIdx.x + GEN_THREADS] = (s > 0.0f) ? s : p.sigma_default;
    }
}

// ---------------------------------------------------------------------------------------------
hipError_t launch_row_norms(const void *W, int dtype, int64_t ldw, int n_rows, const Problem &p, float *norms) {
    if (dtype == 0)
        hipLaunchKernelGGL(k_row_norms<0>, dim3(n_rows), dim3(GEN_THREADS), 0, p.stream, W, ldw, p.d_in, p.chan_scale, norms);
    else
        hipLaunchKernelGGL(k_row_norms<1>, dim3(n_rows), dim3(GEN_THREADS), 0, p.stream, W, ldw, p.d_in, p.chan_scale, norms);
    return hipGetLastError();
}

hipError_t launch_encode_general(const void *W, int dtype, int64_t ldw, const Problem &p, const float *norms,
                                 uint8_t *packed) {
    if (dtype == 0)
        hipLaunchKernelGGL(k_encode_general<0>, dim3(p.d_out), dim3(GEN_THREADS), 0, p.stream, W, ldw, p, norms, packed);
    else
        hipLaunchKernelGGL(k_encode_general<1>, dim3(p.d_out), dim3(GEN_THREADS), 0, p.stream, W, ldw, p, norms, packed);
    return hipGetLastError();
}

hipError_t launch_decode_general(const uint8_t *packed, const float *norms, const Problem &p, void *out, int64_t ldo,
                                 bool out_bf16) {
    if (out_bf16)
        hipLaunchKernelGGL(k_decode_general<true>, dim3(p.d_out), dim3(GEN_THREADS), 0, p.stream, packed, norms, p, out, ldo);
    else
        hipLaunchKernelGGL(k_decode_general<false>, dim3(p.d_out), dim3(GEN_THREADS), 0, p.stream, packed, norms, p, out, ldo);
    return hipGetLastError();
}

hipError_t launch_calibrate_general(const void *W, int dtype, int64_t ldw, int n_rows, const Problem &p,
                                    const float *norms, float *sigma_out) {
    dim3 grid(p.d_in / p.block);
    if (dtype == 0)
        hipLaunchKernelGGL(k_calibrate_general<0>, grid, dim3(GEN_THREADS), 0, p.stream, W, ldw, n_rows, p, norms, sigma_out);
    else
        hipLaunchKernelGGL(k_calibrate_general<1>, grid, dim3(GEN_THREADS), 0, p.stream, W, ldw, n_rows, p, norms, sigma_out);
    return hipGetLastError();
}

}  // namespace qamw
