// Fused dequantise-and-multiply for a few activation rows, Y = X W^T with W the decoded matrix
// (the follow-up the paper names in its Limitations: a fused dequantization-matmul kernel).
//
// The decoder is linear in the codewords (Sec. 3.2, Sec. B.2):
//     w_i = r_i * D_s^-1 S F yhat_i,        yhat_i,k = sigma_k * c[idx_ik]   (pair k of row i)
// and F is symmetric, S and D_s diagonal, so for an activation row x
//     <w_i, x> = r_i * < yhat_i, F S D_s^-1 x > = r_i * sum_k < c[idx_ik], z_k >,
//     z = the pairs of  sigma (.) F S (x / s).
// The weights are never rotated back: the ACTIVATIONS are rotated once (m rows, d_in log b adds
// each), and each packed index then costs one codeword lookup and two multiply-adds per
// activation row.  HBM traffic is the packed matrix, B/8 bytes per pair, against 4 bytes per pair
// for a bf16 matrix.
//
// Kernels: k_rotate_x (one wave per activation row and 1024-column slab, the encoder's register
// transform) and k_qgemv: a workgroup of 4 waves owns 8 rows of one matrix; wave w takes the
// 1024-column slabs w, w+4, ...; per slab it holds the slab's z in registers, requests the packed
// words of a group of rows at once, and per row unpacks 8 indices, gathers 8 codewords from the
// LDS codebook and multiply-adds them into per-row, per-lane accumulators.  Nothing crosses lanes
// until the wave has finished its slabs: then one transposing reduction (two half-swaps that halve
// the number of live sums, a butterfly over the remaining 16 lanes), a sum over the 4 waves in
// LDS in a fixed order, times r_i, and the store of 8 x m outputs.
#include <cmath>

#include "qamw_common.hpp"
#include "qamw_internal.hpp"
#include "qamw_wave_fwht.hpp"

namespace qamw {

constexpr int GV_THREADS = 256;
constexpr int GV_WAVES = GV_THREADS / WAVE;
constexpr int GV_SLAB = 1024;
constexpr int GV_UNIT_ROWS = 8;        // rows per workgroup (8: more, shorter workgroups balance a layer-sized launch better than 16 or 32)
constexpr int GV_MAX_M = 8;

typedef uint32_t gv_u32x4_t __attribute__((ext_vector_type(4)));

// One product of a batch, as the kernels see it.  Z and partial point into the caller's workspace.
struct GemvMat {
    const void *X;
    const uint8_t *packed;
    const float *norms, *chan_scale, *pair_sigma;
    const int8_t *signs;
    float *Z, *Y;
    int64_t ldx, ldy, row_bytes;
    int d_out, d_in, n_slabs;
    float sigma_default;                   // 1/sqrt(d_in), used when pair_sigma is NULL
};
// Work lists of one launch: rotation items (activation row, slab) and row groups (GV_UNIT_ROWS rows), each numbered
// matrix-major.
struct GemvBatch {
    GemvMat mat[QAMW_MATMUL_MAX_BATCH];
    int rot_begin[QAMW_MATMUL_MAX_BATCH + 1];
    int grp_begin[QAMW_MATMUL_MAX_BATCH + 1];
    int n, m, K;
    float inv_sqrt_block;
    const float *codebook;
};
__device__ __forceinline__ int gv_find(const int *begin, int n, int u) {
    int i = 0;
    while (i + 1 < n && u >= begin[i + 1]) ++i;
    return i;
}

// z = sigma (.) F S (x / s) for every activation row, fp32, row-major [m][d_in].
template <int XDTYPE, int B>
__global__ __launch_bounds__(GV_THREADS) void k_rotate_x(GemvBatch bt) {
    const int lane = threadIdx.x & (WAVE - 1);
    const int wid = threadIdx.x >> 6;
    const int item = __builtin_amdgcn_readfirstlane(blockIdx.x * GV_WAVES + wid);
    if (item >= bt.rot_begin[bt.n]) return;
    const int mi = gv_find(bt.rot_begin, bt.n, item);
    const GemvMat &M = bt.mat[mi];
    const int local = item - bt.rot_begin[mi];
    const int n_slabs = M.n_slabs;
    const int tok = __builtin_amdgcn_readfirstlane(local / n_slabs), slab = __builtin_amdgcn_readfirstlane(local % n_slabs);
    const int d_in = M.d_in;
    const float *chan_scale = M.chan_scale, *pair_sigma = M.pair_sigma;
    const int8_t *signs = M.signs;
    const LaneSigns<B> ls(lane);
    const int pos = slab_pos(lane);
    const int col0 = slab * GV_SLAB + 16 * pos;
    const bool active = col0 < d_in;
    const int c = active ? col0 : 0;
    float y[16];
#pragma unroll
    for (int e = 0; e < 16; ++e) y[e] = Elem<XDTYPE>::load(M.X, (int64_t)tok * M.ldx + c + e);
    if (chan_scale) {
#pragma unroll
        for (int e = 0; e < 16; ++e) y[e] = y[e] * (1.0f / chan_scale[c + e]);    // times fl32(1/s_j), as the decoder does
    }
    if (signs) {
#pragma unroll
        for (int e = 0; e < 16; ++e) y[e] = (signs[c + e] < 0) ? -y[e] : y[e];
    }
    fwht_wave<B>(y, ls);
    const float sigma_default = M.sigma_default;
#pragma unroll
    for (int e = 0; e < 16; ++e) {
        const float sg = pair_sigma ? pair_sigma[(c + e) >> 1] : sigma_default;
        y[e] = ((y[e] * ls.parity) * bt.inv_sqrt_block) * sg;
    }
    if (active) {
        float4 *dst = reinterpret_cast<float4 *>(M.Z + (int64_t)tok * d_in + c);
#pragma unroll
        for (int t = 0; t < 4; ++t) dst[t] = make_float4(y[4 * t], y[4 * t + 1], y[4 * t + 2], y[4 * t + 3]);
    }
}

template <int BITS> __device__ __forceinline__ uint32_t gv_field(const uint32_t (&w)[4], int i) {
    const int bit = i * BITS, word = bit >> 5, off = bit & 31;
    uint32_t v = (off + BITS <= 32) ? (w[word] >> off) : __builtin_amdgcn_alignbit(w[word + 1], w[word], off);
    return v & ((1u << BITS) - 1u);
}

// Sums over the 64 lanes of RG per-lane values a[0..RG): two half-swaps leave RG/4 values per lane (lane bits
// 5 and 4 select which), a butterfly over lane bits 0-3 finishes them.  On return a[0 .. RG/4) hold the totals
// of rows  (lane>>5) * RG/2 + ((lane>>4)&1) * RG/4 + j  (the same in all 16 lanes of a row of lanes).
template <int RG> __device__ __forceinline__ void gv_reduce_rows(float (&a)[RG]) {
    static_assert(RG == 4 || RG == 8 || RG == 16, "rows per reduction");
#pragma unroll
    for (int r = 0; r < RG / 2; ++r) {
        auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(a[r]), __float_as_uint(a[r + RG / 2]), false, false);
        a[r] = __uint_as_float(sw[0]) + __uint_as_float(sw[1]);
    }
#pragma unroll
    for (int r = 0; r < RG / 4; ++r) {
        auto sw = __builtin_amdgcn_permlane16_swap(__float_as_uint(a[r]), __float_as_uint(a[r + RG / 4]), false, false);
        a[r] = __uint_as_float(sw[0]) + __uint_as_float(sw[1]);
    }
#pragma unroll
    for (int r = 0; r < RG / 4; ++r) {
#pragma unroll
        for (int s = 1; s < 16; s <<= 1) a[r] += __shfl_xor(a[r], s, WAVE);
    }
}

// Y[t][row] = r_row * sum over the row's pairs of <c[idx], z_t>, GV_UNIT_ROWS rows per workgroup
template <int BITS, int MT, int RG>
__global__ __launch_bounds__(GV_THREADS) void k_qgemv(GemvBatch bt) {
    extern __shared__ __align__(16) float gv_lds[];
    typedef gv_u32x4_t u32x4_a4_t __attribute__((aligned(4)));
    float2 *cb_lds = reinterpret_cast<float2 *>(gv_lds);        // K codewords
    float *red = gv_lds + 2 * bt.K;                             // [waves][rows][MT]
    const int lane = threadIdx.x & (WAVE - 1);
    const int wid = threadIdx.x >> 6;
    const float2 *cbk = reinterpret_cast<const float2 *>(bt.codebook);
    for (int i = threadIdx.x; i < bt.K; i += GV_THREADS) cb_lds[i] = cbk[i];
    __syncthreads();

    const int grp = blockIdx.x;                                 // the grid is exactly the number of row groups
    const int mi = gv_find(bt.grp_begin, bt.n, grp);
    const GemvMat &M = bt.mat[mi];
    const int row0 = (grp - bt.grp_begin[mi]) * GV_UNIT_ROWS;
    const int n_slabs = M.n_slabs, m = bt.m;
    const int d_out = M.d_out, d_in = M.d_in, last_row = M.d_out - 1;
    const int64_t row_bytes = M.row_bytes;
    const uint8_t *packed = M.packed;
    const float *Z = M.Z;
    const unsigned row_dw = (unsigned)(row_bytes >> 2);

    for (int rg = 0; rg < GV_UNIT_ROWS / RG; ++rg) {
        float a[MT][RG];                                        // per-lane sums of this group's rows
#pragma unroll
        for (int t = 0; t < MT; ++t)
#pragma unroll
            for (int r = 0; r < RG; ++r) a[t][r] = 0.0f;
        for (int slab = wid; slab < n_slabs; slab += GV_WAVES) {
            const int col0 = slab * GV_SLAB + 16 * lane;       // no transform here: lanes in natural column order
            const bool active = col0 < d_in;
            const int c = active ? col0 : 0;
            const unsigned lane_off = (unsigned)(c >> 4) * BITS;   // the lane's 8 fields: BITS bytes, same place in every row
            const unsigned lane_b0 = lane_off & ~3u;
            const int sh = (int)(lane_off & 3u) * 8;
            // packed words of the group's rows, all requested before any is used
            uint32_t d[RG][4];
#pragma unroll
            for (int r = 0; r < RG; ++r) {
                const int row = min(row0 + rg * RG + r, last_row);  // rows past the end re-read the last row
                const uint8_t *rowp = packed + (int64_t)row * row_bytes;
                if (row != last_row) {
                    // 16 bytes from a 4-byte-aligned address; may run a few bytes into the next row
                    const gv_u32x4_t v = *reinterpret_cast<const u32x4_a4_t *>(rowp + lane_b0);
                    d[r][0] = v[0]; d[r][1] = v[1]; d[r][2] = v[2]; d[r][3] = v[3];
                } else {
                    // last row of the matrix: stay inside it (the clamped words are beyond the lane's fields)
                    const uint32_t *rw = reinterpret_cast<const uint32_t *>(rowp);
#pragma unroll
                    for (int k = 0; k < 4; ++k) d[r][k] = rw[min((lane_b0 >> 2) + k, row_dw - 1u)];
                }
            }
            // the slab's rotated activations, zero for missing tokens and idle lanes
            float z[MT][16];
#pragma unroll
            for (int t = 0; t < MT; ++t) {
                const bool have = active && t < m;
                const float4 *src = reinterpret_cast<const float4 *>(Z + (int64_t)(t < m ? t : 0) * d_in + c);
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const float4 v = src[q];
                    z[t][4 * q] = have ? v.x : 0.0f;
                    z[t][4 * q + 1] = have ? v.y : 0.0f;
                    z[t][4 * q + 2] = have ? v.z : 0.0f;
                    z[t][4 * q + 3] = have ? v.w : 0.0f;
                }
            }
#pragma unroll
            for (int r = 0; r < RG; ++r) {
                uint32_t w[4];
                w[0] = __builtin_amdgcn_alignbit(d[r][1], d[r][0], sh);
                w[1] = __builtin_amdgcn_alignbit(d[r][2], d[r][1], sh);
                w[2] = __builtin_amdgcn_alignbit(d[r][3], d[r][2], sh);
                w[3] = d[r][3] >> sh;
#pragma unroll
                for (int k = 0; k < 8; ++k) {
                    const float2 cw = cb_lds[gv_field<BITS>(w, k)];
#pragma unroll
                    for (int t = 0; t < MT; ++t)
                        a[t][r] = __builtin_fmaf(cw.y, z[t][2 * k + 1], __builtin_fmaf(cw.x, z[t][2 * k], a[t][r]));
                }
            }
        }
        // totals over the lanes; one lane of each 16-lane row stores its RG/4 rows
        const int first = rg * RG + (lane >> 5) * (RG / 2) + ((lane >> 4) & 1) * (RG / 4);
#pragma unroll
        for (int t = 0; t < MT; ++t) {
            gv_reduce_rows<RG>(a[t]);
            if ((lane & 15) == 0) {
#pragma unroll
                for (int j = 0; j < RG / 4; ++j) red[(wid * GV_UNIT_ROWS + first + j) * MT + t] = a[t][j];
            }
        }
    }
    __syncthreads();
    // the 4 waves' sums in wave order, times the row norm
    const int o = threadIdx.x;
    if (o < GV_UNIT_ROWS * MT) {
        const int row = o / MT, t = o - row * MT;
        if (t < m && row0 + row <= last_row) {
            float s = 0.0f;
#pragma unroll
            for (int w = 0; w < GV_WAVES; ++w) s += red[(w * GV_UNIT_ROWS + row) * MT + t];
            M.Y[(int64_t)t * M.ldy + row0 + row] = M.norms[row0 + row] * s;
        }
    }
}

bool matmul_supported(const Problem &p, int m) {
    const int unit = p.block > 16 ? p.block : 16;
    if (p.d_in % unit || p.block < 64) return false;
    if (p.bits != 7 && p.bits != 8 && p.bits != 11) return false;
    return m >= 1 && m <= GV_MAX_M;
}

size_t matmul_workspace_bytes(int d_in, int d_out, int m) {
    (void)d_out;
    const size_t bytes = (size_t)m * d_in * sizeof(float);     // the rotated activations
    return (bytes + 15) / 16 * 16;
}

template <int XDTYPE>
static hipError_t launch_rotate(const GemvBatch &bt, int block, hipStream_t stream) {
    const unsigned blocks = (unsigned)((bt.rot_begin[bt.n] + GV_WAVES - 1) / GV_WAVES);
#define QAMW_ROT(BB) \
    case BB: hipLaunchKernelGGL((k_rotate_x<XDTYPE, BB>), dim3(blocks), dim3(GV_THREADS), 0, stream, bt); break;
    switch (block) {
        QAMW_ROT(64) QAMW_ROT(128) QAMW_ROT(256) QAMW_ROT(512) QAMW_ROT(1024)
        default: return hipErrorNotSupported;
    }
#undef QAMW_ROT
    return hipGetLastError();
}

template <int BITS>
static hipError_t launch_qgemv(const GemvBatch &bt, hipStream_t stream) {
    const unsigned blocks = (unsigned)bt.grp_begin[bt.n];
#define QAMW_GV(MM, RR)                                                                                              \
    hipLaunchKernelGGL((k_qgemv<BITS, MM, RR>), dim3(blocks), dim3(GV_THREADS),                                        \
                       ((size_t)bt.K * 2 + (size_t)GV_WAVES * GV_UNIT_ROWS * MM) * sizeof(float), stream, bt)
    if (bt.m == 1) QAMW_GV(1, 8);
    else if (bt.m == 2) QAMW_GV(2, 8);
    else if (bt.m <= 4) QAMW_GV(4, 8);
    else QAMW_GV(8, 4);
#undef QAMW_GV
    return hipGetLastError();
}

// Y_i = X_i W_i^T for n <= QAMW_MATMUL_MAX_BATCH matrices that share codebook, bits, block, m and the element type
// of X.  workspace: the sum of matmul_workspace_bytes() over the items, 16-byte aligned.
// Returns hipErrorNotSupported (nothing launched) outside the supported shapes.
hipError_t launch_matmul_batch(const MatmulItem *items, int n, int xdtype, int m, const Problem &p, void *workspace) {
    if (n < 1 || n > QAMW_MATMUL_MAX_BATCH) return hipErrorNotSupported;
    GemvBatch bt;
    int64_t rot = 0, groups = 0;
    char *ws = static_cast<char *>(workspace);
    for (int i = 0; i < n; ++i) {
        Problem q = p;
        q.d_in = items[i].d_in;
        q.d_out = items[i].d_out;
        if (!matmul_supported(q, m) || (reinterpret_cast<uintptr_t>(items[i].packed) & 3)) return hipErrorNotSupported;
        GemvMat &M = bt.mat[i];
        M.X = items[i].X;
        M.packed = items[i].packed;
        M.norms = items[i].norms;
        M.chan_scale = items[i].chan_scale;
        M.pair_sigma = items[i].pair_sigma;
        M.signs = items[i].signs;
        M.Y = items[i].Y;
        M.ldx = items[i].ldx;
        M.ldy = items[i].ldy;
        M.d_out = items[i].d_out;
        M.d_in = items[i].d_in;
        M.n_slabs = (M.d_in + GV_SLAB - 1) / GV_SLAB;
        M.sigma_default = (float)(1.0 / std::sqrt((double)M.d_in));
        M.row_bytes = (((int64_t)(M.d_in / 2) * p.bits + 31) / 32) * 4;
        M.Z = reinterpret_cast<float *>(ws);
        ws += matmul_workspace_bytes(M.d_in, M.d_out, m);
        bt.rot_begin[i] = (int)rot;
        bt.grp_begin[i] = (int)groups;
        rot += (int64_t)m * M.n_slabs;
        groups += (M.d_out + GV_UNIT_ROWS - 1) / GV_UNIT_ROWS;
        if (groups > 0x3fffffff || rot > 0x3fffffff) return hipErrorNotSupported;
    }
    for (int i = n; i <= QAMW_MATMUL_MAX_BATCH; ++i) {
        bt.rot_begin[i] = (int)rot;
        bt.grp_begin[i] = (int)groups;
    }
    for (int i = n; i < QAMW_MATMUL_MAX_BATCH; ++i) bt.mat[i] = bt.mat[0];
    bt.n = n;
    bt.m = m;
    bt.K = p.K;
    bt.inv_sqrt_block = p.inv_sqrt_block;
    bt.codebook = p.codebook;
    hipError_t e = xdtype == 0 ? launch_rotate<0>(bt, p.block, p.stream) : launch_rotate<1>(bt, p.block, p.stream);
    if (e != hipSuccess) return e;
    if (p.bits == 11) e = launch_qgemv<11>(bt, p.stream);
    else if (p.bits == 8) e = launch_qgemv<8>(bt, p.stream);
    else e = launch_qgemv<7>(bt, p.stream);
    return e;
}

}  // namespace qamw
