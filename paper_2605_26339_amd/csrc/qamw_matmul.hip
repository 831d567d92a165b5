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
// transform) and k_qgemv: a workgroup of 4 waves owns up to 64 rows of one matrix; its work is cut
// into (1024-column slab, 8-row group) steps, slab-major, and each wave takes a quarter of them; a
// wave holds the current slab's z in registers (the group's packed words requested together); per row it unpacks 8 indices,
// gathers 8 codewords from the LDS codebook and multiply-adds them into per-row, per-lane
// accumulators.  After each group one transposing reduction (each step
// trades half of the live sums with the lane whose number differs in one bit, so 8 sums per lane end
// as one row total per lane) adds the group's totals to the wave's running totals in LDS; at the end
// the 4 waves' totals are summed in a fixed order, times r_i, and stored.  The row count per
// workgroup is chosen per matrix so that every wave of a launch walks about the same, small number of
// (slab, row group) steps (about 4): a product alone in a launch -- as a forward pass issues most of them --
// takes as long as one wave's chain of dependent loads.
#include <algorithm>
#include <cmath>

#include "qamw_common.hpp"
#include "qamw_internal.hpp"
#include "qamw_wave_fwht.hpp"

namespace qamw {

constexpr int GV_THREADS = 256;
constexpr int GV_WAVES = GV_THREADS / WAVE;
constexpr int GV_SLAB = 1024;
constexpr int GV_RG = 8;                // rows per group: requested together, accumulated together
constexpr int GV_STEPS_PER_WG = 16;     // target number of (slab, 8-row group) steps per workgroup: 4 per wave
constexpr int GV_MIN_WGS = 256;         // a matrix is cut into at least this many workgroups when it has the rows
constexpr int GV_MAX_ROWS_PER_WG = 64;
constexpr int GV_AHEAD_MAX_WGS_2 = 512;        // two activation rows: launches of at most this many workgroups keep two steps' packed words in registers
constexpr int GV_SELF_ROTATE_MAX_WGS = 1024;   // launches of at most this many workgroups (and one or two activation rows) skip k_rotate_x
constexpr int GV_MAX_M = 8;                // activation rows of the vector-ALU kernel
constexpr int GM_MAX_M = 64;               // ... of the matrix-core kernel (QAMW_MATMUL_MAX_ROWS of the public header)
constexpr int GM_ROWS = 32;                // weight rows of a workgroup: one tile of the matrix instruction
constexpr int GM_HALF_TILE_MAX_WGS = 256;  // launches that would make at most this many 32-row workgroups use 16-row ones
constexpr int GM_WAVES = 8;                // waves of a workgroup: each takes every eighth chunk of the rows
constexpr int GM_THREADS = GM_WAVES * WAVE;
constexpr int GM_CHUNK = 256;              // columns of one step of a wave: 2 halves x 16 instructions x 8 columns

typedef uint32_t gv_u32x4_t __attribute__((ext_vector_type(4)));
typedef uint32_t gv_u32x2_t __attribute__((ext_vector_type(2)));
typedef float gv_f32x2_t __attribute__((ext_vector_type(2)));
typedef __bf16 gv_bf16x2_t __attribute__((ext_vector_type(2)));
typedef __bf16 gv_bf16x8_t __attribute__((ext_vector_type(8)));
typedef float gv_f32x16_t __attribute__((ext_vector_type(16)));

// One product of a batch, as the kernels see it.  Z and partial point into the caller's workspace.
struct GemvMat {
    const void *X;
    const uint8_t *packed;
    const float *norms, *chan_scale, *pair_sigma;
    const int8_t *signs;
    float *Z, *Y;
    int64_t ldx, ldy, row_bytes;
    int d_out, d_in, n_slabs;
    int rows_per_wg;                       // rows one workgroup takes: a multiple of GV_RG, at most GV_MAX_ROWS_PER_WG
    float sigma_default;                   // 1/sqrt(d_in), used when pair_sigma is NULL
};
// Work lists of one launch: rotation items (activation row, slab) and workgroups (rows_per_wg rows), each numbered
// matrix-major.
struct GemvBatch {
    GemvMat mat[QAMW_MATMUL_MAX_BATCH];
    int rot_begin[QAMW_MATMUL_MAX_BATCH + 1];
    int grp_begin[QAMW_MATMUL_MAX_BATCH + 1];
    int n, m, K;
    int xdtype;                            // element type of X: 0 fp32, 1 bf16
    int z_bf16;                            // 1: k_rotate_x writes bf16 rows, padded with zero rows to a multiple of 32 (matrix-core kernel)
    int gm_rows;                           // matrix-core kernel: weight rows per workgroup, 32 (a whole tile) or 16 (its upper half unused)
    float inv_sqrt_block;
    const float *codebook;
};
__device__ __forceinline__ int gv_find(const int *begin, int n, int u) {
    int i = 0;
    while (i + 1 < n && u >= begin[i + 1]) ++i;
    return i;
}

// Where the matrix-core kernel keeps 8 consecutive bf16 columns col .. col+7 (col a multiple of 8) of activation row tok:
// in the order its B operand is read -- [32-row tile][256-column chunk][half of the chunk][instruction 0..15][row in the
// tile][8 columns] -- so that the 32 lanes of a half-wave load 512 consecutive bytes.  In elements.
__device__ __forceinline__ int64_t gm_z_offset(int tok, int col, int d_in) {
    const int tile = tok >> 5, r = tok & 31, ch = col >> 8, within = col & 255, h = within >> 7, j = (within & 127) >> 3;
    return ((((int64_t)tile * (d_in >> 8) + ch) * 2 + h) * 16 + j) * 256 + r * 8;
}

// z = sigma (.) F S (x / s) of activation row tok for one 1024-column slab: lane l returns the 16 columns of sub-block
// slab_pos(l) (the order of the register transform); all 64 lanes of the wave call it together.  Lanes past the end of
// the row work on columns 0..15 (their blocks hold no lane that counts) and return values nobody uses.
// In two halves, so that a caller can have other memory requests on their way between the loads and the arithmetic.
template <int MT> struct GvRotIn {          // what one lane loads: 16 values of each of MT activation rows and their columns' constants
    float x[MT][16], scale[16], sigma[8];
    int8_t sign[16];
};
// tok[t]: the activation row that goes into x[t]
template <int XDTYPE, int MT>
__device__ __forceinline__ void gv_rotate_load(GvRotIn<MT> &in, const GemvMat &M, const int (&tok)[MT], int slab, int lane) {
    const int col0 = slab * GV_SLAB + 16 * slab_pos(lane);
    const int c = col0 < M.d_in ? col0 : 0;
#pragma unroll
    for (int t = 0; t < MT; ++t)
#pragma unroll
        for (int e = 0; e < 16; ++e) in.x[t][e] = Elem<XDTYPE>::load(M.X, (int64_t)tok[t] * M.ldx + c + e);
    if (M.chan_scale) {
#pragma unroll
        for (int e = 0; e < 16; ++e) in.scale[e] = M.chan_scale[c + e];
    }
    if (M.signs) {
#pragma unroll
        for (int e = 0; e < 16; ++e) in.sign[e] = M.signs[c + e];
    }
    if (M.pair_sigma) {
#pragma unroll
        for (int e = 0; e < 8; ++e) in.sigma[e] = M.pair_sigma[(c >> 1) + e];
    }
}
// The arithmetic: x times the reciprocal of the channel scale (the decoder's reciprocal, one Newton step), the sign mask,
// the transform, and one factor per pair -- lane sign of the transform x 1/sqrt(b) x sigma.
template <int B, int MT>
__device__ __forceinline__ void gv_rotate_compute(float (&y)[16], const GvRotIn<MT> &in, int t, const GemvBatch &bt, const GemvMat &M, int lane) {
    const LaneSigns<B> ls(lane);
#pragma unroll
    for (int e = 0; e < 16; ++e) y[e] = in.x[t][e];
    if (M.chan_scale) {
#pragma unroll
        for (int e = 0; e < 16; ++e) y[e] = y[e] * fast_recip(in.scale[e]);
    }
    if (M.signs) {
#pragma unroll
        for (int e = 0; e < 16; ++e) y[e] = (in.sign[e] < 0) ? -y[e] : y[e];
    }
    fwht_wave<B>(y, ls);
    const float k = ls.parity * bt.inv_sqrt_block;
    float g[8];
#pragma unroll
    for (int q = 0; q < 8; ++q) g[q] = k * (M.pair_sigma ? in.sigma[q] : M.sigma_default);
#pragma unroll
    for (int e = 0; e < 16; ++e) y[e] = y[e] * g[e >> 1];
}
template <int XDTYPE, int B>
__device__ __forceinline__ void gv_rotate_slab(float (&y)[16], const GemvBatch &bt, const GemvMat &M, int tok, int slab, int lane) {
    GvRotIn<1> in;
    const int toks[1] = {tok};
    gv_rotate_load<XDTYPE, 1>(in, M, toks, slab, lane);
    gv_rotate_compute<B, 1>(y, in, 0, bt, M, lane);
}

// z = sigma (.) F S (x / s) for every activation row: fp32, row-major [m][d_in], or bf16 in the order above.
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
    if (tok >= bt.m) {                                          // a padding row of the bf16 layout: zeros
        const int col = slab * GV_SLAB + 16 * lane;
        if (col < d_in) {
            uint16_t *zb = reinterpret_cast<uint16_t *>(M.Z);
            *reinterpret_cast<uint4 *>(zb + gm_z_offset(tok, col, d_in)) = make_uint4(0, 0, 0, 0);
            *reinterpret_cast<uint4 *>(zb + gm_z_offset(tok, col + 8, d_in)) = make_uint4(0, 0, 0, 0);
        }
        return;
    }
    const int col0 = slab * GV_SLAB + 16 * slab_pos(lane);
    const bool active = col0 < d_in;
    const int c = active ? col0 : 0;
    float y[16];
    gv_rotate_slab<XDTYPE, B>(y, bt, M, tok, slab, lane);
    if (active && !bt.z_bf16) {
        float4 *dst = reinterpret_cast<float4 *>(M.Z + (int64_t)tok * d_in + c);
#pragma unroll
        for (int t = 0; t < 4; ++t) dst[t] = make_float4(y[4 * t], y[4 * t + 1], y[4 * t + 2], y[4 * t + 3]);
    } else if (active) {                                        // bf16, round to nearest even
        uint32_t o[8];
#pragma unroll
        for (int e = 0; e < 16; e += 2) {
            const gv_f32x2_t v = {y[e], y[e + 1]};
            o[e >> 1] = __builtin_bit_cast(uint32_t, __builtin_convertvector(v, gv_bf16x2_t));
        }
        uint16_t *zb = reinterpret_cast<uint16_t *>(M.Z);
        *reinterpret_cast<uint4 *>(zb + gm_z_offset(tok, c, d_in)) = make_uint4(o[0], o[1], o[2], o[3]);
        *reinterpret_cast<uint4 *>(zb + gm_z_offset(tok, c + 8, d_in)) = make_uint4(o[4], o[5], o[6], o[7]);
    }
}

template <int BITS> __device__ __forceinline__ uint32_t gv_field(const uint32_t (&w)[4], int i) {
    const int bit = i * BITS, word = bit >> 5, off = bit & 31;
    uint32_t v = (off + BITS <= 32) ? (w[word] >> off) : __builtin_amdgcn_alignbit(w[word + 1], w[word], off);
    return v & ((1u << BITS) - 1u);
}

// Sums over the 64 lanes of N per-lane values a[0..N), N a power of two <= 64, leaving ONE total per lane:
// each step pairs lane l with lane l ^ 2^bit (bit = 5, 4, ..., ), every lane keeps the half of the live values
// selected by that bit of its number and adds what its partner held for that half.  When one value is left
// the remaining bits are summed in the ordinary way.  On return a[0] is the total of row gv_lane_row<N>(lane).
template <int N> __device__ __forceinline__ int gv_lane_row(int lane) {
    int row = 0, n = N;
#pragma unroll
    for (int bit = 5; bit >= 0 && n > 1; --bit) {
        n >>= 1;
        row += ((lane >> bit) & 1) * n;
    }
    return row;
}
// one step: LIVE values are live in a[0..LIVE); lane l pairs with lane l ^ 2^BIT
template <int N, int LIVE, int BIT> __device__ __forceinline__ void gv_reduce_step(float (&a)[N], int lane) {
    if constexpr (LIVE > 1) {
        constexpr int H = LIVE / 2;
#pragma unroll
        for (int r = 0; r < H; ++r) {
            if constexpr (BIT == 5) {
                auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(a[r]), __float_as_uint(a[r + H]), false, false);
                a[r] = __uint_as_float(sw[0]) + __uint_as_float(sw[1]);
            } else if constexpr (BIT == 4) {
                auto sw = __builtin_amdgcn_permlane16_swap(__float_as_uint(a[r]), __float_as_uint(a[r + H]), false, false);
                a[r] = __uint_as_float(sw[0]) + __uint_as_float(sw[1]);
            } else {
                const bool up = (lane >> BIT) & 1;
                const float send = up ? a[r] : a[r + H], keep = up ? a[r + H] : a[r];
                a[r] = keep + __shfl_xor(send, 1 << BIT, WAVE);
            }
        }
    } else {
        a[0] += __shfl_xor(a[0], 1 << BIT, WAVE);
    }
}
template <int N> __device__ __forceinline__ void gv_reduce_rows(float (&a)[N], int lane) {
    static_assert(N >= 1 && N <= 64 && (N & (N - 1)) == 0, "rows per reduction");
    gv_reduce_step<N, N, 5>(a, lane);
    gv_reduce_step<N, (N > 1 ? N / 2 : 1), 4>(a, lane);
    gv_reduce_step<N, (N > 2 ? N / 4 : 1), 3>(a, lane);
    gv_reduce_step<N, (N > 4 ? N / 8 : 1), 2>(a, lane);
    gv_reduce_step<N, (N > 8 ? N / 16 : 1), 1>(a, lane);
    gv_reduce_step<N, (N > 16 ? N / 32 : 1), 0>(a, lane);
}

// Y[t][row] = r_row * sum over the row's pairs of <c[idx], z_t>.  RB == 0: z comes from the workspace (k_rotate_x ran
// before).  RB > 0 (the block size): every wave rotates the slabs it needs itself, with the same arithmetic, and moves
// the result from the transform's lane order to the natural one -- the same z in the same lanes, so the same Y, bit for
// bit, without the first launch; for launches so small that a second launch costs more than the repeated rotations.
// AHEAD (self-rotating kernels only): the wave keeps two steps' packed words in registers; one activation row fits
// three waves per SIMD (768 resident workgroups: a launch of up to 1024 finishes its last quarter in a second round),
// two rows fit two (512 workgroups: the host picks the plain form for larger two-row launches).
#define QAMW_GV_WAVES_PER_EU (AHEAD ? (MT == 1 ? 3 : 2) : 1)
template <int BITS, int MT, int RB, int AHEAD>
__global__ __launch_bounds__(GV_THREADS) __attribute__((amdgpu_waves_per_eu(QAMW_GV_WAVES_PER_EU)))
void k_qgemv(GemvBatch bt) {
    constexpr int RG = MT == 8 ? 4 : GV_RG, UR = GV_MAX_ROWS_PER_WG;
    // statically sized, so that a codeword's address is its index times 8 with nothing to add (bt.K == 2^BITS)
    __shared__ float2 cb_lds[1 << BITS];                        // the codewords
    __shared__ float red[GV_WAVES * UR * MT];                   // [waves][UR rows][MT]
    typedef gv_u32x4_t u32x4_a4_t __attribute__((aligned(4)));
    const int lane = threadIdx.x & (WAVE - 1);
    const int wid = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // uniform over the wave: keeps the step bookkeeping scalar

    const int grp = blockIdx.x;                                 // the grid is exactly the number of workgroups
    const int mi = gv_find(bt.grp_begin, bt.n, grp);
    const GemvMat &M = bt.mat[mi];
    const int rpw = M.rows_per_wg;
    const int row0 = (grp - bt.grp_begin[mi]) * rpw;
    const int n_g = rpw / RG;                                   // row groups of this workgroup
    const int n_slabs = M.n_slabs, m = bt.m;
    const int d_in = M.d_in, last_row = M.d_out - 1;
    const int64_t row_bytes = M.row_bytes;
    const uint8_t *packed = M.packed;
    const float *Z = M.Z;
    const unsigned row_dw = (unsigned)(row_bytes >> 2);

    auto lane_col = [&](int slab) {                             // first of the lane's 16 columns (0 for idle lanes)
        const int col0 = slab * GV_SLAB + 16 * lane;           // no transform here: lanes in natural column order
        return col0 < d_in ? col0 : 0;
    };
    auto fetch = [&](int slab, int g, uint32_t (&d)[RG][4]) {
        const unsigned lane_b0 = ((unsigned)(lane_col(slab) >> 4) * BITS) & ~3u;   // the lane's 8 fields: BITS bytes, same place in every row
        const int r0 = row0 + g * RG;
        if (r0 + RG - 1 < last_row) {
            // 16 bytes from a 4-byte-aligned address; may run a few bytes into the next row
            const uint8_t *base = packed + (int64_t)r0 * row_bytes + lane_b0;
#pragma unroll
            for (int r = 0; r < RG; ++r) {
                const gv_u32x4_t v = *reinterpret_cast<const u32x4_a4_t *>(base + (int64_t)r * row_bytes);
                d[r][0] = v[0]; d[r][1] = v[1]; d[r][2] = v[2]; d[r][3] = v[3];
            }
        } else {
            // the group reaches the matrix's last row: rows past the end re-read the last row, and every
            // load stays inside its row (the clamped words are beyond the lane's fields)
#pragma unroll
            for (int r = 0; r < RG; ++r) {
                const uint32_t *rw = reinterpret_cast<const uint32_t *>(packed + (int64_t)min(r0 + r, last_row) * row_bytes);
#pragma unroll
                for (int k = 0; k < 4; ++k) d[r][k] = rw[min((lane_b0 >> 2) + k, row_dw - 1u)];
            }
        }
    };
    // the lane whose transform sub-block is this lane's natural one (slab_pos permutes inside groups of 16 lanes)
    int z_from = 0;
    if (RB > 0) {
#pragma unroll
        for (int l = 0; l < 16; ++l) z_from = (slab_pos(l) == (lane & 15)) ? l : z_from;
        z_from = ((lane & ~15) | z_from) << 2;
    }
    // The slab's rotated activations, zero for missing rows of X and idle lanes: the self-rotating kernels load the
    // inputs (rot_load) and rotate (rot_finish) in two steps, the others read the rotation kernel's output.
    auto rot_load = [&](int slab, GvRotIn<MT> &in) {
        int toks[MT];
#pragma unroll
        for (int t = 0; t < MT; ++t) toks[t] = t < m ? t : 0;
        if (bt.xdtype == 0) gv_rotate_load<0, MT>(in, M, toks, slab, lane);
        else gv_rotate_load<1, MT>(in, M, toks, slab, lane);
    };
    auto rot_finish = [&](int slab, const GvRotIn<MT> &in, float (&z)[MT][16]) {
        const bool active = slab * GV_SLAB + 16 * lane < d_in;
#pragma unroll
        for (int t = 0; t < MT; ++t) {
            const bool have = active && t < m;
            float y[16];
            constexpr int B = RB > 0 ? RB : 64;
            gv_rotate_compute<B, MT>(y, in, t, bt, M, lane);
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const float v = __int_as_float(__builtin_amdgcn_ds_bpermute(z_from, __float_as_int(y[e])));
                z[t][e] = have ? v : 0.0f;
            }
        }
    };
    auto load_z = [&](int slab, float (&z)[MT][16]) {
        if constexpr (RB > 0) {
            GvRotIn<MT> in;
            rot_load(slab, in);
            rot_finish(slab, in, z);
        } else {
            const bool active = slab * GV_SLAB + 16 * lane < d_in;
            const int c = lane_col(slab);
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
        }
    };

    // The workgroup's work is n_slabs x n_g steps (slab-major: one slab's row groups are consecutive); wave w takes
    // the w-th quarter of them, so the waves are equally loaded whatever the slab count is.
    const int n_steps = n_slabs * n_g;
    const int per_wave = (n_steps + GV_WAVES - 1) / GV_WAVES;
    const int step0 = wid * per_wave, step1 = min(n_steps, step0 + per_wave);
    float z[MT][16];
    int cur_slab = step0 < step1 ? step0 / n_g : -1;
    const int my_row = gv_lane_row<RG>(lane);                   // after the reduction: which of the group's rows this lane holds
    float *my_red = red + wid * UR * MT;                        // this wave's running row totals (only this wave touches them until the last barrier)

    // one step: the group's 8 x 64 x 8 codeword gathers and multiply-adds, the totals over the lanes, into my_red
    auto work = [&](int step, const uint32_t (&d)[RG][4]) {
        const int slab = step / n_g, g = step - slab * n_g;
        const int sh = (int)(((unsigned)(lane_col(slab) >> 4) * BITS) & 3u) * 8;
        float acc[MT][RG];
#pragma unroll
        for (int t = 0; t < MT; ++t)
#pragma unroll
            for (int r = 0; r < RG; ++r) acc[t][r] = 0.0f;
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
                    acc[t][r] = __builtin_fmaf(cw.y, z[t][2 * k + 1], __builtin_fmaf(cw.x, z[t][2 * k], acc[t][r]));
            }
        }
        // totals over the lanes: every lane ends with one of the group's RG rows (64 / RG lanes hold each, the ones that
        // share the lane number's upper bits); the first of them adds it in
#pragma unroll
        for (int t = 0; t < MT; ++t) gv_reduce_rows<RG>(acc[t], lane);
        if ((lane & (WAVE / RG - 1)) == 0) {
#pragma unroll
            for (int t = 0; t < MT; ++t) my_red[(g * RG + my_row) * MT + t] += acc[t][0];
        }
    };
    auto fetch_step = [&](int step, uint32_t (&d)[RG][4]) {
        const int slab = step / n_g;
        fetch(slab, step - slab * n_g, d);
    };

    static_assert(!AHEAD || RB > 0, "only the self-rotating kernels run ahead");
    if constexpr (!AHEAD) {
        if (cur_slab >= 0) load_z(cur_slab, z);                 // on its way while the codebook is staged
        // For more than one activation row the codebook goes from memory straight into LDS: wave w copies the 1 KB
        // pieces w, w + 4, ..., lane l the 16 bytes l of a piece (the instruction places lane l's bytes at base + 16 l);
        // measured 6 % faster at m = 4, 1-3 % slower at m = 1, where it goes through registers.
        if (MT > 1) {
            const char *src = reinterpret_cast<const char *>(bt.codebook);
            const int bytes = bt.K * (int)sizeof(float2);
            for (int off = wid * 1024; off < bytes; off += GV_WAVES * 1024) {
                if (off + 16 * lane < bytes)
                    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(src + off + 16 * lane),
                                                     (__attribute__((address_space(3))) void *)(reinterpret_cast<char *>(cb_lds) + off),
                                                     16, 0, 0);
            }
            __builtin_amdgcn_s_waitcnt(0x0F70);                // vmcnt(0): this wave's pieces have landed before the barrier
        } else {
            const float2 *cbk = reinterpret_cast<const float2 *>(bt.codebook);
            for (int i = threadIdx.x; i < bt.K; i += GV_THREADS) cb_lds[i] = cbk[i];
        }
        for (int i = lane; i < UR * MT; i += WAVE) my_red[i] = 0.0f;
        __syncthreads();
#pragma unroll 1
        for (int step = step0; step < step1; ++step) {
            const int slab = step / n_g;
            if (slab != cur_slab) {
                load_z(slab, z);
                cur_slab = slab;
            }
            uint32_t d[RG][4];
            fetch_step(step, d);
            work(step, d);
        }
    } else {
        // A launch that rotates the activations itself is a small one -- one to three waves per SIMD, two to four steps
        // per wave -- and lasts as long as one wave's chain of memory round trips.  So the chain is kept short: the
        // rotation's inputs, the workgroup's share of the codebook and the packed words of the wave's first two steps
        // are requested before anything is waited for (the rotation's first: it has arithmetic to do while the rest
        // arrives), and from then on the next step's packed words are on their way while a step is worked on.
        // bt.K == 2^BITS here.
        constexpr int KC = 1 << BITS, CB_PER_THREAD = (KC + GV_THREADS - 1) / GV_THREADS;
        GvRotIn<MT> rin;
        rot_load(cur_slab >= 0 ? cur_slab : 0, rin);
        float2 cbv[CB_PER_THREAD];
        const float2 *cbk = reinterpret_cast<const float2 *>(bt.codebook);
#pragma unroll
        for (int j = 0; j < CB_PER_THREAD; ++j) cbv[j] = cbk[min((int)threadIdx.x + j * GV_THREADS, KC - 1)];
        uint32_t da[RG][4], db[RG][4];
        if (step0 < step1) fetch_step(step0, da);
        if (step0 + 1 < step1) fetch_step(step0 + 1, db);
        if (cur_slab >= 0) rot_finish(cur_slab, rin, z);
#pragma unroll
        for (int j = 0; j < CB_PER_THREAD; ++j)
            if ((int)threadIdx.x + j * GV_THREADS < KC) cb_lds[threadIdx.x + j * GV_THREADS] = cbv[j];
        for (int i = lane; i < UR * MT; i += WAVE) my_red[i] = 0.0f;
        __syncthreads();
        auto keep_z = [&](int step) {
            const int slab = step / n_g;
            if (slab != cur_slab) {
                load_z(slab, z);
                cur_slab = slab;
            }
        };
#pragma unroll 1
        for (int step = step0; step < step1; step += 2) {
            keep_z(step);
            work(step, da);
            if (step + 2 < step1) fetch_step(step + 2, da);
            if (step + 1 < step1) {
                keep_z(step + 1);
                work(step + 1, db);
                if (step + 3 < step1) fetch_step(step + 3, db);
            }
        }
    }
    __syncthreads();
    // the 4 waves' sums in wave order, times the row norm
    for (int o = threadIdx.x; o < rpw * MT; o += GV_THREADS) {
        const int row = o / MT, t = o - row * MT;
        if (t < m && row0 + row <= last_row) {
            float s = 0.0f;
#pragma unroll
            for (int w = 0; w < GV_WAVES; ++w) s += red[(w * UR + row) * MT + t];
            M.Y[(int64_t)t * M.ldy + row0 + row] = M.norms[row0 + row] * s;
        }
    }
}

// ---------------------------------------------------------------------------------------------------------
// More than 8 activation rows: the products go to the bf16 matrix cores.
//   Y[t][i] = r_i * sum_k < bf16(c[idx_ik]), bf16(z_tk) >,   fp32 accumulation,
// z as above but rounded to bf16 (round to nearest even) by k_rotate_x, the codewords rounded to bf16 when the
// workgroup stages them: what a bf16 matmul on a bf16 copy of the rotated-domain operands computes.
//
// v_mfma_f32_32x32x16_bf16 with A = 32 weight rows x 16 columns, B = 16 columns x 32 activation rows: lane
// (r, h) supplies row r's 8 columns of half h to A -- exactly 4 pairs, i.e. 4 codewords, each one 32-bit
// LDS gather of (bf16 c0, bf16 c1) -- and activation row r's same 8 columns to B (16 bytes of z).
// A workgroup of 8 waves owns 32 weight rows (one tile); the 256-column chunks of the rows are dealt to the
// waves round-robin; within a chunk half h of the wave covers columns 128h .. 128h+127, so a lane walks 64
// consecutive pairs of its row: 8*BITS consecutive bytes, read as BITS 8-byte words from the wave's LDS copy
// of the chunk and unpacked at compile-time bit offsets.  No barrier inside the loop; the eight waves' tiles
// are summed through LDS in wave order at the end.  The shape follows from what bounds a launch: the chain of
// dependent chunk loads of its longest workgroup (a wave has one chunk in flight), so short chains -- many
// waves per row, few rows per workgroup -- beat shared operands; 128 registers keep 16 waves on a CU.
template <int BITS> __device__ __forceinline__ uint32_t gm_field_x4(const uint32_t (&w)[2 * BITS], int i) {
    // 4 * (field i of the lane's 64-field stream): the byte offset of the codeword in the bf16 table
    const int bit = i * BITS, word = bit >> 5, off = bit & 31;
    const uint32_t v = (off + BITS <= 32) ? (w[word] >> off) : __builtin_amdgcn_alignbit(w[word + 1], w[word], off);
    return (v & ((1u << BITS) - 1u)) << 2;
}

template <int BITS, int MT>
__global__ __launch_bounds__(GM_THREADS) __attribute__((amdgpu_waves_per_eu(4, 8)))   // two workgroups per CU: at most 128 registers
void k_qgemm(GemvBatch bt) {
    extern __shared__ __align__(16) uint32_t gm_lds[];
    uint32_t *cbh = gm_lds;                                     // K codewords as (bf16 c0) | (bf16 c1) << 16
    // after the codebook: per wave a 32-row tile of packed bytes (pitch PITCH) during the loop, and, after it, the
    // partial tiles of waves 1..7: [7 waves][MT][16][64 lanes]
    float *red = reinterpret_cast<float *>(gm_lds + bt.K);
    constexpr int PITCH = 16 * BITS + 8;                        // bytes; an odd number of 8-byte words: the lanes' 8-byte reads spread over all banks
    const int lane = threadIdx.x & (WAVE - 1);
    const int wid = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int r = lane & 31, h = lane >> 5;
    char *tile = reinterpret_cast<char *>(gm_lds + bt.K) + (size_t)wid * (GM_ROWS * PITCH);

    const int grp = blockIdx.x;
    const int mi = gv_find(bt.grp_begin, bt.n, grp);
    const GemvMat &M = bt.mat[mi];
    // rows of the tile this workgroup fills: all 32, or the first 16 (a launch of few workgroups is cut finer so that it
    // covers the chip; a row's sum is the same chunks in the same waves in the same order either way, bit for bit)
    const int rows = bt.gm_rows;
    const bool row_used = r < rows;
    const int row0 = (grp - bt.grp_begin[mi]) * rows;
    const int d_in = M.d_in, last_row = M.d_out - 1, m = bt.m;
    const int64_t row_bytes = M.row_bytes;
    const uint16_t *Zb = reinterpret_cast<const uint16_t *>(M.Z);
    const int n_chunks = d_in / GM_CHUNK;

    {   // stage the codebook, rounded to bf16
        const float2 *cbk = reinterpret_cast<const float2 *>(bt.codebook);
        for (int i = threadIdx.x; i < bt.K; i += GM_THREADS) {
            const float2 c = cbk[i];
            const gv_f32x2_t v = {c.x, c.y};
            cbh[i] = __builtin_bit_cast(uint32_t, __builtin_convertvector(v, gv_bf16x2_t));
        }
        __syncthreads();
    }

    // The chunk's packed bytes of the workgroup's 32 rows -- BITS 16-byte pieces per row -- are loaded with consecutive
    // lanes on consecutive pieces (piece 64 i + lane of the row-major 32 x BITS array) and laid down in LDS row by row.
    // Rows past the end of the matrix re-read the last row (their results are not stored); the pieces past the tile's
    // last row (rows x BITS is not always a multiple of 64) are neither loaded nor written to LDS.
    // (the offsets are recomputed where they are used: the vector ALU is idle here and the registers are not)
    constexpr int PIECES = (GM_ROWS * BITS + 63) / 64;
    const int tile_pieces = rows * BITS;
    auto src_off = [&](int i) {
        const int piece = 64 * i + lane, row = piece / BITS, c16 = piece - row * BITS;
        return min(row0 + row, last_row) * (int)row_bytes + 16 * c16;
    };
    auto dst_off = [&](int i) {
        const int piece = 64 * i + lane, row = piece / BITS, c16 = piece - row * BITS;
        return row * PITCH + 16 * c16;
    };
    const uint16_t *zrow[MT];
#pragma unroll
    for (int t = 0; t < MT; ++t) zrow[t] = Zb + ((int64_t)t * n_chunks * 2 + h) * 16 * 256 + r * 8;   // padded rows exist and are zero

    gv_f32x16_t acc[MT];
#pragma unroll
    for (int t = 0; t < MT; ++t)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[t][i] = 0.0f;

    // Wave w takes the chunks w, w + 8, ...: at any time the eight waves read neighbouring pieces of the same rows.
    // The packed bytes of the wave's next chunk are requested before the current chunk's matrix instructions start.
    typedef gv_u32x4_t u32x4_a4_t __attribute__((aligned(4)));
    gv_u32x4_t v[PIECES];
#pragma unroll
    for (int i = 0; i < PIECES; ++i) v[i] = gv_u32x4_t{0u, 0u, 0u, 0u};
    if (wid < n_chunks) {
        const uint8_t *src = M.packed + (int64_t)wid * (16 * BITS);
#pragma unroll
        for (int i = 0; i < PIECES; ++i)
            if (64 * i + lane < tile_pieces) v[i] = *reinterpret_cast<const u32x4_a4_t *>(src + src_off(i));
    }
#pragma unroll 1
    for (int ch = wid; ch < n_chunks; ch += GM_WAVES) {
        // the chunk's packed bytes go through LDS: written piece by piece, read back as the lane's stream of 64 pairs
#pragma unroll
        for (int i = 0; i < PIECES; ++i) {
            if (64 * i + lane >= tile_pieces) continue;
            gv_u32x2_t *dst = reinterpret_cast<gv_u32x2_t *>(tile + dst_off(i));
            dst[0] = gv_u32x2_t{v[i][0], v[i][1]};
            dst[1] = gv_u32x2_t{v[i][2], v[i][3]};
        }
        uint32_t w[2 * BITS];
        if (row_used) {
            const gv_u32x2_t *src = reinterpret_cast<const gv_u32x2_t *>(tile + r * PITCH + 8 * BITS * h);
#pragma unroll
            for (int q = 0; q < BITS; ++q) {
                const gv_u32x2_t x2 = src[q];
                w[2 * q] = x2[0];
                w[2 * q + 1] = x2[1];
            }
        }
        // activations of this chunk, ZB instructions' worth at a time: 8, or 2 with two tiles of activation rows (the
        // kernel has 128 registers)
        constexpr int ZB = 8 / (MT * MT);
        gv_u32x4_t zb[MT][ZB];
        auto load_zb = [&](int first) {
#pragma unroll
            for (int t = 0; t < MT; ++t) {
                const uint16_t *src = zrow[t] + ((int64_t)ch * 2 * 16 + first) * 256;
#pragma unroll
                for (int j = 0; j < ZB; ++j) zb[t][j] = *reinterpret_cast<const gv_u32x4_t *>(src + j * 256);
            }
        };
        load_zb(0);
        if (ch + GM_WAVES < n_chunks) {                         // the next chunk's packed bytes
            const uint8_t *src = M.packed + (int64_t)(ch + GM_WAVES) * (16 * BITS);
#pragma unroll
            for (int i = 0; i < PIECES; ++i)
                if (64 * i + lane < tile_pieces) v[i] = *reinterpret_cast<const u32x4_a4_t *>(src + src_off(i));
        }
#pragma unroll
        for (int step = 0; step < 16; ++step) {                 // instruction of the chunk: pairs 4 step .. 4 step + 3 of the lane's 64
            if (step > 0 && step % ZB == 0) load_zb(step);
            gv_u32x4_t a = {0u, 0u, 0u, 0u};                    // the unused half of a 16-row workgroup's tile: zeros, no gathers
            if (row_used) {
#pragma unroll
                for (int f = 0; f < 4; ++f)
                    a[f] = *reinterpret_cast<const uint32_t *>(reinterpret_cast<const char *>(cbh) + gm_field_x4<BITS>(w, 4 * step + f));
            }
            const gv_bf16x8_t av = __builtin_bit_cast(gv_bf16x8_t, a);
#pragma unroll
            for (int t = 0; t < MT; ++t)
                acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av, __builtin_bit_cast(gv_bf16x8_t, zb[t][step % ZB]), acc[t], 0, 0, 0);
        }
    }

    // the eight waves' tiles, summed in wave order by wave 0 (the buffer overlies the packed tiles: everybody is done with those)
    __syncthreads();
    if (wid > 0) {
        float *dst = red + (size_t)(wid - 1) * (MT * 16 * WAVE);
#pragma unroll
        for (int t = 0; t < MT; ++t)
#pragma unroll
            for (int i = 0; i < 16; ++i) dst[(t * 16 + i) * WAVE + lane] = acc[t][i];
    }
    __syncthreads();
    if (wid == 0) {
#pragma unroll
        for (int t = 0; t < MT; ++t) {
            const int tok = 32 * t + r;                         // the accumulator's column is the activation row
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                float s = acc[t][i];
#pragma unroll
                for (int w2 = 0; w2 < GM_WAVES - 1; ++w2) s += red[(size_t)w2 * (MT * 16 * WAVE) + (t * 16 + i) * WAVE + lane];
                const int tile_row = 8 * (i >> 2) + 4 * h + (i & 3);    // accumulator i of half h
                const int row = row0 + tile_row;
                if (tok < m && tile_row < rows && row <= last_row) M.Y[(int64_t)tok * M.ldy + row] = M.norms[row] * s;
            }
        }
    }
}

bool matmul_supported(const Problem &p, int m) {
    const int unit = p.block > 16 ? p.block : 16;
    if (p.d_in % unit || p.block < 64) return false;
    if (p.bits != 7 && p.bits != 8 && p.bits != 11) return false;
    if (m > GV_MAX_M) return m <= GM_MAX_M && p.d_in % GM_CHUNK == 0;      // the matrix-core kernel walks 256-column chunks
    return m >= 1;
}

size_t matmul_workspace_bytes(int d_in, int d_out, int m) {
    (void)d_out;
    // the rotated activations: fp32 rows, or (matrix-core kernel) bf16 rows padded to a multiple of 32 rows
    const size_t bytes = m <= GV_MAX_M ? (size_t)m * d_in * sizeof(float) : (size_t)((m + 31) / 32 * 32) * d_in * sizeof(uint16_t);
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

template <int BITS, int RB>
static hipError_t launch_qgemv_rb(const GemvBatch &bt, hipStream_t stream) {
    const unsigned blocks = (unsigned)bt.grp_begin[bt.n];
#define QAMW_GV(MM, AH) hipLaunchKernelGGL((k_qgemv<BITS, MM, RB, AH>), dim3(blocks), dim3(GV_THREADS), 0, stream, bt)
    if constexpr (RB > 0) {                                     // the self-rotating kernels exist for one and two rows
        if (bt.m == 1) QAMW_GV(1, 1);
        else if (bt.m == 2 && blocks <= GV_AHEAD_MAX_WGS_2) QAMW_GV(2, 1);
        else if (bt.m == 2) QAMW_GV(2, 0);
        else return hipErrorNotSupported;
    } else {
        if (bt.m == 1) QAMW_GV(1, 0);
        else if (bt.m == 2) QAMW_GV(2, 0);
        else if (bt.m <= 4) QAMW_GV(4, 0);
        else QAMW_GV(8, 0);
    }
#undef QAMW_GV
    return hipGetLastError();
}
// rotate_block: 0, or the block size when the product kernel is to rotate the activations itself
template <int BITS>
static hipError_t launch_qgemv(const GemvBatch &bt, int rotate_block, hipStream_t stream) {
    switch (rotate_block) {
        case 0: return launch_qgemv_rb<BITS, 0>(bt, stream);
        case 64: return launch_qgemv_rb<BITS, 64>(bt, stream);
        case 128: return launch_qgemv_rb<BITS, 128>(bt, stream);
        case 256: return launch_qgemv_rb<BITS, 256>(bt, stream);
        case 512: return launch_qgemv_rb<BITS, 512>(bt, stream);
        case 1024: return launch_qgemv_rb<BITS, 1024>(bt, stream);
        default: return hipErrorNotSupported;
    }
}

template <int BITS>
static hipError_t launch_qgemm(const GemvBatch &bt, hipStream_t stream) {
    const unsigned blocks = (unsigned)bt.grp_begin[bt.n];
    const int mt = (bt.m + 31) / 32;
    const size_t red_bytes = (size_t)(GM_WAVES - 1) * mt * 16 * WAVE * sizeof(float);
    const size_t tile_bytes = (size_t)GM_WAVES * GM_ROWS * (16 * BITS + 8);
    const size_t lds = (size_t)bt.K * sizeof(uint32_t) + (red_bytes > tile_bytes ? red_bytes : tile_bytes);
    if (mt == 1) hipLaunchKernelGGL((k_qgemm<BITS, 1>), dim3(blocks), dim3(GM_THREADS), lds, stream, bt);
    else hipLaunchKernelGGL((k_qgemm<BITS, 2>), dim3(blocks), dim3(GM_THREADS), lds, stream, bt);
    return hipGetLastError();
}

// Y_i = X_i W_i^T for n <= QAMW_MATMUL_MAX_BATCH matrices that share codebook, bits, block, m and the element type
// of X.  workspace: the sum of matmul_workspace_bytes() over the items, 16-byte aligned.
// Returns hipErrorNotSupported (nothing launched) outside the supported shapes.  variant: 0, or 1 / 2 to force the
// two-launch / the self-rotating form of the vector kernel.
hipError_t launch_matmul_batch(const MatmulItem *items, int n, int xdtype, int m, const Problem &p, void *workspace, int variant) {
    if (n < 1 || n > QAMW_MATMUL_MAX_BATCH || p.K != (1 << p.bits)) return hipErrorNotSupported;   // the kernels size the codebook from the bit width
    GemvBatch bt;
    int64_t rot = 0, groups = 0;
    char *ws = static_cast<char *>(workspace);
    // Matrix-core kernel: the products with the longest rows go first in the grid.  Their workgroups take longest (one
    // workgroup walks whole rows); started last, they would run on alone after everything else has finished.  The
    // order inside a launch changes no result.
    int order[QAMW_MATMUL_MAX_BATCH];
    for (int i = 0; i < n; ++i) order[i] = i;
    if (m > GV_MAX_M)
        std::stable_sort(order, order + n, [&](int a, int b) { return items[a].d_in > items[b].d_in; });
    // Matrix-core kernel: a launch whose matrices make at most GM_HALF_TILE_MAX_WGS workgroups of 32 rows (one 4096-row
    // projection makes 128) is cut into workgroups of 16 rows, so that it reaches every CU; a row's result does not
    // depend on the cut.
    int64_t tiles32 = 0;
    for (int i = 0; i < n; ++i) tiles32 += (items[i].d_out + GM_ROWS - 1) / GM_ROWS;
    bt.gm_rows = tiles32 <= GM_HALF_TILE_MAX_WGS ? GM_ROWS / 2 : GM_ROWS;
    for (int i = 0; i < n; ++i) {
        const MatmulItem &it = items[order[i]];
        Problem q = p;
        q.d_in = it.d_in;
        q.d_out = it.d_out;
        if (!matmul_supported(q, m) || (reinterpret_cast<uintptr_t>(it.packed) & 3)) return hipErrorNotSupported;
        GemvMat &M = bt.mat[i];
        M.X = it.X;
        M.packed = it.packed;
        M.norms = it.norms;
        M.chan_scale = it.chan_scale;
        M.pair_sigma = it.pair_sigma;
        M.signs = it.signs;
        M.Y = it.Y;
        M.ldx = it.ldx;
        M.ldy = it.ldy;
        M.d_out = it.d_out;
        M.d_in = it.d_in;
        M.n_slabs = (M.d_in + GV_SLAB - 1) / GV_SLAB;
        M.sigma_default = (float)(1.0 / std::sqrt((double)M.d_in));
        M.row_bytes = (((int64_t)(M.d_in / 2) * p.bits + 31) / 32) * 4;
        M.Z = reinterpret_cast<float *>(ws);
        ws += matmul_workspace_bytes(M.d_in, M.d_out, m);
        // Rows per workgroup, from the matrix's own shape only (so a product gives the same bits alone and in a
        // batch): about GV_STEPS_PER_WG (slab, row group) steps per workgroup, halved while the matrix would
        // otherwise make fewer than GV_MIN_WGS workgroups.
        int groups_per_wg = GV_STEPS_PER_WG / M.n_slabs;
        if (groups_per_wg < 1) groups_per_wg = 1;
        if (groups_per_wg > GV_MAX_ROWS_PER_WG / GV_RG) groups_per_wg = GV_MAX_ROWS_PER_WG / GV_RG;
        while (groups_per_wg > 1 && (M.d_out + groups_per_wg * GV_RG - 1) / (groups_per_wg * GV_RG) < GV_MIN_WGS) groups_per_wg >>= 1;
        M.rows_per_wg = groups_per_wg * GV_RG;
        if (m > GV_MAX_M) {                                     // matrix-core kernel: one tile, or half of one, per workgroup
            if ((int64_t)M.d_out * M.row_bytes > 0x7fffffff) return hipErrorNotSupported;   // 32-bit byte offsets into the packed matrix
            M.rows_per_wg = bt.gm_rows;
        }
        bt.rot_begin[i] = (int)rot;
        bt.grp_begin[i] = (int)groups;
        rot += (int64_t)(m > GV_MAX_M ? (m + 31) / 32 * 32 : m) * M.n_slabs;
        groups += (M.d_out + M.rows_per_wg - 1) / M.rows_per_wg;
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
    bt.z_bf16 = m > GV_MAX_M ? 1 : 0;
    bt.xdtype = xdtype;
    // One or two activation rows in a small launch (a forward pass issues one product, or the few that share an input,
    // per call): the product kernel rotates the activations itself.  Same results, one launch less.
    // (variant 1: never, 2: whenever there are one or two rows -- for tests and measurements)
    const bool self_rotate = m <= 2 && variant != 1 && (variant == 2 || groups <= GV_SELF_ROTATE_MAX_WGS);
    hipError_t e = hipSuccess;
    if (!self_rotate) e = xdtype == 0 ? launch_rotate<0>(bt, p.block, p.stream) : launch_rotate<1>(bt, p.block, p.stream);
    if (e != hipSuccess) return e;
    if (m > GV_MAX_M) {
        if (p.bits == 11) return launch_qgemm<11>(bt, p.stream);
        if (p.bits == 8) return launch_qgemm<8>(bt, p.stream);
        return launch_qgemm<7>(bt, p.stream);
    }
    const int rb = self_rotate ? p.block : 0;
    if (p.bits == 11) e = launch_qgemv<11>(bt, rb, p.stream);
    else if (p.bits == 8) e = launch_qgemv<8>(bt, rb, p.stream);
    else e = launch_qgemv<7>(bt, rb, p.stream);
    return e;
}

}  // namespace qamw
