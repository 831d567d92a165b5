// Encoder front half shared by the fast encode and calibration kernels (Sec. 3.1 steps 1-2 on
// the channel-scaled row of Sec. B.2): a lane loads its 16 consecutive columns, scales them,
// divides by the row norm, applies the sign mask and the wave runs the block Walsh-Hadamard
// transform.  On return y[e] = (F S u)[col0 + e] exactly as the library's fp32 arithmetic defines it.
#pragma once
#include "qamw_common.hpp"
#include "qamw_internal.hpp"
#include "qamw_wave_fwht.hpp"

namespace qamw {

// The lane's 16 weights as loaded: 16 fp32 (DTYPE 0) or 16 bf16 in 8 dwords (DTYPE 1).  Split from the arithmetic so that
// a kernel can request the next row before it works on the current one.
template <int DTYPE> struct RawRow {
    uint32_t w[DTYPE == 0 ? 16 : 8];
};
template <int DTYPE>
__device__ __forceinline__ void load_raw_row(RawRow<DTYPE> &raw, const void *__restrict__ W, int64_t row_base, int c) {
    const int64_t base = row_base + c;
    if (DTYPE == 0) {
        const uint4 *w4 = reinterpret_cast<const uint4 *>(reinterpret_cast<const float *>(W) + base);
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const uint4 v = w4[t];
            raw.w[4 * t] = v.x; raw.w[4 * t + 1] = v.y; raw.w[4 * t + 2] = v.z; raw.w[4 * t + 3] = v.w;
        }
    } else {
        const uint4 *w4 = reinterpret_cast<const uint4 *>(reinterpret_cast<const uint16_t *>(W) + base);
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            const uint4 v = w4[t];
            raw.w[4 * t] = v.x; raw.w[4 * t + 1] = v.y; raw.w[4 * t + 2] = v.z; raw.w[4 * t + 3] = v.w;
        }
    }
}

// c: first of the lane's 16 columns (multiple of 16, < d_in); r: the row's norm.
// Requires 16-byte aligned rows and side arrays (checked on the host).
template <int DTYPE, int B>
__device__ __forceinline__ void rotated_unit_row_from(float (&y)[16], const RawRow<DTYPE> &raw, int c, float r, const Problem &p,
                                                      const LaneSigns<B> &ls) {
    if (DTYPE == 0) {
#pragma unroll
        for (int e = 0; e < 16; ++e) y[e] = __uint_as_float(raw.w[e]);
    } else {
#pragma unroll
        for (int q = 0; q < 8; ++q) {                           // bf16 is the upper half of an fp32
            y[2 * q] = __uint_as_float(raw.w[q] << 16);
            y[2 * q + 1] = __uint_as_float(raw.w[q] & 0xFFFF0000u);
        }
    }
    if (p.chan_scale) {
        const float4 *s4 = reinterpret_cast<const float4 *>(p.chan_scale + c);
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            float4 v = s4[t];
            y[4 * t] *= v.x; y[4 * t + 1] *= v.y; y[4 * t + 2] *= v.z; y[4 * t + 3] *= v.w;
        }
    }
    // u = ws / r, the correctly rounded quotient.  With q = fl(1/r) correctly rounded, q0 = fl(ws q) and the exact
    // remainder rem = ws - q0 r (one fused multiply-add), fl(q0 + rem q) IS the correctly rounded ws / r (Markstein's
    // division theorem) as long as nothing under- or overflows on the way: r within 2^+-60 and every |ws| at least
    // 2^-100.  A wave that holds anything else (an exact zero included) takes the plain division for all its lanes.
    if (r > 0.0f) {
        float amin = fminf(fabsf(y[0]), fabsf(y[1]));
#pragma unroll
        for (int e = 2; e < 16; e += 2) amin = fminf(amin, fminf(fabsf(y[e]), fabsf(y[e + 1])));
        const bool plain = !(amin >= 7.8886090522e-31f) || !(r >= 8.6736173799e-19f && r <= 1.1529215046e18f);
        if (__ballot(plain) != 0ull) {
#pragma unroll
            for (int e = 0; e < 16; ++e) y[e] = y[e] / r;                       // IEEE division
        } else {
            const float q = 1.0f / r;                                           // IEEE division, once
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const float q0 = y[e] * q;
                const float rem = __builtin_fmaf(-q0, r, y[e]);
                y[e] = __builtin_fmaf(rem, q, q0);
            }
        }
    } else {
#pragma unroll
        for (int e = 0; e < 16; ++e) y[e] = 0.0f;
    }
    if (p.signs) {
        const uint4 sg = *reinterpret_cast<const uint4 *>(p.signs + c);
        const uint32_t wds[4] = {sg.x, sg.y, sg.z, sg.w};
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            uint32_t neg = (wds[e >> 2] >> (8 * (e & 3) + 7)) & 1u;             // int8 -1: sign bit of the byte
            y[e] = __uint_as_float(__float_as_uint(y[e]) ^ (neg << 31));
        }
    }
    fwht_wave<B>(y, ls);
#pragma unroll
    for (int e = 0; e < 16; ++e) y[e] = (y[e] * ls.parity) * p.inv_sqrt_block;
}

template <int DTYPE, int B>
__device__ __forceinline__ void rotated_unit_row(float (&y)[16], const void *__restrict__ W, int64_t row_base, int c,
                                                 float r, const Problem &p, const LaneSigns<B> &ls) {
    RawRow<DTYPE> raw;
    load_raw_row<DTYPE>(raw, W, row_base, c);
    rotated_unit_row_from<DTYPE, B>(y, raw, c, r, p, ls);
}

// ---------------------------------------------------------------------------------------------
// Row norms inside the kernels that need them (Sec. 3.1 step 1 on the channel-scaled row of Sec. B.2), so that the
// matrix is fetched from memory once per entry point instead of once by a norm kernel and once more by the kernel
// proper.
//
// A workgroup of NWAVES waves owns NWAVES consecutive (row, slab) items, which touch a few consecutive rows.  For every
// slab of every such row one wave sums the squares of the slab's 1024 scaled weights in fp64 (products of fp32 are
// exact in fp64; 16 per lane in column order, then the fixed butterfly of wave_sum) and leaves the sum in LDS; after
// the workgroup's barrier every wave adds its row's slab sums in slab order and takes the square root.  The value of a
// row's norm therefore does not depend on which workgroup computes it.  Rows shared by neighbouring workgroups are
// summed by each of them; fused_norm_block() numbers the workgroups so that neighbours run on the same XCD and
// find each other's rows in its L2.
// ---------------------------------------------------------------------------------------------
constexpr int FUSED_NORM_MAX_SLABS = 64;                       // rows of up to 65536 columns
constexpr int FUSED_NORM_XCDS = 8;

// Hardware workgroup b runs on XCD b mod 8.  Workgroup number used by the kernel: XCD x takes the x-th eighth of the
// work, in order.  A value >= n_blocks means: nothing to do.
__device__ __forceinline__ int fused_norm_block(int b, int n_blocks) {
    const int per = (n_blocks + FUSED_NORM_XCDS - 1) / FUSED_NORM_XCDS;
    return (b % FUSED_NORM_XCDS) * per + b / FUSED_NORM_XCDS;
}
inline int fused_norm_grid(int n_blocks) {                       // workgroups to launch for n_blocks of work
    return (n_blocks + FUSED_NORM_XCDS - 1) / FUSED_NORM_XCDS * FUSED_NORM_XCDS;
}

// Sum of squares of the scaled weights of columns [1024 slab, 1024 slab + 1024) of one row, the same in every lane.
template <int DTYPE>
__device__ __forceinline__ double slab_sum_of_squares(const void *__restrict__ W, int64_t row_base, int slab, const Problem &p,
                                                       int lane) {
    const int c = slab * 1024 + 16 * lane;
    double acc = 0.0;
    if (c < p.d_in) {
        RawRow<DTYPE> raw;
        load_raw_row<DTYPE>(raw, W, row_base, c);
        float w[16];
        if (DTYPE == 0) {
#pragma unroll
            for (int e = 0; e < 16; ++e) w[e] = __uint_as_float(raw.w[e]);
        } else {
#pragma unroll
            for (int q = 0; q < 8; ++q) {
                w[2 * q] = __uint_as_float(raw.w[q] << 16);
                w[2 * q + 1] = __uint_as_float(raw.w[q] & 0xFFFF0000u);
            }
        }
        if (p.chan_scale) {
            const float4 *s4 = reinterpret_cast<const float4 *>(p.chan_scale + c);
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const float4 v = s4[t];
                w[4 * t] *= v.x; w[4 * t + 1] *= v.y; w[4 * t + 2] *= v.z; w[4 * t + 3] *= v.w;
            }
        }
#pragma unroll
        for (int e = 0; e < 16; ++e) acc += (double)w[e] * (double)w[e];
    }
    return wave_sum(acc);
}

// Slab sums of every row touched by the items [item0, item0 + NWAVES) (clipped to n_items) into part[], dealt to
// the workgroup's waves.  The caller's barrier follows; then row_norm_from_slab_sums().
// part: LDS, 2 * max(n_slabs, NWAVES) doubles.  All waves of the workgroup call this.
template <int DTYPE, int NWAVES>
__device__ __forceinline__ void block_slab_sums(double *part, const void *__restrict__ W, int64_t ldw, const Problem &p, int item0,
                                                int n_items, int n_slabs, int lane, int wid) {
    const int last = min(item0 + NWAVES, n_items) - 1;
    const int r0 = item0 / n_slabs, r1 = last / n_slabs;
    const int tasks = (r1 - r0 + 1) * n_slabs;
    for (int t = __builtin_amdgcn_readfirstlane(wid); t < tasks; t += NWAVES) {
        const int dr = t / n_slabs, slab = t - dr * n_slabs;
        const double s2 = slab_sum_of_squares<DTYPE>(W, (int64_t)(r0 + dr) * ldw, slab, p, lane);
        if (lane == 0) part[t] = s2;
    }
}

// The norm of `row` from the slab sums left by block_slab_sums() (after the barrier): slab order, fp64, one rounding
// to fp32 after the square root.
__device__ __forceinline__ float row_norm_from_slab_sums(const double *part, int row, int item0, int n_slabs) {
    const double *src = part + (row - item0 / n_slabs) * n_slabs;
    double s2 = 0.0;
    for (int s = 0; s < n_slabs; ++s) s2 += src[s];
    return (float)sqrt(s2);
}

// Exact squared distance as every encoder decides with it: fma(e1, e1, e0 * e0), e = x - c.
__device__ __forceinline__ float exact_dist2(float x0, float x1, float2 c) {
    const float e0 = x0 - c.x, e1 = x1 - c.y;
    return __builtin_fmaf(e1, e1, e0 * e0);
}

// The nearest of the K codewords in LDS to the point (x0, x1) (the same in all lanes), found by the whole wave: lane l
// scans the codewords l, l + 64, ..., then a lexicographic (distance, index) reduction over the lanes; the lowest index
// wins a tie.  Every lane returns the index (0 if every distance is NaN).
__device__ __forceinline__ int wave_exact_scan(float x0, float x1, const float2 *cb_lds, int K, int lane) {
    float bd = 3.0e38f;
    int bi = 0x7fffffff;
    for (int k = lane; k < K; k += WAVE) {
        const float dd = exact_dist2(x0, x1, cb_lds[k]);
        if (dd < bd) {
            bd = dd;
            bi = k;
        }
    }
#pragma unroll
    for (int m = 1; m < WAVE; m <<= 1) {
        const float od = __shfl_xor(bd, m, WAVE);
        const int oi = __shfl_xor(bi, m, WAVE);
        if (od < bd || (od == bd && oi < bi)) {
            bd = od;
            bi = oi;
        }
    }
    return bi == 0x7fffffff ? 0 : bi;
}

// The lane's 8 pair gains g_k = 1 / sigma_k (IEEE division), or sqrt(d_in) when no pair scales are given; c = first of
// the lane's 16 columns.
__device__ __forceinline__ void load_pair_gains(float (&g)[8], const Problem &p, int c) {
    if (p.pair_sigma) {
        const float4 *g4 = reinterpret_cast<const float4 *>(p.pair_sigma + (c >> 1));
        const float4 a = g4[0], b = g4[1];
        const float sg8[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
#pragma unroll
        for (int k = 0; k < 8; ++k) g[k] = 1.0f / sg8[k];                         // IEEE division
    } else {
#pragma unroll
        for (int k = 0; k < 8; ++k) g[k] = p.g_default;
    }
}

// Writes the lane's 8 indices into the row's bit stream: 8 fields of p.bits bits are exactly p.bits bytes, byte aligned
// at byte (c / 16) * bits of the row.  The lane that holds the row's last 16 columns (col0 + 16 == d_in) zeroes the
// padding bytes of the row.
__device__ __forceinline__ void store_packed_fields(uint8_t *__restrict__ packed, int row, int c, int col0,
                                                    const unsigned (&idx)[8], const Problem &p) {
    const int bits = p.bits;
    uint8_t *dst = packed + (int64_t)row * p.row_bytes + (int64_t)(c >> 4) * bits;
    unsigned __int128 acc = 0;
#pragma unroll
    for (int k = 0; k < 8; ++k) acc |= (unsigned __int128)idx[k] << (k * bits);
    for (int t = 0; t < bits; ++t) dst[t] = (uint8_t)(acc >> (8 * t));
    if (col0 + 16 == p.d_in) {
        const int64_t used = (int64_t)(p.d_in >> 4) * bits;
        uint8_t *rowp = packed + (int64_t)row * p.row_bytes;
        for (int64_t t = used; t < p.row_bytes; ++t) rowp[t] = 0;
    }
}

// Host-side check of what the vector loads above assume.
inline bool front_alignment_ok(const void *W, int dtype, int64_t ldw, const Problem &p) {
    const int64_t row_align = dtype == 0 ? 4 : 8;
    return (ldw % row_align == 0) && ((reinterpret_cast<uintptr_t>(W) & 15) == 0) &&
           (((reinterpret_cast<uintptr_t>(p.chan_scale) | reinterpret_cast<uintptr_t>(p.signs) |
              reinterpret_cast<uintptr_t>(p.pair_sigma)) & 15) == 0);
}

}  // namespace qamw
