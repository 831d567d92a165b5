// QAM-W encoder whose shortlist scores come from the matrix cores (Sec. 3.1 / Sec. 3.5).
//
// The score matrix  S[c][x] = ||c||^2 - 2 x.c  of a block of 32 codewords against a block of 32
// points is a (32 x 2)(2 x 32) product plus a bias: a dense contraction with inner dimension 2.
// The fp32 matrix instruction runs on the same FMA lanes as the vector ALU and buys nothing, but
// the bf16 matrix cores are separate hardware.  Every fp32 operand is split EXACTLY into three
// bf16 pieces (8 + 8 + 8 significant bits, by truncation), and one v_mfma_f32_32x32x16_bf16
// evaluates, per coordinate, the eight piece products hh, hm, mh, hl, mm, lh, ml, lm (only ll,
// below 2^-32 relative, is dropped) on top of ||c||^2 supplied in the fp32 accumulator.  Piece
// products are exact in fp32; the only error is the accumulation's rounding, bounded for any
// summation order by 16 x 2^-24 x (sum of magnitudes) <= 2^-20 (||c|| + |x0| + |x1|)^2 (measured
// worst case over 2e6 random evaluations: 2^-22.6).  That bound is all the shortlist needs: as in
// the vector-ALU encoder, the index is decided by exact fp32 squared distances inside the best
// 16-codeword chunk when the runner-up chunk is provably out of reach, and by an exact scan of
// the whole codebook otherwise.  The vector ALU is left with the min-reduction of the scores.
//
// Work split: a wave owns 512 pairs (one row's 1024-column slab).  Front half in registers as in
// the vector-ALU encoder; the pairs are then transposed through LDS into the matrix layout
// (lane = point of a 32-point block, lanes 0-31 / 32-63 = the two coordinates).  A lane's 16
// accumulator rows {8q + 4h + t} of a 32-codeword block are its shortlist chunk.
#include "qamw_front.hpp"

namespace qamw {

constexpr int MF_THREADS = 256;
constexpr int MF_WAVES = MF_THREADS / WAVE;
constexpr int MSLAB = 1024;
constexpr int NPB = 8;                 // 32-point blocks whose operands and state a wave holds at a time
constexpr int PB_TOTAL = 16;           // 512 pairs / 32
constexpr float MBIG = 3.0e38f;
constexpr int MF_WAVE_LDS_FLOATS = 1024 + 512;   // per wave: 512 points (x0, x1) + 512 indices

typedef float f16v_t __attribute__((ext_vector_type(16)));
typedef __bf16 bf8v_t __attribute__((ext_vector_type(8)));
typedef uint32_t u4v_t __attribute__((ext_vector_type(4)));

__device__ __forceinline__ float mmin3(float a, float b, float c) { return __builtin_fminf(__builtin_fminf(a, b), c); }

// x = h + m + l exactly, each piece with at most 8 significant bits (a bf16 value held as fp32).
__device__ __forceinline__ void split3(float x, uint32_t &h, uint32_t &m, uint32_t &l) {
    h = __float_as_uint(x) & 0xFFFF0000u;
    const float r1 = x - __uint_as_float(h);
    m = __float_as_uint(r1) & 0xFFFF0000u;
    const float r2 = r1 - __uint_as_float(m);
    l = __float_as_uint(r2) & 0xFFFF0000u;
}
// two bf16 (given as fp32 bit patterns with a zero low half) into one dword: `even` in the low half
__device__ __forceinline__ uint32_t pack2(uint32_t even, uint32_t odd) { return (even >> 16) | odd; }

__device__ __forceinline__ float mdist2(float x0, float x1, float2 c) {
    float e0 = x0 - c.x, e1 = x1 - c.y;
    return __builtin_fmaf(e1, e1, e0 * e0);
}

template <int DTYPE, int B>
__global__ __launch_bounds__(MF_THREADS) void k_encode_mfma(const void *__restrict__ W, int64_t ldw, Problem p,
                                                            const float *__restrict__ norms,
                                                            uint8_t *__restrict__ packed, int n_slabs, int n_items) {
    extern __shared__ __align__(16) float lds_raw[];
    float2 *c01 = reinterpret_cast<float2 *>(lds_raw);          // K x (c0, c1)
    float *cn = lds_raw + 2 * p.K;                              // K x ||c||^2
    __shared__ float red[MF_WAVES];

    const int lane = threadIdx.x & (WAVE - 1);
    const int wid = threadIdx.x >> 6;
    const int K = p.K;
    float *wave_area = lds_raw + 3 * K + wid * MF_WAVE_LDS_FLOATS;
    float2 *pts = reinterpret_cast<float2 *>(wave_area);        // the wave's 512 points, pair order
    int *idxl = reinterpret_cast<int *>(wave_area + 1024);      // their indices

    const float2 *cbk = reinterpret_cast<const float2 *>(p.codebook);
    float rmax2 = 0.0f;
    for (int i = threadIdx.x; i < K; i += MF_THREADS) {
        float2 c = cbk[i];
        float n2 = __builtin_fmaf(c.y, c.y, c.x * c.x);
        c01[i] = c;
        cn[i] = n2;
        rmax2 = fmaxf(rmax2, n2);
    }
#pragma unroll
    for (int m = 1; m < WAVE; m <<= 1) rmax2 = fmaxf(rmax2, __shfl_xor(rmax2, m, WAVE));
    if (lane == 0) red[wid] = rmax2;
    __syncthreads();
    rmax2 = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
    const float R = sqrtf(rmax2) * 1.000001f;

    const int item = __builtin_amdgcn_readfirstlane(blockIdx.x * MF_WAVES + wid);
    if (item >= n_items) return;
    const int row = item / n_slabs, slab = item - row * n_slabs;
    const LaneSigns<B> ls(lane);
    const int pos = slab_pos(lane);
    const int col0 = slab * MSLAB + 16 * pos;
    const bool active = col0 < p.d_in;
    const int c = active ? col0 : 0;

    // ---------------- front half, then the pairs go to LDS in pair order
    {
        float x[16];
        rotated_unit_row<DTYPE, B>(x, W, (int64_t)row * ldw, c, norms[row], p, ls);
        float g[8];
        if (p.pair_sigma) {
            const float4 *g4 = reinterpret_cast<const float4 *>(p.pair_sigma + (c >> 1));
            float4 a = g4[0], b = g4[1];
            const float sg8[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
#pragma unroll
            for (int k = 0; k < 8; ++k) g[k] = 1.0f / sg8[k];                     // IEEE division
        } else {
#pragma unroll
            for (int k = 0; k < 8; ++k) g[k] = p.g_default;
        }
        float4 *dst = reinterpret_cast<float4 *>(pts + 8 * pos);
#pragma unroll
        for (int k = 0; k < 8; k += 2)
            dst[k >> 1] = make_float4(x[2 * k] * g[k], x[2 * k + 1] * g[k], x[2 * k + 2] * g[k + 1], x[2 * k + 3] * g[k + 1]);
    }
    __builtin_amdgcn_wave_barrier();

    const int j = lane & 31, hs = lane >> 5;
    const float *ptsf = reinterpret_cast<const float *>(pts);
    const float *c01f = reinterpret_cast<const float *>(c01);
    const float4 *cnv = reinterpret_cast<const float4 *>(cn);
    const int n_cblk = K / 32;

    for (int pass = 0; pass < PB_TOTAL / NPB; ++pass) {
        // point-side operands: lane (j, hs) supplies coordinate hs of point j of each block, times -2
        bf8v_t bop[NPB];
        float m1[NPB], m2[NPB];
        int best[NPB];
#pragma unroll
        for (int pb = 0; pb < NPB; ++pb) {
            const float v = -2.0f * ptsf[(32 * (pass * NPB + pb) + j) * 2 + hs];
            uint32_t h, m, l;
            split3(v, h, m, l);
            const u4v_t u = {pack2(h, m), pack2(h, l), pack2(m, h), pack2(l, m)};      // h m h l m h l m
            bop[pb] = __builtin_bit_cast(bf8v_t, u);
            m1[pb] = MBIG;
            m2[pb] = MBIG;
            best[pb] = 0;
        }
        for (int cb = 0; cb < n_cblk; ++cb) {
            // codeword-side operand: coordinate hs of codeword cb*32 + j, pieces ordered to pair with h m h l m h l m
            uint32_t h, m, l;
            split3(c01f[(cb * 32 + j) * 2 + hs], h, m, l);
            const u4v_t ua = {pack2(h, h), pack2(m, h), pack2(m, l), pack2(m, l)};     // h h m h m l m l
            const bf8v_t aop = __builtin_bit_cast(bf8v_t, ua);
            // accumulator input: ||c||^2 of the lane's 16 rows 8q + 4hs + t
            f16v_t cop;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const float4 v = cnv[cb * 8 + 2 * q + hs];
                cop[4 * q] = v.x; cop[4 * q + 1] = v.y; cop[4 * q + 2] = v.z; cop[4 * q + 3] = v.w;
            }
#pragma unroll
            for (int pb = 0; pb < NPB; ++pb) {
                const f16v_t d = __builtin_amdgcn_mfma_f32_32x32x16_bf16(aop, bop[pb], cop, 0, 0, 0);
                const float t0 = mmin3(d[0], d[1], d[2]), t1 = mmin3(d[3], d[4], d[5]), t2 = mmin3(d[6], d[7], d[8]);
                const float t3 = mmin3(d[9], d[10], d[11]), t4 = mmin3(d[12], d[13], d[14]);
                const float cm = __builtin_fminf(mmin3(t0, t1, t2), mmin3(t3, t4, d[15]));
                best[pb] = (cm < m1[pb]) ? cb : best[pb];
                m2[pb] = __builtin_amdgcn_fmed3f(m1[pb], m2[pb], cm);   // m1 <= m2: second smallest chunk minimum
                m1[pb] = __builtin_fminf(m1[pb], cm);
            }
        }

        // ---------------- merge the two half-chunks of every point, then decide as the vector-ALU encoder does
        unsigned flagged = 0;
#pragma unroll
        for (int pb = 0; pb < NPB; ++pb) {
            const int pbg = pass * NPB + pb;
            const float o1 = __shfl_xor(m1[pb], 32, WAVE), o2 = __shfl_xor(m2[pb], 32, WAVE);
            const int ob = __shfl_xor(best[pb], 32, WAVE);
            const bool other = o1 < m1[pb];
            const float M1 = __builtin_fminf(m1[pb], o1);
            const float M2 = __builtin_fminf(__builtin_fmaxf(m1[pb], o1), __builtin_fminf(m2[pb], o2));
            const int cbb = other ? ob : best[pb];                 // best 32-codeword block ...
            const int hb = other ? (hs ^ 1) : hs;                  // ... and which 16 of its rows
            const float2 x = pts[32 * pbg + j];
            const float n1 = fabsf(x.x) + fabsf(x.y);
            const float emax = 9.54e-7f * (R + n1) * (R + n1);                   // 2^-20 (R + n1)^2
            const float xx = __builtin_fmaf(x.y, x.y, x.x * x.x);
            const float d2 = fmaxf(M1 + xx * 1.000001f + emax, 0.0f);            // >= true best squared distance
            const float rho = sqrtf(d2) * 1.000001f + 0.0625f;
            const float eps = 9.55e-7f * (2.0f * n1 + rho) * (2.0f * n1 + rho);
            const bool safe = (M2 - M1 > 2.0f * eps) && (emax < 1.0e-3f);
            // this lane checks rows 8q + 4hb + t for q = 2hs, 2hs+1 (ascending index), its partner the other two q
            float bd = MBIG;
            int bi = 0x7fffffff;
#pragma unroll
            for (int qq = 0; qq < 2; ++qq) {
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    const int ci = cbb * 32 + 8 * (2 * hs + qq) + 4 * hb + t;
                    const float dd = mdist2(x.x, x.y, c01[ci]);
                    if (dd < bd) {
                        bd = dd;
                        bi = ci;
                    }
                }
            }
            const float od = __shfl_xor(bd, 32, WAVE);
            const int oi = __shfl_xor(bi, 32, WAVE);
            if (od < bd || (od == bd && oi < bi)) bi = oi;
            if (hs == 0) idxl[32 * pbg + j] = bi;
            if (!safe && hs == 0) flagged |= 1u << pb;
            asm volatile("" ::: "memory");
        }
#pragma unroll
        for (int pb = 0; pb < NPB; ++pb) {
            const int pbg = pass * NPB + pb;
            unsigned long long mask = __ballot((flagged >> pb) & 1u);
            while (mask) {
                const int src = __ffsll((long long)mask) - 1;      // a lane below 32: point src of block pbg
                mask &= mask - 1;
                const float2 x = pts[32 * pbg + src];
                float bd = MBIG;
                int bi = 0x7fffffff;
                for (int k = lane; k < K; k += WAVE) {
                    float dd = mdist2(x.x, x.y, c01[k]);
                    if (dd < bd) {
                        bd = dd;
                        bi = k;
                    }
                }
#pragma unroll
                for (int m = 1; m < WAVE; m <<= 1) {
                    float od = __shfl_xor(bd, m, WAVE);
                    int oi = __shfl_xor(bi, m, WAVE);
                    if (od < bd || (od == bd && oi < bi)) {
                        bd = od;
                        bi = oi;
                    }
                }
                if (lane == src) idxl[32 * pbg + src] = bi;
            }
        }
    }
    __builtin_amdgcn_wave_barrier();

    // ---------------- pack: the lane's 8 fields are exactly `bits` bytes, byte aligned in the row
    if (active) {
        const int bits = p.bits;
        const int4 ia = *reinterpret_cast<const int4 *>(idxl + 8 * pos), ib = *reinterpret_cast<const int4 *>(idxl + 8 * pos + 4);
        const int idx[8] = {ia.x, ia.y, ia.z, ia.w, ib.x, ib.y, ib.z, ib.w};
        uint8_t *dst = packed + (int64_t)row * p.row_bytes + (int64_t)(c >> 4) * bits;
        unsigned __int128 acc = 0;
#pragma unroll
        for (int k = 0; k < 8; ++k) acc |= (unsigned __int128)(unsigned)idx[k] << (k * bits);
        for (int t = 0; t < bits; ++t) dst[t] = (uint8_t)(acc >> (8 * t));
        if (col0 + 16 == p.d_in) {                              // last lane of the row zeroes the padding
            const int64_t used = (int64_t)(p.d_in >> 4) * bits;
            uint8_t *rowp = packed + (int64_t)row * p.row_bytes;
            for (int64_t t = used; t < p.row_bytes; ++t) rowp[t] = 0;
        }
    }
}

bool mfma_encode_supported(const Problem &p) {
    const int unit = p.block > 16 ? p.block : 16;
    if (p.d_in % unit) return false;
    if (p.K % 32 || p.bits > 11) return false;
    return p.block >= 64;
}

template <int DTYPE, int B>
static hipError_t launch_mdb(const void *W, int64_t ldw, const Problem &p, const float *norms, uint8_t *packed) {
    const int n_slabs = (p.d_in + MSLAB - 1) / MSLAB;
    const int64_t n_items = (int64_t)p.d_out * n_slabs;
    if (n_items > 0x7fffffff) return hipErrorNotSupported;
    const unsigned blocks = (unsigned)((n_items + MF_WAVES - 1) / MF_WAVES);
    const size_t lds = ((size_t)p.K * 3 + (size_t)MF_WAVES * MF_WAVE_LDS_FLOATS) * sizeof(float);
    hipLaunchKernelGGL((k_encode_mfma<DTYPE, B>), dim3(blocks), dim3(MF_THREADS), lds, p.stream, W, ldw, p, norms, packed,
                       n_slabs, (int)n_items);
    return hipGetLastError();
}

template <int DTYPE>
static hipError_t launch_md(const void *W, int64_t ldw, const Problem &p, const float *norms, uint8_t *packed) {
    switch (p.block) {
        case 64: return launch_mdb<DTYPE, 64>(W, ldw, p, norms, packed);
        case 128: return launch_mdb<DTYPE, 128>(W, ldw, p, norms, packed);
        case 256: return launch_mdb<DTYPE, 256>(W, ldw, p, norms, packed);
        case 512: return launch_mdb<DTYPE, 512>(W, ldw, p, norms, packed);
        case 1024: return launch_mdb<DTYPE, 1024>(W, ldw, p, norms, packed);
        default: return hipErrorNotSupported;
    }
}

// Returns hipErrorNotSupported (nothing launched) when the shape or alignment is outside this kernel's range.
hipError_t launch_encode_mfma(const void *W, int dtype, int64_t ldw, const Problem &p, const float *norms,
                              uint8_t *packed) {
    const bool ok = mfma_encode_supported(p) && front_alignment_ok(W, dtype, ldw, p) &&
                    ((reinterpret_cast<uintptr_t>(p.codebook) & 15) == 0);
    if (!ok) return hipErrorNotSupported;
    return dtype == 0 ? launch_md<0>(W, ldw, p, norms, packed) : launch_md<1>(W, ldw, p, norms, packed);
}

}  // namespace qamw
