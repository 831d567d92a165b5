// Shape-specialised QAM-W encoder (Sec. 3.1 with the channel scaling of Sec. B.2).
//
// A wave owns one row's slab of 1024 columns = 512 pairs, 8 pairs per lane.  The front half
// (scale, normalise, sign, block Walsh-Hadamard, pair gain) runs in registers and reproduces
// the library's fp32 arithmetic bit for bit.  The nearest-codeword search then scores all K
// codewords for the lane's 8 points with the expansion  ||c||^2 - 2 x.c  (2 FMA per evaluation,
// codewords broadcast from LDS), keeping per point the best 16-codeword chunk and the best
// score outside it.  The expansion only SHORTLISTS: the winner is decided by exact fp32 squared
// distances inside the best chunk when the runner-up chunk is provably out of reach, and by an
// exact wave-cooperative scan of the whole codebook otherwise (rare).  Lowest index wins ties.
#include "qamw_front.hpp"

namespace qamw {

constexpr int EF_THREADS = 256;
constexpr int EF_WAVES = EF_THREADS / WAVE;
constexpr int ESLAB = 1024;
constexpr float BIG = 3.0e38f; // larger than any score or squared distance of finite inputs
constexpr int NPT = 8;        // points (pairs) per lane
constexpr int CHUNK = 16;     // codewords per shortlist chunk: scored together, rechecked together

__device__ __forceinline__ float min3(float a, float b, float c) { return __builtin_fminf(__builtin_fminf(a, b), c); }

template <int DTYPE, int B>
__global__ __launch_bounds__(EF_THREADS) void k_encode_fast(const void *__restrict__ W, int64_t ldw, Problem p,
                                                            const float *__restrict__ norms_in, float *__restrict__ norms_out,
                                                            uint8_t *__restrict__ packed, int n_slabs, int n_items,
                                                            int n_blocks) {
    extern __shared__ float lds_raw[];
    float2 *c01 = reinterpret_cast<float2 *>(lds_raw);          // K x (c0, c1)
    float *cn = lds_raw + 2 * p.K;                              // K x ||c||^2
    __shared__ float red[EF_WAVES];
    __shared__ double norm_part[2 * FUSED_NORM_MAX_SLABS];

    const int lane = threadIdx.x & (WAVE - 1);
    const int wid = threadIdx.x >> 6;
    const int K = p.K;
    // norms_in == NULL: the workgroup computes the norms of the rows its items touch (and writes them out); the
    // barrier after the codebook staging below also publishes the slab sums.
    const bool fused = norms_in == nullptr;
    const int item0 = (fused ? fused_norm_block(blockIdx.x, n_blocks) : (int)blockIdx.x) * EF_WAVES;
    if (fused && item0 < n_items) block_slab_sums<DTYPE, EF_WAVES>(norm_part, W, ldw, p, item0, n_items, n_slabs, lane, wid);

    // stage the codebook; R^2 = max ||c||^2 enters the shortlist's error bound
    const float2 *cbk = reinterpret_cast<const float2 *>(p.codebook);
    float rmax2 = 0.0f;
    for (int i = threadIdx.x; i < K; i += EF_THREADS) {
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
    const int col0 = slab * ESLAB + 16 * pos;
    const bool active = col0 < p.d_in;
    const int c = active ? col0 : 0;

    // ---------------- front half: x_k = (F S (W D_s / r))_pair k / sigma_k, in registers
    float x[16];
    rotated_unit_row<DTYPE, B>(x, W, (int64_t)row * ldw, c, rnorm, p, ls);
    {
        float g[NPT];
        load_pair_gains(g, p, c);
#pragma unroll
        for (int e = 0; e < 16; ++e) x[e] = x[e] * g[e >> 1];
    }

    // ---------------- shortlist: best chunk by the expansion score
    float a0[NPT], a1[NPT], m1[NPT], m2[NPT];
    int best[NPT];
#pragma unroll
    for (int j = 0; j < NPT; ++j) {
        a0[j] = -2.0f * x[2 * j];
        a1[j] = -2.0f * x[2 * j + 1];
        m1[j] = BIG;
        m2[j] = BIG;
        best[j] = 0;
    }
    const float4 *c01v = reinterpret_cast<const float4 *>(c01);  // two codewords per float4
    const float4 *cnv = reinterpret_cast<const float4 *>(cn);    // four norms per float4
    const int n_chunks = K / CHUNK;
    for (int ch = 0; ch < n_chunks; ++ch) {
        float cx[CHUNK], cy[CHUNK], cq[CHUNK];
#pragma unroll
        for (int t = 0; t < CHUNK / 2; ++t) {
            float4 v = c01v[ch * (CHUNK / 2) + t];
            cx[2 * t] = v.x; cy[2 * t] = v.y; cx[2 * t + 1] = v.z; cy[2 * t + 1] = v.w;
        }
#pragma unroll
        for (int t = 0; t < CHUNK / 4; ++t) {
            float4 v = cnv[ch * (CHUNK / 4) + t];
            cq[4 * t] = v.x; cq[4 * t + 1] = v.y; cq[4 * t + 2] = v.z; cq[4 * t + 3] = v.w;
        }
#pragma unroll
        for (int j = 0; j < NPT; ++j) {
            float s[CHUNK];
#pragma unroll
            for (int k = 0; k < CHUNK; ++k) s[k] = __builtin_fmaf(a0[j], cx[k], __builtin_fmaf(a1[j], cy[k], cq[k]));
            float t0 = min3(s[0], s[1], s[2]);
            float t1 = min3(s[3], s[4], s[5]);
            float t2 = min3(s[6], s[7], s[8]);
            float t3 = min3(s[9], s[10], s[11]);
            float t4 = min3(s[12], s[13], s[14]);
            float cm = __builtin_fminf(min3(t0, t1, t2), min3(t3, t4, s[15]));
            best[j] = (cm < m1[j]) ? ch : best[j];
            m2[j] = __builtin_amdgcn_fmed3f(m1[j], m2[j], cm);   // m1 <= m2: second smallest chunk minimum
            m1[j] = __builtin_fminf(m1[j], cm);
        }
    }

    // ---------------- decide: exact distances inside the best chunk, or the full exact scan
    // Error model.  n1 = |x0|+|x1| >= ||x||.  Every computed score differs from the true
    // ||c||^2 - 2 x.c by at most E(c) = 2^-21 (||c|| + n1)^2.  The true nearest codeword and every
    // codeword that could be mistaken for it lie within rho = d_best + 1/16 of x, i.e. have norm at
    // most n1 + rho, so for them E <= eps = 2^-21 (2 n1 + rho)^2; codewords further out score at least
    // 2^-8 worse than the minimum and cannot interfere.  If the second-best chunk's minimum
    // exceeds the best by more than 2 eps, the nearest codeword is inside the best chunk.
    int idx[NPT];
    unsigned flagged = 0;
#pragma unroll
    for (int j = 0; j < NPT; ++j) {
        const float x0 = x[2 * j], x1 = x[2 * j + 1];
        const float n1 = fabsf(x0) + fabsf(x1);
        const float emax = 4.77e-7f * (R + n1) * (R + n1);                     // 2^-21 (R + n1)^2
        const float xx = __builtin_fmaf(x1, x1, x0 * x0);
        const float d2 = fmaxf(m1[j] + xx * 1.000001f + emax, 0.0f);           // >= true best squared distance
        const float rho = sqrtf(d2) * 1.000001f + 0.0625f;
        const float eps = 4.78e-7f * (2.0f * n1 + rho) * (2.0f * n1 + rho);
        const bool safe = (m2[j] - m1[j] > 2.0f * eps) && (emax < 1.0e-3f);
        float bd = BIG;
        int bi = best[j] * CHUNK;
#pragma unroll
        for (int k = 0; k < CHUNK; ++k) {
            float dd = exact_dist2(x0, x1, c01[best[j] * CHUNK + k]);
            if (dd < bd) {
                bd = dd;
                bi = best[j] * CHUNK + k;
            }
        }
        idx[j] = bi;
        if (!safe) flagged |= 1u << j;
        asm volatile("" ::: "memory");                          // keep one point's gathers in flight at a time (register budget)
    }
    int n_scans = 0;                                            // uniform: pairs of this wave that took the whole-codebook scan
#pragma unroll
    for (int j = 0; j < NPT; ++j) {
        unsigned long long mask = __ballot((flagged >> j) & 1u);
        n_scans += __popcll(mask);
        while (mask) {
            const int src = __ffsll((long long)mask) - 1;
            mask &= mask - 1;
            const float x0 = __uint_as_float(__builtin_amdgcn_readlane(__float_as_uint(x[2 * j]), src));
            const float x1 = __uint_as_float(__builtin_amdgcn_readlane(__float_as_uint(x[2 * j + 1]), src));
            float bd = BIG;
            int bi = 0x7fffffff;
            for (int k = lane; k < K; k += WAVE) {
                float dd = exact_dist2(x0, x1, c01[k]);
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
            if (lane == src) idx[j] = bi;
        }
    }

    // one update of the counter per wave, after the search (an atomic inside the loops above costs the whole kernel
    // its register allocation)
    if (p.full_scans && n_scans && lane == 0) atomicAdd(p.full_scans, (unsigned long long)n_scans);

    // ---------------- pack: the lane's 8 fields are exactly `bits` bytes, byte aligned in the row
    if (active) {
        const int bits = p.bits;
        uint8_t *dst = packed + (int64_t)row * p.row_bytes + (int64_t)(c >> 4) * bits;
        unsigned __int128 acc = 0;
#pragma unroll
        for (int j = 0; j < NPT; ++j) acc |= (unsigned __int128)(unsigned)idx[j] << (j * bits);
        for (int t = 0; t < bits; ++t) dst[t] = (uint8_t)(acc >> (8 * t));
        if (col0 + 16 == p.d_in) {                              // last lane of the row zeroes the padding
            const int64_t used = (int64_t)(p.d_in >> 4) * bits;
            uint8_t *rowp = packed + (int64_t)row * p.row_bytes;
            for (int64_t t = used; t < p.row_bytes; ++t) rowp[t] = 0;
        }
    }
}

bool fast_encode_supported(const Problem &p) {
    const int unit = p.block > 16 ? p.block : 16;
    if (p.d_in % unit) return false;
    if (p.K % CHUNK || p.bits > 11) return false;
    return p.block >= 64;
}

template <int DTYPE, int B>
static hipError_t launch_db(const void *W, int64_t ldw, const Problem &p, float *norms, bool norms_ready, uint8_t *packed) {
    const int n_slabs = (p.d_in + ESLAB - 1) / ESLAB;
    const int64_t n_items = (int64_t)p.d_out * n_slabs;
    if (n_items > 0x7fffffff) return hipErrorNotSupported;
    if (!norms_ready && n_slabs > FUSED_NORM_MAX_SLABS) return hipErrorNotSupported;
    const int n_blocks = (int)((n_items + EF_WAVES - 1) / EF_WAVES);
    const unsigned blocks = (unsigned)(norms_ready ? n_blocks : fused_norm_grid(n_blocks));
    const size_t lds = (size_t)p.K * 3 * sizeof(float);
    hipLaunchKernelGGL((k_encode_fast<DTYPE, B>), dim3(blocks), dim3(EF_THREADS), lds, p.stream, W, ldw, p,
                       norms_ready ? norms : nullptr, norms, packed, n_slabs, (int)n_items, n_blocks);
    return hipGetLastError();
}

template <int DTYPE>
static hipError_t launch_d(const void *W, int64_t ldw, const Problem &p, float *norms, bool norms_ready, uint8_t *packed) {
    switch (p.block) {
        case 64: return launch_db<DTYPE, 64>(W, ldw, p, norms, norms_ready, packed);
        case 128: return launch_db<DTYPE, 128>(W, ldw, p, norms, norms_ready, packed);
        case 256: return launch_db<DTYPE, 256>(W, ldw, p, norms, norms_ready, packed);
        case 512: return launch_db<DTYPE, 512>(W, ldw, p, norms, norms_ready, packed);
        case 1024: return launch_db<DTYPE, 1024>(W, ldw, p, norms, norms_ready, packed);
        default: return hipErrorNotSupported;
    }
}

// norms_ready: the row norms are already in `norms`; otherwise the kernel computes them itself and writes them there.
// Returns hipErrorNotSupported (nothing launched) when the shape or alignment is outside this kernel's range.
hipError_t launch_encode_fast(const void *W, int dtype, int64_t ldw, const Problem &p, float *norms, bool norms_ready,
                              uint8_t *packed) {
    // vector loads: rows and side arrays must be 16-byte aligned
    const bool ok = fast_encode_supported(p) && front_alignment_ok(W, dtype, ldw, p) &&
                    ((reinterpret_cast<uintptr_t>(p.codebook) & 15) == 0);
    if (!ok) return hipErrorNotSupported;
    return dtype == 0 ? launch_d<0>(W, ldw, p, norms, norms_ready, packed) : launch_d<1>(W, ldw, p, norms, norms_ready, packed);
}

}  // namespace qamw
