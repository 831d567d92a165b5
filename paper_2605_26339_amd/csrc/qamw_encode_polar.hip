// Polar-baseline encoder (Sec. 3 "Polar Baseline"): the QAM-W front half, then amplitude and phase
// of every pair quantised independently instead of a joint nearest-codeword search.
//
// Front half exactly as the joint encoders (a wave owns one row's slab of 1024 columns, 8 pairs per
// lane, everything in registers).  Per pair x = (x0, x1):
//   amplitude index = number of thresholds below |x|, thresholds at the midpoints of neighbouring
//                     Lloyd-Max levels; decided on squares, a2 = fma(x1, x1, x0 x0) against
//                     T_i = t_i^2, by binary search over the sorted thresholds (no square root);
//   phase index     = the bin [2kh, 2(k+1)h), h = pi/Np, that holds atan2(x1, x0) taken in
//                     [0, 2pi): the half-plane by the sign of x1, then binary search with the
//                     sign of the cross product against the boundary directions (cos 2kh, sin 2kh)
//                     (no arctangent).  The origin has phase bin 0.
// Index = amplitude index * Np + phase index, packed like the joint code, so the decoder is the
// joint decoder with the 2^B-entry table {level_ia * (cos, sin)((2 ip + 1) h)}.
#include "qamw_front.hpp"

namespace qamw {

constexpr int PF_THREADS = 256;
constexpr int PF_WAVES = PF_THREADS / WAVE;
constexpr int PSLAB = 1024;
constexpr int PF_MAX_LEVELS = 64;      // amplitude levels
constexpr int PF_MAX_BINS = 4096;      // phase bins

template <int DTYPE, int B>
__global__ __launch_bounds__(PF_THREADS) void k_encode_polar(const void *__restrict__ W, int64_t ldw, Problem p,
                                                             const float *__restrict__ levels, int bits_a, int bits_p,
                                                             const float *__restrict__ norms_in, float *__restrict__ norms_out,
                                                             uint8_t *__restrict__ packed, int n_slabs, int n_items,
                                                             int n_blocks) {
    extern __shared__ __align__(16) float lds_raw[];
    const int Na = 1 << bits_a, Np = 1 << bits_p;
    float *thr2 = lds_raw;                                      // Na: thr2[i] = (midpoint of levels i-1, i)^2, i >= 1
    float2 *bdir = reinterpret_cast<float2 *>(lds_raw + (Na < 2 ? 2 : Na));   // Np boundary directions (cos, sin)(2 k h), 8-byte aligned
    __shared__ double norm_part[2 * FUSED_NORM_MAX_SLABS];
    const int lane = threadIdx.x & (WAVE - 1);
    const int wid = threadIdx.x >> 6;
    // norms_in == NULL: the workgroup computes the norms of the rows its items touch (and writes them out); the
    // barrier after the table set-up below also publishes the slab sums.
    const bool fused = norms_in == nullptr;
    const int item0 = (fused ? fused_norm_block(blockIdx.x, n_blocks) : (int)blockIdx.x) * PF_WAVES;
    if (fused && item0 < n_items) block_slab_sums<DTYPE, PF_WAVES>(norm_part, W, ldw, p, item0, n_items, n_slabs, lane, wid);

    for (int i = threadIdx.x; i < Na; i += PF_THREADS) {
        const float t = (i > 0) ? 0.5f * (levels[i - 1] + levels[i]) : 0.0f;
        thr2[i] = t * t;
    }
    for (int k = threadIdx.x; k < Np; k += PF_THREADS) {
        float sn, cs;
        sincospif(2.0f * (float)k / (float)Np, &sn, &cs);      // the angle 2 k h = pi * (2k / Np), argument exact
        bdir[k] = make_float2(cs, sn);
    }
    __syncthreads();

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
    const int col0 = slab * PSLAB + 16 * pos;
    const bool active = col0 < p.d_in;
    const int c = active ? col0 : 0;

    // ---------------- front half: x_k = (F S (W D_s / r))_pair k / sigma_k, in registers
    float x[16];
    rotated_unit_row<DTYPE, B>(x, W, (int64_t)row * ldw, c, rnorm, p, ls);
    {
        float g[8];
        load_pair_gains(g, p, c);
#pragma unroll
        for (int e = 0; e < 16; ++e) x[e] = x[e] * g[e >> 1];
    }

    // ---------------- amplitude level and phase bin of the lane's 8 pairs
    unsigned idx[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        const float x0 = x[2 * k], x1 = x[2 * k + 1];
        const float a2 = __builtin_fmaf(x1, x1, x0 * x0);
        int ia = 0;
        for (int step = Na >> 1; step; step >>= 1) {
            const int cand = ia + step;
            ia = (a2 > thr2[cand]) ? cand : ia;                 // on the threshold: the lower level
        }
        const bool upper = (x1 < 0.0f) || (x1 == 0.0f && x0 < 0.0f);   // angle in [pi, 2 pi)
        int ip = upper ? (Np >> 1) : 0;
        for (int step = Np >> 2; step; step >>= 1) {
            const int cand = ip + step;
            const float2 b = bdir[cand];
            const float cr = __builtin_fmaf(b.x, x1, -(b.y * x0));     // sin(angle - 2 cand h) * |x|
            ip = (cr >= 0.0f) ? cand : ip;
        }
        if (a2 == 0.0f) ip = 0;
        idx[k] = (unsigned)(ia * Np + ip);
    }

    // ---------------- pack: the lane's 8 fields are exactly `bits` bytes, byte aligned in the row
    if (active) {
        store_packed_fields(packed, row, c, col0, idx, p);
    }
}

static bool polar_encode_supported(const Problem &p, int bits_a, int bits_p) {
    const int unit = p.block > 16 ? p.block : 16;
    if (p.d_in % unit || p.block < 64) return false;
    return bits_a >= 0 && bits_p >= 0 && (1 << bits_a) <= PF_MAX_LEVELS && (1 << bits_p) <= PF_MAX_BINS &&
           bits_a + bits_p == p.bits;
}

template <int DTYPE, int B>
static hipError_t launch_pdb(const void *W, int64_t ldw, const Problem &p, const float *levels, int bits_a, int bits_p,
                             float *norms, bool norms_ready, uint8_t *packed) {
    const int n_slabs = (p.d_in + PSLAB - 1) / PSLAB;
    const int64_t n_items = (int64_t)p.d_out * n_slabs;
    if (n_items > 0x7fffffff) return hipErrorNotSupported;
    if (!norms_ready && n_slabs > FUSED_NORM_MAX_SLABS) return hipErrorNotSupported;
    const int n_blocks = (int)((n_items + PF_WAVES - 1) / PF_WAVES);
    const unsigned blocks = (unsigned)(norms_ready ? n_blocks : fused_norm_grid(n_blocks));
    const size_t lds = ((size_t)(bits_a ? (1 << bits_a) : 2) + 2 * (size_t)(1 << bits_p)) * sizeof(float);
    hipLaunchKernelGGL((k_encode_polar<DTYPE, B>), dim3(blocks), dim3(PF_THREADS), lds, p.stream, W, ldw, p, levels, bits_a,
                       bits_p, norms_ready ? norms : nullptr, norms, packed, n_slabs, (int)n_items, n_blocks);
    return hipGetLastError();
}

template <int DTYPE>
static hipError_t launch_pd(const void *W, int64_t ldw, const Problem &p, const float *levels, int bits_a, int bits_p,
                            float *norms, bool norms_ready, uint8_t *packed) {
    switch (p.block) {
        case 64: return launch_pdb<DTYPE, 64>(W, ldw, p, levels, bits_a, bits_p, norms, norms_ready, packed);
        case 128: return launch_pdb<DTYPE, 128>(W, ldw, p, levels, bits_a, bits_p, norms, norms_ready, packed);
        case 256: return launch_pdb<DTYPE, 256>(W, ldw, p, levels, bits_a, bits_p, norms, norms_ready, packed);
        case 512: return launch_pdb<DTYPE, 512>(W, ldw, p, levels, bits_a, bits_p, norms, norms_ready, packed);
        case 1024: return launch_pdb<DTYPE, 1024>(W, ldw, p, levels, bits_a, bits_p, norms, norms_ready, packed);
        default: return hipErrorNotSupported;
    }
}

bool polar_encode_launchable(const void *W, int dtype, int64_t ldw, const Problem &p, int bits_a, int bits_p) {
    return polar_encode_supported(p, bits_a, bits_p) && front_alignment_ok(W, dtype, ldw, p) &&
           (reinterpret_cast<uintptr_t>(W) != 0);
}

// Returns hipErrorNotSupported (nothing launched) when the shape or alignment is outside this kernel's range.
hipError_t launch_encode_polar(const void *W, int dtype, int64_t ldw, const Problem &p, const float *levels, int bits_a,
                               int bits_p, float *norms, bool norms_ready, uint8_t *packed) {
    if (!polar_encode_launchable(W, dtype, ldw, p, bits_a, bits_p)) return hipErrorNotSupported;
    return dtype == 0 ? launch_pd<0>(W, ldw, p, levels, bits_a, bits_p, norms, norms_ready, packed)
                      : launch_pd<1>(W, ldw, p, levels, bits_a, bits_p, norms, norms_ready, packed);
}

}  // namespace qamw
