// Shape-specialised QAM-W decoder (Sec. 3.2 + Sec. B.2): HBM-bound, everything between the packed
// load and the bf16 store stays in registers.
//
// A wave owns a slab of 1024 columns and walks down a range of rows.  Per row a lane unpacks its
// 8 indices (8*bits bits = `bits` bytes, always byte aligned), gathers 8 codewords from the
// LDS-resident codebook, scales them by sigma_k, runs the block Walsh-Hadamard butterflies
// across the wave (qamw_wave_fwht.hpp), applies row and column factors and stores 16 bf16.
// Column constants (1/s_j with the sign mask and the transform's lane sign folded in, sigma_k)
// are loaded once per slab and reused for every row.
#include "qamw_common.hpp"
#include "qamw_internal.hpp"
#include "qamw_wave_fwht.hpp"

namespace qamw {

constexpr int DF_THREADS = 256;
constexpr int DF_WAVES = DF_THREADS / WAVE;
constexpr int SLAB = 1024;

typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float floatx2_t __attribute__((ext_vector_type(2)));

// Field i (i = 0..7) of a lane's 8*BITS-bit group, the group starting at bit 0 of w[0..2].
template <int BITS> __device__ __forceinline__ uint32_t field(const uint32_t (&w)[4], int i) {
    const int bit = i * BITS, word = bit >> 5, off = bit & 31;
    uint32_t v = (off + BITS <= 32) ? (w[word] >> off) : __builtin_amdgcn_alignbit(w[word + 1], w[word], off);
    return v & ((1u << BITS) - 1u);
}

// Reciprocal with one Newton step: the correctly rounded quotient in all but a few rare cases
// (then one ulp off), at a third of the cost of the IEEE division sequence.
__device__ __forceinline__ float fast_recip(float s) {
    float q = __builtin_amdgcn_rcpf(s);
    float e = __builtin_fmaf(-s, q, 1.0f);
    return __builtin_fmaf(q, e, q);
}

__device__ __forceinline__ void load_group(uint32_t (&d)[4], const uint32_t *pk32, int64_t b0, int64_t total_dw) {
    const int64_t d0 = b0 >> 2;
    if (d0 + 3 < total_dw) {
#pragma unroll
        for (int t = 0; t < 4; ++t) d[t] = pk32[d0 + t];
    } else {
#pragma unroll
        for (int t = 0; t < 4; ++t) d[t] = pk32[min(d0 + t, total_dw - 1)];
    }
}

// Per-lane column constants of 16 consecutive columns starting at c (a multiple of 16):
// qs[e] = parity / s_j with the sign mask folded in, sig[k] = sigma of the lane's 8 pairs.
// Vector loads: the host checks that the arrays are 16-byte aligned.
__device__ __forceinline__ void load_column_constants(float (&qs)[16], float (&sig)[8], const Problem &p, int c,
                                                      float parity) {
    if (p.chan_scale) {
        const float4 *s4 = reinterpret_cast<const float4 *>(p.chan_scale + c);
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            float4 v = s4[t];
            qs[4 * t] = fast_recip(v.x) * parity;
            qs[4 * t + 1] = fast_recip(v.y) * parity;
            qs[4 * t + 2] = fast_recip(v.z) * parity;
            qs[4 * t + 3] = fast_recip(v.w) * parity;
        }
    } else {
#pragma unroll
        for (int e = 0; e < 16; ++e) qs[e] = parity;
    }
    if (p.signs) {
        const uint4 sg = *reinterpret_cast<const uint4 *>(p.signs + c);
        const uint32_t wds[4] = {sg.x, sg.y, sg.z, sg.w};
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            // int8 -1 = 0xFF: bit 7 of the byte is the sign; move it onto the float's sign bit
            uint32_t neg = (wds[e >> 2] >> (8 * (e & 3) + 7)) & 1u;
            qs[e] = __uint_as_float(__float_as_uint(qs[e]) ^ (neg << 31));
        }
    }
    if (p.pair_sigma) {
        const float4 *g4 = reinterpret_cast<const float4 *>(p.pair_sigma + (c >> 1));
        float4 a = g4[0], b = g4[1];
        sig[0] = a.x; sig[1] = a.y; sig[2] = a.z; sig[3] = a.w;
        sig[4] = b.x; sig[5] = b.y; sig[6] = b.z; sig[7] = b.w;
    } else {
#pragma unroll
        for (int k = 0; k < 8; ++k) sig[k] = p.sigma_default;
    }
}

// Persistent kernel.  The grid is sized to the machine (not to the matrix); a block stages the
// codebook into LDS once, then each wave keeps one slab (so its column constants load once) and
// walks over groups of R rows with a grid stride, fetching the next group's packed indices and
// norms while it works on the current one.  The 16 bf16 a lane produces are 32 consecutive
// bytes; a row chunk is therefore bounced through LDS so that each store instruction writes
// 1 KB of consecutive bytes (full cache lines) instead of every other 16 bytes.
template <int BITS, int B, bool OUT_BF16, int R>
__global__ __launch_bounds__(DF_THREADS) void k_decode_fast(const uint8_t *__restrict__ packed,
                                                            const float *__restrict__ norms, Problem p,
                                                            void *__restrict__ out, int64_t ldo, int n_slabs,
                                                            int waves_per_slab) {
    extern __shared__ float2 cb_lds[];                          // K codewords, then the per-wave bounce buffers
    const int lane = threadIdx.x & (WAVE - 1);
    const int wid = threadIdx.x >> 6;
    const int wave = __builtin_amdgcn_readfirstlane(blockIdx.x * DF_WAVES + wid);
    const int slab = wave % n_slabs;
    const int first_group = wave / n_slabs;                     // >= waves_per_slab: nothing to do
    const int n_groups = (p.d_out + R - 1) / R;
    const int last_row = p.d_out - 1;

    const LaneSigns<B> ls(lane);
    const int pos = slab_pos(lane);
    const int col0 = slab * SLAB + 16 * pos;
    const int c = (col0 < p.d_in) ? col0 : 0;                   // idle lanes compute on valid data, store nothing
    const int slab_cols = min(SLAB, p.d_in - slab * SLAB);      // valid columns of this slab
    const int64_t byte_off = (int64_t)(c >> 4) * BITS;          // 8 fields of BITS bits = BITS bytes per lane
    const uint32_t *pk32 = reinterpret_cast<const uint32_t *>(packed);
    const int64_t total_dw = (int64_t)p.d_out * (p.row_bytes >> 2);

    uint32_t nxt[R][4];
    float rn_nxt[R];
    int group = (first_group < waves_per_slab) ? first_group : n_groups;   // surplus waves of the last block idle
    if (group < n_groups) {
#pragma unroll
        for (int t = 0; t < R; ++t) {
            const int row = min(group * R + t, last_row);       // rows past the end re-read the last row
            load_group(nxt[t], pk32, (int64_t)row * p.row_bytes + byte_off, total_dw);
            rn_nxt[t] = norms[row];
        }
    }
    float qs[16], sig[8];
    load_column_constants(qs, sig, p, c, ls.parity);

    const float2 *cbk = reinterpret_cast<const float2 *>(p.codebook);
    for (int i = threadIdx.x; i < p.K; i += DF_THREADS) cb_lds[i] = cbk[i];
    __syncthreads();
    uint4 *bounce = reinterpret_cast<uint4 *>(cb_lds + p.K) + wid * (OUT_BF16 ? 128 : 256);

    for (; group < n_groups; group += waves_per_slab) {
        uint32_t d[R][4];
        float rn[R];
#pragma unroll
        for (int t = 0; t < R; ++t) {
            rn[t] = rn_nxt[t];
#pragma unroll
            for (int q = 0; q < 4; ++q) d[t][q] = nxt[t][q];
        }
        if (group + waves_per_slab < n_groups) {
#pragma unroll
            for (int t = 0; t < R; ++t) {
                const int row = min((group + waves_per_slab) * R + t, last_row);
                load_group(nxt[t], pk32, (int64_t)row * p.row_bytes + byte_off, total_dw);
                rn_nxt[t] = norms[row];
            }
        }
#pragma unroll
        for (int t = 0; t < R; ++t) {
            const int row = group * R + t;
            const int sh = (int)(((int64_t)min(row, last_row) * p.row_bytes + byte_off) & 3) * 8;
            uint32_t w[4];
            w[0] = __builtin_amdgcn_alignbit(d[t][1], d[t][0], sh);
            w[1] = __builtin_amdgcn_alignbit(d[t][2], d[t][1], sh);
            w[2] = __builtin_amdgcn_alignbit(d[t][3], d[t][2], sh);
            w[3] = d[t][3] >> sh;
            float x[16];
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                float2 cw = cb_lds[field<BITS>(w, k)];
                x[2 * k] = sig[k] * cw.x;
                x[2 * k + 1] = sig[k] * cw.y;
            }
            fwht_wave<B>(x, ls);
            const float a = rn[t] * p.inv_sqrt_block;           // row factor r * block^-1/2
            if (OUT_BF16) {
                uint32_t o[8];
#pragma unroll
                for (int e = 0; e < 16; e += 2) {
                    floatx2_t v = {(x[e] * a) * qs[e], (x[e + 1] * a) * qs[e + 1]};
                    o[e >> 1] = __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
                }
                // lane `pos` owns bytes [32 pos, 32 pos + 32) of the chunk; lane l stores bytes [16 l, +16) and [1024 + 16 l, +16)
                bounce[2 * pos] = make_uint4(o[0], o[1], o[2], o[3]);
                bounce[2 * pos + 1] = make_uint4(o[4], o[5], o[6], o[7]);
                __builtin_amdgcn_wave_barrier();
                const uint4 lo = bounce[lane], hi = bounce[64 + lane];
                __builtin_amdgcn_wave_barrier();
                if (row <= last_row) {
                    uint4 *dst = reinterpret_cast<uint4 *>(reinterpret_cast<uint16_t *>(out) + (int64_t)row * ldo + slab * SLAB);
                    if (8 * lane < slab_cols) dst[lane] = lo;
                    if (512 + 8 * lane < slab_cols) dst[64 + lane] = hi;
                }
            } else {
#pragma unroll
                for (int e = 0; e < 16; e += 4)
                    bounce[4 * pos + (e >> 2)] = __builtin_bit_cast(uint4, make_float4((x[e] * a) * qs[e], (x[e + 1] * a) * qs[e + 1],
                                                                                      (x[e + 2] * a) * qs[e + 2], (x[e + 3] * a) * qs[e + 3]));
                __builtin_amdgcn_wave_barrier();
                uint4 v[4];
#pragma unroll
                for (int q = 0; q < 4; ++q) v[q] = bounce[64 * q + lane];
                __builtin_amdgcn_wave_barrier();
                if (row <= last_row) {
                    uint4 *dst = reinterpret_cast<uint4 *>(reinterpret_cast<float *>(out) + (int64_t)row * ldo + slab * SLAB);
#pragma unroll
                    for (int q = 0; q < 4; ++q)
                        if (256 * q + 4 * lane < slab_cols) dst[64 * q + lane] = v[q];
                }
            }
        }
    }
}

bool fast_decode_supported(const Problem &p) {
    const int unit = p.block > 16 ? p.block : 16;
    if (p.d_in % unit) return false;
    if (p.bits != 7 && p.bits != 8 && p.bits != 11) return false;
    return p.block >= 64;                                        // 64, 128, 256, 512, 1024
}

constexpr int DF_ROWS = 4;            // rows a wave handles per step
constexpr int DF_BLOCKS_PER_CU = 6;    // resident blocks per compute unit the grid is sized for

template <int BITS, int B>
static hipError_t launch_bb(const uint8_t *packed, const float *norms, const Problem &p, void *out, int64_t ldo,
                            bool out_bf16) {
    // vector stores need 16-byte aligned rows
    const int64_t align_elems = out_bf16 ? 8 : 4;
    if (ldo % align_elems || (reinterpret_cast<uintptr_t>(out) & 15)) return hipErrorNotSupported;
    if ((reinterpret_cast<uintptr_t>(p.chan_scale) | reinterpret_cast<uintptr_t>(p.signs) |
         reinterpret_cast<uintptr_t>(p.pair_sigma)) & 15)
        return hipErrorNotSupported;
    if ((reinterpret_cast<uintptr_t>(packed) & 3)) return hipErrorNotSupported;
    const int n_slabs = (p.d_in + SLAB - 1) / SLAB;
    const int n_groups = (p.d_out + DF_ROWS - 1) / DF_ROWS;
    // waves that share a slab: enough to fill the machine (256 CUs x DF_BLOCKS_PER_CU blocks), no more than the work
    int max_wps = (256 * DF_BLOCKS_PER_CU * DF_WAVES) / n_slabs;
    if (max_wps < 1) max_wps = 1;
    const int steps = (n_groups + max_wps - 1) / max_wps;           // row groups each wave walks through
    const int waves_per_slab = (n_groups + steps - 1) / steps;     // evened out: no wave does more than `steps`
    const int64_t n_waves = (int64_t)waves_per_slab * n_slabs;
    const unsigned blocks = (unsigned)((n_waves + DF_WAVES - 1) / DF_WAVES);
    const size_t lds = (size_t)p.K * sizeof(float2) + (size_t)DF_WAVES * (out_bf16 ? 2048 : 4096);
    if (out_bf16)
        hipLaunchKernelGGL((k_decode_fast<BITS, B, true, DF_ROWS>), dim3(blocks), dim3(DF_THREADS), lds, p.stream, packed,
                           norms, p, out, ldo, n_slabs, waves_per_slab);
    else
        hipLaunchKernelGGL((k_decode_fast<BITS, B, false, DF_ROWS>), dim3(blocks), dim3(DF_THREADS), lds, p.stream, packed,
                           norms, p, out, ldo, n_slabs, waves_per_slab);
    return hipGetLastError();
}

template <int BITS>
static hipError_t launch_b(const uint8_t *packed, const float *norms, const Problem &p, void *out, int64_t ldo,
                           bool out_bf16) {
    switch (p.block) {
        case 64: return launch_bb<BITS, 64>(packed, norms, p, out, ldo, out_bf16);
        case 128: return launch_bb<BITS, 128>(packed, norms, p, out, ldo, out_bf16);
        case 256: return launch_bb<BITS, 256>(packed, norms, p, out, ldo, out_bf16);
        case 512: return launch_bb<BITS, 512>(packed, norms, p, out, ldo, out_bf16);
        case 1024: return launch_bb<BITS, 1024>(packed, norms, p, out, ldo, out_bf16);
        default: return hipErrorNotSupported;
    }
}

hipError_t launch_decode_fast(const uint8_t *packed, const float *norms, const Problem &p, void *out, int64_t ldo,
                              bool out_bf16) {
    hipError_t e = hipErrorNotSupported;
    if (p.bits == 11) e = launch_b<11>(packed, norms, p, out, ldo, out_bf16);
    else if (p.bits == 8) e = launch_b<8>(packed, norms, p, out, ldo, out_bf16);
    else if (p.bits == 7) e = launch_b<7>(packed, norms, p, out, ldo, out_bf16);
    if (e == hipErrorNotSupported) return launch_decode_general(packed, norms, p, out, ldo, out_bf16);
    return e;
}

}  // namespace qamw
