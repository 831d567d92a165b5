// Shape-specialised QAM-W decoder (Sec. 3.2 + Sec. B.2): HBM-bound, everything between the packed
// load and the bf16 store stays in registers.
//
// A wave owns a slab of 1024 columns and walks down a range of rows.  Per row a lane unpacks its
// 8 indices (8*bits bits = `bits` bytes, always byte aligned), gathers 8 codewords from the
// LDS-resident codebook, scales them by sigma_k, runs the block Walsh-Hadamard butterflies
// across the wave (qamw_wave_fwht.hpp), applies row and column factors and stores 16 bf16.
// Column constants (1/s_j with the sign mask and the transform's lane sign folded in, sigma_k)
// are loaded once per slab and reused for every row.
#include <cmath>
#include <type_traits>

#include "qamw_common.hpp"
#include "qamw_internal.hpp"
#include "qamw_wave_fwht.hpp"

namespace qamw {

#ifndef QAMW_DF_THREADS
#define QAMW_DF_THREADS 256
#endif
constexpr int DF_THREADS = QAMW_DF_THREADS;
constexpr int DF_WAVES = DF_THREADS / WAVE;
constexpr int SLAB = 1024;
constexpr int DF_MAX_BATCH = QAMW_DECODE_MAX_BATCH;
constexpr int DF_MAX_K = 2048;
// Rows of one unit of work: a wave requests the packed words of all of them at the start, in two halves, and
// computes and stores one half while the other is still on its way.  Small units mean many waves per launch and a
// short dependent chain per wave; measured best (7B and 13B shapes): 8 rows at 11 bits (704 packed bytes per row
// and slab), 16 rows at 7 and 8 bits (448 / 512 bytes).
constexpr int df_unit_rows(int bits) { return bits >= 10 ? 8 : 16; }

typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float floatx2_t __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));

// Field i (i = 0..7) of a lane's 8*BITS-bit group (the group starts at bit 0 of w[0..2]) as a byte offset into the
// codebook: index * 8 = (stream >> (bit - 3)) & mask8, one shift or funnel shift and one AND with the mask held in a
// register (an AND of two registers issues at twice the rate of one with a literal operand).
template <int BITS> __device__ __forceinline__ uint32_t field_x8(const uint32_t (&w)[4], int i, uint32_t mask8) {
    const int bit = i * BITS, word = bit >> 5, off = bit & 31, s = off - 3;
    uint32_t v;
    if (s < 0)
        v = w[word] << (-s);
    else if (off + BITS <= 32)
        v = w[word] >> s;
    else
        v = __builtin_amdgcn_alignbit(w[word + 1], w[word], s);
    return v & mask8;
}

// Per-lane column constants of 16 consecutive columns starting at c (a multiple of 16):
// qs[e] = 1 / s_j carrying the sign mask in its sign bit, sig[k] = sigma of the lane's 8 pairs.
// (The transform's lane sign is not folded in here: it rides on the row factor, one multiply per row instead of 16
// per unit.)  Vector loads: the host checks that the arrays are 16-byte aligned.
__device__ __forceinline__ void load_column_constants(float (&qs)[16], float (&sig)[8], const Problem &p, int c) {
    if (p.chan_scale) {
        const float4 *s4 = reinterpret_cast<const float4 *>(p.chan_scale + c);
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            float4 v = s4[t];
            qs[4 * t] = fast_recip(v.x);
            qs[4 * t + 1] = fast_recip(v.y);
            qs[4 * t + 2] = fast_recip(v.z);
            qs[4 * t + 3] = fast_recip(v.w);
        }
    } else {
#pragma unroll
        for (int e = 0; e < 16; ++e) qs[e] = 1.0f;
    }
    if (p.signs) {
        const uint4 sg = *reinterpret_cast<const uint4 *>(p.signs + c);
        const uint32_t wds[4] = {sg.x, sg.y, sg.z, sg.w};
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            // int8 -1 = 0xFF: bit 7 of the byte is the sign.  A shift brings it to bit 31 and a bit-field insert
            // replaces the sign bit of the (positive) reciprocal with it.  s_j > 0 is the contract.
            const uint32_t at31 = wds[e >> 2] << (24 - 8 * (e & 3));
            qs[e] = __uint_as_float((__float_as_uint(qs[e]) & 0x7FFFFFFFu) | (at31 & 0x80000000u));
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

// One matrix of a decode batch, as the kernel sees it.
struct DecodeMat {
    const uint8_t *packed;
    const float *norms;
    const float *chan_scale;
    const int8_t *signs;
    const float *pair_sigma;
    void *out;
    int64_t ldo;
    int64_t row_bytes;
    int d_out, d_in, n_slabs;
    float sigma_default;                  // 1/sqrt(d_in), used when pair_sigma is NULL
};

// Work list of one launch.  A unit is (matrix, group of df_unit_rows(bits) rows, slab), numbered matrix-major,
// then row-group-major, slab fastest: unit numbers follow memory order.
struct DecodeBatch {
    DecodeMat m[DF_MAX_BATCH];
    int unit_begin[DF_MAX_BATCH + 1];     // first unit of each matrix; unit_begin[n] = total
    int n;
    int K;
    float inv_sqrt_block;
    const float *codebook;
};

// Decode kernel over a batch of matrices.  A block (4 waves) stages the codebook into LDS once; wave w
// of the grid takes unit w: 2R rows of one 1024-column slab, with the slab's column constants
// loaded once.  Units are numbered in memory order and blocks are dispatched in that order, which
// keeps the reads and writes in flight close together in HBM.  The packed words of both halves of
// the unit are requested before anything is stored, so a wave never waits for its own stores to
// drain before its loads are under way (loads and stores retire through one in-order counter on
// this chip).
// TRAFFIC_ONLY: the same loads and stores (addresses, widths, order, launch shape) with the arithmetic between them
// left out -- what is stored is a meaningless mix of what was loaded.  It measures what the memory system gives this
// access pattern, i.e. the ceiling of the decoder proper.
// Register budget: the bf16 kernel with 8-row units fits 80 registers (6 waves per SIMD) without spilling; the
// 16-row units, the fp32 output and blocks beyond 256 (their swap stages) need more and are left at 4.
#define QAMW_DF_WAVES_PER_EU ((R > 4 || !OUT_BF16 || B > 256) ? 4 : 6)
template <int BITS, int B, bool OUT_BF16, int R, bool TRAFFIC_ONLY = false>
__global__ __launch_bounds__(DF_THREADS) __attribute__((amdgpu_waves_per_eu(QAMW_DF_WAVES_PER_EU))) void k_decode_fast(DecodeBatch bt, int n_waves) {
    constexpr int UNIT = 2 * R;                                 // rows of a unit: two halves of R rows
    __shared__ float2 cb_lds[DF_MAX_K];                         // K <= DF_MAX_K codewords; a static array: its address folds into the gathers' offset field
    typedef u32x4_t u32x4_a4_t __attribute__((aligned(4)));     // a 16-byte load that is only 4-byte aligned
    const int lane = threadIdx.x & (WAVE - 1);
    const int wid = threadIdx.x >> 6;
    const int wave_id = __builtin_amdgcn_readfirstlane(blockIdx.x * DF_WAVES + wid);
    const LaneSigns<B> ls(lane);
    const int pos = slab_pos(lane);
    // after the half exchange: whose sub-block this lane stores in the first / second store instruction, and which half
    const int pos_a = slab_pos(lane & 31), pos_b = slab_pos((lane & 31) + 32), half = lane >> 5;
    const uint32_t off_a = (uint32_t)(2 * pos_a + half) * 16u, off_b = (uint32_t)(2 * pos_b + half) * 16u;   // byte offsets inside the slab's 2 KB

    // n_waves = number of units.  A surplus wave of the last block goes through the motions on the last unit
    // (it has to reach the barrier below) and stores nothing.
    const bool surplus = wave_id >= n_waves;
    const int wave = surplus ? n_waves - 1 : wave_id;

    // which matrix, slab and rows (all uniform over the wave)
    int mi = 0;
    while (mi + 1 < bt.n && wave >= bt.unit_begin[mi + 1]) ++mi;
    const DecodeMat &M = bt.m[mi];
    const int local = wave - bt.unit_begin[mi];
    const int n_slabs = M.n_slabs;
    // the division runs on the vector ALU; readfirstlane returns the (uniform) results to scalar registers
    const int slab = __builtin_amdgcn_readfirstlane(local % n_slabs);
    const int row0 = __builtin_amdgcn_readfirstlane((local / n_slabs) * UNIT);
    const int d_in = M.d_in, last_row = M.d_out - 1;
    const int64_t row_bytes = M.row_bytes, ldo = M.ldo;
    const uint8_t *packed = M.packed;
    // the row norms are the same for every lane: read through the scalar data path (constant address space)
    typedef const float __attribute__((address_space(4))) *const_f32_ptr;
    const_f32_ptr norms = (const_f32_ptr)(uintptr_t)M.norms;
    void *out = M.out;

    const int col0 = slab * SLAB + 16 * pos;
    const int c = (col0 < d_in) ? col0 : 0;                     // first of the lane's 16 columns (0 for idle lanes)
    const int slab_cols = min(SLAB, d_in - slab * SLAB);        // valid columns of this slab
    // The lane's 8 fields are BITS bytes at byte (c/16)*BITS of the row: rows are multiples of 4 bytes, so the
    // position inside a dword is the same in every row.
    const unsigned lane_off = (unsigned)(c >> 4) * BITS;
    const unsigned lane_b0 = lane_off & ~3u;
    const int sh = (int)(lane_off & 3u) * 8;
    const unsigned row_dw = (unsigned)(row_bytes >> 2);

    const float isb_parity = bt.inv_sqrt_block * ls.parity;     // exact: parity is +-1
    uint32_t mask8;                                             // ((1 << BITS) - 1) * 8 in a register the optimiser cannot fold back into a literal
    asm volatile("v_mov_b32 %0, %1" : "=v"(mask8) : "n"(((1 << BITS) - 1) * 8));
    float qs[16], sig[8];
    {
        Problem pc;
        pc.chan_scale = M.chan_scale;
        pc.signs = M.signs;
        pc.pair_sigma = M.pair_sigma;
        pc.sigma_default = M.sigma_default;
        load_column_constants(qs, sig, pc, c);
    }

    // FULL: every row of the unit exists and is not the matrix's last row, and the slab has all 1024
    // columns.  Then every load and store below is unconditional, which lets the compiler count them
    // (s_waitcnt vmcnt(N) with N > 0) instead of draining the stores before each wait for loads.
    const bool full = slab_cols == SLAB && row0 + UNIT <= last_row && !surplus;
    const bool second = full || row0 + R <= last_row;           // the unit's second half has at least one row
    auto fetch = [&](auto full_tag, int sub, uint32_t (&d)[R][4], float (&rn)[R]) {
        constexpr bool FULL = decltype(full_tag)::value;
#pragma unroll
        for (int t = 0; t < R; ++t) {
            const int row = FULL ? row0 + sub + t : min(row0 + sub + t, last_row);   // rows past the end re-read the last row
            const uint8_t *rowp = packed + (int64_t)row * row_bytes;
            if (FULL || row != last_row) {
                // 16 bytes from a 4-byte-aligned address; may run a few bytes into the next row
                const u32x4_t v = *reinterpret_cast<const u32x4_a4_t *>(rowp + lane_b0);
                d[t][0] = v[0]; d[t][1] = v[1]; d[t][2] = v[2]; d[t][3] = v[3];
            } else {
                // last row of the matrix: stay inside it (the clamped words are beyond the lane's fields)
                const uint32_t *rw = reinterpret_cast<const uint32_t *>(rowp);
#pragma unroll
                for (int k = 0; k < 4; ++k) d[t][k] = rw[min((lane_b0 >> 2) + k, row_dw - 1u)];
            }
            rn[t] = norms[row];
        }
    };
    // Both halves of the unit are requested before anything is computed: the second arrives while the first is
    // computed and stored.  With the longer units (7 and 8 bits) the requests go out even before the block stages
    // the codebook; with 8-row units that would cost registers (5 instead of 6 waves per SIMD), so there they are
    // issued after the barrier (inside run()).
    constexpr bool EARLY = R > 4;
    // The codebook goes from memory straight into LDS (no registers on the way): wave w copies the 1 KB pieces
    // w, w + 4, ..., lane l the 16 bytes l of a piece (the instruction places lane l's bytes at base + 16 l).
    auto stage = [&]() {
        const char *src = reinterpret_cast<const char *>(bt.codebook);
        const int bytes = bt.K * (int)sizeof(float2);
        for (int off = __builtin_amdgcn_readfirstlane(wid) * 1024; off < bytes; off += DF_WAVES * 1024) {
            if (off + 16 * lane < bytes)
                __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(src + off + 16 * lane),
                                                 (__attribute__((address_space(3))) void *)(reinterpret_cast<char *>(cb_lds) + off),
                                                 16, 0, 0);
        }
        __builtin_amdgcn_s_waitcnt(0x0F70);                    // vmcnt(0): this wave's pieces have landed before the barrier
        __syncthreads();
    };
    uint32_t d0[R][4], d1[R][4];
    float rn0[R], rn1[R];
    if (EARLY) {
        if (full) {
            fetch(std::true_type{}, 0, d0, rn0);
            fetch(std::true_type{}, R, d1, rn1);
        } else {
            fetch(std::false_type{}, 0, d0, rn0);
            if (second) fetch(std::false_type{}, R, d1, rn1);
        }
    }
    stage();
    if (surplus) return;

    auto run = [&](auto full_tag) {
        constexpr bool FULL = decltype(full_tag)::value;
        auto rows = [&](int sub, const uint32_t (&d)[R][4], const float (&rn)[R]) {
#pragma unroll
            for (int t = 0; t < R; ++t) {
                const int row = row0 + sub + t;
                if (TRAFFIC_ONLY) {
                    const uint32_t mix = __float_as_uint(rn[t]) ^ __float_as_uint(qs[t]) ^ __float_as_uint(sig[t & 7]);
                    const u32x4_t va = {d[t][0] ^ mix, d[t][1], d[t][2], d[t][3]}, vb = {d[t][3], d[t][2] ^ mix, d[t][1], d[t][0]};
                    if (FULL || row <= last_row) {
                        u32x4_t *dst = reinterpret_cast<u32x4_t *>(reinterpret_cast<uint16_t *>(out) + (int64_t)row * ldo + slab * SLAB);
                        if (FULL || 16 * pos_a < slab_cols) __builtin_nontemporal_store(va, dst + 2 * pos_a + half);
                        if (FULL || 16 * pos_b < slab_cols) __builtin_nontemporal_store(vb, dst + 2 * pos_b + half);
                    }
                    continue;
                }
                uint32_t w[4];
                w[0] = __builtin_amdgcn_alignbit(d[t][1], d[t][0], sh);
                w[1] = __builtin_amdgcn_alignbit(d[t][2], d[t][1], sh);
                w[2] = __builtin_amdgcn_alignbit(d[t][3], d[t][2], sh);
                w[3] = d[t][3] >> sh;
                float x[16];
#pragma unroll
                for (int k = 0; k < 8; ++k) {
                    const float2 cw = *reinterpret_cast<const float2 *>(reinterpret_cast<const char *>(cb_lds) + field_x8<BITS>(w, k, mask8));
                    x[2 * k] = sig[k] * cw.x;
                    x[2 * k + 1] = sig[k] * cw.y;
                }
                fwht_wave<B>(x, ls);
                const float a = rn[t] * isb_parity;             // row factor r * block^-1/2, with the transform's lane sign
                if (OUT_BF16) {
                    uint32_t o[8];
#pragma unroll
                    for (int e = 0; e < 16; e += 2) {
                        floatx2_t v = {(x[e] * a) * qs[e], (x[e + 1] * a) * qs[e + 1]};
                        o[e >> 1] = __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
                    }
                    // A lane's 16 bf16 are 32 consecutive bytes.  Storing them as they are would make each store
                    // instruction write every other 16 bytes; instead lanes i and i+32 trade one half each
                    // (v_permlane32_swap), after which lanes 0-31 hold the first halves and lanes 32-63 the second
                    // halves of 32 neighbouring sub-blocks: each store instruction then covers 1 KB without holes.
                    uint32_t lo[4] = {o[0], o[1], o[2], o[3]}, hi[4] = {o[4], o[5], o[6], o[7]};
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        auto r = __builtin_amdgcn_permlane32_swap(lo[q], hi[q], false, false);   // upper lanes' lo <-> lower lanes' hi
                        lo[q] = r[0];
                        hi[q] = r[1];
                    }
                    if (FULL || row <= last_row) {
                        char *dst = reinterpret_cast<char *>(reinterpret_cast<uint16_t *>(out) + (int64_t)row * ldo + slab * SLAB);
                        // instruction A: sub-blocks of lanes 0-31; instruction B: sub-blocks of lanes 32-63.
                        // The output is written once and not read again by this kernel: streaming stores.
                        const u32x4_t va = {lo[0], lo[1], lo[2], lo[3]}, vb = {hi[0], hi[1], hi[2], hi[3]};
                        if (FULL || 16 * pos_a < slab_cols) __builtin_nontemporal_store(va, reinterpret_cast<u32x4_t *>(dst + off_a));
                        if (FULL || 16 * pos_b < slab_cols) __builtin_nontemporal_store(vb, reinterpret_cast<u32x4_t *>(dst + off_b));
                    }
                } else if (FULL || (row <= last_row && 16 * pos < slab_cols)) {   // fp32 output (accuracy checks): plain per-lane stores
                    float4 *dst = reinterpret_cast<float4 *>(reinterpret_cast<float *>(out) + (int64_t)row * ldo + slab * SLAB + 16 * pos);
#pragma unroll
                    for (int e = 0; e < 16; e += 4)
                        dst[e >> 2] = make_float4((x[e] * a) * qs[e], (x[e + 1] * a) * qs[e + 1], (x[e + 2] * a) * qs[e + 2],
                                                  (x[e + 3] * a) * qs[e + 3]);
                }
            }
        };
        if (!EARLY) {
            fetch(full_tag, 0, d0, rn0);
            if (FULL || second) fetch(full_tag, R, d1, rn1);
        }
        rows(0, d0, rn0);
        if (FULL || second) rows(R, d1, rn1);
    };
    if (full)
        run(std::true_type{});
    else
        run(std::false_type{});
}

bool fast_decode_supported(const Problem &p) {
    const int unit = p.block > 16 ? p.block : 16;
    if (p.d_in % unit) return false;
    if (p.bits != 7 && p.bits != 8 && p.bits != 11) return false;
    return p.block >= 64;                                        // 64, 128, 256, 512, 1024
}

// Alignment the vector loads and stores of the fast kernel assume.
static bool decode_alignment_ok(const DecodeItem &it, bool out_bf16) {
    const int64_t align_elems = out_bf16 ? 8 : 4;
    if (it.ldo % align_elems || (reinterpret_cast<uintptr_t>(it.out) & 15)) return false;
    if ((reinterpret_cast<uintptr_t>(it.chan_scale) | reinterpret_cast<uintptr_t>(it.signs) |
         reinterpret_cast<uintptr_t>(it.pair_sigma)) & 15)
        return false;
    return (reinterpret_cast<uintptr_t>(it.packed) & 3) == 0;
}

template <int BITS, int B>
static hipError_t launch_bb(const DecodeItem *items, int n, const Problem &p, bool out_bf16, bool traffic_only) {
    constexpr int UNIT = df_unit_rows(BITS), R = UNIT / 2;
    DecodeBatch bt;
    int64_t units = 0;
    for (int i = 0; i < n; ++i) {
        DecodeMat &M = bt.m[i];
        M.packed = items[i].packed;
        M.norms = items[i].norms;
        M.chan_scale = items[i].chan_scale;
        M.signs = items[i].signs;
        M.pair_sigma = items[i].pair_sigma;
        M.out = items[i].out;
        M.ldo = items[i].ldo;
        M.d_out = items[i].d_out;
        M.d_in = items[i].d_in;
        M.row_bytes = (((int64_t)(M.d_in / 2) * BITS + 31) / 32) * 4;
        M.n_slabs = (M.d_in + SLAB - 1) / SLAB;
        M.sigma_default = (float)(1.0 / std::sqrt((double)M.d_in));
        bt.unit_begin[i] = (int)units;
        units += (int64_t)M.n_slabs * ((M.d_out + UNIT - 1) / UNIT);
        if (units > 0x3fffffff) return hipErrorNotSupported;
    }
    for (int i = n; i <= DF_MAX_BATCH; ++i) bt.unit_begin[i] = (int)units;
    for (int i = n; i < DF_MAX_BATCH; ++i) bt.m[i] = bt.m[0];
    bt.n = n;
    bt.K = p.K;
    bt.inv_sqrt_block = p.inv_sqrt_block;
    bt.codebook = p.codebook;
    // One unit per wave, blocks dispatched in unit (= memory) order.  (A machine-sized persistent grid with a
    // stride was measured slower on HBM-bound sizes: its waves move in lockstep through read and write phases.)
    const int64_t n_waves = units;
    const unsigned blocks = (unsigned)((n_waves + DF_WAVES - 1) / DF_WAVES);
    if (p.K > DF_MAX_K) return hipErrorNotSupported;
    const size_t lds = 0;
    if (traffic_only)                                            // the access pattern does not depend on the block size
        hipLaunchKernelGGL((k_decode_fast<BITS, 64, true, R, true>), dim3(blocks), dim3(DF_THREADS), lds, p.stream, bt, (int)n_waves);
    else if (out_bf16)
        hipLaunchKernelGGL((k_decode_fast<BITS, B, true, R>), dim3(blocks), dim3(DF_THREADS), lds, p.stream, bt, (int)n_waves);
    else
        hipLaunchKernelGGL((k_decode_fast<BITS, B, false, R>), dim3(blocks), dim3(DF_THREADS), lds, p.stream, bt, (int)n_waves);
    return hipGetLastError();
}

template <int BITS>
static hipError_t launch_b(const DecodeItem *items, int n, const Problem &p, bool out_bf16, bool traffic_only) {
    if (traffic_only) return launch_bb<BITS, 64>(items, n, p, true, true);
    switch (p.block) {
        case 64: return launch_bb<BITS, 64>(items, n, p, out_bf16, false);
        case 128: return launch_bb<BITS, 128>(items, n, p, out_bf16, false);
        case 256: return launch_bb<BITS, 256>(items, n, p, out_bf16, false);
        case 512: return launch_bb<BITS, 512>(items, n, p, out_bf16, false);
        case 1024: return launch_bb<BITS, 1024>(items, n, p, out_bf16, false);
        default: return hipErrorNotSupported;
    }
}

// Decode n <= DF_MAX_BATCH matrices that share codebook, bits and block in one launch.  p carries the shared
// fields only.  Returns hipErrorNotSupported (nothing launched) when any item is outside the fast kernel's shapes.
hipError_t launch_decode_batch_fast(const DecodeItem *items, int n, const Problem &p, bool out_bf16, bool traffic_only) {
    if (n < 1 || n > DF_MAX_BATCH) return hipErrorNotSupported;
    for (int i = 0; i < n; ++i) {
        Problem q = p;
        q.d_in = items[i].d_in;
        if (!fast_decode_supported(q) || !decode_alignment_ok(items[i], out_bf16)) return hipErrorNotSupported;
    }
    if (p.bits == 11) return launch_b<11>(items, n, p, out_bf16, traffic_only);
    if (p.bits == 8) return launch_b<8>(items, n, p, out_bf16, traffic_only);
    if (p.bits == 7) return launch_b<7>(items, n, p, out_bf16, traffic_only);
    return hipErrorNotSupported;
}

hipError_t launch_decode_fast(const uint8_t *packed, const float *norms, const Problem &p, void *out, int64_t ldo,
                              bool out_bf16) {
    DecodeItem it{packed, norms, p.chan_scale, p.signs, p.pair_sigma, out, ldo, p.d_out, p.d_in};
    hipError_t e = launch_decode_batch_fast(&it, 1, p, out_bf16);
    if (e == hipErrorNotSupported) return launch_decode_general(packed, norms, p, out, ldo, out_bf16);
    return e;
}

}  // namespace qamw
