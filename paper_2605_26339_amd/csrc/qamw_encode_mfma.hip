// QAM-W encoder whose shortlist scores come from the matrix cores (Sec. 3.1 / Sec. 3.5).
//
// The score matrix  S[c][x] = ||c||^2 - 2 x.c  of a block of 32 codewords against a block of 32
// points is a (32 x 3)(3 x 32) product: a dense contraction with a tiny inner dimension.  The
// fp32 matrix instruction runs on the same FMA lanes as the vector ALU and buys nothing, but the
// bf16 matrix cores are separate hardware.  Every fp32 operand is split EXACTLY into three bf16
// pieces h + m + l (8 + 8 + 8 significant bits, by truncation), and one
// v_mfma_f32_32x32x16_bf16 sums, per coordinate, the six piece products hh, hm, mh, hl, mm, lh
// and, in the four inner slots left over, the three pieces of ||c||^2 times 1.  Piece products
// are exact in fp32.  What is lost: the products ml, lm, ll (at most 2^-22 n1 ||c|| in all, with
// n1 = |x0| + |x1|) and the rounding of a 15-term fp32 accumulation, which for any summation
// order is at most 14 x 2^-24 x (sum of magnitudes) < 2^-20 (||c||^2 + 2.02 n1 ||c||).  The
// kernel budgets 2^-19 (||c|| + n1)^2; the worst error seen over 3e6 random evaluations on the
// hardware is 2^-21.6 of that scale.  The bound is all the shortlist needs: as in the vector-ALU
// encoder, the index is decided by exact fp32 squared distances inside the best chunk when the
// runner-up chunk is provably out of reach, and by an exact scan of the whole codebook
// otherwise.  The vector ALU is left with the min-reduction of the scores.
//
// Work split: a wave owns 512 pairs (one row's 1024-column slab).  Front half in registers as in
// the vector-ALU encoder; the pairs are then transposed through LDS into the matrix layout
// (lane = point of a 32-point block, lanes 0-31 / 32-63 = the two coordinates).  A chunk is the
// lane's 16 accumulator rows {8q + 4h + t} of two consecutive 32-codeword blocks (of one block for
// codebooks of up to 256 points).
#include <atomic>
#include <cmath>

#include "qamw_front.hpp"

namespace qamw {

constexpr int MF_THREADS = 512;
constexpr int MF_WAVES = MF_THREADS / WAVE;
constexpr int MSLAB = 1024;
constexpr int NPB = 8;                 // 32-point blocks whose operands and state a wave holds at a time
constexpr int PB_TOTAL = 16;           // 512 pairs / 32
constexpr float MBIG = 3.0e38f;
constexpr uint32_t BF16_ONE_ONE = 0x3F803F80u;  // (1.0, 1.0) as two bf16
constexpr int MF_WAVE_LDS_FLOATS = 1024 + 256;   // per wave: 512 points (x0, x1) + 512 16-bit indices
constexpr int MF_MAX_LDS_BYTES = (2048 * 4 + MF_WAVES * MF_WAVE_LDS_FLOATS) * 4;   // K = 2048: 72 KB, two workgroups per CU

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

// CH: 32-codeword blocks per chunk.  Two halve the tracking work of the main loop; one halves the exact distances
// of the decision stage (8 instead of 16 per lane and point), which is what matters for a small codebook.
// One matrix of an encode launch, as the kernel sees it, and the work list of the launch: workgroups are numbered
// matrix-major; a workgroup's MF_WAVES items belong to one matrix.
struct EncodeMat {
    const void *W;
    int64_t ldw;
    const float *chan_scale;
    const int8_t *signs;
    const float *pair_sigma;
    float *norms;
    uint8_t *packed;
    int64_t row_bytes;
    int d_in, n_slabs, n_items;
    float g_default;                      // sqrt(d_in): the pair gain when pair_sigma is NULL
};
struct EncodeBatch {
    EncodeMat m[QAMW_ENCODE_MAX_BATCH];
    int block_begin[QAMW_ENCODE_MAX_BATCH + 1];   // first workgroup of each matrix; block_begin[n] = total
    int n;
    int bits, K;
    float inv_sqrt_block;
    const float *codebook;
    unsigned long long *full_scans;
};

template <int DTYPE, int B, int CH>
__global__ __launch_bounds__(MF_THREADS) void k_encode_mfma(EncodeBatch bt, int fused) {
    extern __shared__ __align__(16) float lds_raw[];
    float2 *c01 = reinterpret_cast<float2 *>(lds_raw);          // K x (c0, c1)
    uint32_t *e67 = reinterpret_cast<uint32_t *>(lds_raw + 2 * bt.K);   // K x 2: bf16 pieces of ||c||^2, (h, m) and (l, 0)
    __shared__ float red[MF_WAVES];
    __shared__ double norm_part[2 * FUSED_NORM_MAX_SLABS];

    const int lane = threadIdx.x & (WAVE - 1);
    const int wid = threadIdx.x >> 6;
    const int K = bt.K;
    // fused: the workgroup computes the norms of the rows its items touch (and writes them out) before anything else;
    // the barrier after the codebook staging below also publishes the slab sums.  Otherwise they are read.
    const int n_blocks = bt.block_begin[bt.n];
    const int blk = min(fused ? fused_norm_block(blockIdx.x, n_blocks) : (int)blockIdx.x, n_blocks);   // n_blocks: nothing to do
    int mi = 0;
    while (mi + 1 < bt.n && blk >= bt.block_begin[mi + 1]) ++mi;
    const EncodeMat &M = bt.m[mi];
    Problem p;
    p.d_in = M.d_in;
    p.bits = bt.bits;
    p.K = K;
    p.chan_scale = M.chan_scale;
    p.signs = M.signs;
    p.pair_sigma = M.pair_sigma;
    p.codebook = bt.codebook;
    p.inv_sqrt_block = bt.inv_sqrt_block;
    p.g_default = M.g_default;
    p.row_bytes = M.row_bytes;
    p.full_scans = bt.full_scans;
    const void *__restrict__ W = M.W;
    const int64_t ldw = M.ldw;
    const int n_slabs = M.n_slabs, n_items = M.n_items;
    float *__restrict__ norms = M.norms;
    uint8_t *__restrict__ packed = M.packed;
    const int item0 = blk < n_blocks ? (blk - bt.block_begin[mi]) * MF_WAVES : n_items;
    if (fused && item0 < n_items) block_slab_sums<DTYPE, MF_WAVES>(norm_part, W, ldw, p, item0, n_items, n_slabs, lane, wid);
    float *wave_area = lds_raw + 4 * K + wid * MF_WAVE_LDS_FLOATS;
    float2 *pts = reinterpret_cast<float2 *>(wave_area);        // the wave's 512 points, pair order
    uint16_t *idxl = reinterpret_cast<uint16_t *>(wave_area + 1024);   // their indices

    const float2 *cbk = reinterpret_cast<const float2 *>(p.codebook);
    float rmax2 = 0.0f;
    for (int i = threadIdx.x; i < K; i += MF_THREADS) {
        float2 c = cbk[i];
        float n2 = __builtin_fmaf(c.y, c.y, c.x * c.x);
        uint32_t h, m, l;
        split3(n2, h, m, l);
        c01[i] = c;
        e67[2 * i] = pack2(h, m);
        e67[2 * i + 1] = pack2(l, 0u);
        rmax2 = fmaxf(rmax2, n2);
    }
#pragma unroll
    for (int m = 1; m < WAVE; m <<= 1) rmax2 = fmaxf(rmax2, __shfl_xor(rmax2, m, WAVE));
    if (lane == 0) red[wid] = rmax2;
    __syncthreads();
    rmax2 = 0.0f;
#pragma unroll
    for (int w = 0; w < MF_WAVES; ++w) rmax2 = fmaxf(rmax2, red[w]);
    const float R = sqrtf(rmax2) * 1.000001f;

    const int item = __builtin_amdgcn_readfirstlane(item0 + wid);
    if (item >= n_items) return;
    const int row = item / n_slabs, slab = item - row * n_slabs;
    float rnorm;
    if (fused) {
        rnorm = row_norm_from_slab_sums(norm_part, row, item0, n_slabs);
        if (slab == 0 && lane == 0) norms[row] = rnorm;
    } else {
        rnorm = norms[row];
    }
    const LaneSigns<B> ls(lane);
    const int pos = slab_pos(lane);
    const int col0 = slab * MSLAB + 16 * pos;
    const bool active = col0 < p.d_in;
    const int c = active ? col0 : 0;

    // ---------------- front half, then the pairs go to LDS in pair order
    {
        float x[16];
        rotated_unit_row<DTYPE, B>(x, W, (int64_t)row * ldw, c, rnorm, p, ls);
        float g[8];
        load_pair_gains(g, p, c);
        float4 *dst = reinterpret_cast<float4 *>(pts + 8 * pos);
#pragma unroll
        for (int k = 0; k < 8; k += 2)
            dst[k >> 1] = make_float4(x[2 * k] * g[k], x[2 * k + 1] * g[k], x[2 * k + 2] * g[k + 1], x[2 * k + 3] * g[k + 1]);
    }
    __builtin_amdgcn_wave_barrier();

    const int j = lane & 31, hs = lane >> 5;
    const float *ptsf = reinterpret_cast<const float *>(pts);
    const float *c01f = reinterpret_cast<const float *>(c01);
    const int n_cblk = K / 32;

    for (int pass = 0; pass < PB_TOTAL / NPB; ++pass) {
        // point-side operands: lane (j, hs) supplies coordinate hs of point j of each block, times -2,
        // and 1 in the two slots that meet the pieces of ||c||^2
        bf8v_t bop[NPB];
        float m1[NPB], m2[NPB];
        int best[NPB];
#pragma unroll
        for (int pb = 0; pb < NPB; ++pb) {
            const float v = -2.0f * ptsf[(32 * (pass * NPB + pb) + j) * 2 + hs];
            uint32_t h, m, l;
            split3(v, h, m, l);
            const u4v_t u = {pack2(h, m), pack2(h, l), pack2(m, h), BF16_ONE_ONE};     // h m h l m h 1 1
            bop[pb] = __builtin_bit_cast(bf8v_t, u);
            m1[pb] = MBIG;
            m2[pb] = MBIG;
            best[pb] = 0;
        }
        const f16v_t zero = {0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f};
        for (int cb = 0; cb < n_cblk; cb += 2) {                   // n_cblk is even
            // codeword-side operands of blocks cb and cb+1: coordinate hs of codeword 32 cb + j in the
            // order h h m h m l that meets h m h l m h, then this half's two pieces of ||c||^2
            bf8v_t aop[2];
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                uint32_t h, m, l;
                split3(c01f[((cb + u) * 32 + j) * 2 + hs], h, m, l);
                const u4v_t ua = {pack2(h, h), pack2(m, h), pack2(m, l), e67[((cb + u) * 32 + j) * 2 + hs]};
                aop[u] = __builtin_bit_cast(bf8v_t, ua);
            }
#pragma unroll
            for (int pb = 0; pb < NPB; ++pb) {
                const f16v_t d = __builtin_amdgcn_mfma_f32_32x32x16_bf16(aop[0], bop[pb], zero, 0, 0, 0);
                const f16v_t e = __builtin_amdgcn_mfma_f32_32x32x16_bf16(aop[1], bop[pb], zero, 0, 0, 0);
                const float t0 = mmin3(d[0], d[1], d[2]), t1 = mmin3(d[3], d[4], d[5]), t2 = mmin3(d[6], d[7], d[8]);
                const float t3 = mmin3(d[9], d[10], d[11]), t4 = mmin3(d[12], d[13], d[14]);
                const float s0 = mmin3(e[0], e[1], e[2]), s1 = mmin3(e[3], e[4], e[5]), s2 = mmin3(e[6], e[7], e[8]);
                const float s3 = mmin3(e[9], e[10], e[11]), s4 = mmin3(e[12], e[13], e[14]);
                const float r0 = mmin3(t0, t1, t2), r1 = mmin3(t3, t4, d[15]), r2 = mmin3(s0, s1, s2), r3 = mmin3(s3, s4, e[15]);
                if (CH == 2) {
                    const float cm = __builtin_fminf(mmin3(r0, r1, r2), r3);
                    best[pb] = (cm < m1[pb]) ? cb : best[pb];
                    m2[pb] = __builtin_amdgcn_fmed3f(m1[pb], m2[pb], cm);   // m1 <= m2: second smallest chunk minimum
                    m1[pb] = __builtin_fminf(m1[pb], cm);
                } else {
                    const float cm0 = __builtin_fminf(r0, r1), cm1 = __builtin_fminf(r2, r3);
                    best[pb] = (cm0 < m1[pb]) ? cb : best[pb];
                    m2[pb] = __builtin_amdgcn_fmed3f(m1[pb], m2[pb], cm0);
                    m1[pb] = __builtin_fminf(m1[pb], cm0);
                    best[pb] = (cm1 < m1[pb]) ? cb + 1 : best[pb];
                    m2[pb] = __builtin_amdgcn_fmed3f(m1[pb], m2[pb], cm1);
                    m1[pb] = __builtin_fminf(m1[pb], cm1);
                }
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
            const int cbb = other ? ob : best[pb];                 // first block of the best chunk ...
            const int hb = other ? (hs ^ 1) : hs;                  // ... and which 16 rows of each of its blocks
            const float2 x = pts[32 * pbg + j];
            const float n1 = fabsf(x.x) + fabsf(x.y);
            const float emax = 1.91e-6f * (R + n1) * (R + n1);                   // 2^-19 (R + n1)^2
            const float xx = __builtin_fmaf(x.y, x.y, x.x * x.x);
            const float d2 = fmaxf(M1 + xx * 1.000001f + emax, 0.0f);            // >= true best squared distance
            const float rho = sqrtf(d2) * 1.000001f + 0.0625f;
            const float eps = 1.92e-6f * (2.0f * n1 + rho) * (2.0f * n1 + rho);
            const bool safe = (M2 - M1 > 2.0f * eps) && (emax < 1.0e-3f);
            // this lane checks rows 8q + 4hb + t of the chunk's blocks for q = 2hs, 2hs+1 (ascending index), its partner the other two q
            float bd = MBIG;
            int bi = 0x7fffffff;
#pragma unroll
            for (int u = 0; u < CH; ++u) {
#pragma unroll
                for (int qq = 0; qq < 2; ++qq) {
#pragma unroll
                    for (int t = 0; t < 4; ++t) {
                        const int ci = (cbb + u) * 32 + 8 * (2 * hs + qq) + 4 * hb + t;
                        const float dd = exact_dist2(x.x, x.y, c01[ci]);
                        if (dd < bd) {
                            bd = dd;
                            bi = ci;
                        }
                    }
                }
            }
            const float od = __shfl_xor(bd, 32, WAVE);
            const int oi = __shfl_xor(bi, 32, WAVE);
            if (od < bd || (od == bd && oi < bi)) bi = oi;
            if (hs == 0) idxl[32 * pbg + j] = (uint16_t)bi;
            if (!safe && hs == 0) flagged |= 1u << pb;
            asm volatile("" ::: "memory");
        }
#pragma unroll
        for (int pb = 0; pb < NPB; ++pb) {
            const int pbg = pass * NPB + pb;
            unsigned long long mask = __ballot((flagged >> pb) & 1u);
            if (p.full_scans && mask && lane == 0) atomicAdd(p.full_scans, (unsigned long long)__popcll(mask));
            while (mask) {
                const int src = __ffsll((long long)mask) - 1;      // a lane below 32: point src of block pbg
                mask &= mask - 1;
                const float2 x = pts[32 * pbg + src];
                const int bi = wave_exact_scan(x.x, x.y, c01, K, lane);
                if (lane == src) idxl[32 * pbg + src] = (uint16_t)bi;
            }
        }
    }
    __builtin_amdgcn_wave_barrier();

    // ---------------- pack: the lane's 8 fields are exactly `bits` bytes, byte aligned in the row
    if (active) {
        const uint4 iv = *reinterpret_cast<const uint4 *>(idxl + 8 * pos);
        const unsigned idx[8] = {iv.x & 0xffffu, iv.x >> 16, iv.y & 0xffffu, iv.y >> 16,
                                 iv.z & 0xffffu, iv.z >> 16, iv.w & 0xffffu, iv.w >> 16};
        store_packed_fields(packed, row, c, col0, idx, p);
    }
}

bool mfma_encode_supported(const Problem &p) {
    const int unit = p.block > 16 ? p.block : 16;
    if (p.d_in % unit) return false;
    if (p.K % 64 || p.bits > 11) return false;          // whole chunks of two 32-codeword blocks
    return p.block >= 64;
}

// More than the default 64 KB of LDS per workgroup has to be asked for: a host-side setting per kernel and device, made
// once per kernel instantiation and device (the devices' bits of `done`).
template <int DTYPE, int B, int CH> static bool allow_large_lds() {
    static std::atomic<uint64_t> done{0};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) {
        (void)hipGetLastError();
        return false;
    }
    if (done.load(std::memory_order_acquire) & (1ull << dev)) return true;
    const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&k_encode_mfma<DTYPE, B, CH>),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, MF_MAX_LDS_BYTES);
    if (e != hipSuccess) {
        (void)hipGetLastError();
        return false;
    }
    done.fetch_or(1ull << dev, std::memory_order_release);
    return true;
}

template <int DTYPE, int B, int CH>
static hipError_t launch_mdbc(const EncodeItem *items, int n, const Problem &p, bool norms_ready) {
    EncodeBatch bt;
    int64_t blocks_total = 0;
    for (int i = 0; i < n; ++i) {
        EncodeMat &M = bt.m[i];
        const int n_slabs = (items[i].d_in + MSLAB - 1) / MSLAB;
        const int64_t n_items = (int64_t)items[i].d_out * n_slabs;
        if (n_items > 0x3fffffff) return hipErrorNotSupported;
        if (!norms_ready && n_slabs > FUSED_NORM_MAX_SLABS) return hipErrorNotSupported;
        M.W = items[i].W;
        M.ldw = items[i].ldw;
        M.chan_scale = items[i].chan_scale;
        M.signs = items[i].signs;
        M.pair_sigma = items[i].pair_sigma;
        M.norms = items[i].norms;
        M.packed = items[i].packed;
        M.row_bytes = (((int64_t)(items[i].d_in / 2) * p.bits + 31) / 32) * 4;
        M.d_in = items[i].d_in;
        M.n_slabs = n_slabs;
        M.n_items = (int)n_items;
        M.g_default = (float)std::sqrt((double)items[i].d_in);
        bt.block_begin[i] = (int)blocks_total;
        blocks_total += (n_items + MF_WAVES - 1) / MF_WAVES;
        if (blocks_total > 0x3fffffff) return hipErrorNotSupported;
    }
    for (int i = n; i <= QAMW_ENCODE_MAX_BATCH; ++i) bt.block_begin[i] = (int)blocks_total;
    for (int i = n; i < QAMW_ENCODE_MAX_BATCH; ++i) bt.m[i] = bt.m[0];
    bt.n = n;
    bt.bits = p.bits;
    bt.K = p.K;
    bt.inv_sqrt_block = p.inv_sqrt_block;
    bt.codebook = p.codebook;
    bt.full_scans = p.full_scans;
    const unsigned blocks = (unsigned)(norms_ready ? blocks_total : fused_norm_grid((int)blocks_total));
    const size_t lds = ((size_t)p.K * 4 + (size_t)MF_WAVES * MF_WAVE_LDS_FLOATS) * sizeof(float);
    if (lds > 64 * 1024 && !allow_large_lds<DTYPE, B, CH>()) return hipErrorNotSupported;
    hipLaunchKernelGGL((k_encode_mfma<DTYPE, B, CH>), dim3(blocks), dim3(MF_THREADS), lds, p.stream, bt, norms_ready ? 0 : 1);
    return hipGetLastError();
}

// one-block chunks for codebooks of up to 256 points, where the decision stage outweighs the main loop
template <int DTYPE, int B>
static hipError_t launch_mdb(const EncodeItem *items, int n, const Problem &p, bool norms_ready) {
    return p.K <= 256 ? launch_mdbc<DTYPE, B, 1>(items, n, p, norms_ready) : launch_mdbc<DTYPE, B, 2>(items, n, p, norms_ready);
}

template <int DTYPE>
static hipError_t launch_md(const EncodeItem *items, int n, const Problem &p, bool norms_ready) {
    switch (p.block) {
        case 64: return launch_mdb<DTYPE, 64>(items, n, p, norms_ready);
        case 128: return launch_mdb<DTYPE, 128>(items, n, p, norms_ready);
        case 256: return launch_mdb<DTYPE, 256>(items, n, p, norms_ready);
        case 512: return launch_mdb<DTYPE, 512>(items, n, p, norms_ready);
        case 1024: return launch_mdb<DTYPE, 1024>(items, n, p, norms_ready);
        default: return hipErrorNotSupported;
    }
}

// n <= QAMW_ENCODE_MAX_BATCH matrices that share codebook, bits, block and element type in ONE launch; p carries the
// shared fields.  Returns hipErrorNotSupported (nothing launched) when any item's shape or alignment is outside this
// kernel's range.  norms_ready: the row norms are already in every item's `norms`; otherwise the kernel computes them
// itself and writes them there.
hipError_t launch_encode_batch_mfma(const EncodeItem *items, int n, int dtype, const Problem &p, bool norms_ready) {
    if (n < 1 || n > QAMW_ENCODE_MAX_BATCH || (reinterpret_cast<uintptr_t>(p.codebook) & 15)) return hipErrorNotSupported;
    for (int i = 0; i < n; ++i) {
        Problem q = p;
        q.d_in = items[i].d_in;
        q.chan_scale = items[i].chan_scale;
        q.signs = items[i].signs;
        q.pair_sigma = items[i].pair_sigma;
        if (!mfma_encode_supported(q) || !front_alignment_ok(items[i].W, dtype, items[i].ldw, q)) return hipErrorNotSupported;
    }
    return dtype == 0 ? launch_md<0>(items, n, p, norms_ready) : launch_md<1>(items, n, p, norms_ready);
}

hipError_t launch_encode_mfma(const void *W, int dtype, int64_t ldw, const Problem &p, float *norms, bool norms_ready,
                              uint8_t *packed) {
    const EncodeItem it{W, ldw, p.chan_scale, p.signs, p.pair_sigma, norms, packed, p.d_out, p.d_in};
    return launch_encode_batch_mfma(&it, 1, dtype, p, norms_ready);
}

}  // namespace qamw
