// QAM-W encoder with a pruned nearest-codeword search (the search step of Sec. 3.1; the result is
// the same index the whole-codebook search returns).
//
// A uniform G x G grid covers the square [-R, R)^2 that holds the codebook.  For every cell the host
// lists, in ascending index order, every codeword that can be nearest to some point of the cell
// (qamw_search_grid_build: a codeword whose smallest distance to the cell exceeds the smallest over
// the codebook of the LARGEST distance to the cell can never win).  The kernel locates the pair's
// cell, reads its record of 8 candidates (one 16-byte load) and takes the minimum of the exact fp32
// squared distances over them, strict comparison in ascending index order, so the lowest index wins
// a tie exactly as in the whole-codebook scan.  A pair outside the square, or in a cell with more
// than 8 candidates, is decided by the exact scan of the whole codebook (64 lanes x K/64 codewords).
//
// Front half as in the other fast encoders: a wave owns one row's slab of 1024 columns, 8 pairs per
// lane, everything in registers; the codebook sits in LDS.  The table is 1 MB at K = 2048 and every
// pair reads a different 128-byte line of it, so a kernel that reads it from global memory
// (k_encode_grid) runs at the rate of L2 round trips.  k_encode_grid_lds keeps the CENTRAL Gc x Gc
// cells (Gc <= 128: the square that holds 99.6 % of Gaussian pairs at K = 2048) in LDS as records of
// 5 candidates (8 bytes): workgroups of 16 waves, one per CU, stage the codebook and that part of
// the table once and then walk (row, slab) items in a strided loop.  A pair outside the central
// square or in a cell with more than 5 candidates (1.3 % of Gaussian pairs at K = 2048) takes the
// global record; a lane reads at most two of them per item and leaves any further such pair to the
// exact scan.
#include <atomic>

#include "qamw_front.hpp"

namespace qamw {

constexpr int GF_THREADS = 256;
constexpr int GF_WAVES = GF_THREADS / WAVE;
constexpr int GSLAB = 1024;
constexpr float GBIG = 3.0e38f;

template <int DTYPE, int B>
__global__ __launch_bounds__(GF_THREADS) void k_encode_grid(const void *__restrict__ W, int64_t ldw, Problem p,
                                                            const uint32_t *__restrict__ table, int G,
                                                            const float *__restrict__ norms,
                                                            uint8_t *__restrict__ packed, int n_slabs, int n_items) {
    extern __shared__ __align__(16) float2 gcb[];               // K codewords
    const int K = p.K;
    const float2 *cbk = reinterpret_cast<const float2 *>(p.codebook);
    for (int i = threadIdx.x; i < K; i += GF_THREADS) gcb[i] = cbk[i];
    __syncthreads();

    const int lane = threadIdx.x & (WAVE - 1);
    const int wid = threadIdx.x >> 6;
    const int item = __builtin_amdgcn_readfirstlane(blockIdx.x * GF_WAVES + wid);
    if (item >= n_items) return;
    // the table: a 32-byte header (word 4 = cells per unit length, as a float), then G x G records of 8 x 16 bits
    const float inv_h = __uint_as_float(table[4]);
    const float half_g = 0.5f * (float)G, g_f = (float)G;
    const uint4 *cells = reinterpret_cast<const uint4 *>(table + 8);
    const int row = item / n_slabs, slab = item - row * n_slabs;
    const LaneSigns<B> ls(lane);
    const int pos = slab_pos(lane);
    const int col0 = slab * GSLAB + 16 * pos;
    const bool active = col0 < p.d_in;
    const int c = active ? col0 : 0;

    // ---------------- front half: x_k = (F S (W D_s / r))_pair k / sigma_k, in registers
    float x[16];
    rotated_unit_row<DTYPE, B>(x, W, (int64_t)row * ldw, c, norms[row], p, ls);
    {
        float g[8];
        load_pair_gains(g, p, c);
#pragma unroll
        for (int e = 0; e < 16; ++e) x[e] = x[e] * g[e >> 1];
    }

    // ---------------- the cells' records: all 8 requested before the first is used
    uint4 rec[8];
    unsigned scan = 0;                                          // bit k: pair k needs the whole-codebook scan
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        // clamped to [-1, G] before the conversion (a NaN becomes -1): outside the square either way
        const int ix = (int)floorf(fminf(fmaxf(__builtin_fmaf(x[2 * k], inv_h, half_g), -1.0f), g_f));
        const int iy = (int)floorf(fminf(fmaxf(__builtin_fmaf(x[2 * k + 1], inv_h, half_g), -1.0f), g_f));
        const bool inside = (unsigned)ix < (unsigned)G && (unsigned)iy < (unsigned)G;
        rec[k] = cells[inside ? iy * G + ix : 0];
        if (!inside) scan |= 1u << k;
    }
    unsigned idx[8];
    const unsigned kmask = (unsigned)K - 1u;
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        const float x0 = x[2 * k], x1 = x[2 * k + 1];
        const unsigned cand[8] = {rec[k].x & 0xffffu, rec[k].x >> 16, rec[k].y & 0xffffu, rec[k].y >> 16,
                                  rec[k].z & 0xffffu, rec[k].z >> 16, rec[k].w & 0xffffu, rec[k].w >> 16};
        if (cand[7] == 0xffffu) scan |= 1u << k;                // more candidates than a record holds
        float bd = GBIG;
        unsigned bi = 0;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const unsigned ci = cand[j] & kmask;                // (the overflow mark stays inside the codebook)
            const float dd = exact_dist2(x0, x1, gcb[ci]);
            if (dd < bd) {
                bd = dd;
                bi = ci;
            }
        }
        idx[k] = bi;
    }

    // ---------------- the exact scan for the pairs that need it: the whole wave works on one pair at a time
    if (!active) scan = 0;
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        unsigned long long mask = __ballot((scan >> k) & 1u);
        if (p.full_scans && mask && lane == 0) atomicAdd(p.full_scans, (unsigned long long)__popcll(mask));
        while (mask) {
            const int src = __ffsll((long long)mask) - 1;
            mask &= mask - 1;
            const float x0 = __shfl(x[2 * k], src, WAVE), x1 = __shfl(x[2 * k + 1], src, WAVE);
            const int bi = wave_exact_scan(x0, x1, gcb, K, lane);
            if (lane == src) idx[k] = (unsigned)bi;
        }
    }

    // ---------------- pack: the lane's 8 fields are exactly `bits` bytes, byte aligned in the row
    if (active) {
        store_packed_fields(packed, row, c, col0, idx, p);
    }
}

constexpr int GL_THREADS = 1024;
constexpr int GL_WAVES = GL_THREADS / WAVE;
constexpr int GL_MAX_CENTRAL = 128;                            // cells per side kept in LDS, at most
constexpr size_t GL_MAX_LDS_BYTES = 144 * 1024;

// cells per side of the central square kept in LDS: a multiple of 32, as large as fits beside the codebook
static int central_cells(int G, int K) {
    int gc = G < GL_MAX_CENTRAL ? G : GL_MAX_CENTRAL;
    while (gc > 32 && (size_t)K * 8 + (size_t)gc * gc * 8 > GL_MAX_LDS_BYTES) gc -= 32;
    return gc;
}

// Central record: five 12-bit candidates in bits 0-59 (ascending, padded with the first), bit 63 set when the
// cell's list is longer and the global record has to be read.
__device__ __forceinline__ uint2 central_record(uint4 r) {
    const unsigned e0 = r.x & 0xffffu, e1 = r.x >> 16, e2 = r.y & 0xffffu, e3 = r.y >> 16, e4 = r.z & 0xffffu;
    const bool fits = (r.z >> 16) == e0 && r.w == (e0 | (e0 << 16));     // slots 5..7 repeat slot 0: at most 5 entries
    const unsigned lo = e0 | (e1 << 12) | (e2 << 24);
    const unsigned hi = (e2 >> 8) | (e3 << 4) | ((e4 & 0xfffu) << 16) | (fits ? 0u : 0x80000000u);
    return make_uint2(lo, hi);
}

// the pair a lane selects by number: x[2k], x[2k+1] for a k that differs from lane to lane
__device__ __forceinline__ float2 pick_pair(const float (&x)[16], int k) {
    float a = x[0], b = x[1];
#pragma unroll
    for (int j = 1; j < 8; ++j) {
        a = (k == j) ? x[2 * j] : a;
        b = (k == j) ? x[2 * j + 1] : b;
    }
    return make_float2(a, b);
}

template <int DTYPE, int B>
__global__ __launch_bounds__(GL_THREADS) void k_encode_grid_lds(const void *__restrict__ W, int64_t ldw, Problem p,
                                                                 const uint32_t *__restrict__ table, int G, int Gc,
                                                                 const float *__restrict__ norms,
                                                                 uint8_t *__restrict__ packed, int n_slabs, int n_items) {
    extern __shared__ __align__(16) float2 gcb[];               // K codewords, then Gc x Gc central records
    const int K = p.K;
    uint2 *central = reinterpret_cast<uint2 *>(gcb + K);
    const uint4 *cells = reinterpret_cast<const uint4 *>(table + 8);
    const int c0 = (G - Gc) >> 1;                               // first central cell, per axis
    const float2 *cbk = reinterpret_cast<const float2 *>(p.codebook);
    for (int i = threadIdx.x; i < K; i += GL_THREADS) gcb[i] = cbk[i];
    for (int i = threadIdx.x; i < Gc * Gc; i += GL_THREADS) {
        const int iy = i / Gc, ix = i - iy * Gc;
        central[i] = central_record(cells[(c0 + iy) * G + c0 + ix]);
    }
    __syncthreads();

    const int lane = threadIdx.x & (WAVE - 1);
    const int wid = threadIdx.x >> 6;
    const float inv_h = __uint_as_float(table[4]);
    const float half_g = 0.5f * (float)G, g_f = (float)G;
    const LaneSigns<B> ls(lane);
    const int pos = slab_pos(lane);
    const unsigned kmask = (unsigned)K - 1u;
    auto cell_coord = [&](float v) {                            // clamped to [-1, G] before the conversion (a NaN becomes -1)
        return (int)floorf(fminf(fmaxf(__builtin_fmaf(v, inv_h, half_g), -1.0f), g_f));
    };

    // The weights of the next item are requested before the current item is searched: a wave has only three
    // others on its SIMD to hide the HBM round trip behind.
    const int stride = (int)gridDim.x * GL_WAVES;
    int item = __builtin_amdgcn_readfirstlane(blockIdx.x * GL_WAVES + wid);
    auto request = [&](int it, RawRow<DTYPE> &raw, float &norm) {
        const int r = it / n_slabs, sl = it - r * n_slabs;
        const int cc = sl * GSLAB + 16 * pos;
        load_raw_row<DTYPE>(raw, W, (int64_t)r * ldw, cc < p.d_in ? cc : 0);
        norm = norms[r];
    };
    RawRow<DTYPE> raw_next;
    float norm_next = 0.0f;
    if (item < n_items) request(item, raw_next, norm_next);
    for (; item < n_items; item += stride) {
        const int row = item / n_slabs, slab = item - row * n_slabs;
        const int col0 = slab * GSLAB + 16 * pos;
        const bool active = col0 < p.d_in;
        const int c = active ? col0 : 0;
        const RawRow<DTYPE> raw = raw_next;
        const float norm = norm_next;
        if (item + stride < n_items) request(item + stride, raw_next, norm_next);

        // ---------------- front half
        float x[16];
        rotated_unit_row_from<DTYPE, B>(x, raw, c, norm, p, ls);
        {
            float g[8];
            load_pair_gains(g, p, c);
#pragma unroll
            for (int e = 0; e < 16; ++e) x[e] = x[e] * g[e >> 1];
        }

        // ---------------- the central records, and which pairs they do not settle
        uint2 lrec[8];
        unsigned more = 0;                                      // bit k: pair k is outside the central square or its list is long
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            const int ix = cell_coord(x[2 * k]) - c0, iy = cell_coord(x[2 * k + 1]) - c0;
            const bool mid = (unsigned)ix < (unsigned)Gc && (unsigned)iy < (unsigned)Gc;
            lrec[k] = central[mid ? iy * Gc + ix : 0];
            if (!mid || (lrec[k].y >> 31)) more |= 1u << k;
        }
        // Such pairs are rare.  The lane's first two get the global record, requested now and used after the
        // central candidates have been evaluated; any further ones go to the exact scan.
        const int k0 = more ? __ffs((int)more) - 1 : -1;
        const unsigned more1 = more & (more - 1u);
        const int k1 = more1 ? __ffs((int)more1) - 1 : -1;
        unsigned scan = more1 & (more1 - 1u);
        uint4 grec[2] = {make_uint4(0, 0, 0, 0), make_uint4(0, 0, 0, 0)};
        float2 gx[2];
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            const int ks = s ? k1 : k0;
            gx[s] = pick_pair(x, ks);
            if (ks >= 0) {
                const int ix = cell_coord(gx[s].x), iy = cell_coord(gx[s].y);
                if ((unsigned)ix < (unsigned)G && (unsigned)iy < (unsigned)G)
                    grec[s] = cells[iy * G + ix];
                else
                    scan |= 1u << ks;                           // outside the square
            }
        }

        // ---------------- five candidates per pair from the central records
        unsigned idx[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            const float x0 = x[2 * k], x1 = x[2 * k + 1];
            const unsigned lo = lrec[k].x, hi = lrec[k].y;
            const unsigned cand[5] = {lo & 0xfffu, (lo >> 12) & 0xfffu, __builtin_amdgcn_alignbit(hi, lo, 24) & 0xfffu,
                                      (hi >> 4) & 0xfffu, (hi >> 16) & 0xfffu};
            float bd = GBIG;
            unsigned bi = 0;
#pragma unroll
            for (int j = 0; j < 5; ++j) {
                const unsigned ci = cand[j] & kmask;
                const float dd = exact_dist2(x0, x1, gcb[ci]);
                if (dd < bd) {
                    bd = dd;
                    bi = ci;
                }
            }
            idx[k] = bi;
            __builtin_amdgcn_sched_barrier(0);                  // one pair's gathers in flight at a time: registers
        }

        // ---------------- eight candidates from the global records
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            const int ks = s ? k1 : k0;
            if (__ballot(ks >= 0) == 0) continue;
            const uint4 r = grec[s];
            const unsigned cand[8] = {r.x & 0xffffu, r.x >> 16, r.y & 0xffffu, r.y >> 16,
                                      r.z & 0xffffu, r.z >> 16, r.w & 0xffffu, r.w >> 16};
            if (ks >= 0 && cand[7] == 0xffffu) scan |= 1u << ks;     // more candidates than a record holds
            float bd = GBIG;
            unsigned bi = 0;
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const unsigned ci = cand[j] & kmask;
                const float dd = exact_dist2(gx[s].x, gx[s].y, gcb[ci]);
                if (dd < bd) {
                    bd = dd;
                    bi = ci;
                }
            }
#pragma unroll
            for (int k = 0; k < 8; ++k) idx[k] = (k == ks) ? bi : idx[k];
            __builtin_amdgcn_sched_barrier(0);
        }

        // ---------------- the exact scan for what is left: the whole wave works on one pair at a time
        if (!active) scan = 0;
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            unsigned long long mask = __ballot((scan >> k) & 1u);
            if (p.full_scans && mask && lane == 0) atomicAdd(p.full_scans, (unsigned long long)__popcll(mask));
            while (mask) {
                const int src = __ffsll((long long)mask) - 1;
                mask &= mask - 1;
                const float x0 = __shfl(x[2 * k], src, WAVE), x1 = __shfl(x[2 * k + 1], src, WAVE);
                const int bi = wave_exact_scan(x0, x1, gcb, K, lane);
                if (lane == src) idx[k] = (unsigned)bi;
            }
        }

        // ---------------- pack: the lane's 8 fields are exactly `bits` bytes, byte aligned in the row
        if (active) {
            store_packed_fields(packed, row, c, col0, idx, p);
        }
    }
}

static bool grid_encode_supported(const Problem &p) {
    const int unit = p.block > 16 ? p.block : 16;
    if (p.d_in % unit || p.block < 64) return false;
    return p.bits >= 1 && p.bits <= 12;
}

// More than the default 64 KB of LDS per workgroup has to be asked for: a host-side setting per kernel and device, made
// once per kernel instantiation and device (the devices' bits of `done`).
template <int DTYPE, int B> static bool grid_allow_large_lds() {
    static std::atomic<uint64_t> done{0};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) {
        (void)hipGetLastError();
        return false;
    }
    if (done.load(std::memory_order_acquire) & (1ull << dev)) return true;
    const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&k_encode_grid_lds<DTYPE, B>),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, (int)GL_MAX_LDS_BYTES);
    if (e != hipSuccess) {
        (void)hipGetLastError();
        return false;
    }
    done.fetch_or(1ull << dev, std::memory_order_release);
    return true;
}

template <int DTYPE, int B>
static hipError_t launch_gdb(const void *W, int64_t ldw, const Problem &p, const SearchGridView &g, const float *norms,
                             uint8_t *packed) {
    const int n_slabs = (p.d_in + GSLAB - 1) / GSLAB;
    const int64_t n_items = (int64_t)p.d_out * n_slabs;
    if (n_items > 0x7fffffff) return hipErrorNotSupported;
    const uint32_t *table = reinterpret_cast<const uint32_t *>(g.table);
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess ||
        cus < 1) {
        (void)hipGetLastError();
        return hipErrorNotSupported;
    }
    const int gc = central_cells(g.G, p.K);
    // The LDS variant pays when the central square is at least half the grid's width (+-3 sigma of the pairs for
    // a Lloyd codebook of the unit Gaussian; at K = 4096 the LDS holds less) and when there is enough work to
    // amortise staging it (at least 4 items per CU); otherwise every record is read from memory.
    if (g.variant == 1 || 2 * gc < g.G || (g.variant == 0 && n_items < 4 * (int64_t)cus)) {
        const unsigned blocks = (unsigned)((n_items + GF_WAVES - 1) / GF_WAVES);
        hipLaunchKernelGGL((k_encode_grid<DTYPE, B>), dim3(blocks), dim3(GF_THREADS), (size_t)p.K * sizeof(float2), p.stream,
                           W, ldw, p, table, g.G, norms, packed, n_slabs, (int)n_items);
        return hipGetLastError();
    }
    // one workgroup of 16 waves per CU, each wave a strided share of the items
    const size_t lds = (size_t)p.K * sizeof(float2) + (size_t)gc * gc * sizeof(uint2);
    if (lds > 64 * 1024 && !grid_allow_large_lds<DTYPE, B>()) return hipErrorNotSupported;
    const int64_t want = (n_items + GL_WAVES - 1) / GL_WAVES;
    const unsigned blocks = (unsigned)(want < cus ? want : cus);
    hipLaunchKernelGGL((k_encode_grid_lds<DTYPE, B>), dim3(blocks), dim3(GL_THREADS), lds, p.stream, W, ldw, p, table, g.G, gc,
                       norms, packed, n_slabs, (int)n_items);
    return hipGetLastError();
}

template <int DTYPE>
static hipError_t launch_gd(const void *W, int64_t ldw, const Problem &p, const SearchGridView &g, const float *norms,
                            uint8_t *packed) {
    switch (p.block) {
        case 64: return launch_gdb<DTYPE, 64>(W, ldw, p, g, norms, packed);
        case 128: return launch_gdb<DTYPE, 128>(W, ldw, p, g, norms, packed);
        case 256: return launch_gdb<DTYPE, 256>(W, ldw, p, g, norms, packed);
        case 512: return launch_gdb<DTYPE, 512>(W, ldw, p, g, norms, packed);
        case 1024: return launch_gdb<DTYPE, 1024>(W, ldw, p, g, norms, packed);
        default: return hipErrorNotSupported;
    }
}

bool grid_encode_launchable(const void *W, int dtype, int64_t ldw, const Problem &p, const SearchGridView &g) {
    return grid_encode_supported(p) && front_alignment_ok(W, dtype, ldw, p) && g.table &&
           ((reinterpret_cast<uintptr_t>(g.table) & 15) == 0) && g.G >= 1 && g.G <= 4096;
}

// Returns hipErrorNotSupported (nothing launched) when the shape or alignment is outside this kernel's range.
hipError_t launch_encode_grid(const void *W, int dtype, int64_t ldw, const Problem &p, const SearchGridView &g,
                              const float *norms, uint8_t *packed) {
    if (!grid_encode_launchable(W, dtype, ldw, p, g)) return hipErrorNotSupported;
    return dtype == 0 ? launch_gd<0>(W, ldw, p, g, norms, packed) : launch_gd<1>(W, ldw, p, g, norms, packed);
}

}  // namespace qamw
