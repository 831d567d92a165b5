// libqamw host side: status strings, storage accounting, sign mask, channel scales and the
// CPU codebook trainer.  Nothing in this file touches the GPU.
#include "qamw.h"

#include <algorithm>
#include <atomic>
#include <cmath>
#include <cstdlib>
#include <cstring>
#include <limits>
#include <thread>
#include <vector>

namespace {

// SplitMix64 output function applied to a counter: word n of stream `seed`.
inline uint64_t stream_word(uint64_t seed, uint64_t n) {
    uint64_t z = seed + (n + 1u) * 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

int worker_count() {
    if (const char *e = std::getenv("QAMW_NUM_THREADS")) {
        int v = std::atoi(e);
        if (v >= 1) return std::min(v, 64);
    }
    unsigned hw = std::thread::hardware_concurrency();
    return (int)std::max(1u, std::min(hw, 16u));
}

// Run fn(task) for task in [0, n_tasks) on a small thread pool.  Tasks write disjoint outputs, so
// the result does not depend on which thread ran which task.
template <class F> void parallel_tasks(int64_t n_tasks, F fn) {
    int nt = (int)std::min<int64_t>(worker_count(), n_tasks);
    if (nt <= 1) {
        for (int64_t t = 0; t < n_tasks; ++t) fn(t);
        return;
    }
    std::atomic<int64_t> next{0};
    std::vector<std::thread> pool;
    for (int w = 0; w < nt; ++w)
        pool.emplace_back([&] {
            for (;;) {
                int64_t t = next.fetch_add(1);
                if (t >= n_tasks) break;
                fn(t);
            }
        });
    for (auto &th : pool) th.join();
}

}  // namespace

extern "C" {

const char *qamw_status_string(int status) {
    switch (status) {
        case QAMW_OK: return "ok";
        case QAMW_ERR_INVALID_ARG: return "invalid argument";
        case QAMW_ERR_SHAPE: return "invalid shape";
        case QAMW_ERR_UNSUPPORTED: return "unsupported configuration";
        case QAMW_ERR_DEVICE: return "device error";
        default: return "unknown status";
    }
}

int qamw_packed_row_bytes(int d_in, int bits, size_t *out) {
    if (!out || bits < 1 || bits > QAMW_MAX_BITS) return QAMW_ERR_INVALID_ARG;
    if (d_in <= 0 || (d_in & 1)) return QAMW_ERR_SHAPE;
    uint64_t nbits = (uint64_t)(d_in / 2) * (uint64_t)bits;
    *out = (size_t)((nbits + 31) / 32 * 4);
    return QAMW_OK;
}

int qamw_paper_block_size(int d_in, int *block_out) {
    if (!block_out) return QAMW_ERR_INVALID_ARG;
    if (d_in <= 0) return QAMW_ERR_SHAPE;
    int b = 1;
    while (b < QAMW_MAX_BLOCK && (d_in & b) == 0) b <<= 1;   // lowest set bit of d_in, capped
    *block_out = b;
    return QAMW_OK;
}

int qamw_bpw(int d_in, int d_out, int bits, int with_f16_scales, double *out) {
    if (!out || bits < 1 || bits > QAMW_MAX_BITS) return QAMW_ERR_INVALID_ARG;
    if (d_in <= 0 || d_out <= 0) return QAMW_ERR_SHAPE;
    double v = 0.5 * bits + 16.0 / d_in;
    if (with_f16_scales) v += 16.0 / d_out;
    *out = v;
    return QAMW_OK;
}

int qamw_sign_mask(uint64_t seed, int d_in, int8_t *signs_out) {
    if (!signs_out) return QAMW_ERR_INVALID_ARG;
    if (d_in <= 0) return QAMW_ERR_SHAPE;
    for (int w = 0; w * 64 < d_in; ++w) {
        uint64_t word = stream_word(seed, (uint64_t)w);
        int n = std::min(64, d_in - w * 64);
        for (int t = 0; t < n; ++t) signs_out[w * 64 + t] = (int8_t)(1 - 2 * (int)((word >> t) & 1u));
    }
    return QAMW_OK;
}

int qamw_channel_scales(const float *act_rms, int d_in, float alpha, float *s_out) {
    if (!act_rms || !s_out || !(alpha >= 0.0f && alpha <= 1.0f)) return QAMW_ERR_INVALID_ARG;
    if (d_in <= 0) return QAMW_ERR_SHAPE;
    std::vector<double> lg((size_t)d_in);
    double mean = 0.0;
    for (int j = 0; j < d_in; ++j) {
        lg[j] = (double)alpha * std::log(std::max((double)act_rms[j], 1e-30));
        mean += lg[j];
    }
    mean /= d_in;
    for (int j = 0; j < d_in; ++j)
        s_out[j] = (float)std::min(16.0, std::max(1.0 / 16.0, std::exp(lg[j] - mean)));
    return QAMW_OK;
}

// ---------------------------------------------------------------------------------------------
// Codebook training.  The assignment step is exact nearest-neighbour search made cheap by a
// uniform grid: for every grid cell the list of codewords that can be nearest to ANY point of the
// cell is those within (distance from the cell centre to its nearest codeword) + (cell diagonal)
// of the centre.  Per-chunk partial sums are reduced in chunk order, so the result is the same
// for any number of threads.
// ---------------------------------------------------------------------------------------------
int qamw_train_codebook(int bits, uint64_t n_samples, uint64_t seed, int max_iters, double tol,
                        float *codebook_out, double *mse_out, int *iters_out) {
    if (!codebook_out || bits < 1 || bits > QAMW_MAX_BITS || max_iters < 1 || !(tol >= 0.0))
        return QAMW_ERR_INVALID_ARG;
    const int K = 1 << bits;
    if (n_samples < (uint64_t)K || n_samples > (1ull << 32)) return QAMW_ERR_INVALID_ARG;
    const int64_t n = (int64_t)n_samples;

    // samples
    std::vector<double> xy((size_t)n * 2);
    const int64_t CH = 4096;
    const int64_t n_chunks = (n + CH - 1) / CH;
    parallel_tasks(n_chunks, [&](int64_t c) {
        const double two_pi = 6.283185307179586476925286766559;
        for (int64_t i = c * CH; i < std::min(n, (c + 1) * CH); ++i) {
            uint64_t a = stream_word(seed, (uint64_t)(2 * i));
            uint64_t b = stream_word(seed, (uint64_t)(2 * i + 1));
            double u1 = ((double)(a >> 11) + 1.0) * (1.0 / 9007199254740992.0);
            double u2 = (double)(b >> 11) * (1.0 / 9007199254740992.0);
            double rad = std::sqrt(-2.0 * std::log(u1));
            xy[2 * i] = rad * std::cos(two_pi * u2);
            xy[2 * i + 1] = rad * std::sin(two_pi * u2);
        }
    });

    // initial points
    std::vector<double> cb((size_t)K * 2);
    {
        const double golden = 2.3999632297286533222315555066336;
        for (int i = 0; i < K; ++i) {
            double q = (i + 0.5) / K;
            double rad = std::sqrt(-4.0 * std::log(1.0 - q));
            cb[2 * i] = rad * std::cos(golden * i);
            cb[2 * i + 1] = rad * std::sin(golden * i);
        }
    }

    const double R = 6.5;                                            // grid covers [-R, R)^2
    const int G = std::max(8, std::min(256, (int)std::lround(4.0 * std::sqrt((double)K))));
    const double h = 2.0 * R / G, inv_h = 1.0 / h, diag = h * std::sqrt(2.0);
    std::vector<int32_t> cell_begin((size_t)G * G + 1);
    std::vector<std::vector<int32_t>> cell_list((size_t)G * G);
    std::vector<int32_t> cand;

    std::vector<int32_t> assign((size_t)n);
    std::vector<double> err((size_t)n);
    std::vector<double> part_sum((size_t)n_chunks * K * 2);
    std::vector<int64_t> part_cnt((size_t)n_chunks * K);
    std::vector<double> part_err((size_t)n_chunks);

    double prev = std::numeric_limits<double>::infinity(), D = prev;
    int it = 0;
    for (;; ++it) {
        // candidate lists per grid cell (ascending codeword index)
        parallel_tasks((int64_t)G, [&](int64_t gy) {
            std::vector<double> dist((size_t)K);
            for (int gx = 0; gx < G; ++gx) {
                double cx = -R + (gx + 0.5) * h, cy = -R + (gy + 0.5) * h;
                double dmin = std::numeric_limits<double>::infinity();
                for (int c = 0; c < K; ++c) {
                    double e0 = cx - cb[2 * c], e1 = cy - cb[2 * c + 1];
                    dist[c] = std::sqrt(e0 * e0 + e1 * e1);
                    dmin = std::min(dmin, dist[c]);
                }
                double lim = dmin + diag * (1.0 + 1e-9) + 1e-12;
                auto &lst = cell_list[(size_t)gy * G + gx];
                lst.clear();
                for (int c = 0; c < K; ++c)
                    if (dist[c] <= lim) lst.push_back(c);
            }
        });
        cell_begin[0] = 0;
        for (size_t c = 0; c < cell_list.size(); ++c) cell_begin[c + 1] = cell_begin[c] + (int32_t)cell_list[c].size();
        cand.resize((size_t)cell_begin.back());
        for (size_t c = 0; c < cell_list.size(); ++c)
            std::copy(cell_list[c].begin(), cell_list[c].end(), cand.begin() + cell_begin[c]);

        // assignment + per-chunk partial sums
        parallel_tasks(n_chunks, [&](int64_t ch) {
            double *ps = &part_sum[(size_t)ch * K * 2];
            int64_t *pc = &part_cnt[(size_t)ch * K];
            std::memset(ps, 0, sizeof(double) * K * 2);
            std::memset(pc, 0, sizeof(int64_t) * K);
            double tot = 0.0;
            for (int64_t s = ch * CH; s < std::min(n, (ch + 1) * CH); ++s) {
                double x = xy[2 * s], y = xy[2 * s + 1];
                double best = std::numeric_limits<double>::infinity();
                int32_t bi = 0;
                int gx = (int)std::floor((x + R) * inv_h), gy = (int)std::floor((y + R) * inv_h);
                if (gx >= 0 && gx < G && gy >= 0 && gy < G) {
                    size_t cell = (size_t)gy * G + gx;
                    for (int32_t q = cell_begin[cell]; q < cell_begin[cell + 1]; ++q) {
                        int32_t c = cand[q];
                        double e0 = x - cb[2 * c], e1 = y - cb[2 * c + 1];
                        double d = e0 * e0 + e1 * e1;
                        if (d < best) { best = d; bi = c; }
                    }
                } else {
                    for (int32_t c = 0; c < K; ++c) {
                        double e0 = x - cb[2 * c], e1 = y - cb[2 * c + 1];
                        double d = e0 * e0 + e1 * e1;
                        if (d < best) { best = d; bi = c; }
                    }
                }
                assign[s] = bi;
                err[s] = best;
                tot += best;
                ps[2 * bi] += x;
                ps[2 * bi + 1] += y;
                pc[bi]++;
            }
            part_err[ch] = tot;
        });
        double tot = 0.0;
        for (int64_t ch = 0; ch < n_chunks; ++ch) tot += part_err[ch];
        D = tot / (double)n;
        if ((it > 0 && std::fabs(prev - D) < tol * prev) || it == max_iters - 1) {
            ++it;
            break;
        }
        prev = D;

        // centroid step
        for (int c = 0; c < K; ++c) {
            double sx = 0.0, sy = 0.0;
            int64_t cnt = 0;
            for (int64_t ch = 0; ch < n_chunks; ++ch) {
                sx += part_sum[((size_t)ch * K + c) * 2];
                sy += part_sum[((size_t)ch * K + c) * 2 + 1];
                cnt += part_cnt[(size_t)ch * K + c];
            }
            if (cnt > 0) {
                cb[2 * c] = sx / (double)cnt;
                cb[2 * c + 1] = sy / (double)cnt;
            } else {
                int64_t worst = 0;
                for (int64_t s = 1; s < n; ++s)
                    if (err[s] > err[worst]) worst = s;
                cb[2 * c] = xy[2 * worst];
                cb[2 * c + 1] = xy[2 * worst + 1];
                err[worst] = 0.0;
            }
        }
    }
    for (int i = 0; i < 2 * K; ++i) codebook_out[i] = (float)cb[i];
    if (mse_out) *mse_out = D;
    if (iters_out) *iters_out = it;
    return QAMW_OK;
}

}  // extern "C"

namespace {

// Running integrals of f(r) = r exp(-r^2/2) times 1, r, r^2 from 0 to r on a uniform grid over
// [0, rmax] (Simpson's rule per grid interval), read back between grid points by cubic Hermite
// interpolation (the derivative of a running integral is its integrand).
struct RayleighTables {
    static constexpr int N = 1 << 15;
    double rmax, h;
    std::vector<double> m[3];
    static double integrand(int k, double r) {
        const double f = r * std::exp(-0.5 * r * r);
        return k == 0 ? f : (k == 1 ? f * r : f * r * r);
    }
    explicit RayleighTables(double rmax_) : rmax(rmax_), h(rmax_ / N) {
        for (int k = 0; k < 3; ++k) {
            m[k].assign(N + 1, 0.0);
            for (int i = 0; i < N; ++i) {
                const double a = h * i, b = a + h;
                m[k][i + 1] = m[k][i] + h / 6.0 * (integrand(k, a) + 4.0 * integrand(k, 0.5 * (a + b)) + integrand(k, b));
            }
        }
    }
    double upto(int k, double r) const {
        if (r <= 0.0) return 0.0;
        if (r >= rmax) return m[k][N];
        const int i = std::min((int)(r / h), N - 1);
        const double a = h * i, t = (r - a) / h;
        const double y0 = m[k][i], y1 = m[k][i + 1], d0 = h * integrand(k, a), d1 = h * integrand(k, a + h);
        const double t2 = t * t, t3 = t2 * t;
        return (2 * t3 - 3 * t2 + 1) * y0 + (t3 - 2 * t2 + t) * d0 + (-2 * t3 + 3 * t2) * y1 + (t3 - t2) * d1;
    }
};

}  // namespace

extern "C" int qamw_polar_codebook(int bits_a, int bits_p, float *levels_out, float *table_out, double *c_lm_out) {
    if (!levels_out || bits_a < 0 || bits_a > QAMW_MAX_POLAR_AMPLITUDE_BITS || bits_p < 0 || bits_p > 12 ||
        bits_a + bits_p < 1 || bits_a + bits_p > QAMW_MAX_BITS)
        return QAMW_ERR_INVALID_ARG;
    const int Na = 1 << bits_a, Np = 1 << bits_p;
    const RayleighTables T(8.0);
    std::vector<double> lv(Na), nx(Na);
    for (int i = 0; i < Na; ++i) lv[i] = 4.0 * (i + 0.5) / Na;   // any increasing start converges; this one is uniform on [0, 4]
    double D = 0.0;
    // the fixed-point iteration contracts slowly when there are many levels (about Na^2 log(1/tol) steps)
    for (int it = 0; it < 1000000; ++it) {
        double move = 0.0;
        D = 0.0;
        for (int i = 0; i < Na; ++i) {
            const double lo = i == 0 ? 0.0 : 0.5 * (lv[i - 1] + lv[i]);
            const double hi = i == Na - 1 ? T.rmax : 0.5 * (lv[i] + lv[i + 1]);
            const double m0 = T.upto(0, hi) - T.upto(0, lo), m1 = T.upto(1, hi) - T.upto(1, lo),
                         m2 = T.upto(2, hi) - T.upto(2, lo);
            nx[i] = m0 > 0.0 ? m1 / m0 : lv[i];
            D += m2 - 2.0 * lv[i] * m1 + lv[i] * lv[i] * m0;     // distortion of the levels before the move
            move = std::max(move, std::fabs(nx[i] - lv[i]));
        }
        lv = nx;
        if (move < 1e-14) break;
    }
    for (int i = 0; i < Na; ++i) levels_out[i] = (float)lv[i];
    if (table_out) {
        const double h = 3.14159265358979323846 / Np;
        for (int ia = 0; ia < Na; ++ia)
            for (int ip = 0; ip < Np; ++ip) {
                const double ph = (2.0 * ip + 1.0) * h;
                table_out[2 * ((size_t)ia * Np + ip)] = (float)((double)levels_out[ia] * std::cos(ph));
                table_out[2 * ((size_t)ia * Np + ip) + 1] = (float)((double)levels_out[ia] * std::sin(ph));
            }
    }
    if (c_lm_out) *c_lm_out = D;
    return QAMW_OK;
}

// ---------------------------------------------------------------------------------------------
// Search grid for the pruned nearest-codeword search.
namespace {
constexpr uint32_t GRID_MAGIC = 0x44524751u;   // "QGRD"
constexpr int GRID_ENTRIES = 8;
constexpr size_t GRID_HEADER_BYTES = 32;
}  // namespace

extern "C" int qamw_search_grid_size(int bits, int *cells_per_side_out, size_t *bytes_out) {
    if (bits < 1 || bits > QAMW_MAX_BITS) return QAMW_ERR_INVALID_ARG;
    const int G = 1 << ((bits + 6) / 2);                        // about 16-32 cells per codeword
    if (cells_per_side_out) *cells_per_side_out = G;
    if (bytes_out) *bytes_out = GRID_HEADER_BYTES + (size_t)G * G * GRID_ENTRIES * sizeof(uint16_t);
    return QAMW_OK;
}

extern "C" int qamw_search_grid_build(const float *codebook, int bits, void *grid_out, size_t grid_bytes,
                                      int *max_candidates_out, uint64_t *overflow_cells_out) {
    int G = 0;
    size_t need = 0;
    if (!codebook || !grid_out || qamw_search_grid_size(bits, &G, &need) != QAMW_OK || grid_bytes < need)
        return QAMW_ERR_INVALID_ARG;
    const int K = 1 << bits;
    double cmax = 0.0;
    for (int i = 0; i < 2 * K; ++i) {
        if (!std::isfinite(codebook[i])) return QAMW_ERR_INVALID_ARG;
        cmax = std::max(cmax, std::fabs((double)codebook[i]));
    }
    // the square [-R, R)^2: a quarter wider than the codebook, so that few points fall outside
    const double R = cmax > 0.0 ? 1.25 * cmax : 1.0;
    const float inv_h = (float)((double)G / (2.0 * R));         // cells per unit length, as the kernel uses it
    const double h = 1.0 / (double)inv_h;
    // The kernel takes floor(fma(x, inv_h, G/2)) in fp32; the rounding of that fma moves a point by at most
    // 2^-24 G cells.  Every cell is widened by four times that on each side, so that a point the kernel
    // assigns to a cell lies in the widened cell.
    const double margin = std::ldexp((double)G * h, -22);
    std::vector<double> lo(G), hi(G);
    for (int i = 0; i < G; ++i) {
        lo[i] = ((double)i - 0.5 * G) * h - margin;
        hi[i] = ((double)(i + 1) - 0.5 * G) * h + margin;
    }
    // per axis and codeword: squared smallest / largest distance from the coordinate to the cell's interval
    std::vector<double> nx((size_t)K * G), fx((size_t)K * G), ny((size_t)K * G), fy((size_t)K * G);
    for (int c = 0; c < K; ++c)
        for (int a = 0; a < 2; ++a) {
            const double v = codebook[2 * c + a];
            double *nn = (a == 0 ? nx : ny).data() + (size_t)c * G, *ff = (a == 0 ? fx : fy).data() + (size_t)c * G;
            for (int i = 0; i < G; ++i) {
                const double dn = std::max(std::max(lo[i] - v, v - hi[i]), 0.0);
                const double df = std::max(std::fabs(v - lo[i]), std::fabs(v - hi[i]));
                nn[i] = dn * dn;
                ff[i] = df * df;
            }
        }
    uint32_t *hdr = static_cast<uint32_t *>(grid_out);
    std::memset(hdr, 0, GRID_HEADER_BYTES);
    hdr[0] = GRID_MAGIC;
    hdr[1] = (uint32_t)bits;
    hdr[2] = (uint32_t)G;
    hdr[3] = (uint32_t)GRID_ENTRIES;
    std::memcpy(&hdr[4], &inv_h, sizeof(float));
    const float Rf = (float)R;
    std::memcpy(&hdr[5], &Rf, sizeof(float));
    uint16_t *cells = reinterpret_cast<uint16_t *>(static_cast<char *>(grid_out) + GRID_HEADER_BYTES);
    std::vector<int> row_max(G, 0);
    std::vector<uint64_t> row_over(G, 0);
    parallel_tasks(G, [&](int64_t iy) {
        std::vector<int> cand;
        for (int ix = 0; ix < G; ++ix) {
            // no codeword farther from every point of the cell than U can be nearest to a point of the cell
            double U = std::numeric_limits<double>::infinity();
            for (int c = 0; c < K; ++c) U = std::min(U, fx[(size_t)c * G + ix] + fy[(size_t)c * G + iy]);
            // fp32 evaluation of a squared distance is within 2^-22 of it, relatively: 1e-5 covers both sides with room
            const double lim = U * (1.0 + 1e-5) + 1e-30;
            cand.clear();
            for (int c = 0; c < K; ++c)
                if (nx[(size_t)c * G + ix] + ny[(size_t)c * G + iy] <= lim) cand.push_back(c);
            uint16_t *rec = cells + ((size_t)iy * G + ix) * GRID_ENTRIES;
            const int n = (int)cand.size();
            row_max[iy] = std::max(row_max[iy], n);
            if (n <= GRID_ENTRIES) {
                for (int j = 0; j < GRID_ENTRIES; ++j) rec[j] = (uint16_t)cand[j < n ? j : 0];
            } else {                                            // too many: the kernel scans the whole codebook
                for (int j = 0; j < GRID_ENTRIES - 1; ++j) rec[j] = (uint16_t)cand[j];
                rec[GRID_ENTRIES - 1] = 0xFFFFu;
                ++row_over[iy];
            }
        }
    });
    int mx = 0;
    uint64_t over = 0;
    for (int i = 0; i < G; ++i) {
        mx = std::max(mx, row_max[i]);
        over += row_over[i];
    }
    if (max_candidates_out) *max_candidates_out = mx;
    if (overflow_cells_out) *overflow_cells_out = over;
    return QAMW_OK;
}
