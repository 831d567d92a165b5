// Runs the host-side functions of libqamw (csrc/qamw_host.cpp: no GPU involved) on small inputs with exactly sized
// heap buffers, for a build with -fsanitize=address,undefined.  The exit status is what the test reads.
#include <cmath>
#include <cstdio>
#include <cstring>
#include <vector>

#include "qamw.h"

static int fails = 0;
#define EXPECT(c) do { if (!(c)) { std::printf("FAILED: %s (line %d)\n", #c, __LINE__); ++fails; } } while (0)

int main() {
    for (int s = -1; s < 7; ++s) EXPECT(qamw_status_string(s) != nullptr && std::strlen(qamw_status_string(s)) > 0);
    size_t rb = 0;
    EXPECT(qamw_packed_row_bytes(2048, 11, &rb) == QAMW_OK && rb == 1408);
    EXPECT(qamw_packed_row_bytes(6, 3, &rb) == QAMW_OK && rb == 4);
    EXPECT(qamw_packed_row_bytes(7, 3, &rb) == QAMW_ERR_SHAPE && qamw_packed_row_bytes(8, 13, &rb) == QAMW_ERR_INVALID_ARG);
    int blk = 0;
    EXPECT(qamw_paper_block_size(5632, &blk) == QAMW_OK && blk == 512);
    EXPECT(qamw_paper_block_size(1 << 20, &blk) == QAMW_OK && blk == 1024);
    double bpw = 0;
    EXPECT(qamw_bpw(2048, 5632, 11, 1, &bpw) == QAMW_OK && bpw > 5.5 && bpw < 5.52);
    for (int d : {1, 63, 64, 65, 1000}) {
        std::vector<int8_t> sg((size_t)d);
        EXPECT(qamw_sign_mask(0xFFFFFFFFFFFFFFFFull, d, sg.data()) == QAMW_OK);
        for (int8_t v : sg) EXPECT(v == 1 || v == -1);
    }
    {
        std::vector<float> a = {1.0f, 1e-38f, 0.0f, 1e30f, 3.0f, 0.5f, 2.0f}, s(a.size());
        EXPECT(qamw_channel_scales(a.data(), (int)a.size(), 0.3f, s.data()) == QAMW_OK);
        for (float v : s) EXPECT(v >= 1.0f / 16 && v <= 16.0f);
        EXPECT(qamw_channel_scales(a.data(), (int)a.size(), 0.0f, s.data()) == QAMW_OK && s[3] == 1.0f);
        EXPECT(qamw_channel_scales(a.data(), (int)a.size(), 1.5f, s.data()) == QAMW_ERR_INVALID_ARG);
    }
    for (int bits : {1, 4, 7}) {
        std::vector<float> cb((size_t)2 << bits);
        double mse = 0;
        int iters = 0;
        EXPECT(qamw_train_codebook(bits, 1 << 12, 5, 8, 1e-6, cb.data(), &mse, &iters) == QAMW_OK && mse > 0 && iters >= 1);
        EXPECT(qamw_train_codebook(bits, (1ull << bits), 5, 3, 0.0, cb.data(), nullptr, nullptr) == QAMW_OK);   // one sample per point
        int G = 0, longest = 0;
        size_t bytes = 0;
        uint64_t over = 0;
        EXPECT(qamw_search_grid_size(bits, &G, &bytes) == QAMW_OK && bytes == 32 + 16 * (size_t)G * G);
        std::vector<unsigned char> grid(bytes);
        EXPECT(qamw_search_grid_build(cb.data(), bits, grid.data(), bytes, &longest, &over) == QAMW_OK && longest >= 1);
        EXPECT(qamw_search_grid_build(cb.data(), bits, grid.data(), bytes - 1, nullptr, nullptr) == QAMW_ERR_INVALID_ARG);
        std::fill(cb.begin(), cb.end(), 0.25f);                                     // every codeword the same point
        EXPECT(qamw_search_grid_build(cb.data(), bits, grid.data(), bytes, &longest, &over) == QAMW_OK);
        cb[1] = NAN;
        EXPECT(qamw_search_grid_build(cb.data(), bits, grid.data(), bytes, nullptr, nullptr) == QAMW_ERR_INVALID_ARG);
    }
    for (int ba = 0; ba <= 3; ++ba)
        for (int bp : {0, 1, 5}) {
            if (ba + bp < 1) continue;
            std::vector<float> lv((size_t)1 << ba), table((size_t)2 << (ba + bp));
            double c_lm = -1;
            EXPECT(qamw_polar_codebook(ba, bp, lv.data(), table.data(), &c_lm) == QAMW_OK && c_lm >= 0);
            for (size_t i = 1; i < lv.size(); ++i) EXPECT(lv[i] > lv[i - 1]);
        }
    EXPECT(qamw_polar_codebook(7, 1, nullptr, nullptr, nullptr) == QAMW_ERR_INVALID_ARG);
    std::printf(fails ? "host driver: %d failed checks\n" : "host driver ok\n", fails);
    return fails ? 1 : 0;
}
