// Block Walsh-Hadamard transform held in the registers of one wavefront (gfx950, wave64).
//
// Layout.  A wave owns 1024 consecutive columns of one row ("slab").  Every lane holds one
// sub-block of 16 consecutive columns in x[0..15].  Which sub-block a lane holds is permuted inside
// each group of 16 lanes so that every cross-lane butterfly partner is reachable with ONE DPP
// operand modifier:
//     logical sub-block  = slab_pos(lane)          (see below)
//     stride 16  <-> quad_perm [1,0,3,2]           (lane ^ 1)
//     stride 32  <-> quad_perm [2,3,0,1]           (lane ^ 2)
//     stride 64  <-> row_half_mirror               (lane -> 7 - lane within 8)
//     stride 128 <-> row_mirror                    (lane -> 15 - lane within 16)
//     stride 256 / 512 <-> v_permlane16_swap / v_permlane32_swap (rows of 16 lanes, halves of 32)
// Mirrors are not XORs, so the upper half of each mirrored group stores its sub-blocks in reversed
// order; slab_pos() is that order.
//
// Arithmetic.  Butterflies run with stride 1, 2, 4, ..., B/2 in this order and every sum and
// difference is one fp32 operation, so the result is bit-identical to the plain in-order loop.
// In a DPP stage a lane computes partner*(+-1) + self in one v_fmac_f32_dpp; lanes on the "minus"
// side therefore hold the NEGATED coefficient afterwards (negation is exact and commutes with
// rounding).  lane_parity_sign() is the factor that undoes it; callers fold it into a multiplier
// they apply anyway.
#pragma once
#include <hip/hip_runtime.h>

namespace qamw {

// Sub-block (0..63) of the slab that physical lane `lane` holds.
__device__ __forceinline__ int slab_pos(int lane) {
    int p = lane & 15;
    int q = p & 7;
    int l8 = (q < 4) ? q : 11 - q;                 // 0 1 2 3 7 6 5 4
    int l16 = (p < 8) ? l8 : 8 + ((7 - q) < 4 ? (7 - q) : 11 - (7 - q));
    return (lane & ~15) | l16;
}

// In-lane stages: stride 1, 2, 4, 8 (as many as fit in min(B,16)).
template <int B> __device__ __forceinline__ void fwht_in_lane(float (&x)[16]) {
#pragma unroll
    for (int h = 1; h < (B < 16 ? B : 16); h <<= 1) {
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            if ((i & h) == 0) {
                float a = x[i], b = x[i + h];
                x[i] = a + b;
                x[i + h] = a - b;
            }
        }
    }
}

#define QAMW_DPP_STAGE(CTRL)                                                                       \
    asm("s_nop 1\n\t"                                                                              \
        "v_fmac_f32_dpp %0, %0, %16 " CTRL " row_mask:0xf bank_mask:0xf\n\t"                       \
        "v_fmac_f32_dpp %1, %1, %16 " CTRL " row_mask:0xf bank_mask:0xf\n\t"                       \
        "v_fmac_f32_dpp %2, %2, %16 " CTRL " row_mask:0xf bank_mask:0xf\n\t"                       \
        "v_fmac_f32_dpp %3, %3, %16 " CTRL " row_mask:0xf bank_mask:0xf\n\t"                       \
        "v_fmac_f32_dpp %4, %4, %16 " CTRL " row_mask:0xf bank_mask:0xf\n\t"                       \
        "v_fmac_f32_dpp %5, %5, %16 " CTRL " row_mask:0xf bank_mask:0xf\n\t"                       \
        "v_fmac_f32_dpp %6, %6, %16 " CTRL " row_mask:0xf bank_mask:0xf\n\t"                       \
        "v_fmac_f32_dpp %7, %7, %16 " CTRL " row_mask:0xf bank_mask:0xf\n\t"                       \
        "v_fmac_f32_dpp %8, %8, %16 " CTRL " row_mask:0xf bank_mask:0xf\n\t"                       \
        "v_fmac_f32_dpp %9, %9, %16 " CTRL " row_mask:0xf bank_mask:0xf\n\t"                       \
        "v_fmac_f32_dpp %10, %10, %16 " CTRL " row_mask:0xf bank_mask:0xf\n\t"                     \
        "v_fmac_f32_dpp %11, %11, %16 " CTRL " row_mask:0xf bank_mask:0xf\n\t"                     \
        "v_fmac_f32_dpp %12, %12, %16 " CTRL " row_mask:0xf bank_mask:0xf\n\t"                     \
        "v_fmac_f32_dpp %13, %13, %16 " CTRL " row_mask:0xf bank_mask:0xf\n\t"                     \
        "v_fmac_f32_dpp %14, %14, %16 " CTRL " row_mask:0xf bank_mask:0xf\n\t"                     \
        "v_fmac_f32_dpp %15, %15, %16 " CTRL " row_mask:0xf bank_mask:0xf"                         \
        : "+v"(x[0]), "+v"(x[1]), "+v"(x[2]), "+v"(x[3]), "+v"(x[4]), "+v"(x[5]), "+v"(x[6]),      \
          "+v"(x[7]), "+v"(x[8]), "+v"(x[9]), "+v"(x[10]), "+v"(x[11]), "+v"(x[12]), "+v"(x[13]),  \
          "+v"(x[14]), "+v"(x[15])                                                                 \
        : "v"(sg))

// Cross-row stage through a register swap: the two lanes of a pair exchange one register each so
// that each ends up with both operands of one butterfly, computes sum and difference, and the
// results are swapped back.  No negation is left behind.
template <bool HALVES> __device__ __forceinline__ void fwht_swap_stage(float (&x)[16]) {
#pragma unroll
    for (int e = 0; e < 16; e += 2) {
        unsigned a = __float_as_uint(x[e]), b = __float_as_uint(x[e + 1]);
        auto r = HALVES ? __builtin_amdgcn_permlane32_swap(a, b, false, false)
                        : __builtin_amdgcn_permlane16_swap(a, b, false, false);
        float lo = __uint_as_float(r[0]), hi = __uint_as_float(r[1]);   // (low side value, high side value)
        float s = lo + hi, d = lo - hi;
        auto w = HALVES ? __builtin_amdgcn_permlane32_swap(__float_as_uint(s), __float_as_uint(d), false, false)
                        : __builtin_amdgcn_permlane16_swap(__float_as_uint(s), __float_as_uint(d), false, false);
        x[e] = __uint_as_float(w[0]);
        x[e + 1] = __uint_as_float(w[1]);
    }
}

// Per-lane constants of the DPP stages for block size B.
template <int B> struct LaneSigns {
    float s16, s32, s64, s128;     // -1 where the lane sits on the "minus" side of that stage
    float parity;                   // product of the above for the stages B uses
    __device__ __forceinline__ explicit LaneSigns(int lane) {
        int pos = slab_pos(lane);
        s16 = (pos & 1) ? -1.f : 1.f;
        s32 = (pos & 2) ? -1.f : 1.f;
        s64 = (pos & 4) ? -1.f : 1.f;
        s128 = (pos & 8) ? -1.f : 1.f;
        float p = 1.f;
        if (B >= 32) p *= s16;
        if (B >= 64) p *= s32;
        if (B >= 128) p *= s64;
        if (B >= 256) p *= s128;
        parity = p;
    }
};

// Unnormalised block-Hadamard transform of the wave's slab, block size B (2..1024), in place.
// On return lane L holds parity(L) * (true coefficient).  All 64 lanes must be active.
template <int B> __device__ __forceinline__ void fwht_wave(float (&x)[16], const LaneSigns<B> &ls) {
    fwht_in_lane<B>(x);
    if (B >= 32) {
        float sg = ls.s16;
        QAMW_DPP_STAGE("quad_perm:[1,0,3,2]");
    }
    if (B >= 64) {
        float sg = ls.s32;
        QAMW_DPP_STAGE("quad_perm:[2,3,0,1]");
    }
    if (B >= 128) {
        float sg = ls.s64;
        QAMW_DPP_STAGE("row_half_mirror");
    }
    if (B >= 256) {
        float sg = ls.s128;
        QAMW_DPP_STAGE("row_mirror");
    }
    if (B >= 512) fwht_swap_stage<false>(x);
    if (B >= 1024) fwht_swap_stage<true>(x);
}

}  // namespace qamw
