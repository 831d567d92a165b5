// Shared device helpers of libqamw's HIP kernels (gfx950, wave64).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace qamw {

constexpr int WAVE = 64;

// Element load widened to fp32.  bf16 storage is the upper half of an fp32: widening is exact.
template <int DTYPE> struct Elem;
template <> struct Elem<0> {
    using type = float;
    static __device__ __forceinline__ float load(const void *base, int64_t i) {
        return reinterpret_cast<const float *>(base)[i];
    }
};
template <> struct Elem<1> {
    using type = uint16_t;
    static __device__ __forceinline__ float load(const void *base, int64_t i) {
        return __uint_as_float((uint32_t) reinterpret_cast<const uint16_t *>(base)[i] << 16);
    }
};

// Reciprocal with one Newton step: the correctly rounded quotient in all but a few rare cases
// (then one ulp off), at a third of the cost of the IEEE division sequence.
__device__ __forceinline__ float fast_recip(float s) {
    float q = __builtin_amdgcn_rcpf(s);
    float e = __builtin_fmaf(-s, q, 1.0f);
    return __builtin_fmaf(q, e, q);
}

// fp32 -> bf16 bits, round to nearest even (NaN stays a quiet NaN).
__device__ __forceinline__ uint32_t bf16_rne_bits(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (u >> 16) | 0x40u;
    return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}

// One B-bit field of a little-endian bit stream held as dwords: field k sits at bit k*bits.
__device__ __forceinline__ uint32_t unpack_field(const uint32_t *row, int row_dwords, int k, int bits) {
    uint32_t bit = (uint32_t)k * (uint32_t)bits;
    uint32_t w = bit >> 5, sh = bit & 31u;
    uint64_t lo = row[w];
    uint64_t hi = (w + 1 < (uint32_t)row_dwords) ? row[w + 1] : 0u;
    return (uint32_t)(((hi << 32) | lo) >> sh) & ((1u << bits) - 1u);
}

// Sum over the 64 lanes of a wave in a fixed butterfly order (the same in every lane).
__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
    for (int m = 1; m < WAVE; m <<= 1) v += __shfl_xor(v, m, WAVE);
    return v;
}

}  // namespace qamw
