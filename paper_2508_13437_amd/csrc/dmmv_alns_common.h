// Device helpers of the ALNS outer loop shared by its translation units: counter-based random
// numbers, the fixed-sequence exponential, the fixed-point impact term, block reductions.
#pragma once

#include "dmmv_common.h"

namespace dmmv {

#ifdef __HIPCC__

// ----------------------------------------------------------------------------------------
// random numbers and the exponential
// ----------------------------------------------------------------------------------------
__device__ __forceinline__ uint64_t alns_mix(uint64_t z) {
    z ^= z >> 30; z *= 0xbf58476d1ce4e5b9ull;
    z ^= z >> 27; z *= 0x94d049bb133111ebull;
    z ^= z >> 31;
    return z;
}

// streams: 0 operator choice (counter 0 destroy, 1 repair), 1 destroy draws, 2 repair bits
__device__ __forceinline__ uint64_t alns_rnd(uint64_t seed, uint64_t inst, uint64_t it, uint64_t stream, uint64_t c) {
    constexpr uint64_t G = 0x9e3779b97f4a7c15ull;
    uint64_t z = alns_mix(seed + G * (inst + 1));
    z = alns_mix(z + G * (it + 1));
    z = alns_mix(z + G * (stream + 1));
    z = alns_mix(z + G * (c + 1));
    return z;
}

__device__ __forceinline__ double alns_unit(uint64_t x) { return (double)(x >> 11) * 0x1.0p-53; }

// e^{-y}, y >= 0: y = k ln2 + z, k = rint(y log2 e); Taylor polynomial of degree 13 of e^{-z} in
// Horner form with fused multiply-adds; scaled by 2^{-k}.  700 and above (and NaN) give 0.
__device__ __forceinline__ double alns_expneg(double y) {
    if (!(y < 700.0)) return 0.0;
    const double kf = __builtin_rint(y * 0x1.71547652b82fep+0);
    double z = __builtin_fma(-kf, 0x1.62e42fee00000p-1, y);
    z = __builtin_fma(-kf, 0x1.a39ef35793c76p-33, z);
    const double w = -z;
    double p = 1.0 / 6227020800.0;
    p = __builtin_fma(p, w, 1.0 / 479001600.0);
    p = __builtin_fma(p, w, 1.0 / 39916800.0);
    p = __builtin_fma(p, w, 1.0 / 3628800.0);
    p = __builtin_fma(p, w, 1.0 / 362880.0);
    p = __builtin_fma(p, w, 1.0 / 40320.0);
    p = __builtin_fma(p, w, 1.0 / 5040.0);
    p = __builtin_fma(p, w, 1.0 / 720.0);
    p = __builtin_fma(p, w, 1.0 / 120.0);
    p = __builtin_fma(p, w, 1.0 / 24.0);
    p = __builtin_fma(p, w, 1.0 / 6.0);
    p = __builtin_fma(p, w, 0.5);
    p = __builtin_fma(p, w, 1.0);
    p = __builtin_fma(p, w, 1.0);
    const int64_t k = (int64_t)kf;
    const double s = __longlong_as_double((long long)((uint64_t)(1023 - k) << 52));
    return p * s;
}

__device__ __forceinline__ int alns_bits(int64_t x) { int b = 0; while (x > 0) { ++b; x >>= 1; } return b; }

// fixed-point term of the impact score of one stored entry (0 for a zero coefficient)
__device__ __forceinline__ uint64_t alns_impact_term(double a_abs, double sk, double t, double alpha,
                                                     double scale) {
    if (a_abs == 0.0) return 0;
    const double slack = t - sk;
    // Shortcut with the same result: slack > a * 18 / alpha makes alpha * R exceed 17.9 whatever
    // the roundings, so exp(-alpha R) < 1.7e-8 and the term, below 2^24 * 1.7e-8 < 1, truncates
    // to 0.  Most rows are far from the maximum, so most terms end here.
    if (slack > a_abs * (18.0 / alpha)) return 0;
    const double R = slack / a_abs;
    const double E = alns_expneg(alpha * R);
    const double g = (sk * E) * scale;
    return (uint64_t)g;
}

// scale 2^24 / 2^e with 2^e > t; 0 when t is below 2^-900 (then every weight is 1)
__device__ __forceinline__ double alns_impact_scale(double t) {
    if (!(t >= 0x1p-900)) return 0.0;
    int e;
    (void)frexp(t, &e);
    return ldexp(1.0, 24 - e);
}

__device__ __forceinline__ uint64_t block_sum_u64(uint64_t v, uint64_t* sh /* blockDim/64 */) {
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) v += (uint64_t)__shfl_xor((long long)v, off, 64);
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6, nw = (blockDim.x + 63) >> 6;
    __syncthreads();
    if (lane == 0) sh[w] = v;
    __syncthreads();
    uint64_t tot = 0;
    for (int q = 0; q < nw; ++q) tot += sh[q];
    return tot;
}

template <class T>
__device__ __forceinline__ T block_max(T v, T* sh /* blockDim/64 */) {
    v = wave_max(v);
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6, nw = (blockDim.x + 63) >> 6;
    __syncthreads();
    if (lane == 0) sh[w] = v;
    __syncthreads();
    T out = sh[0];
    for (int q = 1; q < nw; ++q) out = dmmv_max(out, sh[q]);
    return out;
}

#endif  // __HIPCC__

}  // namespace dmmv
