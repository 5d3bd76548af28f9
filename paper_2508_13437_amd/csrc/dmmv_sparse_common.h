// Device helpers shared by the sparse-path translation units.
#pragma once

#include "dmmv_common.h"

namespace dmmv {

constexpr int SEG_ALIGN = 4;   // entries: segment alignment, and entries per lane per pass

// reservoir metadata slots (Ctx::res_meta)
enum { RES_CNT = 0, RES_FLOOR_ROW = 1, RES_META = 4 };

#ifdef __HIPCC__

// strict total order of rows by |r|: larger value first, lower row first among equal values
template <class T>
__device__ __forceinline__ bool key_before(T a1, int32_t r1, T a2, int32_t r2) {
    return (a1 > a2) || (a1 == a2 && r1 < r2);
}

template <int CTRL>
__device__ __forceinline__ uint32_t dpp_mov_u32(uint32_t v) {
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, 0xF, 0xF, true);
}

// maximum over each row of 16 lanes, result in every lane of the row
template <class T>
__device__ __forceinline__ T row16_max(T v) {
    v = dmmv_max(v, dpp_mov<DPP_QUAD_XOR1>(v));
    v = dmmv_max(v, dpp_mov<DPP_QUAD_XOR2>(v));
    v = dmmv_max(v, dpp_mov<DPP_ROW_HALF_MIRROR>(v));
    v = dmmv_max(v, dpp_mov<DPP_ROW_MIRROR>(v));
    return v;
}
// Same for values known to be >= 0: non-negative floats order like their bit patterns, and an
// unsigned integer max takes the DPP permutation as an operand (one instruction per step, no
// NaN canonicalisation).
__device__ __forceinline__ float row16_max_nonneg(float v) {
    uint32_t u = __float_as_uint(v);
    u = max(u, dpp_mov_u32<DPP_QUAD_XOR1>(u));
    u = max(u, dpp_mov_u32<DPP_QUAD_XOR2>(u));
    u = max(u, dpp_mov_u32<DPP_ROW_HALF_MIRROR>(u));
    u = max(u, dpp_mov_u32<DPP_ROW_MIRROR>(u));
    return __uint_as_float(u);
}
__device__ __forceinline__ double row16_max_nonneg(double v) { return row16_max(v); }

__device__ __forceinline__ uint32_t row16_or(uint32_t v) {
    v |= dpp_mov_u32<DPP_QUAD_XOR1>(v);
    v |= dpp_mov_u32<DPP_QUAD_XOR2>(v);
    v |= dpp_mov_u32<DPP_ROW_HALF_MIRROR>(v);
    v |= dpp_mov_u32<DPP_ROW_MIRROR>(v);
    return v;
}

// maximum / OR over each aligned run of LANES lanes (4, 8 or 16), result in every lane
template <int LANES>
__device__ __forceinline__ float lanes_max_nonneg(float v) {
    uint32_t u = __float_as_uint(v);
    u = max(u, dpp_mov_u32<DPP_QUAD_XOR1>(u));
    u = max(u, dpp_mov_u32<DPP_QUAD_XOR2>(u));
    if (LANES >= 8) u = max(u, dpp_mov_u32<DPP_ROW_HALF_MIRROR>(u));
    if (LANES >= 16) u = max(u, dpp_mov_u32<DPP_ROW_MIRROR>(u));
    return __uint_as_float(u);
}
template <int LANES>
__device__ __forceinline__ double lanes_max_nonneg(double v) {
    v = dmmv_max(v, dpp_mov<DPP_QUAD_XOR1>(v));
    v = dmmv_max(v, dpp_mov<DPP_QUAD_XOR2>(v));
    if (LANES >= 8) v = dmmv_max(v, dpp_mov<DPP_ROW_HALF_MIRROR>(v));
    if (LANES >= 16) v = dmmv_max(v, dpp_mov<DPP_ROW_MIRROR>(v));
    return v;
}
template <int LANES>
__device__ __forceinline__ uint32_t lanes_or(uint32_t v) {
    v |= dpp_mov_u32<DPP_QUAD_XOR1>(v);
    v |= dpp_mov_u32<DPP_QUAD_XOR2>(v);
    if (LANES >= 8) v |= dpp_mov_u32<DPP_ROW_HALF_MIRROR>(v);
    if (LANES >= 16) v |= dpp_mov_u32<DPP_ROW_MIRROR>(v);
    return v;
}

template <class T> struct Vec4;
template <> struct Vec4<float> { typedef float4 type; };
template <> struct Vec4<double> { typedef double4 type; };

// Is `row` stored in column j?  Binary search in the segment of the row's partition (rows are
// ascending inside a segment; pads carry offset mp and sort after every real row).
template <class T>
__device__ __forceinline__ bool column_has_row(const int32_t* __restrict__ segptr,
                                               const uint16_t* __restrict__ row16, int64_t n,
                                               int32_t mp, int64_t j, int32_t row) {
    const int64_t p = row / mp;
    const int32_t loc = row - (int32_t)(p * mp);
    int32_t lo = segptr[p * n + j], hi = segptr[p * n + j + 1];
    const int32_t end = hi;
    while (lo < hi) {
        const int32_t mid = (lo + hi) >> 1;
        if ((int32_t)row16[mid] < loc) lo = mid + 1; else hi = mid;
    }
    return lo < end && (int32_t)row16[lo] == loc;
}

#endif  // __HIPCC__

}  // namespace dmmv
