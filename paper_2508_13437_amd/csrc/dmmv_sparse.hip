// Sparse single-instance path: A given in CSR, scored through a row-partitioned,
// column-compressed copy built on the device at create.
//
// Layout.  Rows are cut into P partitions of at most MP rows, MP chosen so that one
// partition of the residual fits in LDS (128 KiB).  Inside a partition the entries are stored
// column by column, rows ascending, as a 16-bit row offset and a value: 6 bytes per entry
// (fp32).  Segment s = p*n + j holds the entries of column j that fall in partition p; every
// segment starts on a multiple of four entries and is padded to one (pad = row offset MP,
// value 0; LDS slot MP holds 0, so a pad contributes |fma(d, 0, 0)| = 0).
//
// Evaluation (one kernel).  A workgroup owns a range of columns holding an equal share of the
// entries.  For each partition in turn it stages that partition of r in LDS, then its
// wavefronts stream the column segments: a row of 16 lanes takes one column, each lane four
// consecutive entries per pass (one 8-byte and one 16-byte load), gathers r from LDS, keeps
// KT running maxima and reduces them over the 16 lanes with DPP.  Per-column maxima are
// carried across partitions in a small global scratch touched by one fixed lane per column.
//
// The score of a move is a maximum over ALL m rows: rows without an entry in the column keep
// |r_i|.  That outside maximum comes from a reservoir: the rows of largest |r| in a strict
// total order (|r| descending, row ascending), kept sorted on the device and updated
// incrementally by the kernel that applies a move.  While streaming, a lane that meets a row
// at or above the reservoir's 32nd value marks it in a per-column bit mask; the first
// unmarked reservoir entry is the outside maximum.  Columns that contain all of the first 32
// reservoir rows walk the rest of the reservoir, then fall back to an exact scan.
#include "dmmv_common.h"

namespace dmmv {

constexpr int EVAL_BLOCK = 512;    // 8 wavefronts: 256 VGPRs each, room for every load of a chunk
constexpr int EVAL_WAVES = EVAL_BLOCK / 64;
constexpr int SEG_ALIGN = 4;       // entries; also entries per lane per pass
constexpr int MAX_FLAGGED = 64;    // columns per workgroup that may need the slow outside path

// =========================================================================================
// ordering of rows by |r|
// =========================================================================================
template <class T>
__device__ __forceinline__ bool key_before(T a1, int32_t r1, T a2, int32_t r2) {
    return (a1 > a2) || (a1 == a2 && r1 < r2);
}

// =========================================================================================
// CSR -> partitioned, padded CSC (setup)
// =========================================================================================
__global__ void k_cscp_zero(int32_t* a, int64_t count) {
    int64_t q = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
    if (q < count) a[q] = 0;
}

// one thread per row: validate and count entries per segment (into segptr[seg + 1])
__global__ void k_cscp_count(int64_t m, int64_t n, int64_t nnz, int32_t mp,
                             const int64_t* __restrict__ rowptr, const int32_t* __restrict__ col,
                             int32_t* segptr, int32_t* flags) {
    int64_t i = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
    if (i >= m) return;
    const int64_t e0 = rowptr[i], e1 = rowptr[i + 1];
    if (e0 < 0 || e1 < e0 || e1 > nnz || (i == 0 && e0 != 0) || (i == m - 1 && e1 != nnz)) {
        atomicOr(&flags[FLAG_ERROR], ERRBIT_CSR_RANGE);
        return;
    }
    const int64_t p = i / mp;
    for (int64_t e = e0; e < e1; ++e) {
        const int32_t j = col[e];
        if (j < 0 || j >= n) { atomicOr(&flags[FLAG_ERROR], ERRBIT_CSR_RANGE); continue; }
        atomicAdd(&segptr[p * n + j + 1], 1);
    }
}

// single block: a[s+1] holds the length of segment s on entry; on exit a[s] is the padded
// start of segment s (a[count] = padded total) and fillpos[s] = a[s].
__global__ void k_cscp_scan(int64_t count, int32_t* a, int32_t* fillpos) {
    __shared__ int32_t sh[1024];
    __shared__ int32_t carry;
    if (threadIdx.x == 0) carry = 0;
    __syncthreads();
    for (int64_t base = 0; base < count; base += 1024) {
        const int64_t s = base + threadIdx.x;
        const int32_t len = s < count ? a[s + 1] : 0;
        const int32_t v = (len + SEG_ALIGN - 1) / SEG_ALIGN * SEG_ALIGN;
        sh[threadIdx.x] = v;
        __syncthreads();
        for (int off = 1; off < 1024; off <<= 1) {
            const int32_t t = threadIdx.x >= off ? sh[threadIdx.x - off] : 0;
            __syncthreads();
            sh[threadIdx.x] += t;
            __syncthreads();
        }
        const int32_t incl = sh[threadIdx.x] + carry;
        if (s < count) { a[s + 1] = incl; fillpos[s] = incl - v; }
        __syncthreads();
        if (threadIdx.x == 1023) carry = incl;
        __syncthreads();
    }
}

// one thread per row: scatter its entries into their segments (arbitrary order inside a
// segment; k_cscp_sort fixes it).  Afterwards fillpos[s] = start + length of segment s.
template <class T>
__global__ void k_cscp_fill(int64_t m, int64_t n, int32_t mp, const int64_t* __restrict__ rowptr,
                            const int32_t* __restrict__ col, const T* __restrict__ val,
                            int32_t* fillpos, uint16_t* __restrict__ row_tmp,
                            T* __restrict__ val_tmp, const int32_t* flags) {
    int64_t i = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
    if (i >= m || flags[FLAG_ERROR]) return;
    const int64_t p = i / mp;
    const uint16_t loc = (uint16_t)(i - p * mp);
    for (int64_t e = rowptr[i]; e < rowptr[i + 1]; ++e) {
        const int32_t j = col[e];
        if (j < 0 || j >= n) continue;
        const int32_t pos = atomicAdd(&fillpos[p * n + j], 1);
        row_tmp[pos] = loc;
        val_tmp[pos] = val[e];
    }
}

// one wavefront per segment: place every entry at its rank by row (rows ascending), write the
// pads.  Equal rows inside a segment mean the matrix stores an entry twice.
template <class T>
__global__ void k_cscp_sort(int64_t nseg, int32_t mp, const int32_t* __restrict__ segptr,
                            const int32_t* __restrict__ fillpos,
                            const uint16_t* __restrict__ row_tmp, const T* __restrict__ val_tmp,
                            uint16_t* __restrict__ row16, T* __restrict__ cval, int32_t* flags) {
    if (flags[FLAG_ERROR] & ERRBIT_CSR_RANGE) return;
    const int lane = threadIdx.x & 63;
    const int64_t s = blockIdx.x * (int64_t)(blockDim.x >> 6) + (threadIdx.x >> 6);
    if (s >= nseg) return;
    const int32_t e0 = segptr[s], e1 = fillpos[s], epad = segptr[s + 1];
    for (int32_t e = e0 + lane; e < e1; e += 64) {
        const uint16_t row = row_tmp[e];
        int32_t rank = 0;
        bool dup = false;
        for (int32_t f = e0; f < e1; ++f) {
            const uint16_t other = row_tmp[f];
            rank += other < row;
            dup |= (other == row && f != e);
        }
        if (dup) { atomicOr(&flags[FLAG_ERROR], ERRBIT_CSR_DUP); continue; }
        row16[e0 + rank] = row;
        cval[e0 + rank] = val_tmp[e];
    }
    for (int32_t e = e1 + lane; e < epad; e += 64) { row16[e] = (uint16_t)mp; cval[e] = (T)0; }
}

// column range of every evaluation workgroup: equal shares of the padded entries
__global__ void k_cscp_ranges(int64_t n, int32_t P, int32_t gb, const int32_t* __restrict__ segptr,
                              int32_t* __restrict__ blk_lo) {
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b > gb) return;
    if (b == 0) { blk_lo[0] = 0; return; }
    if (b == gb) { blk_lo[gb] = (int32_t)n; return; }
    int64_t total = 0;
    for (int32_t p = 0; p < P; ++p) total += segptr[(int64_t)p * n + n] - segptr[(int64_t)p * n];
    const int64_t want = total * b / gb;
    int64_t lo = 0, hi = n;      // first column j with entries-before(j) >= want
    while (lo < hi) {
        const int64_t mid = (lo + hi) >> 1;
        int64_t before = 0;
        for (int32_t p = 0; p < P; ++p) before += segptr[(int64_t)p * n + mid] - segptr[(int64_t)p * n];
        if (before < want) lo = mid + 1; else hi = mid;
    }
    blk_lo[b] = (int32_t)lo;
}

// =========================================================================================
// residual: one thread per row, entries in stored order
// =========================================================================================
template <class T>
__global__ void k_residual_csr(int64_t m, const int64_t* __restrict__ rowptr,
                               const int32_t* __restrict__ col, const T* __restrict__ val,
                               const T* __restrict__ D, const int32_t* __restrict__ kidx,
                               const T* __restrict__ b, T* __restrict__ r) {
    int64_t i = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
    if (i >= m) return;
    T acc = (T)0;
    for (int64_t e = rowptr[i]; e < rowptr[i + 1]; ++e) acc = dmmv_fma(val[e], D[kidx[col[e]]], acc);
    r[i] = dmmv_fma(acc, (T)1, -b[i]);
}

// =========================================================================================
// reservoir of the rows of largest |r|
//   res_val/res_row [RES_CAP] sorted by key_before; meta[RES_CNT] entries; the reservoir holds
//   EVERY row whose key is before-or-equal the floor key (floor_val[0], meta[RES_FLOOR_ROW]).
// =========================================================================================
enum { RES_CNT = 0, RES_FLOOR_ROW = 1, RES_META = 4 };
constexpr int RES_SEL = 256;     // threads whose strided maxima choose the floor at a rebuild
constexpr int RES_COLLECT = 1024;

// r may have been written earlier in the same kernel by other wavefronts: read past the L1
template <class T>
__device__ __forceinline__ T ld_coherent(const T* p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// LDS work area shared by rebuild and update (both run in one workgroup of >= 256 threads)
template <class T>
struct ResLds {
    T v[RES_COLLECT];
    int32_t r[RES_COLLECT];
    T ov[RES_CAP];
    int32_t orow[RES_CAP];
    T fv;
    int32_t fr;
    int32_t count;
};

// rank-sort the first c entries of L.v/L.r, keep the first RES_CAP, publish them
template <class T>
__device__ void reservoir_publish(ResLds<T>& L, int32_t c, bool set_floor_from_last, T* res_val,
                                  int32_t* res_row, int32_t* meta, T* floor_val) {
    for (int32_t u = threadIdx.x; u < c; u += blockDim.x) {
        const T a = L.v[u];
        const int32_t row = L.r[u];
        int32_t rank = 0;
        for (int32_t q = 0; q < c; ++q) rank += key_before(L.v[q], L.r[q], a, row);
        if (rank < RES_CAP) { L.ov[rank] = a; L.orow[rank] = row; }
    }
    __syncthreads();
    const int32_t keep = c < RES_CAP ? c : RES_CAP;
    for (int32_t u = threadIdx.x; u < keep; u += blockDim.x) { res_val[u] = L.ov[u]; res_row[u] = L.orow[u]; }
    if (threadIdx.x == 0) {
        meta[RES_CNT] = keep;
        if (set_floor_from_last || c > RES_CAP) {
            if (keep > 0) { floor_val[0] = L.ov[keep - 1]; meta[RES_FLOOR_ROW] = L.orow[keep - 1]; }
        }
    }
    __syncthreads();
}

// Full rebuild from r.  Call with every thread of the workgroup.
template <class T>
__device__ void reservoir_rebuild(ResLds<T>& L, int64_t m, const T* r, T* res_val,
                                  int32_t* res_row, int32_t* meta, T* floor_val) {
    if (m <= RES_CAP) {
        // everything fits: the floor admits every row
        for (int32_t u = threadIdx.x; u < (int32_t)m; u += blockDim.x) { L.v[u] = dmmv_abs(ld_coherent(r + u)); L.r[u] = u; }
        __syncthreads();
        reservoir_publish(L, (int32_t)m, false, res_val, res_row, meta, floor_val);
        if (threadIdx.x == 0) { floor_val[0] = (T)-1; meta[RES_FLOOR_ROW] = INT32_MAX; }
        __syncthreads();
        return;
    }
    // strided maxima of the first RES_SEL threads propose a floor with about `target` rows above it
    T mv = (T)-1;
    int32_t mr = INT32_MAX;
    if (threadIdx.x < RES_SEL)
        for (int64_t i = threadIdx.x; i < m; i += RES_SEL) {
            const T a = dmmv_abs(ld_coherent(r + i));
            if (key_before(a, (int32_t)i, mv, mr)) { mv = a; mr = (int32_t)i; }
        }
    int32_t target = RES_CAP / 2;
    for (;;) {
        __syncthreads();
        if (threadIdx.x < RES_SEL) { L.v[threadIdx.x] = mv; L.r[threadIdx.x] = mr; }
        if (threadIdx.x == 0) L.count = 0;
        __syncthreads();
        if (threadIdx.x < RES_SEL) {
            int32_t rank = 0;
            for (int32_t q = 0; q < RES_SEL; ++q) rank += key_before(L.v[q], L.r[q], mv, mr);
            if (rank == target - 1) { L.fv = mv; L.fr = mr; }
        }
        __syncthreads();
        const T fv = L.fv;
        const int32_t fr = L.fr;
        __syncthreads();
        for (int64_t i = threadIdx.x; i < m; i += blockDim.x) {
            const T a = dmmv_abs(ld_coherent(r + i));
            if (!key_before(fv, fr, a, (int32_t)i)) {          // key(i) before-or-equal floor
                const int32_t pos = atomicAdd(&L.count, 1);
                if (pos < RES_COLLECT) { L.v[pos] = a; L.r[pos] = (int32_t)i; }
            }
        }
        __syncthreads();
        if (L.count <= RES_COLLECT || target == 1) break;
        target = target > 1 ? target / 2 : 1;
    }
    const int32_t c = L.count < RES_COLLECT ? L.count : RES_COLLECT;
    __syncthreads();
    reservoir_publish(L, c, true, res_val, res_row, meta, floor_val);
}

template <class T>
__global__ __launch_bounds__(1024) void k_reservoir_build(int64_t m, const T* r,
                                                          T* res_val, int32_t* res_row,
                                                          int32_t* meta, T* floor_val) {
    __shared__ ResLds<T> L;
    reservoir_rebuild(L, m, r, res_val, res_row, meta, floor_val);
}

// =========================================================================================
// evaluation
// =========================================================================================
template <int CTRL>
__device__ __forceinline__ uint32_t dpp_mov_u32(uint32_t v) {
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, 0xF, 0xF, true);
}
// maximum / bit-or over each row of 16 lanes, result in every lane of the row
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

template <class T> struct Vec4;
template <> struct Vec4<float> { typedef float4 type; };
template <> struct Vec4<double> { typedef double4 type; };

template <class T>
__device__ __forceinline__ bool column_has_row(const int32_t* __restrict__ segptr,
                                               const uint16_t* __restrict__ row16, int64_t n,
                                               int32_t mp, int64_t j, int32_t row) {
    const int64_t p = row / mp;
    const int32_t loc = row - (int32_t)(p * mp);
    int32_t lo = segptr[p * n + j], hi = segptr[p * n + j + 1];
    const int32_t end = hi;
    while (lo < hi) {                       // pads (offset mp) sort after every real row
        const int32_t mid = (lo + hi) >> 1;
        if ((int32_t)row16[mid] < loc) lo = mid + 1; else hi = mid;
    }
    return lo < end && (int32_t)row16[lo] == loc;
}

// -----------------------------------------------------------------------------------------
// Evaluation kernel.  The workgroup's columns are taken in chunks of up to CH; for a chunk
// the segment bounds of every partition, the current values and the running per-column
// maxima / masks live in LDS.  Per partition: stage r, then every wavefront consumes the
// entries of its column groups (their loads were issued before the staging barrier, so the
// two latencies overlap) and folds the row-of-16 maxima into the column's LDS slot, which no
// other lane touches.  After the last partition one thread per column finishes the scores.
// -----------------------------------------------------------------------------------------
template <class T, int KT>
struct EvalCfg {
    static constexpr int CH = 160;                           // columns per chunk
    static constexpr int NQW = CH / 4 / EVAL_WAVES;          // column groups per wavefront
    static constexpr int BOUNDS = 2048;                      // ints of LDS for segment bounds
};

// one pass (64 entries) of one column group, as loaded
template <class T>
struct EntryRegs {
    uint2 ix;
    typename Vec4<T>::type av;
    bool ok;
};

// Loads are unconditional (address clamped into the arrays) and the out-of-segment lanes are
// turned into pads afterwards: straight-line code lets the compiler count outstanding loads.
template <class T>
__device__ __forceinline__ void load_entries(EntryRegs<T>& E, const uint16_t* __restrict__ row16,
                                             const T* __restrict__ cval, int32_t e, int32_t s1,
                                             int32_t emax, uint32_t pad) {
    const int32_t ec = e < emax ? e : emax;
    E.ix = *reinterpret_cast<const uint2*>(row16 + ec);
    E.av = *reinterpret_cast<const typename Vec4<T>::type*>(cval + ec);
    E.ok = e < s1;
}

template <class T>
__device__ __forceinline__ void mask_entries(EntryRegs<T>& E, uint32_t pad) {
    const uint32_t pp = pad | (pad << 16);
    E.ix.x = E.ok ? E.ix.x : pp;
    E.ix.y = E.ok ? E.ix.y : pp;
    E.av.x = E.ok ? E.av.x : (T)0;
    E.av.y = E.ok ? E.av.y : (T)0;
    E.av.z = E.ok ? E.av.z : (T)0;
    E.av.w = E.ok ? E.av.w : (T)0;
}

// One pass (up to 64 entries per column) of one group of four columns: gather r from LDS,
// update the running maxima of the KT values, reduce over the row of 16 lanes and fold the
// result into the column's LDS slot (lane sub == 0 is the only writer of column t).
template <class T, int KT>
__device__ __forceinline__ void consume_pass(const EntryRegs<T>& E, const T* lds_r, const T (&delta)[KT],
                                             bool first_tile, T thr, int32_t nfast,
                                             const int32_t* sh_rr, int64_t row0, uint32_t pad,
                                             int sub, bool col_ok, int32_t t, T* sh_cmax,
                                             uint32_t* sh_mask) {
    const uint32_t i0 = E.ix.x & 0xFFFFu, i1 = E.ix.x >> 16, i2 = E.ix.y & 0xFFFFu, i3 = E.ix.y >> 16;
    const T r0 = lds_r[i0], r1 = lds_r[i1], r2 = lds_r[i2], r3 = lds_r[i3];
    uint32_t mask = 0;
    if (first_tile) {
        const T big = dmmv_max(dmmv_max(dmmv_abs(r0), dmmv_abs(r1)), dmmv_max(dmmv_abs(r2), dmmv_abs(r3)));
        if (big >= thr) {      // uncommon: one of these rows may be among the listed ones
            for (int32_t q = 0; q < nfast; ++q) {
                const int64_t loc = (int64_t)sh_rr[q] - row0;      // offset in this partition, if any
                if (loc < 0 || loc >= (int64_t)pad) continue;      // uniform
                const uint32_t l = (uint32_t)loc;
                if (i0 == l || i1 == l || i2 == l || i3 == l) mask |= 1u << q;
            }
        }
    }
    T acc[KT];
#pragma unroll
    for (int q = 0; q < KT; ++q) {
        T a = dmmv_abs(dmmv_fma(delta[q], E.av.x, r0));
        a = dmmv_max(a, dmmv_abs(dmmv_fma(delta[q], E.av.y, r1)));
        a = dmmv_max(a, dmmv_abs(dmmv_fma(delta[q], E.av.z, r2)));
        a = dmmv_max(a, dmmv_abs(dmmv_fma(delta[q], E.av.w, r3)));
        acc[q] = row16_max_nonneg(a);
    }
    if (first_tile) mask = row16_or(mask);
    if (sub == 0 && col_ok) {
#pragma unroll
        for (int q = 0; q < KT; ++q) sh_cmax[t * KT + q] = dmmv_max(sh_cmax[t * KT + q], acc[q]);
        if (first_tile && mask) sh_mask[t] |= mask;
    }
}

template <class T, int KT>
__global__ __launch_bounds__(EVAL_BLOCK, 4) void k_eval_cscp(   // 4 waves per SIMD: two workgroups per CU
    int64_t m, int64_t n, int32_t nd, int32_t mp, int32_t P, const int32_t* __restrict__ segptr,
    const uint16_t* __restrict__ row16, const T* __restrict__ cval,
    const int32_t* __restrict__ blk_lo, const T* __restrict__ D, const int32_t* __restrict__ kidx,
    const T* __restrict__ r, const T* __restrict__ res_val, const int32_t* __restrict__ res_row,
    const int32_t* __restrict__ res_meta, int32_t radius, const uint8_t* __restrict__ var_mask,
    const InstState<T>* __restrict__ st, int32_t honor_done, T* __restrict__ colmax,
    uint32_t* __restrict__ colmask, T* __restrict__ scores, Partial<T>* __restrict__ part) {
    constexpr int CH = EvalCfg<T, KT>::CH;
    constexpr int NQW = EvalCfg<T, KT>::NQW;
    constexpr int BOUNDS = EvalCfg<T, KT>::BOUNDS;
    extern __shared__ __align__(32) unsigned char smem[];
    T* lds_r = reinterpret_cast<T*>(smem);                 // mp + 1 entries (slot mp = 0)
    __shared__ T sh_rv[RES_CAP];
    __shared__ int32_t sh_rr[RES_CAP];
    __shared__ T sh_s[EVAL_WAVES];
    __shared__ int64_t sh_c[EVAL_WAVES];
    __shared__ int32_t sh_flag_n;
    __shared__ int32_t sh_flag_j[MAX_FLAGGED];
    __shared__ int32_t sh_long;
    __shared__ int32_t sh_b[BOUNDS];
    __shared__ T sh_dcur[CH];
    __shared__ uint32_t sh_mask[CH];
    __shared__ T sh_cmax[CH * KT];
    if (honor_done && st[0].done) return;

    const int lane = threadIdx.x & 63;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int sub = lane & 15;                 // position inside the row of 16 lanes
    const int rowid = lane >> 4;               // which of the wavefront's 4 columns
    const int64_t j_lo = blk_lo[blockIdx.x], j_hi = blk_lo[blockIdx.x + 1];
    const int32_t cnt = res_meta[RES_CNT];
    if (threadIdx.x < RES_CAP) {
        sh_rv[threadIdx.x] = threadIdx.x < cnt ? res_val[threadIdx.x] : (T)-1;
        sh_rr[threadIdx.x] = threadIdx.x < cnt ? res_row[threadIdx.x] : -1;
    }
    if (threadIdx.x == 0) sh_flag_n = 0;
    const int32_t nfast = cnt < RES_FAST ? cnt : RES_FAST;
    const uint32_t full = nfast >= 32 ? 0xFFFFFFFFu : ((1u << nfast) - 1u);
    const uint32_t pad = (uint32_t)mp;
    const int32_t emax = segptr[(int64_t)P * n];     // four spare entries follow the arrays
    int32_t ncm = BOUNDS / P - 1;              // columns per chunk that the bounds area allows
    if (ncm > CH) ncm = CH;
    const int32_t bstride = ncm + 1;
    T bs = (T)0;                               // best (score, candidate) seen by this thread
    int64_t bc = -1;

    for (int64_t c0 = j_lo; c0 < j_hi; c0 += ncm) {
        const int32_t nc = (int32_t)(j_hi - c0 < ncm ? j_hi - c0 : ncm);
        const int32_t nq = (nc + 3) >> 2;
        __syncthreads();                       // previous chunk's epilogue done
        if (threadIdx.x == 0) sh_long = 0;
        __syncthreads();
        for (int32_t idx = threadIdx.x; idx < P * (nc + 1); idx += EVAL_BLOCK) {
            const int32_t p = idx / (nc + 1), t = idx - p * (nc + 1);
            const int32_t b0 = segptr[(int64_t)p * n + c0 + t];
            sh_b[p * bstride + t] = b0;
            // a segment of more than one pass (64 entries) anywhere in the chunk?
            if (t < nc && segptr[(int64_t)p * n + c0 + t + 1] - b0 > 64) sh_long = 1;
        }
        for (int32_t t = threadIdx.x; t < nc; t += EVAL_BLOCK) sh_dcur[t] = D[kidx[c0 + t]];
        for (int32_t k0 = 0; k0 < nd; k0 += KT) {
            __syncthreads();                   // bounds visible; previous tile's epilogue done
            for (int32_t t = threadIdx.x; t < nc; t += EVAL_BLOCK) {
                if (k0 == 0) sh_mask[t] = 0u;
#pragma unroll
                for (int q = 0; q < KT; ++q) sh_cmax[t * KT + q] = (T)0;
            }
            T dk[KT];
#pragma unroll
            for (int q = 0; q < KT; ++q) dk[q] = D[k0 + q < nd ? k0 + q : nd - 1];
            const T thr = nfast > 0 ? sh_rv[nfast - 1] : Limits<T>::inf();
            const bool any_long = sh_long != 0;
            // first partition's entries: issued now, consumed after r is staged
            EntryRegs<T> ent[NQW];
            int32_t qe[NQW], qs1[NQW];
#pragma unroll
            for (int u = 0; u < NQW; ++u) {
                const int32_t t = (w + u * EVAL_WAVES) * 4 + rowid;
                const bool okc = t < nc;
                qe[u] = (okc ? sh_b[t] : 0) + sub * SEG_ALIGN;
                qs1[u] = okc ? sh_b[t + 1] : 0;
                load_entries<T>(ent[u], row16, cval, qe[u], qs1[u], emax, pad);
            }
            for (int32_t p = 0; p < P; ++p) {
                __syncthreads();               // everyone is done with the previous partition of r
                const int64_t row0 = (int64_t)p * mp;
                const int32_t rows_here = (int32_t)((m - row0) < mp ? (m - row0) : mp);
                if ((row0 & 3) == 0) {
                    const int32_t nvec = rows_here >> 2;
                    const typename Vec4<T>::type* __restrict__ src = reinterpret_cast<const typename Vec4<T>::type*>(r + row0);
                    typename Vec4<T>::type* dst = reinterpret_cast<typename Vec4<T>::type*>(lds_r);
                    for (int32_t i = threadIdx.x; i < nvec; i += EVAL_BLOCK) dst[i] = src[i];
                    for (int32_t i = (nvec << 2) + threadIdx.x; i < rows_here; i += EVAL_BLOCK) lds_r[i] = r[row0 + i];
                } else {
                    for (int32_t i = threadIdx.x; i < rows_here; i += EVAL_BLOCK) lds_r[i] = r[row0 + i];
                }
                if (threadIdx.x == 0) lds_r[mp] = (T)0;
                __syncthreads();
                // first pass of every group (straight-line)
#pragma unroll
                for (int u = 0; u < NQW; ++u) {
                    if (w + u * EVAL_WAVES >= nq) continue;    // uniform: no such group in this chunk
                    const int32_t t = (w + u * EVAL_WAVES) * 4 + rowid;
                    const bool col_ok = t < nc;
                    const T dcur = sh_dcur[col_ok ? t : 0];
                    T delta[KT];
#pragma unroll
                    for (int q = 0; q < KT; ++q) delta[q] = step_of(dk[q], dcur, (T)1);
                    mask_entries<T>(ent[u], pad);
                    consume_pass<T, KT>(ent[u], lds_r, delta, k0 == 0, thr, nfast, sh_rr, row0, pad, sub,
                                        col_ok, col_ok ? t : 0, sh_cmax, sh_mask);
                }
                // segments longer than one pass (64 entries): the rest, loaded in place
#pragma unroll 1
                for (int u = 0; u < (any_long ? NQW : 0); ++u) {
                    int32_t left = qs1[u] - (qe[u] - sub * SEG_ALIGN);
                    left = max(left, __shfl_xor(left, 16, 64));
                    left = max(left, __shfl_xor(left, 32, 64));
                    const int32_t passes = __builtin_amdgcn_readfirstlane((left + 63) >> 6);
                    if (passes <= 1) continue;                 // uniform
                    const int32_t t = (w + u * EVAL_WAVES) * 4 + rowid;
                    const bool col_ok = t < nc;
                    const T dcur = sh_dcur[col_ok ? t : 0];
                    T delta[KT];
#pragma unroll
                    for (int q = 0; q < KT; ++q) delta[q] = step_of(dk[q], dcur, (T)1);
                    for (int32_t ps = 1; ps < passes; ++ps) {
                        EntryRegs<T> more;
                        load_entries<T>(more, row16, cval, qe[u] + ps * 64, qs1[u], emax, pad);
                        mask_entries<T>(more, pad);
                        consume_pass<T, KT>(more, lds_r, delta, k0 == 0, thr, nfast, sh_rr, row0, pad, sub,
                                            col_ok, col_ok ? t : 0, sh_cmax, sh_mask);
                    }
                }
                // next partition's entries, in flight during the next staging
                if (p + 1 < P) {
#pragma unroll
                    for (int u = 0; u < NQW; ++u) {
                        const int32_t t = (w + u * EVAL_WAVES) * 4 + rowid;
                        const bool okc = t < nc;
                        qe[u] = (okc ? sh_b[(p + 1) * bstride + t] : 0) + sub * SEG_ALIGN;
                        qs1[u] = okc ? sh_b[(p + 1) * bstride + t + 1] : 0;
                        load_entries<T>(ent[u], row16, cval, qe[u], qs1[u], emax, pad);
                    }
                }
            }
            __syncthreads();
            // ---- one thread per column: finish the scores of this tile ----
            for (int32_t t = threadIdx.x; t < nc; t += EVAL_BLOCK) {
                const int64_t j = c0 + t;
                const uint32_t cm = sh_mask[t];
                T outside = (T)0;
                bool defer = false;
                const uint32_t missing = full & ~cm;
                if (missing) outside = sh_rv[__builtin_ctz(missing)];
                else if ((int64_t)nfast >= m) outside = (T)0;      // the column holds every row
                else defer = true;
                const int32_t kcur = kidx[j];
                const bool var_ok = var_mask ? var_mask[j] != 0 : true;
#pragma unroll
                for (int q = 0; q < KT; ++q) {
                    const int32_t k = k0 + q;
                    if (k >= nd) break;
                    const int64_t cidx = j * (int64_t)nd + k;
                    T v = sh_cmax[t * KT + q];
                    if (defer) { colmax[cidx] = v; continue; }
                    v = dmmv_max(v, outside);
                    if (!cand_allowed(kcur, k, radius, var_ok)) v = Limits<T>::inf();
                    if (scores) scores[cidx] = v;
                    if (rec_less(v, cidx, bs, bc)) { bs = v; bc = cidx; }
                }
                if (k0 == 0) {
                    colmask[j] = defer ? 1u : 0u;
                    if (defer) {
                        const int32_t slot = atomicAdd(&sh_flag_n, 1);
                        if (slot < MAX_FLAGGED) sh_flag_j[slot] = (int32_t)j;
                    }
                }
            }
        }
    }
    __syncthreads();
    // ---- rare: columns that contain every one of the first RES_FAST reservoir rows ----
    const int32_t nflag = sh_flag_n;
    if (nflag > 0) {
        // more than MAX_FLAGGED: rescan this workgroup's columns for the deferred ones
        // (colmask[j] = 1 marks a deferred column; its maxima are in colmax)
        const int64_t scan_lo = nflag > MAX_FLAGGED ? j_lo : 0;
        const int64_t scan_hi = nflag > MAX_FLAGGED ? j_hi : nflag;
        for (int64_t it = scan_lo; it < scan_hi; ++it) {
            int64_t j;
            if (nflag > MAX_FLAGGED) {
                j = it;
                if (colmask[j] == 0u) continue;                // uniform
            } else {
                j = sh_flag_j[it];
            }
            __syncthreads();
            // 1) the rest of the reservoir, in order: first entry whose row is not in the column
            if (threadIdx.x == 0) sh_flag_n = INT32_MAX;
            __syncthreads();
            for (int32_t q = RES_FAST + threadIdx.x; q < cnt; q += EVAL_BLOCK)
                if (!column_has_row<T>(segptr, row16, n, mp, j, sh_rr[q])) atomicMin(&sh_flag_n, q);
            __syncthreads();
            T outside;
            if (sh_flag_n != INT32_MAX) {
                outside = sh_rv[sh_flag_n];
            } else if ((int64_t)cnt >= m) {
                outside = (T)0;
            } else {
                // 2) exact scan over all rows
                T o = (T)0;
                for (int64_t i = threadIdx.x; i < m; i += EVAL_BLOCK)
                    if (!column_has_row<T>(segptr, row16, n, mp, j, (int32_t)i)) o = dmmv_max(o, dmmv_abs(r[i]));
                o = wave_max(o);
                __syncthreads();
                if (lane == 0) sh_s[w] = o;
                __syncthreads();
                o = sh_s[0];
                for (int q = 1; q < EVAL_WAVES; ++q) o = dmmv_max(o, sh_s[q]);
                outside = o;
            }
            __syncthreads();
            if (threadIdx.x == 0) {
                const int32_t kcur = kidx[j];
                const bool var_ok = var_mask ? var_mask[j] != 0 : true;
                for (int32_t k = 0; k < nd; ++k) {
                    const int64_t cidx = j * (int64_t)nd + k;
                    T v = dmmv_max(colmax[cidx], outside);
                    if (!cand_allowed(kcur, k, radius, var_ok)) v = Limits<T>::inf();
                    if (scores) scores[cidx] = v;
                    if (rec_less(v, cidx, bs, bc)) { bs = v; bc = cidx; }
                }
            }
        }
        __syncthreads();
    }
    if (part) {
        block_argmin(bs, bc, sh_s, sh_c);
        if (threadIdx.x == 0) { Partial<T> pr; pr.s = bs; pr.c = bc; part[blockIdx.x] = pr; }
    }
}

// =========================================================================================
// apply
// =========================================================================================
// Plain apply of a staged move (dmmv_apply_move): the reservoir is rebuilt afterwards.
template <class T>
__global__ void k_apply_cscp(int64_t n, int32_t mp, int32_t P, const int32_t* __restrict__ segptr,
                             const uint16_t* __restrict__ row16, const T* __restrict__ cval,
                             T* __restrict__ r, int32_t* __restrict__ kidx, InstState<T>* st) {
    const int32_t j = st[0].apply_j;
    if (j < 0) return;
    const T delta = st[0].delta;
    const int32_t k = st[0].apply_k;
    const int32_t moves = st[0].moves;
    __syncthreads();
    for (int32_t p = 0; p < P; ++p) {
        const int32_t e0 = segptr[(int64_t)p * n + j], e1 = segptr[(int64_t)p * n + j + 1];
        for (int32_t e = e0 + threadIdx.x; e < e1; e += blockDim.x) {
            const uint32_t loc = row16[e];
            if (loc == (uint32_t)mp) continue;
            const int64_t i = (int64_t)p * mp + loc;
            r[i] = dmmv_fma(delta, cval[e], r[i]);
        }
    }
    if (threadIdx.x == 0) { kidx[j] = k; st[0].moves = moves + 1; }
}

// The loop's fused step: reduce the evaluation's arg-min records, decide, apply the move to r
// and x, and update the reservoir for the rows that changed.  One workgroup.
constexpr int SA_BLOCK = 1024;
constexpr int SA_MAXCOL = RES_COLLECT - RES_CAP;   // changed rows handled incrementally

template <class T>
__global__ __launch_bounds__(SA_BLOCK) void k_select_apply_cscp(
    int64_t m, int64_t n, int32_t nd, int32_t mp, int32_t P, const int32_t* __restrict__ segptr,
    const uint16_t* __restrict__ row16, const T* __restrict__ cval, const T* __restrict__ D,
    T* __restrict__ r, int32_t* __restrict__ kidx, const Partial<T>* __restrict__ part,
    int64_t n_part, InstState<T>* st, int32_t keep_going, T* res_val, int32_t* res_row,
    int32_t* res_meta, T* floor_val, int32_t iters, dmmv_move* trace, T* trace_t) {
    __shared__ ResLds<T> L;
    __shared__ T sh_s[SA_BLOCK / 64];
    __shared__ int64_t sh_c[SA_BLOCK / 64];
    __shared__ int32_t sh_srow[SA_MAXCOL];      // rows changed by the move, ascending
    __shared__ T sh_sval[SA_MAXCOL];            // their new |r|
    __shared__ int32_t sh_ns, sh_j, sh_k;
    __shared__ T sh_delta, sh_best;
    if (st[0].done) return;
    T s = (T)0;
    int64_t c = -1;
    for (int64_t q = threadIdx.x; q < n_part; q += SA_BLOCK) {
        const Partial<T> pr = part[q];
        if (rec_less(pr.s, pr.c, s, c)) { s = pr.s; c = pr.c; }
    }
    block_argmin(s, c, sh_s, sh_c);
    if (threadIdx.x == 0) {
        InstState<T> z = st[0];
        int32_t j = -1, k = -1;
        if (c >= 0) { j = (int32_t)(c / nd); k = (int32_t)(c % nd); }
        const bool improving = c >= 0 && s < z.t;
        z.best_s = s;
        z.apply_j = -1; z.apply_k = -1; z.delta = (T)0;      // applied right here
        sh_j = improving ? j : -1;
        sh_k = k;
        sh_best = s;
        if (improving) {
            sh_delta = step_of(D[k], D[kidx[j]], (T)1);
            if (z.moves < iters) {
                if (trace) { trace[z.moves].j = j; trace[z.moves].k = k; }
                if (trace_t) trace_t[z.moves] = s;
            }
            z.t = s;
            z.moves += 1;
            kidx[j] = k;
        } else if (!keep_going) {
            z.done = 1;
        }
        st[0] = z;
        sh_ns = 0;
    }
    __syncthreads();
    const int32_t j = sh_j;
    if (j < 0) return;
    const T delta = sh_delta;
    // ---- rank-1 update of the rows of column j; remember them (ascending by row) ----
    int32_t col_len = 0;
    for (int32_t p = 0; p < P; ++p) col_len += segptr[(int64_t)p * n + j + 1] - segptr[(int64_t)p * n + j];
    const bool incremental = col_len <= SA_MAXCOL && m > RES_CAP;
    int32_t base = 0;
    for (int32_t p = 0; p < P; ++p) {
        const int32_t e0 = segptr[(int64_t)p * n + j], e1 = segptr[(int64_t)p * n + j + 1];
        for (int32_t e = e0 + threadIdx.x; e < e1; e += SA_BLOCK) {
            const uint32_t loc = row16[e];
            const bool pad = loc == (uint32_t)mp;
            const int64_t i = (int64_t)p * mp + loc;
            T nv = (T)0;
            if (!pad) { nv = dmmv_fma(delta, cval[e], r[i]); r[i] = nv; }
            if (incremental) {
                // pads sit at the end of a segment: give them row INT32_MAX-ish keys past the real ones
                sh_srow[base + (e - e0)] = pad ? INT32_MAX : (int32_t)i;
                sh_sval[base + (e - e0)] = dmmv_abs(nv);
            }
        }
        base += e1 - e0;
    }
    __syncthreads();
    if (!incremental) {
        __threadfence_block();
        reservoir_rebuild(L, m, r, res_val, res_row, res_meta, floor_val);
        return;
    }
    // ---- incremental reservoir update ----
    // (pads make sh_srow non-monotone across partitions only at segment ends; membership
    //  below therefore searches each partition's slice separately)
    const int32_t cnt = res_meta[RES_CNT];
    const T fv = floor_val[0];
    const int32_t fr = res_meta[RES_FLOOR_ROW];
    if (threadIdx.x == 0) L.count = 0;
    __syncthreads();
    // survivors: reservoir rows that the move did not touch
    if (threadIdx.x < cnt) {
        const int32_t row = res_row[threadIdx.x];
        const int32_t p = row / mp;
        int32_t lo = 0;
        for (int32_t pp = 0; pp < p; ++pp) lo += segptr[(int64_t)pp * n + j + 1] - segptr[(int64_t)pp * n + j];
        int32_t hi = lo + (segptr[(int64_t)p * n + j + 1] - segptr[(int64_t)p * n + j]);
        const int32_t end = hi;
        while (lo < hi) {
            const int32_t mid = (lo + hi) >> 1;
            if (sh_srow[mid] < row) lo = mid + 1; else hi = mid;
        }
        const bool touched = lo < end && sh_srow[lo] == row;
        if (!touched) {
            const int32_t pos = atomicAdd(&L.count, 1);
            L.v[pos] = res_val[threadIdx.x];
            L.r[pos] = row;
        }
    }
    // entrants: changed rows whose new key is before-or-equal the floor
    for (int32_t u = threadIdx.x; u < col_len; u += SA_BLOCK) {
        const int32_t row = sh_srow[u];
        if (row == INT32_MAX) continue;
        const T a = sh_sval[u];
        if (!key_before(fv, fr, a, row)) {
            const int32_t pos = atomicAdd(&L.count, 1);
            L.v[pos] = a;
            L.r[pos] = row;
        }
    }
    __syncthreads();
    const int32_t cnew = L.count;
    __syncthreads();
    reservoir_publish(L, cnew, false, res_val, res_row, res_meta, floor_val);
    if (res_meta[RES_CNT] < RES_MIN) {
        __threadfence_block();
        reservoir_rebuild(L, m, r, res_val, res_row, res_meta, floor_val);
    }
}

// =========================================================================================
// host dispatch
// =========================================================================================
template <class T>
static dmmv_status build_t(Ctx* c) {
    const int64_t m = c->p.m, n = c->p.n, nnz = c->p.nnz;
    const int64_t nseg = (int64_t)c->csc_P * n;
    hipLaunchKernelGGL(k_cscp_zero, dim3((unsigned)ceil_div(nseg + 1, 256)), dim3(256), 0, c->stream, c->segptr, nseg + 1);
    if (m > 0)
        hipLaunchKernelGGL(k_cscp_count, dim3((unsigned)ceil_div(m, 256)), dim3(256), 0, c->stream, m, n, nnz, c->csc_mp, c->p.csr_rowptr, c->p.csr_col, c->segptr, c->flags);
    hipLaunchKernelGGL(k_cscp_scan, dim3(1), dim3(1024), 0, c->stream, nseg, c->segptr, c->fillpos);
    if (m > 0)
        hipLaunchKernelGGL(k_cscp_fill<T>, dim3((unsigned)ceil_div(m, 256)), dim3(256), 0, c->stream, m, n, c->csc_mp, c->p.csr_rowptr, c->p.csr_col, (const T*)c->p.csr_val, c->fillpos, c->row16_tmp, (T*)c->cval_tmp, (const int32_t*)c->flags);
    if (nseg > 0)
        hipLaunchKernelGGL(k_cscp_sort<T>, dim3((unsigned)ceil_div(nseg, 4)), dim3(256), 0, c->stream, nseg, c->csc_mp, (const int32_t*)c->segptr, (const int32_t*)c->fillpos, (const uint16_t*)c->row16_tmp, (const T*)c->cval_tmp, c->row16, (T*)c->cval, c->flags);
    hipLaunchKernelGGL(k_cscp_ranges, dim3((unsigned)ceil_div(c->csc_gb + 1, 256)), dim3(256), 0, c->stream, n, c->csc_P, c->csc_gb, (const int32_t*)c->segptr, c->blk_lo);
    DMMV_LAUNCH_CHECK();
    return DMMV_OK;
}

template <class T>
static dmmv_status residual_t(Ctx* c) {
    if (c->p.m == 0) return DMMV_OK;
    hipLaunchKernelGGL(k_residual_csr<T>, dim3((unsigned)ceil_div(c->p.m, 256)), dim3(256), 0, c->stream,
                       c->p.m, c->p.csr_rowptr, c->p.csr_col, (const T*)c->p.csr_val, (const T*)c->D_dev,
                       (const int32_t*)c->kidx, (const T*)c->p.b, (T*)c->r);
    DMMV_LAUNCH_CHECK();
    return DMMV_OK;
}

template <class T>
static dmmv_status reservoir_t(Ctx* c) {
    hipLaunchKernelGGL(k_reservoir_build<T>, dim3(1), dim3(1024), 0, c->stream, c->p.m, (const T*)c->r,
                       (T*)c->res_val, c->res_row, c->res_meta, (T*)c->res_floor);
    DMMV_LAUNCH_CHECK();
    return DMMV_OK;
}

template <class T, int KT>
static dmmv_status eval_launch(Ctx* c, void* scores, bool want_partials, bool honor_done) {
    if ((int64_t)c->csc_gb != c->n_partials) return fail(DMMV_ERR_STATE, "sparse evaluation grid does not match the partial-record buffer");
    if (c->csc_P > CSC_MAX_PARTITIONS) return fail(DMMV_ERR_UNSUPPORTED, "sparse path: %d row partitions exceed the limit of %d (raise sparse_partition_rows)", c->csc_P, CSC_MAX_PARTITIONS);
    const size_t lds = ((size_t)c->csc_mp + 1) * sizeof(T);
    static bool attr_set = false;
    if (!attr_set) {
        DMMV_HIP_CHECK(hipFuncSetAttribute(reinterpret_cast<const void*>(&k_eval_cscp<T, KT>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, CSC_LDS_BYTES + 256));
        attr_set = true;
    }
    hipLaunchKernelGGL((k_eval_cscp<T, KT>), dim3((unsigned)c->csc_gb), dim3(EVAL_BLOCK), lds, c->stream,
                       c->p.m, c->p.n, c->p.nd, c->csc_mp, c->csc_P, (const int32_t*)c->segptr,
                       (const uint16_t*)c->row16, (const T*)c->cval, (const int32_t*)c->blk_lo,
                       (const T*)c->D_dev, (const int32_t*)c->kidx, (const T*)c->r,
                       (const T*)c->res_val, (const int32_t*)c->res_row, (const int32_t*)c->res_meta,
                       c->o.radius, c->o.var_mask, (const InstState<T>*)c->state, (int32_t)honor_done,
                       (T*)c->colmax, c->colmask, (T*)scores,
                       want_partials ? (Partial<T>*)c->partials : nullptr);
    DMMV_LAUNCH_CHECK();
    return DMMV_OK;
}

template <class T>
static dmmv_status eval_t(Ctx* c, void* scores, bool want_partials, bool honor_done) {
    if (c->p.nd <= 2) return eval_launch<T, 2>(c, scores, want_partials, honor_done);
    if (c->p.nd == 3) return eval_launch<T, 3>(c, scores, want_partials, honor_done);
    if (c->p.nd <= 4) return eval_launch<T, 4>(c, scores, want_partials, honor_done);
    return eval_launch<T, 8>(c, scores, want_partials, honor_done);
}

template <class T>
static dmmv_status apply_t(Ctx* c) {
    hipLaunchKernelGGL(k_apply_cscp<T>, dim3(1), dim3(256), 0, c->stream, c->p.n, c->csc_mp, c->csc_P,
                       (const int32_t*)c->segptr, (const uint16_t*)c->row16, (const T*)c->cval, (T*)c->r,
                       c->kidx, (InstState<T>*)c->state);
    DMMV_LAUNCH_CHECK();
    return DMMV_OK;
}

template <class T>
static dmmv_status select_apply_t(Ctx* c, int32_t iters, dmmv_move* trace, void* trace_t) {
    hipLaunchKernelGGL(k_select_apply_cscp<T>, dim3(1), dim3(SA_BLOCK), 0, c->stream, c->p.m, c->p.n,
                       c->p.nd, c->csc_mp, c->csc_P, (const int32_t*)c->segptr, (const uint16_t*)c->row16,
                       (const T*)c->cval, (const T*)c->D_dev, (T*)c->r, c->kidx,
                       (const Partial<T>*)c->partials, c->p.n > 0 ? c->n_partials : 0,
                       (InstState<T>*)c->state, c->o.keep_going, (T*)c->res_val, c->res_row, c->res_meta,
                       (T*)c->res_floor, iters, trace, (T*)trace_t);
    DMMV_LAUNCH_CHECK();
    return DMMV_OK;
}

dmmv_status csc_build(Ctx* c) { return c->p.dtype == DMMV_F64 ? build_t<double>(c) : build_t<float>(c); }
dmmv_status csc_residual(Ctx* c) { return c->p.dtype == DMMV_F64 ? residual_t<double>(c) : residual_t<float>(c); }
dmmv_status csc_reservoir(Ctx* c) { return c->p.dtype == DMMV_F64 ? reservoir_t<double>(c) : reservoir_t<float>(c); }
dmmv_status csc_eval(Ctx* c, void* scores_out, bool want_partials, bool honor_done) {
    return c->p.dtype == DMMV_F64 ? eval_t<double>(c, scores_out, want_partials, honor_done)
                                  : eval_t<float>(c, scores_out, want_partials, honor_done);
}
dmmv_status csc_apply(Ctx* c) { return c->p.dtype == DMMV_F64 ? apply_t<double>(c) : apply_t<float>(c); }
dmmv_status csc_select_apply(Ctx* c, int32_t iters, dmmv_move* trace, void* trace_t) {
    return c->p.dtype == DMMV_F64 ? select_apply_t<double>(c, iters, trace, trace_t)
                                  : select_apply_t<float>(c, iters, trace, trace_t);
}

}  // namespace dmmv
