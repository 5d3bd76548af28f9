// Sparse single-instance path, part 1: building the row-partitioned, column-compressed copy
// of a CSR matrix on the device, the residual, the reservoir of the rows of largest |r|, and
// the kernels that apply a move, and the layout-dependent kernels of the ALNS outer loop
// (impact weights, repair).  The evaluation kernels are in dmmv_sparse_eval.hip.
//
// Layout.  Rows are cut into P partitions of at most MP rows, MP chosen so that one partition
// of the residual fits the LDS budget of an evaluation workgroup.  Inside a partition the
// entries are stored column by column, rows ascending, as a 16-bit row offset and a value
// (6 bytes per entry in fp32).  Segment s = p*n + j holds the entries of column j that fall in
// partition p; every segment starts on a multiple of four entries, is padded to one and holds
// at least four (pad = row offset MP, value 0).
//
// Reservoir.  The rows of largest |r| in a strict total order (|r| descending, row ascending),
// kept sorted on the device together with a floor key: the reservoir holds EVERY row at or
// before the floor.  It is rebuilt from r after a residual computation and updated
// incrementally by the kernel that applies a move (drop the rows the move touched, insert the
// changed rows that are at or before the floor, sort, truncate; rebuild when it runs low).
#include "dmmv_sparse_common.h"
#include "dmmv_alns_common.h"

namespace dmmv {

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
    atomicMax(&flags[FLAG_MAXROW], (int32_t)(e1 - e0 < INT32_MAX ? e1 - e0 : INT32_MAX));
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
        // padded to whole groups of SEG_ALIGN, and never empty: the streaming kernel's lanes
        // re-read a segment's last group when they have nothing of their own
        const int32_t v = s < count ? (len > 0 ? (len + SEG_ALIGN - 1) / SEG_ALIGN * SEG_ALIGN : SEG_ALIGN) : 0;
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

// most entries of one column over all its segments, padding included
__global__ void k_cscp_maxcol(int64_t n, int32_t P, const int32_t* __restrict__ segptr, int32_t* flags) {
    const int64_t j = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
    if (j >= n) return;
    int64_t len = 0;
    for (int32_t p = 0; p < P; ++p) len += segptr[(int64_t)p * n + j + 1] - segptr[(int64_t)p * n + j];
    atomicMax(&flags[FLAG_MAXCOL], (int32_t)(len < INT32_MAX ? len : INT32_MAX));
}

// column range of every evaluation workgroup: per partition, equal shares of its entries.
// blk_lo[p*(gbp+1) + b] = first column of workgroup b of partition p.
__global__ void k_cscp_ranges(int64_t n, int32_t P, int32_t gbp, const int32_t* __restrict__ segptr,
                              int32_t* __restrict__ blk_lo) {
    const int64_t t = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
    if (t >= (int64_t)P * (gbp + 1)) return;
    const int32_t p = (int32_t)(t / (gbp + 1)), b = (int32_t)(t % (gbp + 1));
    const int32_t* __restrict__ sp = segptr + (int64_t)p * n;
    if (b == 0) { blk_lo[t] = 0; return; }
    if (b == gbp) { blk_lo[t] = (int32_t)n; return; }
    const int64_t base = sp[0], total = sp[n] - base;
    const int64_t want = base + total * b / gbp;
    int64_t lo = 0, hi = n;      // first column whose segment starts at or after `want`
    while (lo < hi) {
        const int64_t mid = (lo + hi) >> 1;
        if (sp[mid] < want) lo = mid + 1; else hi = mid;
    }
    blk_lo[t] = (int32_t)lo;
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
constexpr int RES_SEL = 256;     // threads whose strided maxima choose the floor at a rebuild
constexpr int RES_COLLECT = 1024;
constexpr int RES_BATCH = 8;     // rows a thread requests before it waits, in the scans of a rebuild (16: slower)

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
        // eight entries per step, so that their LDS reads are in flight together (one at a time
        // the loop runs at the LDS latency: 4.5 us for 150 entries)
        int32_t rank = 0, q = 0;
        for (; q + 8 <= c; q += 8) {
            T v8[8];
            int32_t r8[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) { v8[e] = L.v[q + e]; r8[e] = L.r[q + e]; }
#pragma unroll
            for (int e = 0; e < 8; ++e) rank += key_before(v8[e], r8[e], a, row);
        }
        for (; q < c; ++q) rank += key_before(L.v[q], L.r[q], a, row);
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
    // The maxima of the RES_SEL residue classes of the row number propose a floor with about
    // `target` rows above it.  Every thread scans (the workgroup's size is a multiple of RES_SEL,
    // so a thread's rows t, t + blockDim, ... belong to one class), RES_BATCH rows per step so that
    // their loads are in flight together; the partial maxima of a class are joined through LDS.
    T mv = (T)-1;
    int32_t mr = INT32_MAX;
    {
        const int64_t step = blockDim.x;
        int64_t i = threadIdx.x;
        for (; i + (RES_BATCH - 1) * step < m; i += RES_BATCH * step) {
            T a8[RES_BATCH];
#pragma unroll
            for (int e = 0; e < RES_BATCH; ++e) a8[e] = dmmv_abs(ld_coherent(r + i + e * step));
#pragma unroll
            for (int e = 0; e < RES_BATCH; ++e)
                if (key_before(a8[e], (int32_t)(i + e * step), mv, mr)) { mv = a8[e]; mr = (int32_t)(i + e * step); }
        }
        for (; i < m; i += step) {
            const T a = dmmv_abs(ld_coherent(r + i));
            if (key_before(a, (int32_t)i, mv, mr)) { mv = a; mr = (int32_t)i; }
        }
    }
    L.v[threadIdx.x] = mv;
    L.r[threadIdx.x] = mr;
    __syncthreads();
    if (threadIdx.x < RES_SEL) {
        for (int32_t o = threadIdx.x + RES_SEL; o < (int32_t)blockDim.x; o += RES_SEL) {
            const T ov = L.v[o];
            const int32_t orow = L.r[o];
            if (key_before(ov, orow, mv, mr)) { mv = ov; mr = orow; }
        }
    }
    int32_t target = RES_CAP / 2;
    for (;;) {
        __syncthreads();
        if (threadIdx.x < RES_SEL) { L.v[threadIdx.x] = mv; L.r[threadIdx.x] = mr; }
        if (threadIdx.x == 0) L.count = 0;
        __syncthreads();
        if (threadIdx.x < RES_SEL) {
            int32_t rank = 0;
            static_assert(RES_SEL % 8 == 0, "ranking loop step");
            for (int32_t q = 0; q < RES_SEL; q += 8) {
                T v8[8];
                int32_t r8[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) { v8[e] = L.v[q + e]; r8[e] = L.r[q + e]; }
#pragma unroll
                for (int e = 0; e < 8; ++e) rank += key_before(v8[e], r8[e], mv, mr);
            }
            if (rank == target - 1) { L.fv = mv; L.fr = mr; }
        }
        __syncthreads();
        const T fv = L.fv;
        const int32_t fr = L.fr;
        __syncthreads();
        {
            const int64_t step = blockDim.x;
            int64_t i = threadIdx.x;
            for (; i + (RES_BATCH - 1) * step < m; i += RES_BATCH * step) {
                T a8[RES_BATCH];
#pragma unroll
                for (int e = 0; e < RES_BATCH; ++e) a8[e] = dmmv_abs(ld_coherent(r + i + e * step));
#pragma unroll
                for (int e = 0; e < RES_BATCH; ++e)
                    if (!key_before(fv, fr, a8[e], (int32_t)(i + e * step))) {      // key before-or-equal floor
                        const int32_t pos = atomicAdd(&L.count, 1);
                        if (pos < RES_COLLECT) { L.v[pos] = a8[e]; L.r[pos] = (int32_t)(i + e * step); }
                    }
            }
            for (; i < m; i += step) {
                const T a = dmmv_abs(ld_coherent(r + i));
                if (!key_before(fv, fr, a, (int32_t)i)) {
                    const int32_t pos = atomicAdd(&L.count, 1);
                    if (pos < RES_COLLECT) { L.v[pos] = a; L.r[pos] = (int32_t)i; }
                }
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
constexpr int SA_DCAP = SA_BLOCK;                  // levels kept in LDS: one per thread

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
    __shared__ int32_t sh_e0[CSC_MAX_PARTITIONS], sh_len[CSC_MAX_PARTITIONS];   // column j's segments
    __shared__ T sh_D[SA_DCAP];                 // the levels, when they fit: requested with the first loads
    // Everything that depends on nothing is fetched together (one memory latency, not one per
    // use): the loop state, the records, and the reservoir this kernel will update.  From one
    // workgroup every dependent access to memory costs about a microsecond.
    const InstState<T> z0 = st[0];
    const int32_t cnt = res_meta[RES_CNT];
    const int32_t fr = res_meta[RES_FLOOR_ROW];
    const T fv = floor_val[0];
    int32_t my_row = -1;
    T my_val = (T)0;
    if (threadIdx.x < RES_CAP) { my_row = res_row[threadIdx.x]; my_val = res_val[threadIdx.x]; }
    const bool d_lds = nd <= SA_DCAP;
    T my_d = (T)0;
    if (d_lds && (int32_t)threadIdx.x < nd) my_d = D[threadIdx.x];
    T s = (T)0;
    int64_t c = -1;
    for (int64_t q = threadIdx.x; q < n_part; q += SA_BLOCK) {
        const Partial<T> pr = part[q];
        if (rec_less(pr.s, pr.c, s, c)) { s = pr.s; c = pr.c; }
    }
    if (z0.done) return;
    if (d_lds && (int32_t)threadIdx.x < nd) sh_D[threadIdx.x] = my_d;     // (the reduction's barriers order it)
    block_argmin(s, c, sh_s, sh_c);
    if (threadIdx.x == 0) {
        InstState<T> z = z0;
        int32_t j = -1, k = -1;
        if (c >= 0) { j = (int32_t)(c / nd); k = (int32_t)(c % nd); }
        const bool improving = c >= 0 && s < z.t;
        z.best_s = s;
        z.apply_j = -1; z.apply_k = -1; z.delta = (T)0;      // applied right here
        sh_j = improving ? j : -1;
        sh_k = k;
        sh_best = s;
        if (improving) {
            const int32_t kc = kidx[j];
            sh_delta = d_lds ? step_of(sh_D[k], sh_D[kc], (T)1) : step_of(D[k], D[kc], (T)1);
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
    for (int32_t p = threadIdx.x; p < P; p += SA_BLOCK) {
        const int32_t e0 = segptr[(int64_t)p * n + j], e1 = segptr[(int64_t)p * n + j + 1];
        sh_e0[p] = e0;
        sh_len[p] = e1 - e0;
    }
    __syncthreads();
    int32_t col_len = 0;
    for (int32_t p = 0; p < P; ++p) col_len += sh_len[p];
    const bool incremental = col_len <= SA_MAXCOL && m > RES_CAP;
    // The segments of all partitions are taken as one list (position u = entries of the earlier
    // partitions + offset in its own), one entry per thread: the entries of the whole column are
    // requested together and so are its rows of r - two trips to memory, not two per partition.
    for (int32_t u = threadIdx.x; u < col_len; u += SA_BLOCK) {
        int32_t p = 0, lo = 0, len = sh_len[0];
        while (u >= lo + len) { lo += len; len = sh_len[++p]; }       // u < col_len: ends inside the table
        const int32_t e = sh_e0[p] + (u - lo);
        const uint32_t loc = row16[e];
        const T a = cval[e];
        const bool pad = loc == (uint32_t)mp;
        const int64_t i = (int64_t)p * mp + loc;
        T nv = (T)0;
        if (!pad) { nv = dmmv_fma(delta, a, r[i]); r[i] = nv; }
        if (incremental) {
            // pads sit at the end of a segment: give them row INT32_MAX-ish keys past the real ones
            sh_srow[u] = pad ? INT32_MAX : (int32_t)i;
            sh_sval[u] = dmmv_abs(nv);
        }
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
    if (threadIdx.x == 0) L.count = 0;
    __syncthreads();
    // survivors: reservoir rows that the move did not touch
    if (threadIdx.x < cnt) {
        const int32_t row = my_row;
        const int32_t p = row / mp;
        int32_t lo = 0;
        for (int32_t pp = 0; pp < p; ++pp) lo += sh_len[pp];
        int32_t hi = lo + sh_len[p];
        const int32_t end = hi;
        while (lo < hi) {
            const int32_t mid = (lo + hi) >> 1;
            if (sh_srow[mid] < row) lo = mid + 1; else hi = mid;
        }
        const bool touched = lo < end && sh_srow[lo] == row;
        if (!touched) {
            const int32_t pos = atomicAdd(&L.count, 1);
            L.v[pos] = my_val;
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
    if ((cnew < RES_CAP ? cnew : RES_CAP) < RES_MIN) {      // what publish left in meta[RES_CNT]
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
    hipLaunchKernelGGL(k_cscp_ranges, dim3((unsigned)ceil_div((int64_t)c->csc_P * (c->csc_gb + 1), 256)), dim3(256), 0, c->stream, n, c->csc_P, c->csc_gb, (const int32_t*)c->segptr, c->blk_lo);
    if (n > 0)
        hipLaunchKernelGGL(k_cscp_maxcol, dim3((unsigned)ceil_div(n, 256)), dim3(256), 0, c->stream, n, c->csc_P, (const int32_t*)c->segptr, c->flags);
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

template <class T>
static dmmv_status apply_t(Ctx* c) {
    hipLaunchKernelGGL(k_apply_cscp<T>, dim3(1), dim3(256), 0, c->stream, c->p.n, c->csc_mp, c->csc_P,
                       (const int32_t*)c->segptr, (const uint16_t*)c->row16, (const T*)c->cval, (T*)c->r,
                       c->kidx, (InstState<T>*)c->state);
    DMMV_LAUNCH_CHECK();
    return DMMV_OK;
}

template <class T>
static dmmv_status select_apply_t(Ctx* c, int32_t iters, dmmv_move* trace, void* trace_t, bool pruned) {
    hipLaunchKernelGGL(k_select_apply_cscp<T>, dim3(1), dim3(SA_BLOCK), 0, c->stream, c->p.m, c->p.n,
                       c->p.nd, c->csc_mp, c->csc_P, (const int32_t*)c->segptr, (const uint16_t*)c->row16,
                       (const T*)c->cval, (const T*)c->D_dev, (T*)c->r, c->kidx,
                       pruned ? (const Partial<T>*)c->prune_part : (const Partial<T>*)c->partials,
                       pruned ? (int64_t)c->csc_max_row : (c->p.n > 0 ? c->n_partials : 0),
                       (InstState<T>*)c->state, c->o.keep_going, (T*)c->res_val, c->res_row, c->res_meta,
                       (T*)c->res_floor, iters, trace, (T*)trace_t);
    DMMV_LAUNCH_CHECK();
    return DMMV_OK;
}

dmmv_status csc_build(Ctx* c) { return c->p.dtype == DMMV_F64 ? build_t<double>(c) : build_t<float>(c); }
dmmv_status csc_residual(Ctx* c) { return c->p.dtype == DMMV_F64 ? residual_t<double>(c) : residual_t<float>(c); }
dmmv_status csc_reservoir(Ctx* c) { return c->p.dtype == DMMV_F64 ? reservoir_t<double>(c) : reservoir_t<float>(c); }
dmmv_status csc_apply(Ctx* c) { return c->p.dtype == DMMV_F64 ? apply_t<double>(c) : apply_t<float>(c); }
dmmv_status csc_select_apply(Ctx* c, int32_t iters, dmmv_move* trace, void* trace_t, bool pruned) {
    return c->p.dtype == DMMV_F64 ? select_apply_t<double>(c, iters, trace, trace_t, pruned)
                                  : select_apply_t<float>(c, iters, trace, trace_t, pruned);
}

// =========================================================================================
// ALNS outer loop: the kernels that depend on the sparse layout
// =========================================================================================
// worst-remove operator: integer sampling weight of every variable, one wavefront per column
template <class T>
__global__ __launch_bounds__(256) void k_alns_impact_cscp(int64_t m, int64_t n, int32_t mp, int32_t P,
                                                         const int32_t* __restrict__ segptr,
                                                         const uint16_t* __restrict__ row16,
                                                         const T* __restrict__ cval, const T* __restrict__ r,
                                                         const InstState<T>* st, double alpha,
                                                         uint64_t* __restrict__ weight, const AlnsState* S) {
    if (S->d_op != 1) return;
    const int lane = threadIdx.x & 63;
    const int64_t j = blockIdx.x * 4ll + (threadIdx.x >> 6);
    if (j >= n) return;
    const double t = (double)st[0].t;
    const double scale = alns_impact_scale(t);
    uint64_t sum = 0;
    if (scale != 0.0) {
        for (int32_t p = 0; p < P; ++p) {
            const int32_t e0 = segptr[(int64_t)p * n + j], e1 = segptr[(int64_t)p * n + j + 1];
            for (int32_t e = e0 + lane; e < e1; e += 64) {
                const uint32_t loc = row16[e];
                if (loc == (uint32_t)mp) continue;
                const double sk = __builtin_fabs((double)r[(int64_t)p * mp + loc]);
                sum += alns_impact_term(__builtin_fabs((double)cval[e]), sk, t, alpha, scale);
            }
        }
    }
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) sum += (uint64_t)__shfl_xor((long long)sum, off, 64);
    if (lane == 0) {
        int shift = alns_bits(m) + 24 + alns_bits(n) - 62;
        if (shift < 0) shift = 0;
        weight[j] = 1 + (sum >> shift);
    }
}

// repair: single workgroup, the picked variables one after the other.  A greedy choice needs
// the worst-case error over ALL rows for both neighbouring levels: the rows of the column are
// marked, the others contribute their |r| as it stands.
template <class T>
__global__ __launch_bounds__(1024) void k_alns_repair_cscp_general(int64_t m, int64_t n, int32_t nd, int32_t mp, int32_t P,
                                                          const int32_t* __restrict__ segptr,
                                                          const uint16_t* __restrict__ row16,
                                                          const T* __restrict__ cval, const T* __restrict__ D,
                                                          T* r, int32_t* kidx, int32_t count,
                                                          const int32_t* __restrict__ picked, uint8_t* touched,
                                                          InstState<T>* st, const AlnsState* S, uint64_t seed,
                                                          uint64_t inst) {
    __shared__ T sh[16];
    const int32_t it = S->it;
    const bool greedy = S->r_op == 1;
    for (int32_t pos = 0; pos < count; ++pos) {
        const int64_t j = picked[pos];
        const int32_t kc = kidx[j];
        const bool has_lo = kc > 0, has_hi = kc < nd - 1;
        int32_t knew;
        if (has_lo && has_hi) {
            if (greedy) {
                for (int32_t p = 0; p < P; ++p) {
                    const int32_t e0 = segptr[(int64_t)p * n + j], e1 = segptr[(int64_t)p * n + j + 1];
                    for (int32_t e = e0 + threadIdx.x; e < e1; e += blockDim.x) {
                        const uint32_t loc = row16[e];
                        if (loc != (uint32_t)mp) touched[(int64_t)p * mp + loc] = 1;
                    }
                }
                __syncthreads();
                const T dlo = step_of(D[kc - 1], D[kc], (T)1), dhi = step_of(D[kc + 1], D[kc], (T)1);
                T rest = (T)0;
                for (int64_t i = threadIdx.x; i < m; i += blockDim.x)
                    if (!touched[i]) rest = dmmv_max(rest, dmmv_abs(r[i]));
                T elo = rest, ehi = rest;
                for (int32_t p = 0; p < P; ++p) {
                    const int32_t e0 = segptr[(int64_t)p * n + j], e1 = segptr[(int64_t)p * n + j + 1];
                    for (int32_t e = e0 + threadIdx.x; e < e1; e += blockDim.x) {
                        const uint32_t loc = row16[e];
                        if (loc == (uint32_t)mp) continue;
                        const T a = cval[e], ri = r[(int64_t)p * mp + loc];
                        elo = dmmv_max(elo, dmmv_abs(dmmv_fma(dlo, a, ri)));
                        ehi = dmmv_max(ehi, dmmv_abs(dmmv_fma(dhi, a, ri)));
                    }
                }
                elo = block_max(elo, sh);
                ehi = block_max(ehi, sh);
                knew = ehi < elo ? kc + 1 : kc - 1;
                for (int32_t p = 0; p < P; ++p) {
                    const int32_t e0 = segptr[(int64_t)p * n + j], e1 = segptr[(int64_t)p * n + j + 1];
                    for (int32_t e = e0 + threadIdx.x; e < e1; e += blockDim.x) {
                        const uint32_t loc = row16[e];
                        if (loc != (uint32_t)mp) touched[(int64_t)p * mp + loc] = 0;
                    }
                }
            } else {
                knew = (alns_rnd(seed, inst, (uint64_t)it, 2, (uint64_t)pos) & 1) ? kc + 1 : kc - 1;
            }
        } else {
            knew = has_lo ? kc - 1 : kc + 1;
        }
        const T delta = step_of(D[knew], D[kc], (T)1);
        for (int32_t p = 0; p < P; ++p) {
            const int32_t e0 = segptr[(int64_t)p * n + j], e1 = segptr[(int64_t)p * n + j + 1];
            for (int32_t e = e0 + threadIdx.x; e < e1; e += blockDim.x) {
                const uint32_t loc = row16[e];
                if (loc == (uint32_t)mp) continue;
                const int64_t i = (int64_t)p * mp + loc;
                r[i] = dmmv_fma(delta, cval[e], r[i]);
            }
        }
        __syncthreads();                      // r and the marks are settled; kidx[j] was read by all
        if (threadIdx.x == 0) kidx[j] = knew;
    }
    T tmax = (T)0;
    for (int64_t i = threadIdx.x; i < m; i += blockDim.x) tmax = dmmv_max(tmax, dmmv_abs(r[i]));
    tmax = block_max(tmax, sh);
    if (threadIdx.x == 0) { st[0].t = tmax; st[0].done = 0; st[0].moves = 0; }
}

// Repair without the chain of dependent loads.  From one workgroup every dependent access to
// memory costs about half a microsecond, and the general kernel needs three to five per picked
// variable (segment bounds, entries, residuals, ...).  Here the entries of all picked columns are
// first gathered, by many workgroups, into a scratch array with a fixed stride per column
// (k_alns_gather: global row and value, row -1 for padding), so the repair kernel knows the
// address of a pick's entries without loading anything and fetches the next pick's entries, pick
// number and level index while it works on the current one; the levels sit in LDS.  What is left
// per pick is one trip for the residuals and one for the acknowledgement of their stores.
// Greedy: a thread keeps one entry (row, value, residual) in registers for the whole step; the
// column's rows are marked in an LDS bitmap; the maxima of |r| over chunks of 16 rows live in LDS,
// so "the largest |r| outside the column" is the kept maximum of the chunks the column does not
// touch and a row-by-row look at those it does - one row of 16 lanes per chunk, all loads of a
// pass issued together on clamped indices (a load inside a branch is waited for inside it);
// the touched chunks get their new maxima from that look and from the new residuals.
// One workgroup of 1024 threads issues one wavefront instruction per clock at best, so the
// step is written for few instructions: 32-bit indices, reductions as a DPP pass over 16 lanes
// plus one LDS atomic per row of lanes (|.| >= 0: the bit patterns order like the values).
// Maxima are exact in any order, so the choices are those of the general kernel.
constexpr int RP_CHUNK = 16;              // rows per chunk = lanes of a DPP row
constexpr int RP_CMAX_BYTES = 32768;      // LDS for the chunk maxima: 131072 rows in fp32, 65536 in fp64
constexpr int RP_BLOCK = 1024;            // longest column (padding included) the kernel takes
constexpr int RP_DCAP = 1024;             // levels kept in LDS (more are read from memory)
constexpr int RP_LOOK = 4;                // passes of 64 touched chunks whose loads are in flight together
constexpr int64_t RP_GATHER_CAP = 1 << 20;   // entries of the scratch array

template <class T>
constexpr int rp_max_chunks() { return RP_CMAX_BYTES / (int)sizeof(T); }

template <class T>
__global__ void k_alns_gather(int64_t n, int32_t mp, int32_t P, int32_t stride, const int32_t* __restrict__ segptr,
                              const uint16_t* __restrict__ row16, const T* __restrict__ cval,
                              const int32_t* __restrict__ picked, int32_t* __restrict__ g_row,
                              T* __restrict__ g_val) {
    const int64_t q = blockIdx.x;
    const int64_t j = picked[q];
    int32_t base = 0;
    for (int32_t p = 0; p < P; ++p) {
        const int32_t e0 = segptr[(int64_t)p * n + j], e1 = segptr[(int64_t)p * n + j + 1];
        for (int32_t e = e0 + threadIdx.x; e < e1; e += blockDim.x) {
            const uint32_t loc = row16[e];
            const bool pad = loc == (uint32_t)mp;
            g_row[q * stride + base + (e - e0)] = pad ? -1 : (int32_t)((int64_t)p * mp + loc);
            g_val[q * stride + base + (e - e0)] = pad ? (T)0 : cval[e];
        }
        base += e1 - e0;
    }
    for (int32_t t = base + threadIdx.x; t < stride; t += blockDim.x) { g_row[q * stride + t] = -1; g_val[q * stride + t] = (T)0; }
}

// LDS maximum of values >= 0
__device__ __forceinline__ void lds_max_nonneg(float* p, float v) {
    atomicMax(reinterpret_cast<unsigned int*>(p), __float_as_uint(v));
}
__device__ __forceinline__ void lds_max_nonneg(double* p, double v) {
    atomicMax(reinterpret_cast<unsigned long long*>(p), (unsigned long long)__double_as_longlong(v));
}

template <class T>
__global__ __launch_bounds__(RP_BLOCK) void k_alns_repair_gathered(
    int32_t m, int32_t nd, int32_t stride, const int32_t* __restrict__ g_row, const T* __restrict__ g_val,
    const T* __restrict__ D, T* r, int32_t* kidx, int32_t count, const int32_t* __restrict__ picked,
    InstState<T>* st, const AlnsState* S, uint64_t seed, uint64_t inst) {
    constexpr int MAXCH = rp_max_chunks<T>();
    __shared__ T sh[16];
    __shared__ __align__(32) T sh_cmax[MAXCH];                 // max |r| of every chunk
    __shared__ unsigned int sh_rowbit[MAXCH * RP_CHUNK / 32];  // rows of the current column
    __shared__ unsigned int sh_dirtybit[MAXCH / 32];           // chunks the column touches
    __shared__ int32_t sh_dirty[RP_BLOCK];                     // the same as a list, each once
    __shared__ int32_t sh_ndirty;
    __shared__ T sh_red[2][4];                                 // per pick parity: outside, column low, column high
    __shared__ T sh_D[RP_DCAP];                                // the levels, when they fit
    const int32_t it = S->it;
    const bool greedy = S->r_op == 1;
    const int32_t tid = threadIdx.x;
    const int lane = tid & 63, w = tid >> 6, sub = lane & 15;
    const int32_t nch = (m + RP_CHUNK - 1) / RP_CHUNK;
    const int32_t nch4 = (nch + 3) & ~3;
    const bool d_lds = nd <= RP_DCAP;
    if (d_lds)
        for (int32_t k = tid; k < nd; k += RP_BLOCK) sh_D[k] = D[k];
#define RP_LEVEL(k) (d_lds ? sh_D[k] : D[k])
    if (greedy) {
        // rows i0 + tid: the 16 lanes of a DPP row hold one chunk
        for (int32_t i0 = 0; i0 < nch4 * RP_CHUNK; i0 += 8 * RP_BLOCK) {
            T v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) v[u] = r[min(i0 + u * RP_BLOCK + tid, m - 1)];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int32_t i = i0 + u * RP_BLOCK + tid;
                const T cm = row16_max(i < m ? dmmv_abs(v[u]) : (T)0);
                if (sub == 0 && i < nch4 * RP_CHUNK) sh_cmax[i / RP_CHUNK] = cm;
            }
        }
        for (int32_t q = tid; q < nch4 * RP_CHUNK / 32; q += RP_BLOCK) sh_rowbit[q] = 0u;
        for (int32_t q = tid; q < (nch4 + 31) / 32; q += RP_BLOCK) sh_dirtybit[q] = 0u;
        if (tid < 8) sh_red[tid >> 2][tid & 3] = (T)0;
        if (tid == 0) sh_ndirty = 0;
    }
    const bool mine = tid < stride;
    const bool entry_wave = w * 64 < stride;                 // wavefronts that hold entries
    // entry of the first pick; picks two ahead, level index one ahead: no load of the chain
    // picked -> kidx is waited for inside a step (the picks are distinct, so kidx[j] of a later
    // pick is final already)
    int32_t row_n = -1;
    T a_n = (T)0;
    if (mine && count > 0) { row_n = g_row[tid]; a_n = g_val[tid]; }
    int32_t j_cur = count > 0 ? picked[0] : 0;
    int32_t j_n = count > 1 ? picked[1] : 0;
    int32_t j_nn = 0;
    int32_t kc_n = count > 0 ? kidx[j_cur] : 0;
    __syncthreads();                                         // the LDS tables
    for (int32_t pos = 0; pos < count; ++pos) {
        const int32_t j = j_cur;
        const int32_t kc = kc_n;
        const int32_t row = row_n;
        const T a = a_n;
        const int par = pos & 1;
        const bool real = row >= 0;
        const bool has_lo = kc > 0, has_hi = kc < nd - 1;
        const bool evaluate = greedy && has_lo && has_hi;
        if (greedy) {
            if (real) {
                atomicOr(&sh_rowbit[row >> 5], 1u << (row & 31));
                const int32_t c = row / RP_CHUNK;
                const unsigned int bit = 1u << (c & 31);
                if ((atomicOr(&sh_dirtybit[c >> 5], bit) & bit) == 0u) {   // first to touch the chunk: list it, restart its maximum
                    sh_dirty[atomicAdd(&sh_ndirty, 1)] = c;
                    sh_cmax[c] = (T)0;
                }
            }
            __syncthreads();
        }
        // the entry's residual and the look at the touched chunks are requested together
        const T ri = real ? r[row] : (T)0;
        T rest = (T)0;
        if (greedy) {
            const int32_t ndirty = sh_ndirty;
            for (int32_t d0 = 0; d0 < ndirty; d0 += 64 * RP_LOOK) {
                T v[RP_LOOK];
                int32_t row_u[RP_LOOK];
                unsigned int bits[RP_LOOK];
#pragma unroll
                for (int u = 0; u < RP_LOOK; ++u)
                    row_u[u] = sh_dirty[min(d0 + u * 64 + 4 * w + (lane >> 4), ndirty - 1)] * RP_CHUNK + sub;
#pragma unroll
                for (int u = 0; u < RP_LOOK; ++u) {
                    const int32_t ic = min(row_u[u], m - 1);
                    bits[u] = sh_rowbit[ic >> 5];
                    v[u] = r[ic];
                }
#pragma unroll
                for (int u = 0; u < RP_LOOK; ++u) {
                    const bool valid = d0 + u * 64 + 4 * w + (lane >> 4) < ndirty;
                    const bool in_col = (bits[u] >> (row_u[u] & 31)) & 1u;
                    const T val = (valid && row_u[u] < m && !in_col) ? dmmv_abs(v[u]) : (T)0;
                    rest = dmmv_max(rest, val);
                    // the chunk's maximum restarts from its rows outside the column; the
                    // column's rows join below
                    const T rm = row16_max(val);
                    if (valid && sub == 0) lds_max_nonneg(&sh_cmax[row_u[u] / RP_CHUNK], rm);
                }
            }
        }
        int32_t knew;
        if (evaluate) {
            // untouched chunks: four kept maxima per thread
            for (int32_t g = tid; 4 * g < nch4; g += RP_BLOCK) {
                const unsigned int db = sh_dirtybit[g >> 3] >> ((g & 7) * 4);
                const typename Vec4<T>::type c4 = *reinterpret_cast<const typename Vec4<T>::type*>(&sh_cmax[4 * g]);
                rest = dmmv_max(rest, (db & 1u) ? (T)0 : c4.x);
                rest = dmmv_max(rest, (db & 2u) ? (T)0 : c4.y);
                rest = dmmv_max(rest, (db & 4u) ? (T)0 : c4.z);
                rest = dmmv_max(rest, (db & 8u) ? (T)0 : c4.w);
            }
            const T rm = row16_max(rest);
            if (sub == 0) lds_max_nonneg(&sh_red[par][0], rm);
            if (entry_wave) {
                const T dlo = step_of(RP_LEVEL(kc - 1), RP_LEVEL(kc), (T)1), dhi = step_of(RP_LEVEL(kc + 1), RP_LEVEL(kc), (T)1);
                const T lo = row16_max(real ? dmmv_abs(dmmv_fma(dlo, a, ri)) : (T)0);
                const T hi = row16_max(real ? dmmv_abs(dmmv_fma(dhi, a, ri)) : (T)0);
                if (sub == 0) { lds_max_nonneg(&sh_red[par][1], lo); lds_max_nonneg(&sh_red[par][2], hi); }
            }
            __syncthreads();
            const T outside = sh_red[par][0];
            const T elo = dmmv_max(outside, sh_red[par][1]), ehi = dmmv_max(outside, sh_red[par][2]);
            knew = ehi < elo ? kc + 1 : kc - 1;
        } else {
            if (has_lo && has_hi) knew = (alns_rnd(seed, inst, (uint64_t)it, 2, (uint64_t)pos) & 1) ? kc + 1 : kc - 1;
            else knew = has_lo ? kc - 1 : kc + 1;
            if (greedy) __syncthreads();                    // the look's chunk maxima are in place
        }
        // the next pick: requested here, so that only the step's last barrier waits for it
        if (pos + 1 < count) {
            if (mine) { row_n = g_row[(int64_t)(pos + 1) * stride + tid]; a_n = g_val[(int64_t)(pos + 1) * stride + tid]; }
            kc_n = kidx[j_n];
            if (pos + 2 < count) j_nn = picked[pos + 2];
        }
        // reassign: r follows; greedy: the touched chunks take in the new residuals, the marks go
        const T delta = step_of(RP_LEVEL(knew), RP_LEVEL(kc), (T)1);
        if (real) {
            const T nv = dmmv_fma(delta, a, ri);
            r[row] = nv;
            if (greedy) {
                const int32_t c = row / RP_CHUNK;
                lds_max_nonneg(&sh_cmax[c], dmmv_abs(nv));
                atomicAnd(&sh_rowbit[row >> 5], ~(1u << (row & 31)));
                atomicAnd(&sh_dirtybit[c >> 5], ~(1u << (c & 31)));
            }
        }
        if (tid == 0) { kidx[j] = knew; sh_ndirty = 0; }
        if (tid < 4) sh_red[par ^ 1][tid] = (T)0;            // last read before the previous step's end
        j_cur = j_n;
        j_n = j_nn;
        __syncthreads();                                     // r, kidx and the tables are settled
    }
#undef RP_LEVEL
    T tmax = (T)0;
    if (greedy) {
        for (int32_t c = tid; c < nch; c += RP_BLOCK) tmax = dmmv_max(tmax, sh_cmax[c]);
    } else {
        for (int32_t i = tid; i < m; i += RP_BLOCK) tmax = dmmv_max(tmax, dmmv_abs(r[i]));
    }
    tmax = block_max(tmax, sh);
    if (tid == 0) { st[0].t = tmax; st[0].done = 0; st[0].moves = 0; }
}

// after a rejected iteration r was restored: the reservoir has to follow
template <class T>
__global__ __launch_bounds__(1024) void k_reservoir_build_if_rejected(int64_t m, const T* r, T* res_val,
                                                                      int32_t* res_row, int32_t* meta,
                                                                      T* floor_val, const AlnsState* S) {
    __shared__ ResLds<T> L;
    if (S->accepted) return;
    reservoir_rebuild(L, m, r, res_val, res_row, meta, floor_val);
}

__global__ void k_alns_clear_touched(int64_t m, uint8_t* touched) {
    const int64_t i = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
    if (i < m) touched[i] = 0;
}

template <class T>
static dmmv_status alns_impact_t(Ctx* c, double alpha) {
    hipLaunchKernelGGL(k_alns_impact_cscp<T>, dim3((unsigned)ceil_div(c->p.n, 4)), dim3(256), 0, c->stream,
                       c->p.m, c->p.n, c->csc_mp, c->csc_P, (const int32_t*)c->segptr, (const uint16_t*)c->row16,
                       (const T*)c->cval, (const T*)c->r, (const InstState<T>*)c->state, alpha, c->alns_weight,
                       (const AlnsState*)c->alns_state);
    DMMV_LAUNCH_CHECK();
    return DMMV_OK;
}

template <class T>
static dmmv_status alns_repair_t(Ctx* c, int32_t count, uint64_t seed) {
    // where the tables and the scratch array fit: gather the picked columns, then the kernel
    // without dependent loads; else the general kernel
    const int32_t stride = (int32_t)(ceil_div(c->csc_max_col > 0 ? c->csc_max_col : 1, 64) * 64);
    const bool fast = c->p.m >= 1 && ceil_div(c->p.m, RP_CHUNK) <= rp_max_chunks<T>() && stride <= RP_BLOCK &&
                      (int64_t)count * stride <= RP_GATHER_CAP && c->alns_g_row && c->alns_g_val;
    if (fast) {
        if (count > 0)
            hipLaunchKernelGGL(k_alns_gather<T>, dim3((unsigned)count), dim3(128), 0, c->stream, c->p.n, c->csc_mp,
                               c->csc_P, stride, (const int32_t*)c->segptr, (const uint16_t*)c->row16,
                               (const T*)c->cval, (const int32_t*)c->alns_picked, c->alns_g_row, (T*)c->alns_g_val);
        hipLaunchKernelGGL(k_alns_repair_gathered<T>, dim3(1), dim3(RP_BLOCK), 0, c->stream, (int32_t)c->p.m, c->p.nd, stride,
                           (const int32_t*)c->alns_g_row, (const T*)c->alns_g_val, (const T*)c->D_dev, (T*)c->r,
                           c->kidx, count, (const int32_t*)c->alns_picked, (InstState<T>*)c->state,
                           (const AlnsState*)c->alns_state, seed, (uint64_t)0);
    } else {
        if (c->p.m > 0)
            hipLaunchKernelGGL(k_alns_clear_touched, dim3((unsigned)ceil_div(c->p.m, 256)), dim3(256), 0, c->stream,
                               c->p.m, c->alns_touched);
        hipLaunchKernelGGL(k_alns_repair_cscp_general<T>, dim3(1), dim3(1024), 0, c->stream, c->p.m, c->p.n, c->p.nd,
                           c->csc_mp, c->csc_P, (const int32_t*)c->segptr, (const uint16_t*)c->row16,
                           (const T*)c->cval, (const T*)c->D_dev, (T*)c->r, c->kidx, count,
                           (const int32_t*)c->alns_picked, c->alns_touched, (InstState<T>*)c->state,
                           (const AlnsState*)c->alns_state, seed, (uint64_t)0);
    }
    DMMV_LAUNCH_CHECK();
    return reservoir_t<T>(c);
}

template <class T>
static dmmv_status alns_after_copy_t(Ctx* c) {
    hipLaunchKernelGGL(k_reservoir_build_if_rejected<T>, dim3(1), dim3(1024), 0, c->stream, c->p.m,
                       (const T*)c->r, (T*)c->res_val, c->res_row, c->res_meta, (T*)c->res_floor,
                       (const AlnsState*)c->alns_state);
    DMMV_LAUNCH_CHECK();
    return DMMV_OK;
}

dmmv_status csc_alns_impact(Ctx* c, double alpha) {
    return c->p.dtype == DMMV_F64 ? alns_impact_t<double>(c, alpha) : alns_impact_t<float>(c, alpha);
}
dmmv_status csc_alns_repair(Ctx* c, int32_t count, uint64_t seed) {
    return c->p.dtype == DMMV_F64 ? alns_repair_t<double>(c, count, seed) : alns_repair_t<float>(c, count, seed);
}
dmmv_status csc_alns_after_copy(Ctx* c) {
    return c->p.dtype == DMMV_F64 ? alns_after_copy_t<double>(c) : alns_after_copy_t<float>(c);
}

}  // namespace dmmv
