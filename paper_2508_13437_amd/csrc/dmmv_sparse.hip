// Sparse single-instance path: A given in CSR, scored through a column-compressed (CSC) copy.
//
// The score of a move on variable j is still a maximum over ALL m rows: the rows stored in
// column j change, every other row keeps |r_i|.  The largest |r_i| over the rows outside a
// column is found without scanning them: the TOPK rows of largest |r| are kept in a short
// list (refreshed after every residual change); while a wavefront streams its column it marks
// which listed rows it meets, and the first unmarked list entry is the outside maximum.  Only
// a column that contains all TOPK listed rows needs the exact fallback scan.
#include "dmmv_common.h"

namespace dmmv {

// =========================================================================================
// CSR -> CSC (setup)
// =========================================================================================
__global__ void k_csc_zero(int64_t* colptr, int64_t n1) {
    int64_t j = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
    if (j < n1) colptr[j] = 0;
}

// one thread per row: validate and count entries per column (into colptr[col + 1])
__global__ void k_csc_count(int64_t m, int64_t n, int64_t nnz, const int64_t* __restrict__ rowptr,
                            const int32_t* __restrict__ col, int64_t* colptr, int32_t* flags) {
    int64_t i = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
    if (i >= m) return;
    int64_t e0 = rowptr[i], e1 = rowptr[i + 1];
    if (e0 < 0 || e1 < e0 || e1 > nnz || (i == 0 && e0 != 0) || (i == m - 1 && e1 != nnz)) {
        atomicOr(&flags[FLAG_ERROR], ERRBIT_CSR_RANGE);
        return;
    }
    for (int64_t e = e0; e < e1; ++e) {
        int32_t j = col[e];
        if (j < 0 || j >= n) { atomicOr(&flags[FLAG_ERROR], ERRBIT_CSR_RANGE); continue; }
        atomicAdd((unsigned long long*)&colptr[j + 1], 1ull);
    }
}

// single block: inclusive scan of colptr[1..n] in place (colptr[0] = 0); copy to fillpos
__global__ void k_csc_scan(int64_t n, int64_t* colptr, int64_t* fillpos) {
    __shared__ int64_t sh[1024];
    __shared__ int64_t carry;
    if (threadIdx.x == 0) carry = 0;
    __syncthreads();
    for (int64_t base = 0; base < n; base += 1024) {
        int64_t j = base + threadIdx.x;
        int64_t v = j < n ? colptr[j + 1] : 0;
        sh[threadIdx.x] = v;
        __syncthreads();
        for (int off = 1; off < 1024; off <<= 1) {
            int64_t t = threadIdx.x >= off ? sh[threadIdx.x - off] : 0;
            __syncthreads();
            sh[threadIdx.x] += t;
            __syncthreads();
        }
        int64_t incl = sh[threadIdx.x] + carry;
        if (j < n) { colptr[j + 1] = incl; fillpos[j] = incl - v; }
        __syncthreads();
        if (threadIdx.x == 1023) carry = incl;
        __syncthreads();
    }
}

// one thread per row: scatter its entries into the column segments (order inside a segment
// is arbitrary here; k_csc_sort fixes it)
template <class T>
__global__ void k_csc_fill(int64_t m, int64_t n, const int64_t* __restrict__ rowptr,
                           const int32_t* __restrict__ col, const T* __restrict__ val,
                           int64_t* fillpos, int32_t* __restrict__ rowidx_tmp,
                           T* __restrict__ cval_tmp, const int32_t* flags) {
    int64_t i = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
    if (i >= m || flags[FLAG_ERROR]) return;
    for (int64_t e = rowptr[i]; e < rowptr[i + 1]; ++e) {
        int32_t j = col[e];
        if (j < 0 || j >= n) continue;
        int64_t p = (int64_t)atomicAdd((unsigned long long*)&fillpos[j], 1ull);
        rowidx_tmp[p] = (int32_t)i;
        cval_tmp[p] = val[e];
    }
}

// one wavefront per column: place every entry at its rank by row (rows ascending).  Equal
// rows inside a column mean the matrix stores an entry twice.
template <class T>
__global__ void k_csc_sort(int64_t n, const int64_t* __restrict__ colptr,
                           const int32_t* __restrict__ rowidx_tmp, const T* __restrict__ cval_tmp,
                           int32_t* __restrict__ rowidx, T* __restrict__ cval, int32_t* flags) {
    if (flags[FLAG_ERROR] & ERRBIT_CSR_RANGE) return;
    const int lane = threadIdx.x & 63;
    const int64_t j = blockIdx.x * (int64_t)(blockDim.x >> 6) + (threadIdx.x >> 6);
    if (j >= n) return;
    const int64_t e0 = colptr[j], e1 = colptr[j + 1];
    for (int64_t e = e0 + lane; e < e1; e += 64) {
        const int32_t row = rowidx_tmp[e];
        int64_t rank = 0;
        bool dup = false;
        for (int64_t f = e0; f < e1; ++f) {
            const int32_t other = rowidx_tmp[f];
            rank += other < row;
            dup |= (other == row && f != e);
        }
        if (dup) { atomicOr(&flags[FLAG_ERROR], ERRBIT_CSR_DUP); continue; }
        rowidx[e0 + rank] = row;
        cval[e0 + rank] = cval_tmp[e];
    }
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
// top-K rows by |r| (value descending, row ascending among equals)
// =========================================================================================
template <class T>
__device__ __forceinline__ bool topk_before(T a1, int32_t r1, T a2, int32_t r2) {
    return (a1 > a2) || (a1 == a2 && r1 < r2);
}

// TOPK rounds of block-wide arg-max over PER_THREAD candidates held per thread.
// Candidate with value < 0 is empty.  Thread 0 writes winner q to out_val[q], out_row[q]
// (value -1 / row -1 once the candidates run out).
template <class T, int PER_THREAD, int BLOCK>
__device__ void topk_rounds(T (&a)[PER_THREAD], int32_t (&row)[PER_THREAD], T* out_val,
                            int32_t* out_row) {
    constexpr int NW = BLOCK / 64;
    __shared__ T sh_a[2][NW];
    __shared__ int32_t sh_r[2][NW];
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    for (int round = 0; round < TOPK; ++round) {
        T ba = (T)-1;
        int32_t br = INT32_MAX;
#pragma unroll
        for (int q = 0; q < PER_THREAD; ++q)
            if (a[q] >= (T)0 && topk_before(a[q], row[q], ba, br)) { ba = a[q]; br = row[q]; }
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            T oa = __shfl_xor(ba, off, 64);
            int32_t orow = __shfl_xor(br, off, 64);
            if (topk_before(oa, orow, ba, br)) { ba = oa; br = orow; }
        }
        const int buf = round & 1;
        if (lane == 0) { sh_a[buf][w] = ba; sh_r[buf][w] = br; }
        __syncthreads();
        T wa = sh_a[buf][0];
        int32_t wr = sh_r[buf][0];
#pragma unroll
        for (int q = 1; q < NW; ++q)
            if (topk_before(sh_a[buf][q], sh_r[buf][q], wa, wr)) { wa = sh_a[buf][q]; wr = sh_r[buf][q]; }
        if (threadIdx.x == 0) {
            out_val[round] = wa;
            out_row[round] = wa >= (T)0 ? wr : -1;
        }
        // retire the winner (rows are unique among candidates)
#pragma unroll
        for (int q = 0; q < PER_THREAD; ++q)
            if (a[q] >= (T)0 && row[q] == wr && a[q] == wa) a[q] = (T)-1;
    }
}

template <class T>
__global__ __launch_bounds__(256) void k_topk_stage1(int64_t m, const T* __restrict__ r,
                                                     T* __restrict__ sval, int32_t* __restrict__ srow) {
    constexpr int PER = TOPK_GROUP / 256;
    T a[PER];
    int32_t row[PER];
    const int64_t base = blockIdx.x * (int64_t)TOPK_GROUP;
#pragma unroll
    for (int q = 0; q < PER; ++q) {
        int64_t i = base + q * 256 + threadIdx.x;
        a[q] = i < m ? dmmv_abs(r[i]) : (T)-1;
        row[q] = (int32_t)i;
    }
    topk_rounds<T, PER, 256>(a, row, sval + blockIdx.x * (int64_t)TOPK, srow + blockIdx.x * (int64_t)TOPK);
}

// single block: merge the stage-1 lists; also publishes t = largest |r| (0 when m = 0)
template <class T>
__global__ __launch_bounds__(256) void k_topk_stage2(int64_t ncand, const T* __restrict__ sval,
                                                     const int32_t* __restrict__ srow,
                                                     T* __restrict__ tval, int32_t* __restrict__ trow,
                                                     InstState<T>* st) {
    constexpr int PER = 8;   // candidates per thread per pass: 2048 per pass
    __shared__ T cur_val[TOPK];
    __shared__ int32_t cur_row[TOPK];
    __shared__ T new_val[TOPK];
    __shared__ int32_t new_row[TOPK];
    if (threadIdx.x < TOPK) { cur_val[threadIdx.x] = (T)-1; cur_row[threadIdx.x] = -1; }
    __syncthreads();
    for (int64_t base = 0; base < ncand; base += (PER - 1) * 256) {
        T a[PER];
        int32_t row[PER];
#pragma unroll
        for (int q = 0; q < PER - 1; ++q) {
            int64_t i = base + q * 256 + threadIdx.x;
            a[q] = i < ncand ? sval[i] : (T)-1;
            row[q] = i < ncand ? srow[i] : -1;
        }
        // the running list competes as the last candidate slot of the first TOPK threads
        a[PER - 1] = threadIdx.x < TOPK ? cur_val[threadIdx.x] : (T)-1;
        row[PER - 1] = threadIdx.x < TOPK ? cur_row[threadIdx.x] : -1;
        __syncthreads();
        topk_rounds<T, PER, 256>(a, row, new_val, new_row);
        __syncthreads();
        if (threadIdx.x < TOPK) { cur_val[threadIdx.x] = new_val[threadIdx.x]; cur_row[threadIdx.x] = new_row[threadIdx.x]; }
        __syncthreads();
    }
    if (threadIdx.x < TOPK) { tval[threadIdx.x] = cur_val[threadIdx.x]; trow[threadIdx.x] = cur_row[threadIdx.x]; }
    if (threadIdx.x == 0) st[0].t = cur_val[0] >= (T)0 ? cur_val[0] : (T)0;
}

// =========================================================================================
// evaluation: one wavefront per column, KT values of D per pass
// =========================================================================================
template <class T, int KT>
__global__ __launch_bounds__(256) void k_eval_csc(
    int64_t m, int64_t n, int32_t nd, const int64_t* __restrict__ colptr,
    const int32_t* __restrict__ rowidx, const T* __restrict__ cval, const T* __restrict__ D,
    const int32_t* __restrict__ kidx, const T* __restrict__ r, const T* __restrict__ topk_val,
    const int32_t* __restrict__ topk_row, int32_t radius, const uint8_t* __restrict__ var_mask,
    const InstState<T>* __restrict__ st, T* __restrict__ scores, Partial<T>* __restrict__ part) {
    __shared__ T sh_tv[TOPK];
    __shared__ int32_t sh_tr[TOPK];
    __shared__ T sh_s[4];
    __shared__ int64_t sh_c[4];
    if (part && !scores && st[0].done) return;
    if (threadIdx.x < TOPK) { sh_tv[threadIdx.x] = topk_val[threadIdx.x]; sh_tr[threadIdx.x] = topk_row[threadIdx.x]; }
    __syncthreads();
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    // number of valid list entries and the smallest listed value
    int32_t cnt = 0;
    for (int q = 0; q < TOPK; ++q) cnt += sh_tr[q] >= 0;
    const T thr = cnt > 0 ? sh_tv[cnt - 1] : Limits<T>::inf();
    const uint32_t full = cnt >= 32 ? 0xFFFFFFFFu : ((1u << cnt) - 1u);

    T bs = (T)0;
    int64_t bc = -1;
    constexpr int CPW = CSC_COLS_PER_BLOCK / 4;   // columns per wavefront
    for (int cc = 0; cc < CPW; ++cc) {
        const int64_t j = blockIdx.x * (int64_t)CSC_COLS_PER_BLOCK + w * CPW + cc;
        if (j >= n) break;                         // uniform per wavefront
        const int64_t e0 = colptr[j], e1 = colptr[j + 1];
        const int32_t kcur = kidx[j];
        const T dcur = D[kcur];
        const bool var_ok = var_mask ? var_mask[j] != 0 : true;
        T outside = (T)0;
        bool outside_known = false;
        for (int32_t k0 = 0; k0 < nd; k0 += KT) {
            T delta[KT], acc[KT];
#pragma unroll
            for (int q = 0; q < KT; ++q) {
                const int32_t k = k0 + q < nd ? k0 + q : nd - 1;
                delta[q] = step_of(D[k], dcur, (T)1);
                acc[q] = (T)0;
            }
            uint32_t mask = 0;
            for (int64_t e = e0 + lane; e < e1; e += 64) {
                const int32_t i = rowidx[e];
                const T a = cval[e];
                const T ri = r[i];
                if (!outside_known && dmmv_abs(ri) >= thr) {
                    for (int q = 0; q < cnt; ++q)
                        if (sh_tr[q] == i) mask |= 1u << q;
                }
#pragma unroll
                for (int q = 0; q < KT; ++q) acc[q] = dmmv_max(acc[q], dmmv_abs(dmmv_fma(delta[q], a, ri)));
            }
#pragma unroll
            for (int q = 0; q < KT; ++q) acc[q] = wave_max(acc[q]);
            if (!outside_known) {
                mask = wave_or(mask);
                const uint32_t missing = full & ~mask;
                if (missing) {
                    outside = sh_tv[__builtin_ctz(missing)];
                } else if ((int64_t)cnt >= m) {
                    outside = (T)0;                 // the column holds every row
                } else {
                    // every listed row is in this column: exact scan of the rows outside it
                    T o = (T)0;
                    for (int64_t i = lane; i < m; i += 64) {
                        int64_t lo = e0, hi = e1;  // binary search for row i in the column
                        while (lo < hi) {
                            int64_t mid = (lo + hi) >> 1;
                            if (rowidx[mid] < (int32_t)i) lo = mid + 1; else hi = mid;
                        }
                        const bool inside = lo < e1 && rowidx[lo] == (int32_t)i;
                        if (!inside) o = dmmv_max(o, dmmv_abs(r[i]));
                    }
                    outside = wave_max(o);
                }
                outside_known = true;
            }
            if (lane == 0) {
                for (int q = 0; q < KT; ++q) {
                    const int32_t k = k0 + q;
                    if (k >= nd) break;
                    T v = dmmv_max(acc[q], outside);
                    if (!cand_allowed(kcur, k, radius, var_ok)) v = Limits<T>::inf();
                    const int64_t cidx = j * (int64_t)nd + k;
                    if (scores) scores[cidx] = v;
                    if (rec_less(v, cidx, bs, bc)) { bs = v; bc = cidx; }
                }
            }
        }
    }
    if (part) {
        if (lane == 0) { sh_s[w] = bs; sh_c[w] = bc; }
        __syncthreads();
        if (threadIdx.x == 0) {
            T s = sh_s[0];
            int64_t c = sh_c[0];
            for (int q = 1; q < 4; ++q)
                if (rec_less(sh_s[q], sh_c[q], s, c)) { s = sh_s[q]; c = sh_c[q]; }
            Partial<T> p; p.s = s; p.c = c;
            part[blockIdx.x] = p;
        }
    }
}

// =========================================================================================
// apply: one block, the rows of column j
// =========================================================================================
template <class T>
__global__ void k_apply_csc(const int64_t* __restrict__ colptr, const int32_t* __restrict__ rowidx,
                            const T* __restrict__ cval, T* __restrict__ r, int32_t* __restrict__ kidx,
                            InstState<T>* st, int32_t t_from_score, int32_t iters, dmmv_move* trace,
                            T* trace_t) {
    const int32_t j = st[0].apply_j;
    if (j < 0) return;
    const T delta = st[0].delta;
    const int32_t k = st[0].apply_k;
    const T best_s = st[0].best_s;
    const int32_t moves = st[0].moves;
    __syncthreads();
    for (int64_t e = colptr[j] + threadIdx.x; e < colptr[j + 1]; e += blockDim.x) {
        const int32_t i = rowidx[e];
        r[i] = dmmv_fma(delta, cval[e], r[i]);
    }
    if (threadIdx.x == 0) {
        kidx[j] = k;
        if (t_from_score) {
            st[0].t = best_s;
            if (moves < iters) {
                if (trace) { trace[moves].j = j; trace[moves].k = k; }
                if (trace_t) trace_t[moves] = best_s;
            }
        }
        st[0].moves = moves + 1;
    }
}

// =========================================================================================
// host dispatch
// =========================================================================================
template <class T>
static dmmv_status build_t(Ctx* c) {
    const int64_t m = c->p.m, n = c->p.n, nnz = c->p.nnz;
    hipLaunchKernelGGL(k_csc_zero, dim3((unsigned)ceil_div(n + 1, 256)), dim3(256), 0, c->stream, c->colptr, n + 1);
    if (m > 0)
        hipLaunchKernelGGL(k_csc_count, dim3((unsigned)ceil_div(m, 256)), dim3(256), 0, c->stream, m, n, nnz, c->p.csr_rowptr, c->p.csr_col, c->colptr, c->flags);
    hipLaunchKernelGGL(k_csc_scan, dim3(1), dim3(1024), 0, c->stream, n, c->colptr, c->fillpos);
    if (m > 0)
        hipLaunchKernelGGL(k_csc_fill<T>, dim3((unsigned)ceil_div(m, 256)), dim3(256), 0, c->stream, m, n, c->p.csr_rowptr, c->p.csr_col, (const T*)c->p.csr_val, c->fillpos, c->rowidx_tmp, (T*)c->cval_tmp, (const int32_t*)c->flags);
    if (n > 0)
        hipLaunchKernelGGL(k_csc_sort<T>, dim3((unsigned)ceil_div(n, 4)), dim3(256), 0, c->stream, n, (const int64_t*)c->colptr, (const int32_t*)c->rowidx_tmp, (const T*)c->cval_tmp, c->rowidx, (T*)c->cval, c->flags);
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
static dmmv_status topk_t(Ctx* c) {
    const int64_t groups = c->topk_groups;
    hipLaunchKernelGGL(k_topk_stage1<T>, dim3((unsigned)groups), dim3(256), 0, c->stream, c->p.m, (const T*)c->r, (T*)c->topk_sval, c->topk_srow);
    hipLaunchKernelGGL(k_topk_stage2<T>, dim3(1), dim3(256), 0, c->stream, groups * TOPK, (const T*)c->topk_sval, (const int32_t*)c->topk_srow, (T*)c->topk_val, c->topk_row, (InstState<T>*)c->state);
    DMMV_LAUNCH_CHECK();
    return DMMV_OK;
}

template <class T>
static dmmv_status eval_t(Ctx* c, void* scores, bool want_partials) {
    const unsigned blocks = (unsigned)ceil_div(c->p.n, CSC_COLS_PER_BLOCK);
    if ((int64_t)blocks != c->n_partials) return fail(DMMV_ERR_STATE, "sparse evaluation grid does not match the partial-record buffer");
#define DMMV_EVAL_CSC(KT)                                                                            \
    hipLaunchKernelGGL((k_eval_csc<T, KT>), dim3(blocks), dim3(256), 0, c->stream, c->p.m, c->p.n,   \
                       c->p.nd, (const int64_t*)c->colptr, (const int32_t*)c->rowidx,                \
                       (const T*)c->cval, (const T*)c->D_dev, (const int32_t*)c->kidx,               \
                       (const T*)c->r, (const T*)c->topk_val, (const int32_t*)c->topk_row,           \
                       c->o.radius, c->o.var_mask, (const InstState<T>*)c->state, (T*)scores,        \
                       want_partials ? (Partial<T>*)c->partials : nullptr)
    if (c->p.nd <= 2) DMMV_EVAL_CSC(2);
    else if (c->p.nd <= 4) DMMV_EVAL_CSC(4);
    else DMMV_EVAL_CSC(8);
#undef DMMV_EVAL_CSC
    DMMV_LAUNCH_CHECK();
    return DMMV_OK;
}

template <class T>
static dmmv_status apply_t(Ctx* c, bool t_from_score, int32_t iters, dmmv_move* trace, void* trace_t) {
    hipLaunchKernelGGL(k_apply_csc<T>, dim3(1), dim3(256), 0, c->stream, (const int64_t*)c->colptr,
                       (const int32_t*)c->rowidx, (const T*)c->cval, (T*)c->r, c->kidx,
                       (InstState<T>*)c->state, (int32_t)t_from_score, iters, trace, (T*)trace_t);
    DMMV_LAUNCH_CHECK();
    return DMMV_OK;
}

dmmv_status csc_build(Ctx* c) { return c->p.dtype == DMMV_F64 ? build_t<double>(c) : build_t<float>(c); }
dmmv_status csc_residual(Ctx* c) { return c->p.dtype == DMMV_F64 ? residual_t<double>(c) : residual_t<float>(c); }
dmmv_status csc_refresh_topk(Ctx* c) { return c->p.dtype == DMMV_F64 ? topk_t<double>(c) : topk_t<float>(c); }
dmmv_status csc_eval(Ctx* c, void* scores_out, bool want_partials) {
    return c->p.dtype == DMMV_F64 ? eval_t<double>(c, scores_out, want_partials) : eval_t<float>(c, scores_out, want_partials);
}
dmmv_status csc_apply(Ctx* c, bool t_from_score, int32_t iters, dmmv_move* trace, void* trace_t) {
    return c->p.dtype == DMMV_F64 ? apply_t<double>(c, t_from_score, iters, trace, trace_t)
                                  : apply_t<float>(c, t_from_score, iters, trace, trace_t);
}

}  // namespace dmmv
