// Swap move of the local search for sparse matrices (paper: section "Search Operators",
// Proposition 1 and Corollary 1; Appendix B "Swap Move", Algorithm 2).
//
// Same definition as for dense matrices: r'_k = fma(Delta, A_kj - A_ki, r_k) over all rows, the
// pair with the smallest t' = max_k |r'_k| (lowest pair number on a tie) if t' < t.  Rows
// stored in neither column keep their residual, so
//     t' = max( max over the rows of the two columns of |r'_k| ,  max over the other rows of |r_k| ).
//
// Filters (necessary conditions, so the result stays that of the full enumeration):
//  - the row k* of largest |r| must change, so one of the two variables has an entry in it:
//    a workgroup takes one such variable u (one per stored entry of row k*), its lanes the
//    partners v;
//  - the second term is known before any arithmetic: it is the residual of the first row, in
//    order of decreasing |r|, that neither column stores.  The reservoir of the rows of largest
//    |r| (rebuilt before the search) gives it with a few binary searches; a pair is dropped if
//    it reaches t or exceeds the best t' found so far by any workgroup;
//  - the walk over the two columns stops as soon as the running maximum does the same.
#include <cstring>
#include <limits>

#include "dmmv_sparse_common.h"

namespace dmmv {

namespace {

constexpr int SS_BLOCK = 256;
constexpr int SS_WAVES = SS_BLOCK / 64;

__device__ __forceinline__ unsigned long long ss_bits(float v) { return (unsigned long long)__float_as_uint(v); }
__device__ __forceinline__ unsigned long long ss_bits(double v) { return (unsigned long long)__double_as_longlong(v); }
__device__ __forceinline__ void ss_from_bits(unsigned long long b, float& v) { v = __uint_as_float((uint32_t)b); }
__device__ __forceinline__ void ss_from_bits(unsigned long long b, double& v) { v = __longlong_as_double((long long)b); }

// Cursor over the stored entries of one column, rows ascending: the segments of the column in
// partition order, the pads that end a segment skipped.  row = INT32_MAX past the end.
template <class T>
struct ColCursor {
    const int32_t* __restrict__ segptr;
    const uint16_t* __restrict__ row16;
    const T* __restrict__ cval;
    int64_t n, j;
    int32_t mp, P;
    int32_t p, e, e_end;
    int32_t row;
    T val;

    __device__ __forceinline__ ColCursor(const int32_t* sp, const uint16_t* r16, const T* cv, int64_t n_,
                                         int32_t mp_, int32_t P_, int64_t j_)
        : segptr(sp), row16(r16), cval(cv), n(n_), j(j_), mp(mp_), P(P_), p(-1), e(0), e_end(0),
          row(INT32_MAX), val((T)0) {
        advance();
    }
    __device__ __forceinline__ void advance() {
        for (;;) {
            if (e < e_end) {
                const uint32_t loc = row16[e];
                if (loc != (uint32_t)mp) {
                    row = p * mp + (int32_t)loc;
                    val = cval[e];
                    ++e;
                    return;
                }
                e = e_end;                                  // pads: the segment is over
            }
            ++p;
            if (p >= P) { row = INT32_MAX; val = (T)0; return; }
            e = segptr[(int64_t)p * n + j];
            e_end = segptr[(int64_t)p * n + j + 1];
        }
    }
};

__global__ void k_swap_csc_begin(unsigned long long* gbest, unsigned long long inf_bits) { gbest[0] = inf_bits; }

// ---- evaluation: grid (entries of the longest row, chunks of partners).  One record per
// workgroup.
template <class T>
__global__ __launch_bounds__(SS_BLOCK) void k_swap_eval_csc(
    int64_t m, int64_t n, int32_t mp, int32_t P, const int64_t* __restrict__ rowptr,
    const int32_t* __restrict__ col, const int32_t* __restrict__ segptr,
    const uint16_t* __restrict__ row16, const T* __restrict__ cval, const T* __restrict__ D,
    const int32_t* __restrict__ kidx, const T* __restrict__ r, const InstState<T>* __restrict__ st,
    const uint8_t* __restrict__ vm, const T* __restrict__ res_val, const int32_t* __restrict__ res_row,
    const int32_t* __restrict__ res_meta, const int32_t* __restrict__ skip,
    unsigned long long* __restrict__ gbest, Partial<T>* __restrict__ part) {
    __shared__ T sh_rv[RES_CAP];
    __shared__ int32_t sh_rr[RES_CAP];
    __shared__ uint8_t sh_uhas[RES_CAP];
    __shared__ unsigned long long sh_best;
    __shared__ T sh_s[SS_WAVES];
    __shared__ int64_t sh_c[SS_WAVES];
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    Partial<T>* out = part + (int64_t)blockIdx.y * gridDim.x + blockIdx.x;
    Partial<T> empty;
    empty.s = (T)0;
    empty.c = -1;
    const int32_t cnt = res_meta[RES_CNT];
    bool idle = (skip && skip[0]) || cnt <= 0;
    int64_t u = 0;
    if (!idle) {
        const int32_t kstar = res_row[0];
        const int64_t e0 = rowptr[kstar], e1 = rowptr[kstar + 1];
        if ((int64_t)blockIdx.x >= e1 - e0) idle = true;
        else u = col[e0 + blockIdx.x];
    }
    if (!idle && vm && !vm[u]) idle = true;
    if (idle) {
        if (threadIdx.x == 0) *out = empty;
        return;
    }
    if ((int32_t)threadIdx.x < cnt) {
        const int32_t row = res_row[threadIdx.x];
        sh_rr[threadIdx.x] = row;
        sh_rv[threadIdx.x] = res_val[threadIdx.x];
        sh_uhas[threadIdx.x] = column_has_row<T>(segptr, row16, n, mp, u, row) ? 1 : 0;
    }
    if (threadIdx.x == 0) sh_best = ss_bits(Limits<T>::inf());
    __syncthreads();

    const T t = st[0].t;
    const T dvu = D[kidx[u]];
    T best_t = Limits<T>::inf();                           // this lane's record
    int64_t best_c = -1;

    for (int64_t v0 = ((int64_t)blockIdx.y * SS_WAVES + w) * 64; v0 < n; v0 += (int64_t)gridDim.y * SS_BLOCK) {
        const int64_t v = v0 + lane;
        bool alive = false;
        T Ds = (T)0, dvv = (T)0;
        if (v < n && v != u) {
            dvv = D[kidx[v]];
            alive = dvu != dvv && (!vm || vm[v]);
            if (dvu > dvv) { const T diff = dvu - dvv; Ds = diff; }             // scale 1: Delta = 1 * diff
            else { const T diff = dvv - dvu; Ds = -diff; }
        }
        if (!__any(alive)) continue;
        T gb, sb;
        ss_from_bits(__atomic_load_n(gbest, __ATOMIC_RELAXED), gb);
        ss_from_bits(__hip_atomic_load(&sh_best, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP), sb);
        const T bnd = dmmv_min(best_t, dmmv_min(gb, sb));
        // residual that stays: the first row, by decreasing |r|, stored in neither column
        T outside = (T)0;
        bool scan = false;
        if (alive) {
            int32_t e = 0;
            for (; e < cnt; ++e) {
                if (sh_uhas[e]) continue;
                if (!column_has_row<T>(segptr, row16, n, mp, v, sh_rr[e])) break;
            }
            if (e < cnt) outside = sh_rv[e];
            else if ((int64_t)cnt >= m) outside = (T)0;     // the two columns store every row
            else scan = true;
            if (!scan) alive = outside < t && !(outside > bnd);
        }
        // rare: the two columns store every row of the reservoir; the wavefront scans all rows
        unsigned long long todo = __ballot(alive && scan);
        while (todo) {
            const int src = __builtin_ctzll(todo);
            todo &= todo - 1;
            const int64_t sv = v0 + src;
            T o = (T)0;
            for (int64_t i = lane; i < m; i += 64)
                if (!column_has_row<T>(segptr, row16, n, mp, u, (int32_t)i) &&
                    !column_has_row<T>(segptr, row16, n, mp, sv, (int32_t)i))
                    o = dmmv_max(o, dmmv_abs(r[i]));
            o = wave_max(o);
            if (lane == src) {
                outside = o;
                alive = outside < t && !(outside > bnd);
            }
        }
        if (alive) {
            ColCursor<T> cu(segptr, row16, cval, n, mp, P, u), cv(segptr, row16, cval, n, mp, P, v);
            T mx = outside;
            while (cu.row != INT32_MAX || cv.row != INT32_MAX) {
                const int32_t k = cu.row < cv.row ? cu.row : cv.row;
                const T au = cu.row == k ? cu.val : (T)0;
                const T av = cv.row == k ? cv.val : (T)0;
                mx = dmmv_max(mx, dmmv_abs(dmmv_fma(Ds, av - au, r[k])));
                if (!(mx < t) || mx > bnd) { alive = false; break; }
                if (cu.row == k) cu.advance();
                if (cv.row == k) cv.advance();
            }
            if (alive && mx < t) {
                const int64_t c = dvu > dvv ? u * n + v : v * n + u;
                if (rec_less(mx, c, best_t, best_c)) {
                    best_t = mx;
                    best_c = c;
                    atomicMin(&sh_best, ss_bits(mx));
                    atomicMin(gbest, ss_bits(mx));
                }
            }
        }
    }
    block_argmin(best_t, best_c, sh_s, sh_c);
    if (threadIdx.x == 0) {
        Partial<T> p;
        p.s = best_c < 0 ? (T)0 : best_t;
        p.c = best_c;
        *out = p;
    }
}

// ---- reduce the records, report, carry the swap out.  One workgroup.
template <class T>
__global__ __launch_bounds__(SS_BLOCK) void k_swap_apply_csc(
    int64_t n, int32_t mp, int32_t P, int64_t n_rec, int32_t apply, const int32_t* __restrict__ segptr,
    const uint16_t* __restrict__ row16, const T* __restrict__ cval, const T* __restrict__ D,
    int32_t* __restrict__ kidx, T* __restrict__ r, InstState<T>* __restrict__ st,
    const Partial<T>* __restrict__ part, int32_t* __restrict__ skip, int32_t mark_skip,
    dmmv_swap* __restrict__ best_out, T* __restrict__ best_t_out) {
    __shared__ T sh_s[SS_WAVES];
    __shared__ int64_t sh_c[SS_WAVES];
    if (skip && skip[0]) {
        if (threadIdx.x == 0) {
            if (best_out) { best_out[0].i = -1; best_out[0].j = -1; }
            if (best_t_out) best_t_out[0] = st[0].t;
        }
        return;
    }
    T s = (T)0;
    int64_t c = -1;
    for (int64_t e = threadIdx.x; e < n_rec; e += SS_BLOCK) {
        const Partial<T> p = part[e];
        if (rec_less(p.s, p.c, s, c)) { s = p.s; c = p.c; }
    }
    block_argmin(s, c, sh_s, sh_c);
    if (threadIdx.x != 0) return;
    if (best_out) { best_out[0].i = c < 0 ? -1 : c / n; best_out[0].j = c < 0 ? -1 : c % n; }
    if (best_t_out) best_t_out[0] = c < 0 ? st[0].t : s;
    if (c < 0 && skip && mark_skip) skip[0] = 1;
    if (c < 0 || !apply) return;
    const int64_t i = c / n, j = c % n;
    const int32_t ki = kidx[i], kj = kidx[j];
    const T Delta = D[ki] - D[kj];                         // scale 1
    ColCursor<T> ci(segptr, row16, cval, n, mp, P, i), cj(segptr, row16, cval, n, mp, P, j);
    while (ci.row != INT32_MAX || cj.row != INT32_MAX) {
        const int32_t k = ci.row < cj.row ? ci.row : cj.row;
        const T ai = ci.row == k ? ci.val : (T)0;
        const T aj = cj.row == k ? cj.val : (T)0;
        r[k] = dmmv_fma(Delta, aj - ai, r[k]);
        if (ci.row == k) ci.advance();
        if (cj.row == k) cj.advance();
    }
    kidx[i] = kj;
    kidx[j] = ki;
    st[0].t = s;
    st[0].moves += 1;
}

template <class T>
dmmv_status swap_csc_t(Ctx* c, int32_t apply, bool use_skip, dmmv_swap* best, void* best_t) {
    const int64_t n = c->p.n, m = c->p.m;
    DMMV_TRY(csc_reservoir(c));
    int32_t* skip = use_skip ? c->swap_skip : nullptr;
    const T inf = std::numeric_limits<T>::infinity();
    unsigned long long inf_bits = 0;
    memcpy(&inf_bits, &inf, sizeof(T));
    hipLaunchKernelGGL(k_swap_csc_begin, dim3(1), dim3(1), 0, c->stream, c->swap_gbest, inf_bits);
    const int64_t X = c->csc_max_row > 0 ? c->csc_max_row : 1;
    int64_t Y = 4096 / X;
    if (Y > ceil_div(n, SS_BLOCK)) Y = ceil_div(n, SS_BLOCK);
    if (Y < 1) Y = 1;
    hipLaunchKernelGGL(k_swap_eval_csc<T>, dim3((unsigned)X, (unsigned)Y), dim3(SS_BLOCK), 0, c->stream, m, n,
                       c->csc_mp, c->csc_P, c->p.csr_rowptr, c->p.csr_col, (const int32_t*)c->segptr,
                       (const uint16_t*)c->row16, (const T*)c->cval, (const T*)c->D_dev, (const int32_t*)c->kidx,
                       (const T*)c->r, (const InstState<T>*)c->state, c->o.var_mask, (const T*)c->res_val,
                       (const int32_t*)c->res_row, (const int32_t*)c->res_meta, (const int32_t*)skip,
                       c->swap_gbest, (Partial<T>*)c->swap_part);
    hipLaunchKernelGGL(k_swap_apply_csc<T>, dim3(1), dim3(SS_BLOCK), 0, c->stream, n, c->csc_mp, c->csc_P, X * Y,
                       apply, (const int32_t*)c->segptr, (const uint16_t*)c->row16, (const T*)c->cval,
                       (const T*)c->D_dev, c->kidx, (T*)c->r, (InstState<T>*)c->state,
                       (const Partial<T>*)c->swap_part, skip, use_skip ? 1 : 0, best, (T*)best_t);
    DMMV_LAUNCH_CHECK();
    if (apply) DMMV_TRY(csc_reservoir(c));
    return DMMV_OK;
}

}  // namespace

int64_t swap_csc_records(const dmmv_problem& p) { return (p.n > 4096 ? p.n : 4096) + 1; }

dmmv_status swap_move_csc(Ctx* c, int32_t apply, bool use_skip, dmmv_swap* best, void* best_t) {
    if (!c->swap_skip || !c->swap_part || !c->swap_gbest)
        return fail(DMMV_ERR_STATE, "swap move: workspace of the sparse swap is missing");
    return c->p.dtype == DMMV_F64 ? swap_csc_t<double>(c, apply, use_skip, best, best_t)
                                  : swap_csc_t<float>(c, apply, use_skip, best, best_t);
}

}  // namespace dmmv
