// Dense single-instance path: A column-major m x n.
//
// Layout: a column of A is one variable's move direction, so lanes map to consecutive rows
// and every load of A or r is a coalesced stream.  One workgroup scores one variable j for
// a tile of KT values of D: each lane keeps KT running maxima in registers, reads A_ij and
// r_i once per row, and the KT maxima are reduced over the wavefront with DPP row
// operations and over the workgroup through LDS.
#include "dmmv_common.h"

namespace dmmv {

// ---- residual: r_i = fma(sum_j fma-chain, 1, -b_i), lanes over rows (coalesced) ----------
template <class T>
__global__ void k_residual_dense(int64_t m, int64_t n, const T* __restrict__ A, int64_t lda,
                                 const T* __restrict__ D, const int32_t* __restrict__ kidx,
                                 const T* __restrict__ b, T* __restrict__ r) {
    int64_t i = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
    if (i >= m) return;
    T acc = (T)0;
    for (int64_t j = 0; j < n; ++j) acc = dmmv_fma(A[i + lda * j], D[kidx[j]], acc);
    r[i] = dmmv_fma(acc, (T)1, -b[i]);
}

// ---- evaluation ---------------------------------------------------------------------------
// grid.x = variable j, grid.y = tile of KT values.  Writes the table entries of its tile
// (scores != NULL) and one partial arg-min record (part != NULL).
template <class T, int KT, int BLOCK>
__global__ __launch_bounds__(BLOCK) void k_eval_dense(
    int64_t m, int32_t nd, const T* __restrict__ A, int64_t lda, const T* __restrict__ D,
    const int32_t* __restrict__ kidx, const T* __restrict__ r, int32_t radius,
    const uint8_t* __restrict__ var_mask, const InstState<T>* __restrict__ st,
    T* __restrict__ scores, Partial<T>* __restrict__ part) {
    constexpr int NW = BLOCK / 64;
    __shared__ T sh[NW][KT];
    if (part && !scores && st[0].done) return;
    const int64_t j = blockIdx.x;
    const int32_t k0 = blockIdx.y * KT;
    const int32_t kcur = kidx[j];
    const T dcur = D[kcur];
    T delta[KT], acc[KT];
#pragma unroll
    for (int q = 0; q < KT; ++q) {
        const int32_t k = k0 + q < nd ? k0 + q : nd - 1;
        delta[q] = step_of(D[k], dcur, (T)1);
        acc[q] = (T)0;
    }
    const T* __restrict__ col = A + lda * j;
    for (int64_t i = threadIdx.x; i < m; i += BLOCK) {
        const T a = col[i];
        const T ri = r[i];
#pragma unroll
        for (int q = 0; q < KT; ++q) acc[q] = dmmv_max(acc[q], dmmv_abs(dmmv_fma(delta[q], a, ri)));
    }
#pragma unroll
    for (int q = 0; q < KT; ++q) acc[q] = wave_max(acc[q]);
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    if (lane == 0) {
#pragma unroll
        for (int q = 0; q < KT; ++q) sh[w][q] = acc[q];
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        const bool var_ok = var_mask ? var_mask[j] != 0 : true;
        T bs = (T)0;
        int64_t bc = -1;
        for (int q = 0; q < KT; ++q) {
            const int32_t k = k0 + q;
            if (k >= nd) break;
            T v = sh[0][q];
            for (int ww = 1; ww < NW; ++ww) v = dmmv_max(v, sh[ww][q]);
            if (!cand_allowed(kcur, k, radius, var_ok)) v = Limits<T>::inf();
            const int64_t cidx = j * (int64_t)nd + k;
            if (scores) scores[cidx] = v;
            if (rec_less(v, cidx, bs, bc)) { bs = v; bc = cidx; }
        }
        if (part) {
            Partial<T> p; p.s = bs; p.c = bc;
            part[j * (int64_t)gridDim.y + blockIdx.y] = p;
        }
    }
}

// ---- apply the staged move: r_i <- fma(delta, A_ij, r_i); block 0 updates x, t, trace -----
template <class T>
__global__ void k_apply_dense(int64_t m, const T* __restrict__ A, int64_t lda, T* __restrict__ r,
                              int32_t* __restrict__ kidx, InstState<T>* st, int32_t t_from_score,
                              int32_t iters, dmmv_move* trace, T* trace_t) {
    const int32_t j = st[0].apply_j;
    if (j < 0) return;
    const T delta = st[0].delta;
    const int32_t k = st[0].apply_k;
    const T best_s = st[0].best_s;
    const int32_t moves = st[0].moves;
    const T* __restrict__ col = A + lda * (int64_t)j;
    for (int64_t i = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; i < m;
         i += (int64_t)gridDim.x * blockDim.x)
        r[i] = dmmv_fma(delta, col[i], r[i]);
    if (blockIdx.x == 0 && threadIdx.x == 0) {
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

// ---- host dispatch ---------------------------------------------------------------------------
template <class T>
static dmmv_status residual_t(Ctx* c) {
    if (c->p.m == 0) return DMMV_OK;
    hipLaunchKernelGGL(k_residual_dense<T>, dim3((unsigned)ceil_div(c->p.m, 256)), dim3(256), 0,
                       c->stream, c->p.m, c->p.n, (const T*)c->p.A_dense, c->p.lda,
                       (const T*)c->D_dev, (const int32_t*)c->kidx, (const T*)c->p.b, (T*)c->r);
    DMMV_LAUNCH_CHECK();
    return DMMV_OK;
}

template <class T, int KT>
static dmmv_status eval_launch(Ctx* c, void* scores, bool want_partials) {
    constexpr int BLOCK = 256;
    dim3 grid((unsigned)c->p.n, (unsigned)ceil_div(c->p.nd, KT));
    if ((int64_t)grid.x * grid.y != c->n_partials)
        return fail(DMMV_ERR_STATE, "dense evaluation grid does not match the partial-record buffer");
    hipLaunchKernelGGL((k_eval_dense<T, KT, BLOCK>), grid, dim3(BLOCK), 0, c->stream, c->p.m,
                       c->p.nd, (const T*)c->p.A_dense, c->p.lda, (const T*)c->D_dev,
                       (const int32_t*)c->kidx, (const T*)c->r, c->o.radius, c->o.var_mask,
                       (const InstState<T>*)c->state, (T*)scores,
                       want_partials ? (Partial<T>*)c->partials : nullptr);
    DMMV_LAUNCH_CHECK();
    return DMMV_OK;
}

template <class T>
static dmmv_status eval_t(Ctx* c, void* scores, bool want_partials) {
    switch (dense_ktile(c->p.nd)) {
        case 16: return eval_launch<T, 16>(c, scores, want_partials);
        case 8: return eval_launch<T, 8>(c, scores, want_partials);
        default: return eval_launch<T, 4>(c, scores, want_partials);
    }
}

template <class T>
static dmmv_status apply_t(Ctx* c, bool t_from_score, int32_t iters, dmmv_move* trace, void* trace_t) {
    int64_t blocks = ceil_div(c->p.m > 0 ? c->p.m : 1, 256);
    if (blocks > 1024) blocks = 1024;
    hipLaunchKernelGGL(k_apply_dense<T>, dim3((unsigned)blocks), dim3(256), 0, c->stream, c->p.m,
                       (const T*)c->p.A_dense, c->p.lda, (T*)c->r, c->kidx,
                       (InstState<T>*)c->state, (int32_t)t_from_score, iters, trace, (T*)trace_t);
    DMMV_LAUNCH_CHECK();
    return DMMV_OK;
}

dmmv_status dense_residual(Ctx* c) {
    return c->p.dtype == DMMV_F64 ? residual_t<double>(c) : residual_t<float>(c);
}
dmmv_status dense_eval(Ctx* c, void* scores_out, bool want_partials) {
    return c->p.dtype == DMMV_F64 ? eval_t<double>(c, scores_out, want_partials)
                                  : eval_t<float>(c, scores_out, want_partials);
}
dmmv_status dense_apply(Ctx* c, bool t_from_score, int32_t iters, dmmv_move* trace, void* trace_t) {
    return c->p.dtype == DMMV_F64 ? apply_t<double>(c, t_from_score, iters, trace, trace_t)
                                  : apply_t<float>(c, t_from_score, iters, trace, trace_t);
}

}  // namespace dmmv
