// Dense single-instance path: A column-major m x n.
//
// A column of A is one variable's move direction, so lanes map to consecutive rows and every
// load of A or r is a coalesced stream.  A workgroup scores one variable j for up to 64 values
// of D: it streams the column and r through two LDS buffers (the next row chunk is in flight
// in registers while the current one is scored), and each of its wavefronts keeps KT = 16
// running maxima per lane while striding over the staged rows.  The
// 16 x 64 lane maxima of a wavefront are reduced through an LDS transpose (each lane folds a
// quarter of one value's 64 entries, two DPP steps finish), so the reduction costs a few dozen
// instructions per 16 x m pairs.  The wavefronts' best candidates become one arg-min record
// per workgroup.
#include "dmmv_common.h"

namespace dmmv {

constexpr int DE_KT = 16;                 // values of D per wavefront
constexpr int DE_MAXW = 4;                // wavefronts (value tiles) per workgroup
constexpr int DE_PF = 4;                  // rows each thread stages per chunk (chunk = PF * threads)
constexpr int DE_SKEW = 65;               // row stride of the transpose scratch (bank skew)
constexpr int64_t DE_FUSED_APPLY_ROWS = 32768;   // up to here one workgroup selects AND applies

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
// grid.x = variable j, grid.y = group of NW value tiles (NW wavefronts per workgroup).  Writes the table entries
// of its values (scores != NULL) and one partial arg-min record (part != NULL).
template <class T, int NW>
__global__ __launch_bounds__(64 * NW) void k_eval_dense(
    int64_t m, int32_t nd, const T* __restrict__ A, int64_t lda,
    const T* __restrict__ D, const int32_t* __restrict__ kidx, const T* __restrict__ r,
    int32_t radius, const uint8_t* __restrict__ var_mask, const InstState<T>* __restrict__ st,
    int32_t honor_done, T* __restrict__ scores, Partial<T>* __restrict__ part) {
    constexpr int KT = DE_KT;
    constexpr int PF = DE_PF;
    extern __shared__ __align__(16) unsigned char smem[];
    constexpr int THREADS = 64 * NW;
    constexpr int rows_per_chunk = PF * THREADS;
    // two buffers of (column chunk, r chunk), rows_per_chunk rows each
    T* lds = reinterpret_cast<T*>(smem);
    __shared__ T sh_s[DE_MAXW];
    __shared__ int64_t sh_c[DE_MAXW];
    if (honor_done && st[0].done) return;
    const int lane = threadIdx.x & 63;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t j = blockIdx.x;
    const int32_t kbase = (blockIdx.y * NW + w) * KT;
    const int32_t kcur = kidx[j];
    const T dcur = D[kcur];
    T delta[KT], acc[KT];
#pragma unroll
    for (int q = 0; q < KT; ++q) {
        const int32_t k = kbase + q < nd ? kbase + q : nd - 1;
        delta[q] = step_of(D[k], dcur, (T)1);
        acc[q] = (T)0;
    }
    const T* __restrict__ col = A + lda * j;
    const int64_t n_chunks = (m + rows_per_chunk - 1) / rows_per_chunk;
    // Rows past m are staged as (a, r) = (0, 0): their |fma| is 0 and never raises a maximum.
    // The loads are unconditional on clamped rows so that a whole chunk is in flight at once.
    T pa[PF], pr[PF];
    auto fetch = [&](int64_t c0) {
#pragma unroll
        for (int u = 0; u < PF; ++u) {
            const int64_t i = c0 + u * THREADS + threadIdx.x;
            const int64_t ic = i < m ? i : m - 1;
            const T a = col[ic];
            const T x = r[ic];
            pa[u] = i < m ? a : (T)0;
            pr[u] = i < m ? x : (T)0;
        }
    };
    auto stash = [&](int buf) {
        T* la = lds + (size_t)buf * 2 * rows_per_chunk;
        T* lr = la + rows_per_chunk;
#pragma unroll
        for (int u = 0; u < PF; ++u) {
            la[u * THREADS + threadIdx.x] = pa[u];
            lr[u * THREADS + threadIdx.x] = pr[u];
        }
    };
    if (n_chunks > 0) {
        fetch(0);
        stash(0);
    }
    __syncthreads();
    for (int64_t ch = 0; ch < n_chunks; ++ch) {
        // rolling prefetch: the next chunk travels while this one is scored (the last pass
        // re-reads row m-1, which is harmless and keeps the loop free of branches)
        fetch((ch + 1) * rows_per_chunk);
        const T* la = lds + (size_t)(ch & 1) * 2 * rows_per_chunk;
        const T* lr = la + rows_per_chunk;
#pragma unroll
        for (int it = 0; it < PF * NW; ++it) {
            const T a = la[it * 64 + lane];
            const T ri = lr[it * 64 + lane];
#pragma unroll
            for (int q = 0; q < KT; ++q) acc[q] = dmmv_max(acc[q], dmmv_abs(dmmv_fma(delta[q], a, ri)));
        }
        stash((int)((ch + 1) & 1));
        __syncthreads();
    }
    // staging area is free (every wavefront passed the loop's last barrier): reuse it as scratch
    T* sc = reinterpret_cast<T*>(smem) + (size_t)w * KT * DE_SKEW;
#pragma unroll
    for (int q = 0; q < KT; ++q) sc[q * DE_SKEW + lane] = acc[q];
    __syncthreads();
    // lane folds a quarter (16 entries) of value q = lane / 4; two DPP steps join the quarters
    const int q = lane >> 2, quarter = lane & 3;
    T v = (T)0;
#pragma unroll
    for (int e = 0; e < 16; ++e) v = dmmv_max(v, sc[q * DE_SKEW + quarter * 16 + e]);
    v = dmmv_max(v, dpp_mov<DPP_QUAD_XOR1>(v));
    v = dmmv_max(v, dpp_mov<DPP_QUAD_XOR2>(v));
    const int32_t k = kbase + q;
    T bs = (T)0;
    int64_t bc = -1;
    if (quarter == 0 && k < nd) {
        const bool var_ok = var_mask ? var_mask[j] != 0 : true;
        if (!cand_allowed(kcur, k, radius, var_ok)) v = Limits<T>::inf();
        const int64_t cidx = j * (int64_t)nd + k;
        if (scores) scores[cidx] = v;
        bs = v;
        bc = cidx;
    }
    if (part) {
        block_argmin(bs, bc, sh_s, sh_c);
        if (threadIdx.x == 0) {
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

// ---- the loop's fused step for matrices of moderate height: one workgroup reduces the
// arg-min records, decides, and applies the move to r and x --------------------------------
template <class T>
__global__ __launch_bounds__(1024) void k_select_apply_dense(
    int64_t m, int32_t nd, const T* __restrict__ A, int64_t lda, const T* __restrict__ D,
    T* __restrict__ r, int32_t* __restrict__ kidx, const Partial<T>* __restrict__ part,
    int64_t n_part, InstState<T>* st, int32_t keep_going, int32_t iters, dmmv_move* trace,
    T* trace_t) {
    __shared__ T sh_s[16];
    __shared__ int64_t sh_c[16];
    __shared__ int32_t sh_j;
    __shared__ T sh_delta;
    if (st[0].done) return;
    T s = (T)0;
    int64_t c = -1;
    for (int64_t q = threadIdx.x; q < n_part; q += blockDim.x) {
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
    }
    __syncthreads();
    const int32_t j = sh_j;
    if (j < 0) return;
    const T delta = sh_delta;
    const T* __restrict__ col = A + lda * (int64_t)j;
    for (int64_t i = threadIdx.x; i < m; i += blockDim.x) r[i] = dmmv_fma(delta, col[i], r[i]);
}

// ---- host dispatch ---------------------------------------------------------------------------
static int dense_wavefronts(int64_t tiles) { return tiles <= 1 ? 1 : tiles == 2 ? 2 : DE_MAXW; }

int64_t dense_num_partials(const dmmv_problem& p) {
    const int64_t tiles = ceil_div(p.nd, DE_KT);
    return p.n * ceil_div(tiles, dense_wavefronts(tiles));
}

template <class T>
static dmmv_status residual_t(Ctx* c) {
    if (c->p.m == 0) return DMMV_OK;
    hipLaunchKernelGGL(k_residual_dense<T>, dim3((unsigned)ceil_div(c->p.m, 256)), dim3(256), 0,
                       c->stream, c->p.m, c->p.n, (const T*)c->p.A_dense, c->p.lda,
                       (const T*)c->D_dev, (const int32_t*)c->kidx, (const T*)c->p.b, (T*)c->r);
    DMMV_LAUNCH_CHECK();
    return DMMV_OK;
}

template <class T>
static dmmv_status eval_t(Ctx* c, void* scores, bool want_partials, bool honor_done) {
    const int64_t tiles = ceil_div(c->p.nd, DE_KT);
    const int nw = dense_wavefronts(tiles);
    dim3 grid((unsigned)c->p.n, (unsigned)ceil_div(tiles, nw));
    if ((int64_t)grid.x * grid.y != c->n_partials)
        return fail(DMMV_ERR_STATE, "dense evaluation grid does not match the partial-record buffer");
    if (grid.y > 65535) return fail(DMMV_ERR_UNSUPPORTED, "dense path: too many values of D for the launch grid");
    const int64_t rows = (int64_t)DE_PF * 64 * nw;           // two (column, r) buffers of this many rows
    size_t lds = (size_t)rows * 4 * sizeof(T);
    const size_t scratch = (size_t)nw * DE_KT * DE_SKEW * sizeof(T);
    if (lds < scratch) lds = scratch;                        // at most 33 KiB: no attribute needed
    auto launch = [&](auto kernel) {
        hipLaunchKernelGGL(kernel, grid, dim3(64 * nw), lds, c->stream, c->p.m, c->p.nd,
                           (const T*)c->p.A_dense, c->p.lda, (const T*)c->D_dev,
                           (const int32_t*)c->kidx, (const T*)c->r, c->o.radius, c->o.var_mask,
                           (const InstState<T>*)c->state, (int32_t)honor_done, (T*)scores,
                           want_partials ? (Partial<T>*)c->partials : nullptr);
    };
    if (nw == 1) launch(k_eval_dense<T, 1>);
    else if (nw == 2) launch(k_eval_dense<T, 2>);
    else launch(k_eval_dense<T, DE_MAXW>);
    DMMV_LAUNCH_CHECK();
    return DMMV_OK;
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

template <class T>
static dmmv_status select_apply_t(Ctx* c, int32_t iters, dmmv_move* trace, void* trace_t) {
    hipLaunchKernelGGL(k_select_apply_dense<T>, dim3(1), dim3(1024), 0, c->stream, c->p.m, c->p.nd,
                       (const T*)c->p.A_dense, c->p.lda, (const T*)c->D_dev, (T*)c->r, c->kidx,
                       (const Partial<T>*)c->partials, c->p.n > 0 ? c->n_partials : 0,
                       (InstState<T>*)c->state, c->o.keep_going, iters, trace, (T*)trace_t);
    DMMV_LAUNCH_CHECK();
    return DMMV_OK;
}

dmmv_status dense_residual(Ctx* c) {
    return c->p.dtype == DMMV_F64 ? residual_t<double>(c) : residual_t<float>(c);
}
dmmv_status dense_eval(Ctx* c, void* scores_out, bool want_partials, bool honor_done) {
    return c->p.dtype == DMMV_F64 ? eval_t<double>(c, scores_out, want_partials, honor_done)
                                  : eval_t<float>(c, scores_out, want_partials, honor_done);
}
dmmv_status dense_apply(Ctx* c, bool t_from_score, int32_t iters, dmmv_move* trace, void* trace_t) {
    return c->p.dtype == DMMV_F64 ? apply_t<double>(c, t_from_score, iters, trace, trace_t)
                                  : apply_t<float>(c, t_from_score, iters, trace, trace_t);
}
bool dense_has_fused_select_apply(const Ctx* c) { return c->p.m <= DE_FUSED_APPLY_ROWS; }
dmmv_status dense_select_apply(Ctx* c, int32_t iters, dmmv_move* trace, void* trace_t) {
    return c->p.dtype == DMMV_F64 ? select_apply_t<double>(c, iters, trace, trace_t)
                                  : select_apply_t<float>(c, iters, trace, trace_t);
}

}  // namespace dmmv
