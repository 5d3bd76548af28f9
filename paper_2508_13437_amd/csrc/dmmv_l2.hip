// The l2 side of a move: change of the squared l2 norm of the residual for every candidate, and the
// arg-min that uses it as second criterion (options.l2_rule).
//
// Paper: section "GPU Acceleration" evaluates the l-infinity and the l2 change of the candidates
// together before the tensor-wide argmin; the quantisation use case checks that the l2 norm does
// not increase (section "Experiment setup and results").  For the move x_j -> D[k] with step delta
// the new residual is r + delta a_j (Appendix A with one basis vector), so
//     dq(j, k) = ||r + delta a_j||^2 - ||r||^2 = 2 delta (a_j . r) + delta^2 ||a_j||^2 .
// Arithmetic contract (what makes the second criterion reproducible bit for bit):
//     g_j = a_j . r   : acc = 0; over the stored entries of column j by ascending row:
//                       acc = fma(A_ij, r_i, acc)
//     c_j = ||a_j||^2 : the same chain with fma(A_ij, A_ij, acc)      (once, at create)
//     dq(j, k)        = delta * fma(delta, c_j, 2 g_j)
// For a batch g is the matrix G = X^T R_mat (n x R), a dense contraction: on fp32 batches it runs on
// the matrix cores in the form that keeps the chain, v_mfma_f32_32x32x1_2b_f32 with K = 1 (one fused
// multiply-add per element and instruction, rows in ascending order), so G carries the same bits
// as the chain on the vector unit.
#include "dmmv_common.h"
#include "dmmv_sparse_common.h"

namespace dmmv {

namespace {

typedef __attribute__((__vector_size__(32 * sizeof(float)))) float floatx32;

// ---- column sums of squares, once per handle ------------------------------------------------
template <class T>
__global__ void k_l2_colsq_dense(int64_t m, int64_t n, const T* __restrict__ A, int64_t lda, T* __restrict__ csq) {
    const int64_t j = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
    if (j >= n) return;
    const T* __restrict__ col = A + lda * j;
    T acc = (T)0;
    for (int64_t i = 0; i < m; ++i) acc = dmmv_fma(col[i], col[i], acc);
    csq[j] = acc;
}

// sparse: the segments of a column in ascending partition hold its entries by ascending row; a
// pad has value 0 and adds nothing to either chain
template <class T>
__global__ void k_l2_sums_csc(int64_t m, int64_t n, int32_t mp, int32_t P, const int32_t* __restrict__ segptr,
                              const uint16_t* __restrict__ row16, const T* __restrict__ cval,
                              const T* __restrict__ r, T* __restrict__ g, T* __restrict__ csq) {
    const int64_t j = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
    if (j >= n) return;
    T acc = (T)0, sq = (T)0;
    for (int32_t p = 0; p < P; ++p) {
        const int32_t e0 = segptr[(int64_t)p * n + j], e1 = segptr[(int64_t)p * n + j + 1];
        for (int32_t e = e0; e < e1; ++e) {
            const uint32_t loc = row16[e];
            if (loc == (uint32_t)mp) continue;
            const T a = cval[e];
            if (g) acc = dmmv_fma(a, r[(int64_t)p * mp + loc], acc);
            if (csq) sq = dmmv_fma(a, a, sq);
        }
    }
    if (g) g[j] = acc;
    if (csq) csq[j] = sq;
}

// ---- g = A^T r -------------------------------------------------------------------------------
template <class T>
__global__ void k_l2_g_dense(int64_t m, int64_t n, const T* __restrict__ A, int64_t lda, const T* __restrict__ r,
                             T* __restrict__ g) {
    const int64_t j = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
    if (j >= n) return;
    const T* __restrict__ col = A + lda * j;
    T acc = (T)0;
    for (int64_t i = 0; i < m; ++i) acc = dmmv_fma(col[i], r[i], acc);
    g[j] = acc;
}

// Batch, vector unit: lane = instance, TJ columns per lane and pass; r is read coalesced over the
// instances, the row of X is the same for every lane (row-major copy, read through the scalar unit).
template <class T, int TJ>
__global__ __launch_bounds__(256) void k_l2_g_batched(int64_t m, int64_t n, int64_t R, const T* __restrict__ Xt,
                                                      const T* __restrict__ r, T* __restrict__ G) {
    const int64_t q = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
    const int64_t j0 = blockIdx.y * (int64_t)TJ;
    const int64_t qc = q < R ? q : R - 1;
    T acc[TJ];
#pragma unroll
    for (int u = 0; u < TJ; ++u) acc[u] = (T)0;
    for (int64_t i = 0; i < m; ++i) {
        const T ri = r[i * R + qc];
        const T* __restrict__ xr = Xt + i * n;
#pragma unroll
        for (int u = 0; u < TJ; ++u) {
            const int64_t j = j0 + u < n ? j0 + u : n - 1;
            acc[u] = dmmv_fma(xr[j], ri, acc[u]);
        }
    }
    if (q < R) {
#pragma unroll
        for (int u = 0; u < TJ; ++u)
            if (j0 + u < n) G[(j0 + u) * R + q] = acc[u];
    }
}

// Batch, matrix cores (fp32).  One wavefront owns a 128 x 64 tile of G (variables x instances) as
// four 2 x (32 x 32) accumulators; row i of the contraction is ONE instruction per accumulator:
//     D = a b^T + C,  a = X[i][64 variables] (lane l: variable l of the tile's half),
//                     b = r[i][32 instances] (lane l: instance l % 32),
// each element one fused multiply-add rounded once, so after row i an accumulator holds exactly
// the chain fma(X_ij, r_iq, .) over the rows 0..i.  Lane l receives, in register v, block v / 16
// (variables 32 (v / 16) ...), instance l % 32 and variable row 8 ((v % 16) / 4) + 4 (l / 32) + v % 4
// of the block.  The operands of the next L2_U rows are loaded before the products of the
// current ones are issued.
constexpr int L2_U = 6;

__global__ __launch_bounds__(256, 2) void k_l2_g_mfma(int64_t m, int64_t n, int64_t R, const float* __restrict__ Xt,
                                                      const float* __restrict__ r, float* __restrict__ G) {
    const int lane = threadIdx.x & 63;
    const int w = threadIdx.x >> 6;
    const int64_t j0 = (blockIdx.x * 2ll + (w & 1)) * 128;
    const int64_t q0 = (blockIdx.y * 2ll + (w >> 1)) * 64;
    if (j0 >= n || q0 >= R) return;                       // whole wavefronts only
    // Vector instructions do not overlap with the matrix cores' (measured: every one of them adds
    // its issue time to the loop), so the loop is written to need none: a row's address is a
    // uniform pointer (scalar unit) plus an unsigned 32-bit lane offset that never changes, and two sets
    // of operand registers take turns, so nothing is copied.
    // (byte offsets inside X and r, 32-bit: the host takes this kernel when both are below 4 GiB)
    const uint32_t ja = 4u * (uint32_t)(j0 + lane < n ? j0 + lane : n - 1);
    const uint32_t jb = 4u * (uint32_t)(j0 + 64 + lane < n ? j0 + 64 + lane : n - 1);
    const uint32_t qa = 4u * (uint32_t)(q0 + (lane & 31) < R ? q0 + (lane & 31) : R - 1);
    const uint32_t qb = 4u * (uint32_t)(q0 + 32 + (lane & 31) < R ? q0 + 32 + (lane & 31) : R - 1);
    floatx32 c00, c01, c10, c11;
#pragma unroll
    for (int v = 0; v < 32; ++v) { c00[v] = 0.0f; c01[v] = 0.0f; c10[v] = 0.0f; c11[v] = 0.0f; }
    const int32_t mrows = (int32_t)m;                       // rows are counted on the scalar unit
    float pa0[L2_U], pa1[L2_U], pb0[L2_U], pb1[L2_U];       // set P
    float qa0[L2_U], qa1[L2_U], qb0[L2_U], qb1[L2_U];       // set Q
    // raw buffer loads: address = descriptor base + scalar row offset + lane offset, no vector
    // instruction involved (a 64-bit global address would cost one vector add per load)
    const __amdgpu_buffer_rsrc_t rs_x = __builtin_amdgcn_make_buffer_rsrc((void*)Xt, 0, (int)(uint32_t)(m * n * 4), 0x00020000);
    const __amdgpu_buffer_rsrc_t rs_r = __builtin_amdgcn_make_buffer_rsrc((void*)r, 0, (int)(uint32_t)(m * R * 4), 0x00020000);
    const uint32_t xstride = (uint32_t)n * 4u, rstride = (uint32_t)R * 4u;
#define L2_AT(rs, off, soff) __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(rs, (int)(off), (int)(soff), 0))
#define L2_LOAD(A0, A1, B0, B1, I0)                                         \
    _Pragma("unroll") for (int u = 0; u < L2_U; ++u) {                       \
        const uint32_t i = (uint32_t)((I0) + u < mrows ? (I0) + u : mrows - 1); \
        A0[u] = L2_AT(rs_x, ja, i * xstride);                                \
        A1[u] = L2_AT(rs_x, jb, i * xstride);                                \
        B0[u] = L2_AT(rs_r, qa, i * rstride);                                \
        B1[u] = L2_AT(rs_r, qb, i * rstride);                                \
    }
#define L2_ROWS(A0, A1, B0, B1, I0)                                                      \
    _Pragma("unroll") for (int u = 0; u < L2_U; ++u) {                                    \
        if ((I0) + u < mrows) { /* uniform */                                             \
            c00 = __builtin_amdgcn_mfma_f32_32x32x1f32(A0[u], B0[u], c00, 0, 0, 0);        \
            c01 = __builtin_amdgcn_mfma_f32_32x32x1f32(A0[u], B1[u], c01, 0, 0, 0);        \
            c10 = __builtin_amdgcn_mfma_f32_32x32x1f32(A1[u], B0[u], c10, 0, 0, 0);        \
            c11 = __builtin_amdgcn_mfma_f32_32x32x1f32(A1[u], B1[u], c11, 0, 0, 0);        \
        }                                                                                 \
    }
    if (mrows > 0) { L2_LOAD(pa0, pa1, pb0, pb1, 0) }
    for (int32_t i0 = 0; i0 < mrows; i0 += 2 * L2_U) {
        if (i0 + L2_U < mrows) { L2_LOAD(qa0, qa1, qb0, qb1, i0 + L2_U) }
        L2_ROWS(pa0, pa1, pb0, pb1, i0)
        if (i0 + 2 * L2_U < mrows) { L2_LOAD(pa0, pa1, pb0, pb1, i0 + 2 * L2_U) }
        L2_ROWS(qa0, qa1, qb0, qb1, i0 + L2_U)
    }
#undef L2_LOAD
#undef L2_ROWS
#undef L2_AT
    const int half = lane >> 5, col = lane & 31;
#pragma unroll
    for (int v = 0; v < 32; ++v) {
        const int row = 32 * (v / 16) + 8 * ((v % 16) / 4) + 4 * half + v % 4;   // variable inside a 64-wide operand
        const int64_t jlo = j0 + row, jhi = j0 + 64 + row;
        const int64_t qlo = q0 + col, qhi = q0 + 32 + col;
        if (jlo < n && qlo < R) G[jlo * R + qlo] = c00[v];
        if (jlo < n && qhi < R) G[jlo * R + qhi] = c01[v];
        if (jhi < n && qlo < R) G[jhi * R + qlo] = c10[v];
        if (jhi < n && qhi < R) G[jhi * R + qhi] = c11[v];
    }
}

// ---- the table dq[q][j*nd + k] -----------------------------------------------------------------
template <class T>
__device__ __forceinline__ T l2_change(T delta, T csq, T g) {
    const T twog = (T)2 * g;
    return delta * dmmv_fma(delta, csq, twog);
}

// one thread per (instance, variable); g and kidx are [n][R]
template <class T>
__global__ void k_l2_table(int64_t n, int64_t R, int32_t nd, const T* __restrict__ D, const T* __restrict__ scale,
                           const int32_t* __restrict__ kidx, const T* __restrict__ g, const T* __restrict__ csq,
                           T* __restrict__ dq) {
    const int64_t t = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
    if (t >= n * R) return;
    const int64_t q = t % R, j = t / R;
    const T sc = scale[q], dcur = D[kidx[j * R + q]], gj = g[j * R + q], cj = csq[j];
    T* __restrict__ out = dq + q * (n * (int64_t)nd) + j * nd;
    for (int32_t k = 0; k < nd; ++k) out[k] = l2_change(step_of(D[k], dcur, sc), cj, gj);
}

// ---- arg-min of a score table with dq as second criterion, one workgroup per instance ----------
template <class T>
__device__ __forceinline__ bool rec3_less(T s1, T q1, int64_t c1, T s2, T q2, int64_t c2) {
    if (c1 < 0) return false;
    if (c2 < 0) return true;
    if (s1 != s2) return s1 < s2;
    if (q1 != q2) return q1 < q2;
    return c1 < c2;
}

template <class T>
__global__ __launch_bounds__(1024) void k_l2_select(int64_t n, int64_t R, int32_t nd, int32_t rule,
                                                    const T* __restrict__ scores, const T* __restrict__ D,
                                                    const T* __restrict__ scale, const int32_t* __restrict__ kidx,
                                                    const T* __restrict__ g, const T* __restrict__ csq,
                                                    InstState<T>* st, int32_t keep_going, dmmv_move* best_out,
                                                    T* best_score_out) {
    __shared__ T sh_s[16], sh_q[16];
    __shared__ int64_t sh_c[16];
    const int64_t q = blockIdx.x;
    InstState<T> z = st[q];
    if (z.done && !best_out) return;
    const T sc = scale[q];
    const T* __restrict__ tab = scores + q * (n * (int64_t)nd);
    T bs = (T)0, bq = (T)0;
    int64_t bc = -1;
    for (int64_t e = threadIdx.x; e < n * (int64_t)nd; e += blockDim.x) {
        const int64_t j = e / nd;
        const int32_t k = (int32_t)(e - j * nd);
        const T dq = l2_change(step_of(D[k], D[kidx[j * R + q]], sc), csq[j], g[j * R + q]);
        if (rule == 2 && !(dq <= (T)0)) continue;
        const T s = tab[e];
        if (rec3_less(s, dq, e, bs, bq, bc)) { bs = s; bq = dq; bc = e; }
    }
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const T os = __shfl_xor(bs, off, 64), oq = __shfl_xor(bq, off, 64);
        const int64_t oc = (int64_t)__shfl_xor((long long)bc, off, 64);
        if (rec3_less(os, oq, oc, bs, bq, bc)) { bs = os; bq = oq; bc = oc; }
    }
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6, nw = (blockDim.x + 63) >> 6;
    if (lane == 0) { sh_s[w] = bs; sh_q[w] = bq; sh_c[w] = bc; }
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int u = 1; u < nw; ++u)
            if (rec3_less(sh_s[u], sh_q[u], sh_c[u], bs, bq, bc)) { bs = sh_s[u]; bq = sh_q[u]; bc = sh_c[u]; }
        int32_t j = -1, k = -1;
        if (bc >= 0) { j = (int32_t)(bc / nd); k = (int32_t)(bc % nd); }
        const bool improving = bc >= 0 && bs < z.t;
        z.best_s = bs;
        z.apply_j = improving ? j : -1;
        z.apply_k = improving ? k : -1;
        z.delta = improving ? step_of(D[k], D[kidx[(int64_t)j * R + q]], sc) : (T)0;
        if (!improving && !keep_going) z.done = 1;
        st[q] = z;
        if (best_out) { best_out[q].j = j; best_out[q].k = k; }
        if (best_score_out) best_score_out[q] = bc >= 0 ? bs : Limits<T>::inf();
    }
}

// sparse: what the loop's fused select-and-apply kernel does besides the update of r
template <class T>
__global__ void k_l2_after_apply_csc(InstState<T>* st, int32_t applied_before, int32_t iters, dmmv_move* trace,
                                     T* trace_t) {
    InstState<T> z = st[0];
    if (z.apply_j < 0) return;
    (void)applied_before;
    z.t = z.best_s;
    const int32_t slot = z.moves - 1;                     // the apply kernel has counted the move
    if (slot >= 0 && slot < iters) {
        if (trace) { trace[slot].j = z.apply_j; trace[slot].k = z.apply_k; }
        if (trace_t) trace_t[slot] = z.best_s;
    }
    st[0] = z;
}

template <class T>
dmmv_status colsq_t(Ctx* c) {
    const int64_t n = c->p.n;
    if (n == 0) return DMMV_OK;
    const dim3 grid((unsigned)ceil_div(n, 64));
    if (c->kind == KIND_CSC)
        hipLaunchKernelGGL(k_l2_sums_csc<T>, grid, dim3(64), 0, c->stream, c->p.m, n, c->csc_mp, c->csc_P,
                           (const int32_t*)c->segptr, (const uint16_t*)c->row16, (const T*)c->cval, (const T*)nullptr,
                           (T*)nullptr, (T*)c->l2_c);
    else
        hipLaunchKernelGGL(k_l2_colsq_dense<T>, grid, dim3(64), 0, c->stream, c->p.m, n, (const T*)c->p.A_dense,
                           c->p.lda, (T*)c->l2_c);
    DMMV_LAUNCH_CHECK();
    return DMMV_OK;
}

template <class T>
dmmv_status update_g_t(Ctx* c) {
    const int64_t m = c->p.m, n = c->p.n, R = c->p.R;
    if (n == 0) return DMMV_OK;
    if (c->kind == KIND_CSC) {
        hipLaunchKernelGGL(k_l2_sums_csc<T>, dim3((unsigned)ceil_div(n, 64)), dim3(64), 0, c->stream, m, n, c->csc_mp,
                           c->csc_P, (const int32_t*)c->segptr, (const uint16_t*)c->row16, (const T*)c->cval,
                           (const T*)c->r, (T*)c->l2_g, (T*)nullptr);
    } else if (c->kind == KIND_DENSE) {
        hipLaunchKernelGGL(k_l2_g_dense<T>, dim3((unsigned)ceil_div(n, 64)), dim3(64), 0, c->stream, m, n,
                           (const T*)c->p.A_dense, c->p.lda, (const T*)c->r, (T*)c->l2_g);
    } else if (sizeof(T) == 4 && m * n < (1ll << 30) && m * R < (1ll << 30)) {     // the kernel's 32-bit byte offsets
        const dim3 grid((unsigned)ceil_div(n, 256), (unsigned)ceil_div(R, 128));
        hipLaunchKernelGGL(k_l2_g_mfma, grid, dim3(256), 0, c->stream, m, n, R, (const float*)c->Xt, (const float*)c->r,
                           (float*)c->l2_g);
    } else {
        constexpr int TJ = 8;
        const dim3 grid((unsigned)ceil_div(R, 256), (unsigned)ceil_div(n, TJ));
        hipLaunchKernelGGL((k_l2_g_batched<T, TJ>), grid, dim3(256), 0, c->stream, m, n, R, (const T*)c->Xt,
                           (const T*)c->r, (T*)c->l2_g);
    }
    DMMV_LAUNCH_CHECK();
    return DMMV_OK;
}

template <class T>
dmmv_status table_t(Ctx* c, void* dq_out) {
    const int64_t n = c->p.n, R = c->p.R;
    if (n == 0) return DMMV_OK;
    hipLaunchKernelGGL(k_l2_table<T>, dim3((unsigned)ceil_div(n * R, 256)), dim3(256), 0, c->stream, n, R, c->p.nd,
                       (const T*)c->D_dev, (const T*)c->scale_dev, (const int32_t*)c->kidx, (const T*)c->l2_g,
                       (const T*)c->l2_c, (T*)dq_out);
    DMMV_LAUNCH_CHECK();
    return DMMV_OK;
}

template <class T>
dmmv_status select_t(Ctx* c, const void* scores, int32_t keep_going, dmmv_move* best_out, void* best_score_out) {
    hipLaunchKernelGGL(k_l2_select<T>, dim3((unsigned)c->p.R), dim3(1024), 0, c->stream, c->p.n, c->p.R, c->p.nd,
                       c->o.l2_rule, (const T*)scores, (const T*)c->D_dev, (const T*)c->scale_dev,
                       (const int32_t*)c->kidx, (const T*)c->l2_g, (const T*)c->l2_c, (InstState<T>*)c->state,
                       keep_going, best_out, (T*)best_score_out);
    DMMV_LAUNCH_CHECK();
    return DMMV_OK;
}

template <class T>
dmmv_status after_apply_csc_t(Ctx* c, int32_t iters, dmmv_move* trace, void* trace_t) {
    hipLaunchKernelGGL(k_l2_after_apply_csc<T>, dim3(1), dim3(1), 0, c->stream, (InstState<T>*)c->state, 0, iters, trace,
                       (T*)trace_t);
    DMMV_LAUNCH_CHECK();
    return DMMV_OK;
}

}  // namespace

#define L2_DISPATCH(fn, ...) (c->p.dtype == DMMV_F64 ? fn<double>(__VA_ARGS__) : fn<float>(__VA_ARGS__))

dmmv_status l2_build(Ctx* c) { return L2_DISPATCH(colsq_t, c); }
dmmv_status l2_update_g(Ctx* c) { return L2_DISPATCH(update_g_t, c); }
dmmv_status l2_table(Ctx* c, void* dq_out) { return L2_DISPATCH(table_t, c, dq_out); }
dmmv_status l2_select(Ctx* c, const void* scores, int32_t keep_going, dmmv_move* best_out, void* best_score_out) {
    return L2_DISPATCH(select_t, c, scores, keep_going, best_out, best_score_out);
}
dmmv_status l2_after_apply_csc(Ctx* c, int32_t iters, dmmv_move* trace, void* trace_t) {
    return L2_DISPATCH(after_apply_csc_t, c, iters, trace, trace_t);
}

}  // namespace dmmv
