// Batched path: R independent instances share the dense matrix X (m x n).  Instance q has
// its own target b_q, scale s_q, index vector and residual.
//
// Mapping: one lane per instance.  Within a wavefront all 64 lanes work on the same entry
// X_ij, so X is read through the scalar unit (one s_load feeds 64 instances) and every
// per-instance array is laid out instance-contiguous ([row][R], [var][R]) so that lane
// accesses coalesce.  The maximum over rows is then a serial loop inside each lane: no
// cross-lane reduction at all.  Each lane keeps KT x TJ running maxima (KT values of D for TJ
// adjacent variables) in registers.
#include "dmmv_common.h"

namespace dmmv {

// ---- layout helpers -------------------------------------------------------------------------
// out[c][r] = in[r][c] for an in matrix of `rows` x `cols` with row stride ld_in
template <class T>
__global__ void k_transpose(const T* __restrict__ in, int64_t rows, int64_t cols, int64_t ld_in,
                            T* __restrict__ out, int64_t ld_out) {
    __shared__ T tile[32][33];
    const int64_t c0 = blockIdx.x * 32ll, r0 = blockIdx.y * 32ll;
    for (int dy = threadIdx.y; dy < 32; dy += blockDim.y) {
        int64_t rr = r0 + dy, cc = c0 + threadIdx.x;
        if (rr < rows && cc < cols) tile[dy][threadIdx.x] = in[rr * ld_in + cc];
    }
    __syncthreads();
    for (int dy = threadIdx.y; dy < 32; dy += blockDim.y) {
        int64_t cc = c0 + dy, rr = r0 + threadIdx.x;
        if (rr < rows && cc < cols) out[cc * ld_out + rr] = tile[threadIdx.x][dy];
    }
}

template <class T>
static void launch_transpose(hipStream_t s, const T* in, int64_t rows, int64_t cols, int64_t ld_in,
                             T* out, int64_t ld_out) {
    if (rows == 0 || cols == 0) return;
    dim3 grid((unsigned)ceil_div(cols, 32), (unsigned)ceil_div(rows, 32));
    hipLaunchKernelGGL(k_transpose<T>, grid, dim3(32, 8), 0, s, in, rows, cols, ld_in, out, ld_out);
}

// x values [R][n] -> kidx [n][R]
template <class T>
__global__ void k_values_to_index_batched(const T* __restrict__ x, const T* __restrict__ D,
                                          int32_t nd, int64_t n, int64_t R,
                                          int32_t* __restrict__ kidx, int32_t* flags) {
    int64_t t = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
    if (t >= n * R) return;
    const int64_t j = t / R, q = t % R;
    const T v = x[q * n + j];
    int32_t lo = 0, hi = nd - 1;
    while (lo < hi) {
        int32_t mid = (lo + hi) >> 1;
        if (D[mid] < v) lo = mid + 1; else hi = mid;
    }
    if (!(D[lo] == v)) { atomicOr(&flags[FLAG_ERROR], ERRBIT_X_NOT_IN_D); lo = 0; }
    kidx[t] = lo;
}

template <class T>
__global__ void k_index_to_values_batched(const int32_t* __restrict__ kidx, const T* __restrict__ D,
                                          int64_t n, int64_t R, T* __restrict__ x) {
    int64_t t = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
    if (t >= n * R) return;
    const int64_t q = t / n, j = t % n;
    x[t] = D[kidx[j * R + q]];
}

// ---- residual -------------------------------------------------------------------------------
// lane = instance, TI rows per lane at a time.  Column-major X: the TI rows of column j are
// contiguous, read with one scalar load.  Order over j is ascending per (row, instance).
template <class T, int TI>
__global__ __launch_bounds__(256) void k_residual_batched(
    int64_t m, int64_t n, int64_t R, const T* __restrict__ X, int64_t ldx, const T* __restrict__ D,
    int32_t nd, const int32_t* __restrict__ kidx, const T* __restrict__ scale,
    const T* __restrict__ Bt, T* __restrict__ r) {
    extern __shared__ unsigned char smem[];
    T* shD = reinterpret_cast<T*>(smem);
    for (int k = threadIdx.x; k < nd; k += blockDim.x) shD[k] = D[k];
    __syncthreads();
    const int lane = threadIdx.x & 63;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t q = blockIdx.x * 64ll + lane;
    const int64_t qc = q < R ? q : R - 1;
    const int64_t i0 = (blockIdx.y * 4ll + w) * TI;
    if (i0 >= m) return;
    T acc[TI];
#pragma unroll
    for (int u = 0; u < TI; ++u) acc[u] = (T)0;
    // the level indices of RJ variables are fetched together (one memory latency for RJ
    // variables); the order of the additions stays j ascending
    constexpr int RJ = 8;
    for (int64_t j0 = 0; j0 < n; j0 += RJ) {
        int32_t kk[RJ];
#pragma unroll
        for (int e = 0; e < RJ; ++e) kk[e] = kidx[(j0 + e < n ? j0 + e : n - 1) * R + qc];
#pragma unroll
        for (int e = 0; e < RJ; ++e) {
            if (j0 + e >= n) break;                          // the same for the whole wavefront
            const T v = shD[kk[e]];
            const T* __restrict__ xp = X + ldx * (j0 + e) + i0;
#pragma unroll
            for (int u = 0; u < TI; ++u) {
                const T a = (i0 + u < m) ? xp[u] : (T)0;
                acc[u] = dmmv_fma(a, v, acc[u]);
            }
        }
    }
    if (q < R) {
        const T sc = scale[q];
#pragma unroll
        for (int u = 0; u < TI; ++u)
            if (i0 + u < m) r[(i0 + u) * R + q] = dmmv_fma(acc[u], sc, -Bt[(i0 + u) * R + q]);
    }
}

// The same sums for large batches: the 4 wavefronts of a workgroup take 4 groups of 64 instances
// and the SAME RT rows, so a tile of X (RC columns x RT rows) is staged once in LDS for all 256
// instances and read back as broadcasts (every lane of a wavefront needs the same entry), instead
// of travelling through the scalar cache once per wavefront.  Order over j ascending as above.
constexpr int RT = 32;                      // rows per lane
constexpr int RC = 32;                      // columns per staged tile

template <class T>
__global__ __launch_bounds__(256) void k_residual_batched_tiled(
    int64_t m, int64_t n, int64_t R, const T* __restrict__ X, int64_t ldx, const T* __restrict__ D,
    int32_t nd, const int32_t* __restrict__ kidx, const T* __restrict__ scale,
    const T* __restrict__ Bt, T* __restrict__ r) {
    extern __shared__ unsigned char smem[];
    T* shD = reinterpret_cast<T*>(smem);
    __shared__ __align__(16) T tile[2][RC][RT];
    for (int k = threadIdx.x; k < nd; k += blockDim.x) shD[k] = D[k];
    const int lane = threadIdx.x & 63;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t q = (blockIdx.x * 4ll + w) * 64 + lane;
    const int64_t qc = q < R ? q : R - 1;
    const int64_t i0 = blockIdx.y * (int64_t)RT;
    // staging: thread t fetches 4 consecutive rows (t % 8) * 4 .. + 3 of column t / 8 of the tile
    const int sc_col = threadIdx.x >> 3, sc_row = (threadIdx.x & 7) * 4;
    T stage[4];
    auto fetch = [&](int64_t j0) {
        const int64_t j = j0 + sc_col < n ? j0 + sc_col : n - 1;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int64_t i = i0 + sc_row + u;
            stage[u] = X[ldx * j + (i < m ? i : m - 1)];     // rows past the end are never stored below
        }
    };
    auto stash = [&](int buf) {
#pragma unroll
        for (int u = 0; u < 4; ++u) tile[buf][sc_col][sc_row + u] = stage[u];
    };
    T acc[RT];
#pragma unroll
    for (int u = 0; u < RT; ++u) acc[u] = (T)0;
    fetch(0);
    stash(0);
    __syncthreads();
    int buf = 0;
    for (int64_t j0 = 0; j0 < n; j0 += RC, buf ^= 1) {
        if (j0 + RC < n) fetch(j0 + RC);                     // the next tile travels while this one is used
        constexpr int RJ = 8;
        for (int jc0 = 0; jc0 < RC; jc0 += RJ) {
            int32_t kk[RJ];
#pragma unroll
            for (int e = 0; e < RJ; ++e) {
                const int64_t j = j0 + jc0 + e;
                kk[e] = kidx[(j < n ? j : n - 1) * R + qc];
            }
#pragma unroll
            for (int e = 0; e < RJ; ++e) {
                if (j0 + jc0 + e >= n) break;                // the same for the whole workgroup
                const T v = shD[kk[e]];
#pragma unroll
                for (int u = 0; u < RT; ++u) acc[u] = dmmv_fma(tile[buf][jc0 + e][u], v, acc[u]);
            }
        }
        if (j0 + RC < n) stash(buf ^ 1);
        __syncthreads();
    }
    if (q < R) {
        const T sc = scale[q];
#pragma unroll
        for (int u = 0; u < RT; ++u)
            if (i0 + u < m) r[(i0 + u) * R + q] = dmmv_fma(acc[u], sc, -Bt[(i0 + u) * R + q]);
    }
}

// per-instance max |r|: lane = instance, the 16 wavefronts of a workgroup share the rows
template <class T>
__global__ __launch_bounds__(1024) void k_maxabs_batched(int64_t m, int64_t R, const T* __restrict__ r,
                                                         InstState<T>* st) {
    __shared__ T sh[16][64];
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int64_t q = blockIdx.x * 64ll + lane;
    T v = (T)0;
    if (q < R)
        for (int64_t i = w; i < m; i += 16) v = dmmv_max(v, dmmv_abs(r[i * R + q]));
    sh[w][lane] = v;
    __syncthreads();
    if (w == 0 && q < R) {
#pragma unroll
        for (int ww = 1; ww < 16; ++ww) v = dmmv_max(v, sh[ww][lane]);
        st[q].t = v;
    }
}

#ifndef DMMV_BATCHED_RB
#define DMMV_BATCHED_RB 8      // rows of X and r whose loads are in flight together
#endif

// ---- evaluation -----------------------------------------------------------------------------
// grid.x = group of 64 instances, grid.y = chunk of `chunk_cols` variables.  A block has four
// wavefronts; each takes tiles of TJ variables of the chunk in turn.  For nd > KT the values
// of D are covered KT at a time.  Xt is the row-major copy of X, so the TJ entries of a row
// are one scalar load.
// ROT (nd = KT + 1): the null move is not computed at all.  Every lane takes the KT values
// AFTER its own current one, cyclically (the steps are per-lane registers anyway), and the null
// move enters the table and the arg-min with its known score t.
template <class T, int KT, int TJ, bool ROT = false, int RB = DMMV_BATCHED_RB>
__global__ __launch_bounds__(256) void k_eval_batched(
    int64_t m, int64_t n, int64_t R, int32_t nd, int32_t chunk_cols, const T* __restrict__ Xt,
    const T* __restrict__ D, const int32_t* __restrict__ kidx, const T* __restrict__ scale,
    const T* __restrict__ r, int32_t radius, const uint8_t* __restrict__ var_mask,
    const InstState<T>* __restrict__ st, T* __restrict__ scores, Partial<T>* __restrict__ part) {
    extern __shared__ unsigned char smem[];
    T* shD = reinterpret_cast<T*>(smem);
    __shared__ T sh_s[4][64];
    __shared__ int64_t sh_c[4][64];
    for (int k = threadIdx.x; k < nd; k += blockDim.x) shD[k] = D[k];
    __syncthreads();
    const int lane = threadIdx.x & 63;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t q = blockIdx.x * 64ll + lane;
    const bool live = q < R;
    const int64_t qc = live ? q : R - 1;
    const T sc = scale[qc];
    const T t_now = st[qc].t;
    const bool skip = part && !scores && st[qc].done;   // stopped instances score nothing
    const int64_t jbeg = blockIdx.y * (int64_t)chunk_cols;
    const int64_t jend = jbeg + chunk_cols < n ? jbeg + chunk_cols : n;

    T bs = (T)0;
    int64_t bc = -1;
    // whole wavefront stopped: nothing to do (uniform branch)
    const bool wave_idle = __builtin_amdgcn_readfirstlane(__ballot(!skip && live) == 0ull ? 1 : 0) != 0;
    if (!wave_idle) {
        for (int64_t j0 = jbeg + w * TJ; j0 < jend; j0 += 4 * TJ) {
            int32_t kcur[TJ];
            T dcur[TJ];
#pragma unroll
            for (int u = 0; u < TJ; ++u) {
                const int64_t j = j0 + u < n ? j0 + u : n - 1;
                kcur[u] = kidx[j * R + qc];
                dcur[u] = shD[kcur[u]];
            }
            for (int32_t k0 = 0; k0 < (ROT ? 1 : nd); k0 += KT) {
                T delta[TJ][KT], acc[TJ][KT];
#pragma unroll
                for (int u = 0; u < TJ; ++u)
#pragma unroll
                    for (int v = 0; v < KT; ++v) {
                        int32_t k;
                        if (ROT) { k = kcur[u] + 1 + v; k = k >= nd ? k - nd : k; }
                        else k = k0 + v < nd ? k0 + v : nd - 1;
                        delta[u][v] = step_of(shD[k], dcur[u], sc);
                        acc[u][v] = (T)0;
                    }
                if (ROT) {
                    // the value indices are recomputed after the row loop rather than kept in
                    // registers across it
#pragma unroll
                    for (int u = 0; u < TJ; ++u) asm volatile("" : "+v"(kcur[u]));
                }
                if (j0 + TJ <= n) {
                    // RB rows per pass: all their loads (r in vector registers, the X tile in
                    // scalar registers) are issued before the first row is scored, so one pass
                    // of a wavefront computes for longer than the loads of the other resident
                    // wavefront take.
                    const T* __restrict__ xrow = Xt + j0;
#pragma unroll RB
                    for (int64_t i = 0; i < m; ++i) {
                        const T ri = r[i * R + qc];
                        const T* __restrict__ xp = xrow + i * n;
#pragma unroll
                        for (int u = 0; u < TJ; ++u) {
                            const T a = xp[u];
#pragma unroll
                            for (int v = 0; v < KT; ++v)
                                acc[u][v] = dmmv_max(acc[u][v], dmmv_abs(dmmv_fma(delta[u][v], a, ri)));
                        }
                    }
                } else {
                    // ragged last tile: element-wise bounds
                    for (int64_t i = 0; i < m; ++i) {
                        const T ri = r[i * R + qc];
#pragma unroll
                        for (int u = 0; u < TJ; ++u) {
                            const int64_t j = j0 + u < n ? j0 + u : n - 1;
                            const T a = Xt[i * n + j];
#pragma unroll
                            for (int v = 0; v < KT; ++v)
                                acc[u][v] = dmmv_max(acc[u][v], dmmv_abs(dmmv_fma(delta[u][v], a, ri)));
                        }
                    }
                }
                if (live && !skip) {
#pragma unroll
                    for (int u = 0; u < TJ; ++u) {
                        const int64_t j = j0 + u;
                        if (j >= jend) continue;                 // (no break: keeps acc in registers)
                        const bool var_ok = var_mask ? var_mask[q * n + j] != 0 : true;
#pragma unroll
                        for (int v = 0; v < KT; ++v) {
                            int32_t k;
                            if (ROT) { k = kcur[u] + 1 + v; k = k >= nd ? k - nd : k; }
                            else { k = k0 + v; if (k >= nd) continue; }
                            T val = acc[u][v];
                            if (!cand_allowed(kcur[u], k, radius, var_ok)) val = Limits<T>::inf();
                            const int64_t cidx = j * (int64_t)nd + k;
                            if (scores) scores[q * (n * (int64_t)nd) + cidx] = val;
                            if (rec_less(val, cidx, bs, bc)) { bs = val; bc = cidx; }
                        }
                        if (ROT) {                               // the null move: fma(0, a, r) = r, score t
                            const int64_t cidx = j * (int64_t)nd + kcur[u];
                            if (scores) scores[q * (n * (int64_t)nd) + cidx] = t_now;
                            if (rec_less(t_now, cidx, bs, bc)) { bs = t_now; bc = cidx; }
                        }
                    }
                }
            }
        }
    }
    if (part) {
        sh_s[w][lane] = bs;
        sh_c[w][lane] = bc;
        __syncthreads();
        if (w == 0 && live) {
            T s = sh_s[0][lane];
            int64_t c = sh_c[0][lane];
#pragma unroll
            for (int ww = 1; ww < 4; ++ww)
                if (rec_less(sh_s[ww][lane], sh_c[ww][lane], s, c)) { s = sh_s[ww][lane]; c = sh_c[ww][lane]; }
            Partial<T> p; p.s = s; p.c = c;
            part[blockIdx.y * R + q] = p;
        }
    }
}

// ---- apply ----------------------------------------------------------------------------------
// lane = instance; each instance updates with its own column of X (a gather).  grid.y splits
// the rows; the block with blockIdx.y == 0 also updates x, t and the trace.
template <class T>
__global__ void k_apply_batched(int64_t m, int64_t n, int64_t R, const T* __restrict__ X,
                                int64_t ldx, T* __restrict__ r, int32_t* __restrict__ kidx,
                                InstState<T>* st, int32_t t_from_score, int32_t iters,
                                dmmv_move* trace, T* trace_t, int32_t rows_per_block,
                                const int32_t* __restrict__ orig) {
    const int64_t q = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
    if (q >= R) return;
    const int32_t j = st[q].apply_j;
    if (j < 0) return;
    const T delta = st[q].delta;
    const T* __restrict__ col = X + ldx * (int64_t)j;
    const int64_t i0 = blockIdx.y * (int64_t)rows_per_block;
    const int64_t i1 = i0 + rows_per_block < m ? i0 + rows_per_block : m;
    for (int64_t i = i0; i < i1; ++i) r[i * R + q] = dmmv_fma(delta, col[i], r[i * R + q]);
    if (blockIdx.y == 0) {
        const int32_t k = st[q].apply_k;
        const int32_t moves = st[q].moves;
        kidx[(int64_t)j * R + q] = k;
        if (t_from_score) {
            const T best_s = st[q].best_s;
            st[q].t = best_s;
            if (moves < iters) {
                const int64_t slot = (orig ? (int64_t)orig[q] : q) * (int64_t)iters + moves;   // caller's instance number
                if (trace) { trace[slot].j = j; trace[slot].k = k; }
                if (trace_t) trace_t[slot] = best_s;
            }
        }
        st[q].moves = moves + 1;
    }
}

// =========================================================================================
// host dispatch
// =========================================================================================
template <class T>
static dmmv_status build_t(Ctx* c) {
    const int64_t m = c->p.m, n = c->p.n, R = c->p.R;
    // X is column-major m x n = row-major n x m with stride lda; Xt[i][j] = X[j][i]
    launch_transpose<T>(c->stream, (const T*)c->p.A_dense, n, m, c->p.lda, (T*)c->Xt, n);
    // B is [R][m]; Bt[i][q]
    launch_transpose<T>(c->stream, (const T*)c->p.b, R, m, m, (T*)c->Bt, R);
    DMMV_LAUNCH_CHECK();
    return DMMV_OK;
}

template <class T>
static dmmv_status residual_t(Ctx* c) {
    const int64_t m = c->p.m, n = c->p.n, R = c->p.R;
    if (m == 0) return DMMV_OK;
    // rows per lane: every variable's level index is read once per TI rows, so tall matrices take
    // many rows per lane (as long as the launch still fills the chip)
    auto launch = [&](auto kernel, int ti) {
        dim3 grid((unsigned)ceil_div(R, 64), (unsigned)ceil_div(m, 4 * ti));
        hipLaunchKernelGGL(kernel, grid, dim3(256), (size_t)c->p.nd * sizeof(T), c->stream,
                           m, n, R, (const T*)c->p.A_dense, c->p.lda, (const T*)c->D_dev, c->p.nd,
                           (const int32_t*)c->kidx, (const T*)c->scale_dev, (const T*)c->Bt, (T*)c->r);
    };
    if (R >= 256 && ceil_div(R, 256) * ceil_div(m, RT) >= 512) {
        dim3 grid((unsigned)ceil_div(R, 256), (unsigned)ceil_div(m, RT));
        hipLaunchKernelGGL(k_residual_batched_tiled<T>, grid, dim3(256), (size_t)c->p.nd * sizeof(T), c->stream,
                           m, n, R, (const T*)c->p.A_dense, c->p.lda, (const T*)c->D_dev, c->p.nd,
                           (const int32_t*)c->kidx, (const T*)c->scale_dev, (const T*)c->Bt, (T*)c->r);
    } else if (ceil_div(R, 64) * ceil_div(m, 4 * 32) >= 512) {
        launch(k_residual_batched<T, 32>, 32);
    } else {
        launch(k_residual_batched<T, 8>, 8);
    }
    DMMV_LAUNCH_CHECK();
    return DMMV_OK;
}

template <class T>
static dmmv_status maxabs_t(Ctx* c) {
    hipLaunchKernelGGL(k_maxabs_batched<T>, dim3((unsigned)ceil_div(c->p.R, 64)), dim3(1024), 0, c->stream,
                       c->p.m, c->p.R, (const T*)c->r, (InstState<T>*)c->state);
    DMMV_LAUNCH_CHECK();
    return DMMV_OK;
}

template <class T, int KT, int TJ, bool ROT = false>
static dmmv_status eval_launch(Ctx* c, void* scores, bool want_partials) {
    dim3 grid((unsigned)ceil_div(c->p.R, 64), (unsigned)c->n_partials);
    hipLaunchKernelGGL((k_eval_batched<T, KT, TJ, ROT>), grid, dim3(256), (size_t)c->p.nd * sizeof(T), c->stream,
                       c->p.m, c->p.n, c->p.R, c->p.nd, c->chunk_cols, (const T*)c->Xt,
                       (const T*)c->D_dev, (const int32_t*)c->kidx, (const T*)c->scale_dev,
                       (const T*)c->r, c->o.radius, c->o.var_mask, (const InstState<T>*)c->state,
                       (T*)scores, want_partials ? (Partial<T>*)c->partials : nullptr);
    DMMV_LAUNCH_CHECK();
    return DMMV_OK;
}

template <class T>
static dmmv_status eval_t(Ctx* c, void* scores, bool want_partials) {
    if ((size_t)c->p.nd * sizeof(T) > 48 * 1024)
        return fail(DMMV_ERR_UNSUPPORTED, "batched path: nd = %d does not fit the LDS value table", c->p.nd);
    // the usual code widths (4, 3 and 2 bits) in fp32: without computing the null move
    // (in fp64 the variant needs more than the 256 registers that two wavefronts per SIMD leave)
    if (sizeof(T) == 4) {
        if (c->p.nd == 16) return eval_launch<float, 15, 4, true>(c, scores, want_partials);
        if (c->p.nd == 8) return eval_launch<float, 7, 8, true>(c, scores, want_partials);
        if (c->p.nd == 4) return eval_launch<float, 3, 8, true>(c, scores, want_partials);
    }
    if (c->p.nd > 8) return eval_launch<T, 16, 4>(c, scores, want_partials);
    if (c->p.nd > 4) return eval_launch<T, 8, 8>(c, scores, want_partials);
    return eval_launch<T, 4, 8>(c, scores, want_partials);
}

template <class T>
static dmmv_status apply_t(Ctx* c, bool t_from_score, int32_t iters, dmmv_move* trace, void* trace_t) {
    const int64_t m = c->p.m, R = c->p.R;
    const int32_t rows_per_block = 256;
    dim3 grid((unsigned)ceil_div(R, 64), (unsigned)(m > 0 ? ceil_div(m, rows_per_block) : 1));
    hipLaunchKernelGGL(k_apply_batched<T>, grid, dim3(64), 0, c->stream, m, c->p.n, R,
                       (const T*)c->p.A_dense, c->p.lda, (T*)c->r, c->kidx, (InstState<T>*)c->state,
                       (int32_t)t_from_score, iters, trace, (T*)trace_t, rows_per_block,
                       c->cmp_on ? (const int32_t*)c->cmp_orig : nullptr);
    DMMV_LAUNCH_CHECK();
    return DMMV_OK;
}

template <class T>
static dmmv_status set_x_t(Ctx* c, const void* x) {
    const int64_t tot = c->p.n * c->p.R;
    hipLaunchKernelGGL(k_values_to_index_batched<T>, dim3((unsigned)ceil_div(tot, 256)), dim3(256), 0, c->stream,
                       (const T*)x, (const T*)c->D_dev, c->p.nd, c->p.n, c->p.R, c->kidx, c->flags);
    DMMV_LAUNCH_CHECK();
    return DMMV_OK;
}

template <class T>
static dmmv_status get_x_t(Ctx* c, void* x) {
    const int64_t tot = c->p.n * c->p.R;
    hipLaunchKernelGGL(k_index_to_values_batched<T>, dim3((unsigned)ceil_div(tot, 256)), dim3(256), 0, c->stream,
                       (const int32_t*)c->kidx, (const T*)c->D_dev, c->p.n, c->p.R, (T*)x);
    DMMV_LAUNCH_CHECK();
    return DMMV_OK;
}

// =========================================================================================
// dropping stopped instances from the descent
// =========================================================================================
// Instances stop at different iterations, and a wavefront works as long as one of its 64
// instances does.  At the host's polling points the instances still running are therefore
// gathered into a dense "virtual" batch of their own (same layouts, stride = their number),
// which the loop's kernels then work on; orig[p] is the caller's number of virtual instance p.
// Before a new gather, and at the end, the virtual batch is scattered back into the full arrays.
template <class T>
__global__ void k_cmp_scatter(int64_t m, int64_t n, int64_t Rv, int64_t Rf, const int32_t* __restrict__ orig,
                              const T* __restrict__ r_v, T* __restrict__ r_f,
                              const int32_t* __restrict__ k_v, int32_t* __restrict__ k_f,
                              const InstState<T>* __restrict__ st_v, InstState<T>* __restrict__ st_f) {
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    const int64_t t0 = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
    for (int64_t e = t0; e < m * Rv; e += stride) r_f[(e / Rv) * Rf + orig[e % Rv]] = r_v[e];
    for (int64_t e = t0; e < n * Rv; e += stride) k_f[(e / Rv) * Rf + orig[e % Rv]] = k_v[e];
    for (int64_t p = t0; p < Rv; p += stride) st_f[orig[p]] = st_v[p];
}

// the running instances in ascending order (single workgroup); their number goes to
// flags[FLAG_ACTIVE]
template <class T>
__global__ __launch_bounds__(1024) void k_cmp_list(int64_t Rf, const InstState<T>* __restrict__ st_f,
                                                   int32_t* __restrict__ orig, int32_t* flags) {
    __shared__ int32_t sh_cnt[16];
    __shared__ int32_t sh_base;
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    if (threadIdx.x == 0) sh_base = 0;
    __syncthreads();
    for (int64_t b0 = 0; b0 < Rf; b0 += 1024) {
        const int64_t q = b0 + threadIdx.x;
        const bool on = q < Rf && !st_f[q].done;
        const unsigned long long bal = __ballot(on);
        if (lane == 0) sh_cnt[w] = __popcll(bal);
        __syncthreads();
        int32_t before = 0, all = 0;
        for (int u = 0; u < 16; ++u) { if (u < w) before += sh_cnt[u]; all += sh_cnt[u]; }
        const int32_t base = sh_base;
        if (on) orig[base + before + __popcll(bal & ((1ull << lane) - 1ull))] = (int32_t)q;
        __syncthreads();
        if (threadIdx.x == 0) sh_base = base + all;
        __syncthreads();
    }
    if (threadIdx.x == 0) flags[FLAG_ACTIVE] = sh_base;
}

template <class T>
__global__ void k_cmp_gather(int64_t m, int64_t n, int64_t Rv, int64_t Rf, const int32_t* __restrict__ orig,
                             const T* __restrict__ r_f, T* __restrict__ r_v,
                             const int32_t* __restrict__ k_f, int32_t* __restrict__ k_v,
                             const InstState<T>* __restrict__ st_f, InstState<T>* __restrict__ st_v,
                             const T* __restrict__ sc_f, T* __restrict__ sc_v) {
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    const int64_t t0 = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
    for (int64_t e = t0; e < m * Rv; e += stride) r_v[e] = r_f[(e / Rv) * Rf + orig[e % Rv]];
    for (int64_t e = t0; e < n * Rv; e += stride) k_v[e] = k_f[(e / Rv) * Rf + orig[e % Rv]];
    for (int64_t p = t0; p < Rv; p += stride) { st_v[p] = st_f[orig[p]]; sc_v[p] = sc_f[orig[p]]; }
}

template <class T>
static dmmv_status compact_scatter_t(Ctx* c) {
    hipLaunchKernelGGL(k_cmp_scatter<T>, dim3(2048), dim3(256), 0, c->stream, c->p.m, c->p.n, c->p.R, c->cmp_full_R,
                       (const int32_t*)c->cmp_orig, (const T*)c->r, (T*)c->cmp_full_r, (const int32_t*)c->kidx,
                       c->cmp_full_kidx, (const InstState<T>*)c->state, (InstState<T>*)c->cmp_full_state);
    DMMV_LAUNCH_CHECK();
    return DMMV_OK;
}

static void compact_to_full(Ctx* c) {
    c->r = c->cmp_full_r; c->kidx = c->cmp_full_kidx; c->state = c->cmp_full_state;
    c->scale_dev = c->cmp_full_scale; c->p.R = c->cmp_full_R;
    c->cmp_on = false;
}

// At a polling point of the descent: how many instances still run (HOST, *active_out), and the
// loop's arrays re-pointed at a virtual batch of just those when that is worth it.
template <class T>
static dmmv_status compact_t(Ctx* c, int32_t* active_out) {
    if (c->cmp_on) {
        DMMV_TRY(compact_scatter_t<T>(c));
        compact_to_full(c);
    }
    const int64_t Rf = c->p.R, m = c->p.m, n = c->p.n;
    hipLaunchKernelGGL(k_cmp_list<T>, dim3(1), dim3(1024), 0, c->stream, Rf, (const InstState<T>*)c->state,
                       c->cmp_orig, c->flags);
    int32_t active = 0;
    DMMV_HIP_CHECK(hipMemcpyAsync(&active, &c->flags[FLAG_ACTIVE], sizeof(int32_t), hipMemcpyDeviceToHost, c->stream));
    DMMV_HIP_CHECK(hipStreamSynchronize(c->stream));
    *active_out = active;
    if (active == 0 || (int64_t)active * 4 > Rf * 3) return DMMV_OK;      // nothing left, or not worth it
    c->cmp_full_r = c->r; c->cmp_full_kidx = c->kidx; c->cmp_full_state = c->state;
    c->cmp_full_scale = c->scale_dev; c->cmp_full_R = Rf;
    hipLaunchKernelGGL(k_cmp_gather<T>, dim3(2048), dim3(256), 0, c->stream, m, n, (int64_t)active, Rf,
                       (const int32_t*)c->cmp_orig, (const T*)c->cmp_full_r, (T*)c->cmp_r,
                       (const int32_t*)c->cmp_full_kidx, c->cmp_kidx, (const InstState<T>*)c->cmp_full_state,
                       (InstState<T>*)c->cmp_state, (const T*)c->cmp_full_scale, (T*)c->cmp_scale);
    DMMV_LAUNCH_CHECK();
    c->r = c->cmp_r; c->kidx = c->cmp_kidx; c->state = c->cmp_state; c->scale_dev = c->cmp_scale;
    c->p.R = active;
    c->cmp_on = true;
    return DMMV_OK;
}

dmmv_status batched_compact(Ctx* c, int32_t* active_out) {
    return c->p.dtype == DMMV_F64 ? compact_t<double>(c, active_out) : compact_t<float>(c, active_out);
}
// back to the caller's batch (no-op when the loop never left it)
dmmv_status batched_compact_end(Ctx* c) {
    if (!c->cmp_on) return DMMV_OK;
    dmmv_status st = c->p.dtype == DMMV_F64 ? compact_scatter_t<double>(c) : compact_scatter_t<float>(c);
    compact_to_full(c);
    return st;
}

// row-major copy of a column-major matrix alone (a dense single instance that uses the batch's
// pruned descent needs nothing else of the batched layouts)
dmmv_status batched_build_xt(Ctx* c) {
    if (c->p.dtype == DMMV_F64)
        launch_transpose<double>(c->stream, (const double*)c->p.A_dense, c->p.n, c->p.m, c->p.lda, (double*)c->Xt, c->p.n);
    else
        launch_transpose<float>(c->stream, (const float*)c->p.A_dense, c->p.n, c->p.m, c->p.lda, (float*)c->Xt, c->p.n);
    DMMV_LAUNCH_CHECK();
    return DMMV_OK;
}

dmmv_status batched_build(Ctx* c) {
    if (c->eval_mfma) DMMV_TRY(batched_eval_mfma_build(c));
    return c->p.dtype == DMMV_F64 ? build_t<double>(c) : build_t<float>(c);
}
dmmv_status batched_residual(Ctx* c) { return c->p.dtype == DMMV_F64 ? residual_t<double>(c) : residual_t<float>(c); }
dmmv_status batched_maxabs(Ctx* c) { return c->p.dtype == DMMV_F64 ? maxabs_t<double>(c) : maxabs_t<float>(c); }
dmmv_status batched_eval(Ctx* c, void* s, bool p) {
    if (c->eval_mfma) return batched_eval_mfma(c, s, p);
    return c->p.dtype == DMMV_F64 ? eval_t<double>(c, s, p) : eval_t<float>(c, s, p);
}
dmmv_status batched_apply(Ctx* c, bool tf, int32_t iters, dmmv_move* trace, void* trace_t) {
    return c->p.dtype == DMMV_F64 ? apply_t<double>(c, tf, iters, trace, trace_t) : apply_t<float>(c, tf, iters, trace, trace_t);
}
dmmv_status batched_set_x(Ctx* c, const void* x) { return c->p.dtype == DMMV_F64 ? set_x_t<double>(c, x) : set_x_t<float>(c, x); }
dmmv_status batched_get_x_from(Ctx* c, const int32_t* kidx, void* x) {
    const int64_t tot = c->p.n * c->p.R;
    if (tot == 0) return DMMV_OK;
    if (c->p.dtype == DMMV_F64)
        hipLaunchKernelGGL(k_index_to_values_batched<double>, dim3((unsigned)ceil_div(tot, 256)), dim3(256), 0, c->stream,
                           kidx, (const double*)c->D_dev, c->p.n, c->p.R, (double*)x);
    else
        hipLaunchKernelGGL(k_index_to_values_batched<float>, dim3((unsigned)ceil_div(tot, 256)), dim3(256), 0, c->stream,
                           kidx, (const float*)c->D_dev, c->p.n, c->p.R, (float*)x);
    DMMV_LAUNCH_CHECK();
    return DMMV_OK;
}
dmmv_status batched_get_x(Ctx* c, void* x) { return c->p.dtype == DMMV_F64 ? get_x_t<double>(c, x) : get_x_t<float>(c, x); }
dmmv_status batched_set_r(Ctx* c, const void* r) {
    // caller layout [R][m] -> internal [m][R]
    if (c->p.dtype == DMMV_F64) launch_transpose<double>(c->stream, (const double*)r, c->p.R, c->p.m, c->p.m, (double*)c->r, c->p.R);
    else launch_transpose<float>(c->stream, (const float*)r, c->p.R, c->p.m, c->p.m, (float*)c->r, c->p.R);
    DMMV_LAUNCH_CHECK();
    return DMMV_OK;
}
dmmv_status batched_get_r(Ctx* c, void* r) {
    if (c->p.dtype == DMMV_F64) launch_transpose<double>(c->stream, (const double*)c->r, c->p.m, c->p.R, c->p.R, (double*)r, c->p.m);
    else launch_transpose<float>(c->stream, (const float*)c->r, c->p.m, c->p.R, c->p.R, (float*)r, c->p.m);
    DMMV_LAUNCH_CHECK();
    return DMMV_OK;
}

}  // namespace dmmv
