// Swap move of the local search (paper: section "Search Operators", Proposition 1 and
// Corollary 1; Appendix B "Swap Move", Algorithm 2) for dense matrices and batches.
//
// A swap exchanges the values of two variables x_i > x_j.  With Delta = s * (D[k_i] - D[k_j])
// the new residual is r'_k = fma(Delta, A_kj - A_ki, r_k) and the swap kept is the one with
// the smallest t' = max_k |r'_k| (lowest pair number c = i*n + j on a tie), if t' < t.
//
// The filter of Corollary 1 tests a necessary condition on the k_eps rows of largest |r_k|.
// Here the condition is the evaluation itself restricted to those rows: a pair whose new
// residual reaches t on one of them cannot improve.  The rows are tried in order of
// decreasing |r_k| and a pair is dropped at the first row that reaches t, or that exceeds the
// best t' found so far; what survives is evaluated on every row.  Dropping only such pairs
// leaves the result that of the full enumeration, whatever the order in which wavefronts
// find their candidates.
//
// Work split: one workgroup handles one instance; each of its wavefronts takes variables u and
// a lane one partner v > u, so every unordered pair is met once.  The first rows of the filter
// are staged in LDS (as many as fit beside the instance's values D[k_j]), the others are read
// from memory; pairs that pass all of them are finished by the whole wavefront, one lane per
// row, so that A is read along its columns.
#include "dmmv_common.h"

namespace dmmv {

namespace {

constexpr int SW_BLOCK = 256;
constexpr int SW_WAVES = SW_BLOCK / 64;
constexpr int SWE_BLOCK = 1024;                // evaluation: many wavefronts share one instance's LDS tile
constexpr int SWE_WAVES = SWE_BLOCK / 64;
constexpr int SWE_QCAP = 128;                  // queue of a wavefront: under 64 waiting plus at most 64 new
constexpr size_t SW_LDS_BUDGET = 68 * 1024;    // dynamic LDS of the evaluation kernel (8 KiB more are static):
                                               // two workgroups share a compute unit's 160 KiB

__device__ __forceinline__ unsigned long long order_bits(float v) { return (unsigned long long)__float_as_uint(v); }
__device__ __forceinline__ unsigned long long order_bits(double v) { return (unsigned long long)__double_as_longlong(v); }
__device__ __forceinline__ void from_order_bits(unsigned long long b, float& v) { v = __uint_as_float((uint32_t)b); }
__device__ __forceinline__ void from_order_bits(unsigned long long b, double& v) { v = __longlong_as_double((long long)b); }
// the largest value below t >= 0 (finite); -1 for t = 0, which no magnitude is at or below
__device__ __forceinline__ float value_below(float t) { return t > 0.0f ? __uint_as_float(__float_as_uint(t) - 1u) : -1.0f; }
__device__ __forceinline__ double value_below(double t) {
    return t > 0.0 ? __longlong_as_double(__double_as_longlong(t) - 1ll) : -1.0;
}

// ---- K rows of large |r| per instance for the filter, in decreasing order.  Which rows the
// filter tries first changes the time a search takes, never its result, so an exact top-K
// selection is not needed: every thread takes the largest |r| among its rows i = thread,
// thread + 256, ... and the 256 maxima are ranked (larger first, lower row first among equal
// values).  The row of largest |r| always comes first; of the next largest most are there.
// One workgroup per instance.
template <class T>
__global__ __launch_bounds__(SW_BLOCK) void k_swap_top(int64_t m, int64_t R, int32_t K,
                                                        const T* __restrict__ r,
                                                        const int32_t* __restrict__ skip,
                                                        int32_t* __restrict__ rows_all) {
    __shared__ T sh_a[SW_BLOCK];
    __shared__ int32_t sh_row[SW_BLOCK];
    const int64_t q = blockIdx.x;
    if (skip && skip[q]) return;
    T a = (T)-1;                                           // no row: ranks after every real one
    int32_t row = INT32_MAX;
    for (int64_t i = threadIdx.x; i < m; i += SW_BLOCK) {
        const T v = dmmv_abs(r[i * R + q]);
        if (v > a) { a = v; row = (int32_t)i; }
    }
    sh_a[threadIdx.x] = a;
    sh_row[threadIdx.x] = row;
    __syncthreads();
    int32_t rank = 0;
    for (int x = 0; x < SW_BLOCK; ++x) {
        const T oa = sh_a[x];
        const int32_t orow = sh_row[x];
        rank += (oa > a || (oa == a && orow < row)) ? 1 : 0;
    }
    if (row != INT32_MAX && rank < K) rows_all[q * K + rank] = row;
}

// ---- evaluation: grid (R, nb).  Writes one record (t', c) per workgroup; c = -1 if the
// workgroup found no pair with t' < t.
//
// A wavefront owns a variable u and walks its partners v > u, 64 at a time, through the filter
// rows held in LDS.  Every such row drops about half of the pairs still alive when many rows
// are close to t (the state a descent leaves), so the survivors are packed into a queue of the
// wavefront and taken through the remaining filter rows (read from memory) 64 at a time, all
// lanes busy.  What passes every filter row is evaluated on all m rows by the whole wavefront,
// one lane per row.
template <class T, bool DVL>
__global__ __launch_bounds__(SWE_BLOCK) void k_swap_eval(
    int64_t m, int64_t n, int64_t R, int32_t nb, int32_t K, int32_t L, const T* __restrict__ A,
    int64_t lda, const T* __restrict__ At, const T* __restrict__ D, const T* __restrict__ scale,
    const int32_t* __restrict__ kidx, const T* __restrict__ r, const InstState<T>* __restrict__ st,
    const uint8_t* __restrict__ var_mask, const int32_t* __restrict__ rows_all,
    const int32_t* __restrict__ skip, Partial<T>* __restrict__ part) {
    extern __shared__ __align__(16) unsigned char sw_smem[];
    // carve: rtop[K] | dv[n] (DVL) | atop[L][n] | rows[K]
    T* rtop = reinterpret_cast<T*>(sw_smem);
    T* sh_dv = rtop + K;
    T* atop = sh_dv + (DVL ? n : 0);
    int32_t* sh_rows = reinterpret_cast<int32_t*>(atop + (int64_t)L * n);
    __shared__ int32_t sh_queue[SWE_WAVES][SWE_QCAP];      // partners v waiting for the later rows
    __shared__ unsigned long long sh_best;                 // order bits of the best t' of the workgroup
    __shared__ T sh_s[SWE_WAVES];
    __shared__ int64_t sh_c[SWE_WAVES];

    const int64_t q = blockIdx.x;
    const int blk = blockIdx.y;
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    Partial<T>* out = part + q * nb + blk;
    if (skip && skip[q]) {
        if (threadIdx.x == 0) { Partial<T> e; e.s = (T)0; e.c = -1; *out = e; }
        return;
    }
    const int32_t* __restrict__ rows_g = rows_all + q * K;
    const uint8_t* __restrict__ vm = var_mask ? var_mask + q * n : nullptr;
    for (int l = threadIdx.x; l < K; l += SWE_BLOCK) {
        const int32_t row = rows_g[l];
        sh_rows[l] = row;
        rtop[l] = r[(int64_t)row * R + q];
    }
    if (DVL)
        for (int64_t j = threadIdx.x; j < n; j += SWE_BLOCK) sh_dv[j] = D[kidx[j * R + q]];
    for (int64_t e = threadIdx.x; e < (int64_t)L * n; e += SWE_BLOCK) {
        const int64_t l = e / n, j = e % n;
        atop[e] = A[(int64_t)rows_g[l] + j * lda];
    }
    if (threadIdx.x == 0) sh_best = order_bits(Limits<T>::inf());
    __syncthreads();
    int32_t* queue = sh_queue[w];                          // written and read by this wavefront only

    auto dv = [&](int64_t j) -> T { return DVL ? sh_dv[j] : D[kidx[j * R + q]]; };
    // Unordered pairs {u, v}, u < v, each taken in the orientation its values give: with
    // Ds = +Delta when x_u > x_v (pair (u, v)) and -Delta when x_v > x_u (pair (v, u)) the new
    // residual of either is fma(Ds, A_kv - A_ku, r_k), bit for bit (a - b = -(b - a) and
    // fma(-x, y, z) = fma(x, -y, z) exactly).
    const T sc = scale[q];
    auto step_of = [&](T dvu, T dvv) -> T {
        if (dvu > dvv) { const T diff = dvu - dvv; return sc * diff; }
        const T diff = dvv - dvu;
        return -(sc * diff);
    };

    const T t = st[q].t;
    T best_t = Limits<T>::inf();
    int64_t best_c = -1;                                   // the wavefront's record (uniform)
    auto bound = [&]() -> T {
        T shared_t;
        from_order_bits(__hip_atomic_load(&sh_best, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP), shared_t);
        return dmmv_min(best_t, shared_t);
    };

    // the first `cnt` queued partners of u: remaining filter rows, then the full evaluation
    auto drain = [&](int64_t u, T dvu, const T* __restrict__ Au, int cnt) {
        bool alive = lane < cnt;
        const int64_t v = alive ? (int64_t)queue[lane] : u;
        const T Ds = alive ? step_of(dvu, dv(v)) : (T)0;
        T bnd = bound();
        const T thr = dmmv_min(bnd, value_below(t));       // val < t and val <= bound in one test
        for (int l = L; l < K && __any(alive); ++l) {
            if (alive) {
                const int64_t row = sh_rows[l];
                const T au = At ? At[row * n + u] : Au[row];
                const T av = At ? At[row * n + v] : A[row + v * lda];
                const T val = dmmv_abs(dmmv_fma(Ds, av - au, rtop[l]));
                alive = val <= thr;
            }
        }
        unsigned long long todo = __ballot(alive);
        while (todo) {
            const int src = __builtin_ctzll(todo);
            todo &= todo - 1;
            const int64_t sv = (int64_t)queue[src];
            const T dvv = dv(sv);
            const T Dl = step_of(dvu, dvv);
            const T* __restrict__ Av = A + sv * lda;
            bnd = bound();
            T val = (T)0, wm = (T)0;
            bool ok = true;
            for (int64_t base = 0; base < m && ok; base += 256) {
#pragma unroll
                for (int x = 0; x < 4; ++x) {
                    const int64_t row = base + x * 64 + lane;
                    if (row < m) val = dmmv_max(val, dmmv_abs(dmmv_fma(Dl, Av[row] - Au[row], r[row * R + q])));
                }
                wm = wave_max(val);
                ok = wm < t && !(wm > bnd);
            }
            if (ok && wm < t) {
                const int64_t c = dvu > dvv ? u * n + sv : sv * n + u;
                if (rec_less(wm, c, best_t, best_c)) {
                    best_t = wm;
                    best_c = c;
                    if (lane == 0) atomicMin(&sh_best, order_bits(wm));
                }
            }
        }
    };

    // n < 2^31 (the variables are numbered with int32 throughout the library), and L * n
    // elements fit in LDS, so 32-bit indices do below.
    const int32_t n32 = (int32_t)n;
    const unsigned long long below = (1ull << lane) - 1ull;
    const T t_below = value_below(t);
    for (int32_t u = blk * SWE_WAVES + w; u < n32; u += nb * SWE_WAVES) {
        if (vm && !vm[u]) continue;
        const T dvu = dv(u);
        const T* __restrict__ Au = A + (int64_t)u * lda;
        int qn = 0;                                        // queued partners (uniform)
        for (int32_t v0 = (u + 1) & ~63; v0 < n32; v0 += 64) {
            const int32_t v = v0 + lane;
            bool alive = false;
            T Ds = (T)0;
            if (v > u && v < n32) {
                const T dvv = dv(v);
                alive = dvu != dvv;
                if (vm) alive = alive && vm[v];
                Ds = step_of(dvu, dvv);
            }
            // One threshold for both tests: val < t and val <= bound  <=>  val <= min(bound, t-),
            // t- the largest value below t.  After the first row (which, far from a local
            // optimum, often leaves no pair of the 64) the rows are taken without a branch: a
            // wavefront instruction costs the same however many lanes still need it.
            const T thr = dmmv_min(bound(), t_below);
            const int32_t vv = alive ? v : u;              // a lane without a pair reads in bounds
            const T* __restrict__ row_l = atop;
            if (L > 0) {
                const T val = dmmv_abs(dmmv_fma(Ds, row_l[vv] - row_l[u], rtop[0]));
                alive = alive & (val <= thr);
                if (!__any(alive)) continue;
                row_l += n32;
            }
            for (int l = 1; l < L; ++l, row_l += n32) {
                const T val = dmmv_abs(dmmv_fma(Ds, row_l[vv] - row_l[u], rtop[l]));
                alive = alive & (val <= thr);
            }
            const unsigned long long bal = __ballot(alive);
            if (!bal) continue;
            if (alive) queue[qn + __popcll(bal & below)] = v;
            qn += __popcll(bal);
            __builtin_amdgcn_wave_barrier();
            if (qn >= 64) {
                drain(u, dvu, Au, 64);
                const int32_t carry = 64 + lane < qn ? queue[64 + lane] : 0;
                __builtin_amdgcn_wave_barrier();
                if (64 + lane < qn) queue[lane] = carry;
                __builtin_amdgcn_wave_barrier();
                qn -= 64;
            }
        }
        if (qn > 0) drain(u, dvu, Au, qn);
    }
    if (lane == 0) { sh_s[w] = best_t; sh_c[w] = best_c; }
    __syncthreads();
    if (threadIdx.x == 0) {
        T bs = sh_s[0];
        int64_t bc = sh_c[0];
        for (int x = 1; x < SWE_WAVES; ++x)
            if (rec_less(sh_s[x], sh_c[x], bs, bc)) { bs = sh_s[x]; bc = sh_c[x]; }
        Partial<T> p;
        p.s = bc < 0 ? (T)0 : bs;
        p.c = bc;
        *out = p;
    }
}

// ---- reduce the records of an instance, report, and carry the swap out.  One workgroup per
// instance.
template <class T>
__global__ __launch_bounds__(SW_BLOCK) void k_swap_apply(
    int64_t m, int64_t n, int64_t R, int32_t nb, int32_t apply, const T* __restrict__ A, int64_t lda,
    const T* __restrict__ D, const T* __restrict__ scale, int32_t* __restrict__ kidx,
    T* __restrict__ r, InstState<T>* __restrict__ st, const Partial<T>* __restrict__ part,
    int32_t* __restrict__ skip, int32_t mark_skip, dmmv_swap* __restrict__ best_out,
    T* __restrict__ best_t_out) {
    __shared__ T sh_s[SW_WAVES];
    __shared__ int64_t sh_c[SW_WAVES];
    __shared__ T sh_bs;
    __shared__ int64_t sh_bc;
    const int64_t q = blockIdx.x;
    if (skip && skip[q]) {
        if (threadIdx.x == 0) {
            if (best_out) { best_out[q].i = -1; best_out[q].j = -1; }
            if (best_t_out) best_t_out[q] = st[q].t;
        }
        return;
    }
    T s = (T)0;
    int64_t c = -1;
    for (int e = threadIdx.x; e < nb; e += SW_BLOCK) {
        const Partial<T> p = part[q * nb + e];
        if (rec_less(p.s, p.c, s, c)) { s = p.s; c = p.c; }
    }
    block_argmin(s, c, sh_s, sh_c);
    if (threadIdx.x == 0) { sh_bs = s; sh_bc = c; }
    __syncthreads();
    s = sh_bs;
    c = sh_bc;
    if (threadIdx.x == 0) {
        if (best_out) { best_out[q].i = c < 0 ? -1 : c / n; best_out[q].j = c < 0 ? -1 : c % n; }
        if (best_t_out) best_t_out[q] = c < 0 ? st[q].t : s;
        if (c < 0 && skip && mark_skip) skip[q] = 1;
    }
    if (c < 0 || !apply) return;
    const int64_t i = c / n, j = c % n;
    const int32_t ki = kidx[i * R + q], kj = kidx[j * R + q];
    const T diff = D[ki] - D[kj];
    const T Delta = scale[q] * diff;
    const T* __restrict__ Ai = A + i * lda;
    const T* __restrict__ Aj = A + j * lda;
    for (int64_t k = threadIdx.x; k < m; k += SW_BLOCK)
        r[k * R + q] = dmmv_fma(Delta, Aj[k] - Ai[k], r[k * R + q]);
    __syncthreads();                                       // every thread has read ki and kj
    if (threadIdx.x == 0) {
        kidx[i * R + q] = kj;
        kidx[j * R + q] = ki;
        st[q].t = s;
        st[q].moves += 1;
    }
}

__global__ void k_swap_clear(int32_t* skip, int64_t R) {
    const int64_t q = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
    if (q < R) skip[q] = 0;
}

template <class T>
dmmv_status swap_t(Ctx* c, int32_t k_eps, int32_t apply, bool use_skip, dmmv_swap* best, void* best_t) {
    const int64_t m = c->p.m, n = c->p.n, R = c->p.R;
    if (R == 0) return DMMV_OK;
    int32_t K = k_eps > 0 ? k_eps : 100;
    if (K > SWAP_KMAX) K = SWAP_KMAX;
    if ((int64_t)K > m) K = (int32_t)m;
    const int32_t nb = c->swap_nb;
    int32_t* skip = use_skip ? c->swap_skip : nullptr;
    // LDS: the K residuals and rows always; then D[k_j] and filter rows of A
    size_t used = (size_t)K * (sizeof(T) + sizeof(int32_t)) + 64;
    const bool dvl = used + (size_t)n * sizeof(T) <= SW_LDS_BUDGET;
    if (dvl) used += (size_t)n * sizeof(T);
    int64_t L = n > 0 ? (int64_t)((SW_LDS_BUDGET - used) / ((size_t)n * sizeof(T))) : 0;
    if (L > K) L = K;
    used += (size_t)L * n * sizeof(T);

    if (K > 0)
        hipLaunchKernelGGL(k_swap_top<T>, dim3((unsigned)R), dim3(SW_BLOCK), 0, c->stream, m, R, K, (const T*)c->r,
                           (const int32_t*)skip, c->swap_rows);
    const dim3 grid((unsigned)R, (unsigned)nb);
    DMMV_TRY(ensure_dynamic_lds(reinterpret_cast<const void*>(&k_swap_eval<T, true>), (int)SW_LDS_BUDGET));
    DMMV_TRY(ensure_dynamic_lds(reinterpret_cast<const void*>(&k_swap_eval<T, false>), (int)SW_LDS_BUDGET));
#define DMMV_SWAP_LAUNCH(DV)                                                                               \
    hipLaunchKernelGGL((k_swap_eval<T, DV>), grid, dim3(SWE_BLOCK), used, c->stream, m, n, R, nb, K,       \
                       (int32_t)L, (const T*)c->p.A_dense, c->p.lda,                                       \
                       (const T*)(c->kind == KIND_BATCHED ? c->Xt : nullptr), (const T*)c->D_dev,          \
                       (const T*)c->scale_dev, (const int32_t*)c->kidx, (const T*)c->r,                    \
                       (const InstState<T>*)c->state, c->o.var_mask, (const int32_t*)c->swap_rows,         \
                       (const int32_t*)skip, (Partial<T>*)c->swap_part)
    if (dvl) DMMV_SWAP_LAUNCH(true);
    else DMMV_SWAP_LAUNCH(false);
#undef DMMV_SWAP_LAUNCH
    hipLaunchKernelGGL(k_swap_apply<T>, dim3((unsigned)R), dim3(SW_BLOCK), 0, c->stream, m, n, R, nb, apply,
                       (const T*)c->p.A_dense, c->p.lda, (const T*)c->D_dev, (const T*)c->scale_dev, c->kidx,
                       (T*)c->r, (InstState<T>*)c->state, (const Partial<T>*)c->swap_part, skip,
                       use_skip ? 1 : 0, best, (T*)best_t);
    DMMV_LAUNCH_CHECK();
    return DMMV_OK;
}

}  // namespace

int32_t swap_blocks_per_instance(const dmmv_problem& p) {
    // about 2048 workgroups in all, at most one per first variable
    int64_t nb = ceil_div(2048, p.R > 0 ? p.R : 1);
    if (nb > p.n) nb = p.n;
    if (nb < 1) nb = 1;
    return (int32_t)nb;
}

dmmv_status swap_clear_skip(Ctx* c) {
    if (!c->swap_skip) return fail(DMMV_ERR_STATE, "swap move: workspace is missing");
    if (c->p.R == 0) return DMMV_OK;
    hipLaunchKernelGGL(k_swap_clear, dim3((unsigned)ceil_div(c->p.R, 256)), dim3(256), 0, c->stream, c->swap_skip,
                       c->p.R);
    DMMV_LAUNCH_CHECK();
    return DMMV_OK;
}

dmmv_status swap_move(Ctx* c, int32_t k_eps, int32_t apply, bool use_skip, dmmv_swap* best, void* best_t) {
    if (c->kind == KIND_CSC) return swap_move_csc(c, apply, use_skip, best, best_t);
    if (!c->swap_skip || !c->swap_rows || !c->swap_part)
        return fail(DMMV_ERR_STATE, "swap move: workspace is missing");
    return c->p.dtype == DMMV_F64 ? swap_t<double>(c, k_eps, apply, use_skip, best, best_t)
                                  : swap_t<float>(c, k_eps, apply, use_skip, best, best_t);
}

}  // namespace dmmv
