// Dense matrices with many values in D: the best value of one variable by bisection instead of
// scoring all nd values (options.value_search; the descent only).
//
// For a fixed variable j the score of value k is g(k) = max_i |x_i(k)|, x_i(k) =
// fma(delta_k, A_ij, r_i), delta_k = s (D[k] - D[k_j]).  D ascends and rounding is monotone, so
// delta_k does not decrease with k, x_i(k) is monotone in k (up if A_ij > 0, down if A_ij < 0)
// and |x_i(k)| falls and then rises: g is a maximum of such sequences, hence quasi-convex - in
// the computed values, not only in exact arithmetic (its sublevel sets are intervals).
//
// At a value k look at the rows that attain g(k).  If one of them is on its rising side
// (x_i > 0 and A_ij > 0, x_i < 0 and A_ij < 0, A_ij = 0, or x_i = 0), no higher value scores
// strictly less: the lowest best value is <= k.  Otherwise all of them are on their falling
// side, no lower value scores strictly less, and g(k + 1) decides: if it is larger, k is a best
// value (quasi-convexity puts everything above k + 1 at least as high); if not, a best value
// lies above k.  The interval halves every step; at the end the value found is walked down while
// its lower neighbour scores the same, which gives the lowest of the best values, i.e. exactly
// the record (score, index) the full evaluation would reduce this variable to.
//
// One workgroup per variable; the thread's rows of the column and of r stay in registers, so a
// step is arithmetic on registers and one reduction over the workgroup.
#include "dmmv_common.h"

namespace dmmv {

namespace {

constexpr int VS_BLOCK = 256;
constexpr int VS_WAVES = VS_BLOCK / 64;
constexpr int VS_RPT = 16;                 // rows per thread kept in registers

template <class T>
struct VsShared {
    T g0[VS_WAVES], g1[VS_WAVES];
    uint32_t up[VS_WAVES];
};

// g(k), g(k + 1) and whether a row attaining g(k) is on its rising side.  REG: rows in registers.
template <class T, bool REG>
__device__ __forceinline__ void vs_probe(int64_t m, const T* __restrict__ col, const T* __restrict__ r,
                                         const T (&a_reg)[VS_RPT], const T (&r_reg)[VS_RPT], T d0, T d1,
                                         VsShared<T>& sh, T& g0, T& g1, bool& up) {
    T m0 = (T)0, m1 = (T)0;
    bool rising = false;
    auto row = [&](T a, T ri) {
        const T x0 = dmmv_fma(d0, a, ri);
        const T v0 = dmmv_abs(x0);
        const bool rise = (x0 > (T)0 && a > (T)0) || (x0 < (T)0 && a < (T)0) || a == (T)0 || x0 == (T)0;
        if (v0 > m0) { m0 = v0; rising = rise; }
        else if (v0 == m0) rising = rising || rise;
        m1 = dmmv_max(m1, dmmv_abs(dmmv_fma(d1, a, ri)));
    };
    if (REG) {
#pragma unroll
        for (int u = 0; u < VS_RPT; ++u) row(a_reg[u], r_reg[u]);
    } else {
        for (int64_t i = threadIdx.x; i < m; i += VS_BLOCK) row(col[i], r[i]);
    }
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const T w0 = wave_max(m0), w1 = wave_max(m1);
    if (lane == 0) { sh.g0[w] = w0; sh.g1[w] = w1; }
    __syncthreads();
    g0 = sh.g0[0];
    g1 = sh.g1[0];
#pragma unroll
    for (int u = 1; u < VS_WAVES; ++u) { g0 = dmmv_max(g0, sh.g0[u]); g1 = dmmv_max(g1, sh.g1[u]); }
    const unsigned long long b = __ballot(rising && m0 == g0);
    if (lane == 0) sh.up[w] = b != 0ull ? 1u : 0u;
    __syncthreads();
    uint32_t any = 0;
#pragma unroll
    for (int u = 0; u < VS_WAVES; ++u) any |= sh.up[u];
    up = any != 0;
    __syncthreads();                                       // sh is rewritten by the next probe
}

template <class T, bool REG>
__global__ __launch_bounds__(VS_BLOCK) void k_eval_dense_search(
    int64_t m, int32_t nd, const T* __restrict__ A, int64_t lda, const T* __restrict__ D,
    const int32_t* __restrict__ kidx, const T* __restrict__ r, int32_t radius,
    const uint8_t* __restrict__ var_mask, const InstState<T>* __restrict__ st, int32_t honor_done,
    Partial<T>* __restrict__ part) {
    __shared__ VsShared<T> sh;
    if (honor_done && st[0].done) return;
    const int64_t j = blockIdx.x;
    const T* __restrict__ col = A + j * lda;
    T a_reg[VS_RPT], r_reg[VS_RPT];
    if (REG) {
#pragma unroll
        for (int u = 0; u < VS_RPT; ++u) {
            const int64_t i = threadIdx.x + (int64_t)u * VS_BLOCK;
            a_reg[u] = i < m ? col[i] : (T)0;              // a row past the end scores |0|
            r_reg[u] = i < m ? r[i] : (T)0;
        }
    }
    const int32_t kcur = kidx[j];
    const T dcur = D[kcur];
    const bool var_ok = var_mask ? var_mask[j] != 0 : true;
    int32_t lo = kcur, hi = kcur;                          // the values this variable may take
    if (var_ok) {
        lo = radius > 0 ? (kcur - radius > 0 ? kcur - radius : 0) : 0;
        hi = radius > 0 ? (kcur + radius < nd - 1 ? kcur + radius : nd - 1) : nd - 1;
    }
    const int32_t klo = lo;
    auto delta = [&](int32_t k) -> T { return step_of(D[k < nd ? k : nd - 1], dcur, (T)1); };
    T g0, g1;
    bool up;
    while (lo < hi) {
        const int32_t mid = (lo + hi) >> 1;                // mid + 1 <= hi
        vs_probe<T, REG>(m, col, r, a_reg, r_reg, delta(mid), delta(mid + 1), sh, g0, g1, up);
        if (up) hi = mid;
        else if (g1 <= g0) lo = mid + 1;
        else { lo = mid; hi = mid; }
    }
    int32_t kbest = lo;
    // its score, and that of its lower neighbour; walk down while they are equal
    vs_probe<T, REG>(m, col, r, a_reg, r_reg, delta(kbest > klo ? kbest - 1 : kbest), delta(kbest), sh, g0, g1, up);
    T best = g1;
    while (kbest > klo && g0 == best) {
        --kbest;
        if (kbest > klo) vs_probe<T, REG>(m, col, r, a_reg, r_reg, delta(kbest - 1), delta(kbest), sh, g0, g1, up);
    }
    if (threadIdx.x == 0) {
        Partial<T> p;
        p.s = best;
        p.c = j * (int64_t)nd + kbest;
        part[j] = p;
    }
}

template <class T>
dmmv_status search_t(Ctx* c, bool honor_done) {
    const int64_t m = c->p.m, n = c->p.n;
    if (n == 0) return DMMV_OK;
    auto launch = [&](auto kernel) {
        hipLaunchKernelGGL(kernel, dim3((unsigned)n), dim3(VS_BLOCK), 0, c->stream, m, c->p.nd,
                           (const T*)c->p.A_dense, c->p.lda, (const T*)c->D_dev, (const int32_t*)c->kidx,
                           (const T*)c->r, c->o.radius, c->o.var_mask, (const InstState<T>*)c->state,
                           (int32_t)honor_done, (Partial<T>*)c->search_part);
    };
    if (m <= (int64_t)VS_BLOCK * VS_RPT) launch(k_eval_dense_search<T, true>);
    else launch(k_eval_dense_search<T, false>);
    DMMV_LAUNCH_CHECK();
    return DMMV_OK;
}

}  // namespace

dmmv_status dense_eval_search(Ctx* c, bool honor_done) {
    if (!c->search_part) return fail(DMMV_ERR_STATE, "value search: workspace is missing");
    return c->p.dtype == DMMV_F64 ? search_t<double>(c, honor_done) : search_t<float>(c, honor_done);
}

}  // namespace dmmv
