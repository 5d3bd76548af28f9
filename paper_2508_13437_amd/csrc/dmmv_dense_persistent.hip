// Dense single instance, small enough that a launch per step costs more than the step: the
// whole descent (score every move, pick the best, apply it, repeat) in ONE launch.
//
// The moves are cut into units of one variable x DP_KT values of D.  A fixed grid of G
// workgroups shares the units; a workgroup keeps its own copy of r, the columns of A its units
// need and the current indices k_j in LDS for the whole call.  Per iteration it scores its
// units (same arithmetic as the evaluation kernel: |fma(delta, A_ij, r_i)|, maximum over the
// rows), publishes one (score, move) record, reads the records of all workgroups and takes
// their minimum - every workgroup arrives at the same move - and applies it to its own r.  One
// exchange per iteration is the only communication; r is never written to memory before the end.
//
// A record travels as four 64-bit words, each carrying the iteration number in its upper half and
// 32 bits of (score, move index) in its lower half.  Every word is written and read with one
// atomic access and names its own iteration, so the writer needs no ordering between its stores
// and a reader needs no separate arrival flag: it polls the four words until all name the
// iteration it is in (one round trip through the L2 instead of two).  Slots alternate with the
// parity of the iteration; a workgroup can be at most one iteration ahead of the slowest, so a
// slot is never overwritten while somebody still waits for it.
//
// The exchange is a wait on other workgroups, so all G must be resident at once (G never
// exceeds the number of compute units, and each needs at most one unit's LDS).  Should the
// device be shared with another kernel that keeps some of them from starting, the wait ends
// after options.wait_limit polls: the kernel raises an error flag, every workgroup leaves, and
// dmmv_solve returns DMMV_ERR_STATE.
#include "dmmv_common.h"

namespace dmmv {

constexpr int DP_KT = 16;                 // values of D per unit
constexpr int DP_MAX_WAVES = 8;            // wavefronts per workgroup: 4 (one per SIMD) or 8, chosen with the grid
constexpr int DP_MAX_THREADS = 64 * DP_MAX_WAVES;
constexpr int DP_SKEW = 65;               // row stride of the per-wavefront transpose scratch
constexpr int DP_MAX_G = 256;
constexpr size_t DP_LDS_LIMIT = 156 * 1024;
constexpr int32_t DP_WAIT_DEFAULT = 1 << 22;
// The loop of launches, for the automatic choice: its two launches take 8.1 us before any work
// is done, and the chip-wide evaluation kernel then needs about 81 ns per million (row, move)
// pairs in fp64 and 40 in fp32 (fitted to the measured iterations of small and large instances).
constexpr double DP_LAUNCH_LOOP_US = 8.1;
constexpr double DP_LAUNCH_LOOP_US_PER_PAIR_F64 = 8.1e-8, DP_LAUNCH_LOOP_US_PER_PAIR_F32 = 4.0e-8;

constexpr int DP_REC_WORDS = 4;
size_t dense_persistent_exchange_bytes() { return (size_t)2 * DP_MAX_G * DP_REC_WORDS * sizeof(uint64_t); }

namespace {

struct Plan {
    int G = 0;            // workgroups (0: not applicable)
    int upw = 0;          // units per workgroup
    int ncols = 0;        // columns of A a workgroup keeps in LDS
    int waves = 0;        // wavefronts per workgroup
    size_t lds = 0;
    double est_us = 0;    // modelled time of one iteration
};

// Picks the grid and the workgroup size: more workgroups shorten the scoring and lengthen the
// exchange; eight wavefronts per workgroup instead of four put two on every SIMD, which share its
// arithmetic but hide each other's latencies (better when a wavefront would otherwise take
// several units in a row, worse for a single short unit).  Measured on MI355X: the exchange
// takes about 2 us + 4 ns per workgroup, the rest of an iteration outside the scoring 1.6 us;
// 64 (row, move) pairs cost a wavefront about 18 cycles in fp64 (the maximum is not a full-rate
// instruction) and 10 in fp32 when it has its SIMD to itself, 32 and 16 when it shares it; the
// reduction of a unit's 16 x 64 lane maxima about 400.
Plan make_plan(const dmmv_problem& p, int cus) {
    Plan best;
    if (p.csr_rowptr || p.R != 1 || p.scale || p.m < 1 || p.n < 1 || p.nd < 1) return best;
    const size_t w = p.dtype == DMMV_F64 ? 8 : 4;
    const int64_t tiles = ceil_div(p.nd, DP_KT);
    const int64_t U = p.n * tiles;
    if (p.m > (int64_t)(DP_LDS_LIMIT / w) || p.n > (1 << 20) || p.nd > (1 << 16)) return best;
    const int gmax = cus < DP_MAX_G ? (cus > 0 ? cus : 1) : DP_MAX_G;
    for (int waves = 4; waves <= DP_MAX_WAVES; waves *= 2) {
        for (int want = 1;; want = want * 2 < gmax ? want * 2 : gmax) {
            const int64_t upw = ceil_div(U, want);
            const int64_t G = ceil_div(U, upw);
            int64_t ncols = 1;
            for (int64_t g = 0; g < G; ++g) {
                const int64_t u0 = g * upw, u1 = (g + 1) * upw < U ? (g + 1) * upw : U;
                const int64_t span = (u1 - 1) / tiles - u0 / tiles + 1;
                if (span > ncols) ncols = span;
            }
            const size_t lds = (size_t)(1 + ncols) * p.m * w + (size_t)waves * DP_KT * DP_SKEW * w + (size_t)p.nd * w +
                               (size_t)p.n * 4;
            if (lds <= DP_LDS_LIMIT) {
                const double per_64 = waves == 4 ? (w == 8 ? 18.0 : 10.0) : (w == 8 ? 32.0 : 16.0);
                const double per_unit = (double)ceil_div(p.m, 64) * DP_KT * per_64 + 400.0;     // cycles
                const double est = 2.0 + 0.004 * (double)G + (double)ceil_div(upw, waves) * per_unit / 2400.0 + 1.6;
                if (best.G == 0 || est < best.est_us) {
                    best.G = (int)G; best.upw = (int)upw; best.ncols = (int)ncols; best.waves = waves; best.lds = lds;
                    best.est_us = est;
                }
            }
            if (want == gmax) break;
        }
    }
    return best;
}

int device_cus() {
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess) return 0;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return 0;
    return cus;
}

__device__ __forceinline__ uint64_t score_bits(double s) { return (uint64_t)__double_as_longlong(s); }
__device__ __forceinline__ uint64_t score_bits(float s) { return (uint64_t)__float_as_uint(s); }
__device__ __forceinline__ void score_from(uint64_t b, double& s) { s = __longlong_as_double((long long)b); }
__device__ __forceinline__ void score_from(uint64_t b, float& s) { s = __uint_as_float((uint32_t)b); }

__global__ void k_zero_words(uint32_t* p, int n) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0;
}

template <class T, int NWAVES>
__global__ __launch_bounds__(64 * NWAVES) void k_descent_dense_persistent(
    int64_t m, int64_t n, int32_t nd, const T* __restrict__ A, int64_t lda, const T* __restrict__ D,
    T* r, int32_t* kidx, int32_t radius, const uint8_t* __restrict__ var_mask, InstState<T>* st,
    int32_t keep_going, int32_t iters, dmmv_move* trace, T* trace_t, int32_t tiles, int32_t upw,
    int32_t ncols, uint64_t* rec /*[2][G][DP_REC_WORDS]*/, int32_t* flags, int32_t wait_limit) {
    constexpr int KT = DP_KT;
    extern __shared__ __align__(16) unsigned char smem[];
    T* sh_r = reinterpret_cast<T*>(smem);                   // [m]
    T* sh_cols = sh_r + m;                                  // [ncols][m]
    constexpr int nthreads = 64 * NWAVES, nwaves = NWAVES;
    T* sh_sc = sh_cols + (int64_t)ncols * m;                // [nwaves][KT * DP_SKEW]
    T* sh_D = sh_sc + nwaves * KT * DP_SKEW;                // [nd]
    int32_t* sh_kidx = reinterpret_cast<int32_t*>(sh_D + nd);   // [n]
    __shared__ T sh_ws[NWAVES];
    __shared__ int64_t sh_wc[NWAVES];
    __shared__ T sh_bs;
    __shared__ int64_t sh_bc;
    __shared__ int32_t sh_fail;

    const int G = gridDim.x, g = blockIdx.x;
    const int tid = threadIdx.x, lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int64_t U = n * tiles;
    const int64_t u0 = (int64_t)g * upw, u1 = u0 + upw < U ? u0 + upw : U;
    const int64_t j_lo = u0 / tiles, j_hi = (u1 - 1) / tiles;

    for (int64_t i = tid; i < m; i += nthreads) sh_r[i] = r[i];
    for (int64_t j = j_lo; j <= j_hi; ++j)
        for (int64_t i = tid; i < m; i += nthreads) sh_cols[(j - j_lo) * m + i] = A[lda * j + i];
    for (int64_t j = tid; j < n; j += nthreads) sh_kidx[j] = kidx[j];
    for (int32_t k = tid; k < nd; k += nthreads) sh_D[k] = D[k];
    if (tid == 0) sh_fail = 0;
    T t = st[0].t;
    int32_t moves = st[0].moves;
    T last_s = st[0].best_s;
    bool stopped = st[0].done != 0, failed = false;
    __syncthreads();

    // A wavefront with a single unit keeps that unit's level index and steps in registers; they
    // change only when a move lands on its variable (the chain level index -> levels -> steps is
    // three LDS latencies that nothing hides with one wavefront per SIMD).
    const bool one_unit = upw <= nwaves;
    bool steps_stale = true;
    int32_t kcur_keep = 0;
    T delta_keep[KT];
#pragma unroll
    for (int q = 0; q < KT; ++q) delta_keep[q] = (T)0;

    for (int32_t it = 0; it < iters && !stopped; ++it) {
        // ---- score this wavefront's units ------------------------------------------------
        T ws = (T)0;
        int64_t wc = -1;
        for (int64_t u = u0 + w; u < u1; u += nwaves) {
            const int64_t j = u / tiles;
            const int32_t kbase = (int32_t)(u % tiles) * KT;
            const T* __restrict__ col = sh_cols + (j - j_lo) * m;
            T delta[KT], acc[KT];
            int32_t kcur;
            if (!one_unit || steps_stale) {
                kcur = sh_kidx[j];
                const T dcur = sh_D[kcur];
#pragma unroll
                for (int q = 0; q < KT; ++q) {
                    const int32_t k = kbase + q < nd ? kbase + q : nd - 1;
                    delta[q] = step_of(sh_D[k], dcur, (T)1);
                }
                if (one_unit) {
                    kcur_keep = kcur;
#pragma unroll
                    for (int q = 0; q < KT; ++q) delta_keep[q] = delta[q];
                    steps_stale = false;
                }
            } else {
                kcur = kcur_keep;
#pragma unroll
                for (int q = 0; q < KT; ++q) delta[q] = delta_keep[q];
            }
#pragma unroll
            for (int q = 0; q < KT; ++q) acc[q] = (T)0;
            // two rows per pass, both requested before the first is used (a row past the end
            // is replaced by the pass's first row: a maximum does not mind the repeat)
            for (int64_t i = lane; i < m; i += 128) {
                const int64_t i2 = i + 64 < m ? i + 64 : i;
                const T a = col[i], ri = sh_r[i], a2 = col[i2], ri2 = sh_r[i2];
#pragma unroll
                for (int q = 0; q < KT; ++q) acc[q] = dmmv_max(acc[q], dmmv_abs(dmmv_fma(delta[q], a, ri)));
#pragma unroll
                for (int q = 0; q < KT; ++q) acc[q] = dmmv_max(acc[q], dmmv_abs(dmmv_fma(delta[q], a2, ri2)));
            }
            // 16 x 64 lane maxima -> 16 scores: lane folds a quarter of value lane / 4, two DPP steps join
            T* sc = sh_sc + w * KT * DP_SKEW;
#pragma unroll
            for (int q = 0; q < KT; ++q) sc[q * DP_SKEW + lane] = acc[q];
            __builtin_amdgcn_wave_barrier();
            const int q = lane >> 2, quarter = lane & 3;
            T v = (T)0;
#pragma unroll
            for (int e = 0; e < 16; ++e) v = dmmv_max(v, sc[q * DP_SKEW + quarter * 16 + e]);
            __builtin_amdgcn_wave_barrier();
            v = dmmv_max(v, dpp_mov<DPP_QUAD_XOR1>(v));
            v = dmmv_max(v, dpp_mov<DPP_QUAD_XOR2>(v));
            // the unit's candidates sit in lanes 0, 4, 8, ... in ascending k: the smallest score,
            // then the first lane that holds it
            const int32_t k = kbase + q;
            const bool cand = quarter == 0 && k < nd;
            T cs = Limits<T>::inf();
            if (cand) {
                const bool var_ok = var_mask ? var_mask[j] != 0 : true;
                if (cand_allowed(kcur, k, radius, var_ok)) cs = v;
            }
            const T smin = wave_min(cs);
            const unsigned long long hit = __ballot(cand && cs == smin);
            if (hit) {
                const int64_t cc = j * (int64_t)nd + kbase + (__builtin_ctzll(hit) >> 2);
                if (rec_less(smin, cc, ws, wc)) { ws = smin; wc = cc; }
            }
        }
        if (lane == 0) { sh_ws[w] = ws; sh_wc[w] = wc; }
        __syncthreads();
        // ---- publish this workgroup's record ------------------------------------------------
        const uint64_t tag = (uint64_t)(uint32_t)(it + 1) << 32;
        if (tid == 0) {
            T bs = (T)0;
            int64_t bc = -1;
            T xs[NWAVES];
            int64_t xc[NWAVES];
#pragma unroll
            for (int x = 0; x < NWAVES; ++x) { xs[x] = sh_ws[x]; xc[x] = sh_wc[x]; }
#pragma unroll
            for (int x = 0; x < NWAVES; ++x)
                if (rec_less(xs[x], xc[x], bs, bc)) { bs = xs[x]; bc = xc[x]; }
            uint64_t* slot = rec + ((int64_t)(it & 1) * G + g) * DP_REC_WORDS;
            const uint64_t sb = score_bits(bs), cb = (uint64_t)bc;
            __hip_atomic_store(&slot[0], tag | (sb >> 32), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __hip_atomic_store(&slot[1], tag | (sb & 0xffffffffull), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __hip_atomic_store(&slot[2], tag | (cb >> 32), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __hip_atomic_store(&slot[3], tag | (cb & 0xffffffffull), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        // ---- read every workgroup's record (wavefront 0; lane q takes workgroups q, q + 64, ..)
        if (w == 0) {
            T gs = (T)0;
            int64_t gc = -1;
            uint32_t fail = 0;
            for (int q = lane; q < G; q += 64) {
                const uint64_t* slot = rec + ((int64_t)(it & 1) * G + q) * DP_REC_WORDS;
                // Two reads of the record are kept in flight (loads return in order): a read
                // samples memory half a round trip after it was issued, so with one read at a
                // time a record that lands just after the sample costs a whole further round
                // trip; the second read halves that.
                const uint64_t hi = 0xffffffff00000000ull;
                uint64_t a0, a1, a2, a3, b0, b1, b2, b3;
#define DP_READ(x0, x1, x2, x3)                                                              \
    x0 = __hip_atomic_load(&slot[0], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);             \
    x1 = __hip_atomic_load(&slot[1], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);             \
    x2 = __hip_atomic_load(&slot[2], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);             \
    x3 = __hip_atomic_load(&slot[3], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
#define DP_THERE(x0, x1, x2, x3) (((x0) & hi) == tag && ((x1) & hi) == tag && ((x2) & hi) == tag && ((x3) & hi) == tag)
                int32_t polls = 0;
                bool there = false;
                DP_READ(a0, a1, a2, a3)
                do {
                    DP_READ(b0, b1, b2, b3)
                    there = DP_THERE(a0, a1, a2, a3);
                    if (there) break;
                    DP_READ(a0, a1, a2, a3)
                    there = DP_THERE(b0, b1, b2, b3);
                    if (there) { a0 = b0; a1 = b1; a2 = b2; a3 = b3; break; }
                    polls += 2;
                    // somebody else has given up already: no point in waiting out the limit
                    if ((polls & 254) == 254 &&
                        __hip_atomic_load(&flags[FLAG_ERROR], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0)
                        polls = wait_limit;
                } while (polls < wait_limit);
#undef DP_READ
#undef DP_THERE
                if (!there) { fail = 1; break; }
                T s;
                score_from((a0 << 32) | (a1 & 0xffffffffull), s);
                const int64_t c = (int64_t)((a2 << 32) | (a3 & 0xffffffffull));
                if (rec_less(s, c, gs, gc)) { gs = s; gc = c; }
            }
            wave_argmin(gs, gc);
            fail = __ballot(fail != 0) != 0ull;
            if (lane == 0) {
                sh_bs = gs;
                sh_bc = gc;
                if (fail) { sh_fail = 1; atomicOr(&flags[FLAG_ERROR], ERRBIT_WAIT_LIMIT); }
            }
        }
        __syncthreads();
        if (sh_fail) { failed = true; break; }
        // ---- the same decision in every workgroup ------------------------------------------
        const T s = sh_bs;
        const int64_t c = sh_bc;
        last_s = s;
        if (c >= 0 && s < t) {
            const int32_t j = (int32_t)(c / nd), k = (int32_t)(c % nd);
            const T delta = step_of(sh_D[k], sh_D[sh_kidx[j]], (T)1);
            if (g == 0 && tid == 0 && moves < iters) {
                if (trace) { trace[moves].j = j; trace[moves].k = k; }
                if (trace_t) trace_t[moves] = s;
            }
            const T* __restrict__ colg = A + lda * (int64_t)j;
            for (int64_t i = tid; i < m; i += nthreads) sh_r[i] = dmmv_fma(delta, colg[i], sh_r[i]);
            __syncthreads();                                  // every thread has read sh_kidx[j]
            if (tid == 0) sh_kidx[j] = k;
            if (one_unit && u0 + w < u1 && (u0 + w) / tiles == j) steps_stale = true;
            t = s;
            moves += 1;
        } else if (!keep_going) {
            stopped = true;
        }
        __syncthreads();
    }
    // ---- workgroup 0 hands the state back (after a failed wait the state is not written) ---
    if (g != 0 || failed) return;
    for (int64_t i = tid; i < m; i += nthreads) r[i] = sh_r[i];
    for (int64_t j = tid; j < n; j += nthreads) kidx[j] = sh_kidx[j];
    if (tid == 0) {
        InstState<T> z = st[0];
        z.t = t;
        z.best_s = last_s;
        z.apply_j = -1; z.apply_k = -1; z.delta = (T)0;
        z.moves = moves;
        z.done = stopped ? 1 : 0;
        st[0] = z;
    }
}

template <class T>
dmmv_status run_t(Ctx* c, const Plan& pl, int32_t iters, dmmv_move* trace, void* trace_t) {
    // iteration numbers start at 1: cleared records name no iteration
    uint64_t* rec = (uint64_t*)c->persist_exchange;
    const int words = 2 * DP_MAX_G * DP_REC_WORDS * 2;       // as 32-bit words
    hipLaunchKernelGGL(k_zero_words, dim3((unsigned)ceil_div(words, 256)), dim3(256), 0, c->stream, (uint32_t*)rec, words);
    const int32_t wait_limit = c->o.wait_limit > 0 ? c->o.wait_limit : DP_WAIT_DEFAULT;
    auto kernel = pl.waves == 8 ? k_descent_dense_persistent<T, 8> : k_descent_dense_persistent<T, 4>;
    DMMV_TRY(ensure_dynamic_lds((const void*)kernel, (int)DP_LDS_LIMIT));
    hipLaunchKernelGGL(kernel, dim3((unsigned)pl.G), dim3(64 * pl.waves), pl.lds, c->stream,
                       c->p.m, c->p.n, c->p.nd, (const T*)c->p.A_dense, c->p.lda, (const T*)c->D_dev, (T*)c->r,
                       c->kidx, c->o.radius, c->o.var_mask, (InstState<T>*)c->state, c->o.keep_going, iters, trace,
                       (T*)trace_t, (int32_t)ceil_div(c->p.nd, DP_KT), (int32_t)pl.upw, (int32_t)pl.ncols, rec,
                       c->flags, wait_limit);
    DMMV_LAUNCH_CHECK();
    return DMMV_OK;
}

}  // namespace

// options.dense_loop: 0 = one launch when the model says its iteration is shorter than that of
// the loop of launches, 1 = always a launch per step, 2 = one launch whenever the instance fits
// (dmmv_create refuses the option otherwise).
bool dense_persistent_fits(const dmmv_problem& p) { return make_plan(p, DP_MAX_G).G > 0; }

bool dense_persistent_applicable(const Ctx* c) {
    if (c->kind != KIND_DENSE || c->o.dense_loop == 1 || !c->persist_exchange) return false;
    if (c->o.l2_rule == 1 || c->o.l2_rule == 2) return false;
    if (!c->o.keep_going && (c->o.value_search || c->o.prune)) return false;      // those have loops of their own
    const Plan pl = make_plan(c->p, device_cus());
    if (pl.G == 0) return false;
    if (c->o.dense_loop == 2) return true;
    const double pairs = (double)c->p.m * (double)c->p.n * (double)c->p.nd;
    const double launches_us = DP_LAUNCH_LOOP_US + pairs * (c->p.dtype == DMMV_F64 ? DP_LAUNCH_LOOP_US_PER_PAIR_F64
                                                                                   : DP_LAUNCH_LOOP_US_PER_PAIR_F32);
    return pl.est_us < launches_us;
}

dmmv_status dense_descent_persistent(Ctx* c, int32_t iters, dmmv_move* trace, void* trace_t) {
    const Plan pl = make_plan(c->p, device_cus());
    if (pl.G == 0) return fail(DMMV_ERR_STATE, "one-launch dense descent: the instance does not fit");
    return c->p.dtype == DMMV_F64 ? run_t<double>(c, pl, iters, trace, trace_t)
                                  : run_t<float>(c, pl, iters, trace, trace_t);
}

}  // namespace dmmv
