// Batched instances: the descent with exact pruning (options.prune), one workgroup per instance.
//
// The score of a move (j, k) is a maximum over all m rows, so the maximum over ANY subset of the
// rows is a lower bound of it, and a move can only win if its lower bound is below the score of
// the best move known (Corollary 1 turns the same observation into a filter for swaps: a move
// that does not fix the rows of largest |r| cannot improve).  Per iteration the workgroup
//   1. picks S = 16 screening rows: the four rows of largest |r| out of each wavefront's share
//      of the rows (the row of largest |r| overall is always one of them);
//   2. computes, for every candidate, the bound lb(j, k) = max_{i in S} |fma(delta, X_ij, r_i)|
//      - 16 rows instead of m - and keeps per variable its best candidate by (lb, k);
//   3. takes candidates in ascending order of (lb, c), c = j nd + k, scores each one over all m
//      rows (the same fma on the same operands as the full evaluation, so the same bits), and
//      stops as soon as the next candidate's (lb, c) is not below the best (score, c) found:
//      every candidate not scored has score >= lb >= that best score, and loses the tie on c;
//   4. applies the move if its score is below t.
// The result is the arg-min of the full table restricted to strictly improving moves, i.e. the
// move the full evaluation + selection would apply - found with a few full scores instead of
// n (nd - 1).  The instance's r (m values) and x (n level indices) live in LDS for the whole
// launch, so a launch can run any number of iterations without touching the other instances;
// an instance stops by itself at a local optimum.
#include "dmmv_common.h"

namespace dmmv {

namespace {

constexpr int BP_BLOCK = 256;
constexpr int BP_WAVES = BP_BLOCK / 64;
constexpr int BP_TOPW = 4;                       // screening rows a wavefront contributes
constexpr int BP_S = BP_WAVES * BP_TOPW;         // screening rows
constexpr int BP_MAX_RPT = 64;                   // rows per thread at most (one bit each in a 64-bit mask)
constexpr size_t BP_LDS_LIMIT = 96 * 1024;       // dynamic LDS a workgroup may ask for

template <class T>
struct BpShared {
    T top_r[BP_S];
    int32_t top_row[BP_S];
    T red_s[BP_WAVES];
    int64_t red_c[BP_WAVES];
    T red_m[BP_WAVES];
    T pop_s;
    int64_t pop_c;
};

template <class T>
__device__ __forceinline__ size_t bp_lds_bytes(int64_t m, int64_t n) {
    return (size_t)(m + n) * sizeof(T) + (size_t)n * 2 * sizeof(uint16_t);
}

// KT: candidate values scored together per variable (register tile).  RAD: the neighbourhood is
// a radius around the current level (candidate levels differ from lane to lane); without it the
// levels are the same for every variable and their values of D are read once per tile.
template <class T, int KT, bool RAD>
__global__ __launch_bounds__(BP_BLOCK) void k_descent_batched_pruned(
    int64_t m, int64_t n, int32_t nd, int64_t R, const T* __restrict__ X, int64_t ldx,
    const T* __restrict__ Xt, const T* __restrict__ D, const T* __restrict__ scale,
    T* __restrict__ r, int32_t* __restrict__ kidx, InstState<T>* __restrict__ st, int32_t radius,
    const uint8_t* __restrict__ var_mask, int32_t steps, int32_t iters,
    dmmv_move* __restrict__ trace, T* __restrict__ trace_t) {
    extern __shared__ __align__(16) unsigned char smem[];
    __shared__ BpShared<T> F;
    T* sh_r = reinterpret_cast<T*>(smem);                  // the instance's residual
    T* sh_jmin = sh_r + m;                                 // per variable: bound of its next candidate
    uint16_t* sh_k = reinterpret_cast<uint16_t*>(sh_jmin + n);   // current level of every variable
    uint16_t* sh_jarg = sh_k + n;                          // per variable: level of its next candidate

    const int64_t q = blockIdx.x;
    InstState<T> z = st[q];
    if (z.done || steps <= 0) return;                      // the same for the whole workgroup
    const int tid = threadIdx.x, lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    for (int64_t i = tid; i < m; i += BP_BLOCK) sh_r[i] = r[i * R + q];
    for (int64_t j = tid; j < n; j += BP_BLOCK) sh_k[j] = (uint16_t)kidx[j * R + q];
    const T sc = scale[q];
    const uint8_t* __restrict__ vm = var_mask ? var_mask + q * n : nullptr;
    const int32_t rpt = (int32_t)((m + BP_BLOCK - 1) / BP_BLOCK);
    // candidate levels of a variable at level kc: k = base + o for o in [olo, ohi], base = kc
    // inside a radius and 0 otherwise; k == kc and k outside [0, nd) are left out
    const int32_t olo = RAD ? -radius : 0;
    const int32_t ohi = RAD ? radius : nd - 1;
    bool dirty = false;
    __syncthreads();

    for (int32_t step = 0; step < steps; ++step) {
        // ---- 1. screening rows -----------------------------------------------------------
        {
            uint64_t taken = 0;
            for (int round = 0; round < BP_TOPW; ++round) {
                T bv = (T)-1;
                int32_t bu = -1;
                for (int32_t u = 0; u < rpt; ++u) {
                    const int64_t i = tid + (int64_t)u * BP_BLOCK;
                    if (i < m && !((taken >> u) & 1ull)) {
                        const T a = dmmv_abs(sh_r[i]);
                        if (a > bv) { bv = a; bu = u; }
                    }
                }
                T s = -bv;                                  // largest |r| = smallest -|r|; ties: lowest row
                int64_t c = bu >= 0 ? tid + (int64_t)bu * BP_BLOCK : (int64_t)-1;
                const int64_t mine = c;
                wave_argmin(s, c);
                if (c >= 0 && c == mine) taken |= 1ull << bu;
                if (lane == 0) {
                    F.top_row[w * BP_TOPW + round] = (int32_t)c;
                    F.top_r[w * BP_TOPW + round] = c >= 0 ? sh_r[c] : (T)0;
                }
            }
        }
        __syncthreads();
        // a share with fewer rows than BP_TOPW repeats the first screening row (row 0 belongs to
        // wavefront 0, so entry 0 exists whenever m > 0); a repeated row changes no maximum
        const int32_t row0 = F.top_row[0];
        const T r0 = F.top_r[0];
        __syncthreads();
        if (tid < BP_S && F.top_row[tid] < 0) { F.top_row[tid] = row0; F.top_r[tid] = r0; }
        __syncthreads();
        if (row0 < 0) {                                    // m == 0: every score is 0 = t, nothing improves
            z.done = 1;
            z.best_s = z.t;
            break;
        }
        T tr[BP_S];
        const T* xrow[BP_S];
#pragma unroll
        for (int u = 0; u < BP_S; ++u) {
            tr[u] = F.top_r[u];
            xrow[u] = Xt + (int64_t)__builtin_amdgcn_readfirstlane(F.top_row[u]) * n;
        }

        // ---- 2. bounds of all candidates; per variable the best one by (lb, k) ------------
        for (int64_t j = tid; j < n; j += BP_BLOCK) {
            const int32_t kc = sh_k[j];
            const bool var_ok = vm ? vm[j] != 0 : true;
            T xs[BP_S];
#pragma unroll
            for (int u = 0; u < BP_S; ++u) xs[u] = xrow[u][j];
            const T dcur = D[kc];
            const int32_t base = RAD ? kc : 0;
            T jbest = Limits<T>::inf();
            int32_t jk = 0;
            for (int32_t o0 = olo; o0 <= ohi; o0 += KT) {
                T delta[KT], lb[KT], dk[KT];
                bool ok[KT];
                // all the tile's values of D are fetched before the first is used (a level outside
                // D reads an end of it and is masked below)
#pragma unroll
                for (int e = 0; e < KT; ++e) {
                    const int32_t k = base + o0 + e;
                    dk[e] = D[k < 0 ? 0 : (k < nd ? k : nd - 1)];
                }
#pragma unroll
                for (int e = 0; e < KT; ++e) {
                    const int32_t k = base + o0 + e;
                    ok[e] = var_ok && o0 + e <= ohi && k >= 0 && k < nd && k != kc;
                    delta[e] = ok[e] ? step_of(dk[e], dcur, sc) : (T)0;
                    lb[e] = (T)0;
                }
#pragma unroll
                for (int u = 0; u < BP_S; ++u)
#pragma unroll
                    for (int e = 0; e < KT; ++e) lb[e] = dmmv_max(lb[e], dmmv_abs(dmmv_fma(delta[e], xs[u], tr[u])));
#pragma unroll
                for (int e = 0; e < KT; ++e)
                    if (ok[e] && lb[e] < jbest) { jbest = lb[e]; jk = base + o0 + e; }   // k ascends: ties keep the lowest
            }
            sh_jmin[j] = jbest;
            sh_jarg[j] = (uint16_t)jk;
        }
        __syncthreads();

        // ---- 3. candidates in ascending (lb, c) until none can beat the best score ---------
        T best_s = z.t;                                    // only scores below t count
        int64_t best_c = -1;
        for (;;) {
            T s = Limits<T>::inf();
            int64_t c = -1;
            for (int64_t j = tid; j < n; j += BP_BLOCK) {
                const T v = sh_jmin[j];
                if (v < s) { s = v; c = j * (int64_t)nd + sh_jarg[j]; }   // j ascends: ties keep the lowest c
            }
            block_argmin(s, c, F.red_s, F.red_c);
            if (tid == 0) { F.pop_s = s; F.pop_c = c; }
            __syncthreads();
            const T ps = F.pop_s;
            const int64_t pc = F.pop_c;
            const bool go = pc >= 0 && (ps < best_s || (ps == best_s && best_c >= 0 && pc < best_c));
            if (!go) break;                                // the same for the whole workgroup
            const int64_t j = pc / nd;
            const int32_t k = (int32_t)(pc % nd);
            const int32_t kc = sh_k[j];
            const T dcur = D[kc];
            const T delta = step_of(D[k], dcur, sc);
            // its score over all rows
            const T* __restrict__ col = X + ldx * j;
            T acc = (T)0;
            for (int64_t i = tid; i < m; i += BP_BLOCK) acc = dmmv_max(acc, dmmv_abs(dmmv_fma(delta, col[i], sh_r[i])));
            acc = wave_max(acc);
            if (lane == 0) F.red_m[w] = acc;
            // meanwhile wavefront 0 looks for this variable's next candidate: the smallest (lb, k)
            // after (ps, k); lanes take the candidate levels
            if (w == 0) {
                const int32_t base = RAD ? kc : 0;
                const bool var_ok = vm ? vm[j] != 0 : true;
                T xs[BP_S];
#pragma unroll
                for (int u = 0; u < BP_S; ++u) xs[u] = xrow[u][j];
                T bl = Limits<T>::inf();
                int64_t bk = -1;
                for (int32_t o0 = olo; o0 <= ohi; o0 += 64) {
                    const int32_t o = o0 + lane;
                    const int32_t kk = base + o;
                    const bool ok = var_ok && o <= ohi && kk >= 0 && kk < nd && kk != kc;
                    const T dl = ok ? step_of(D[ok ? kk : 0], dcur, sc) : (T)0;
                    T lb = (T)0;
#pragma unroll
                    for (int u = 0; u < BP_S; ++u) lb = dmmv_max(lb, dmmv_abs(dmmv_fma(dl, xs[u], tr[u])));
                    const bool after = ok && (lb > ps || (lb == ps && kk > k));
                    if (after && lb < bl) { bl = lb; bk = kk; }       // kk ascends per lane: ties keep the lowest
                }
                wave_argmin(bl, bk);
                if (lane == 0) {
                    sh_jmin[j] = bk >= 0 ? bl : Limits<T>::inf();
                    sh_jarg[j] = (uint16_t)(bk >= 0 ? bk : 0);
                }
            }
            __syncthreads();
            T sfull = F.red_m[0];
#pragma unroll
            for (int u = 1; u < BP_WAVES; ++u) sfull = dmmv_max(sfull, F.red_m[u]);
            if (sfull < best_s || (sfull == best_s && best_c >= 0 && pc < best_c)) { best_s = sfull; best_c = pc; }
            __syncthreads();                               // red_m, pop_* are rewritten by the next round
        }

        // ---- 4. decide and apply ---------------------------------------------------------
        z.best_s = best_s;
        if (best_c < 0) { z.done = 1; break; }
        {
            const int64_t j = best_c / nd;
            const int32_t k = (int32_t)(best_c % nd);
            const T delta = step_of(D[k], D[sh_k[j]], sc);
            const T* __restrict__ col = X + ldx * j;
            for (int64_t i = tid; i < m; i += BP_BLOCK) sh_r[i] = dmmv_fma(delta, col[i], sh_r[i]);
            __syncthreads();                               // everyone has read sh_k[j]
            if (tid == 0) {
                sh_k[j] = (uint16_t)k;
                kidx[j * R + q] = k;
                if (z.moves < iters) {
                    const int64_t slot = q * (int64_t)iters + z.moves;
                    if (trace) { trace[slot].j = (int32_t)j; trace[slot].k = k; }
                    if (trace_t) trace_t[slot] = best_s;
                }
            }
            z.t = best_s;                                  // the applied move's score is the new max |r|, bit for bit
            z.moves += 1;
            dirty = true;
            __syncthreads();
        }
    }

    if (dirty)
        for (int64_t i = tid; i < m; i += BP_BLOCK) r[i * R + q] = sh_r[i];
    if (tid == 0) {
        z.apply_j = -1;
        z.apply_k = -1;
        z.delta = (T)0;
        st[q] = z;
    }
}

template <class T>
dmmv_status descent_t(Ctx* c, int32_t steps, int32_t iters, dmmv_move* trace, void* trace_t) {
    const int64_t m = c->p.m, n = c->p.n, R = c->p.R;
    const size_t lds = (size_t)(m + n) * sizeof(T) + (size_t)n * 2 * sizeof(uint16_t);
    const int32_t span = c->o.radius > 0 ? 2 * c->o.radius + 1 : c->p.nd;
    auto launch = [&](auto kernel) -> dmmv_status {
        DMMV_HIP_CHECK(hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)BP_LDS_LIMIT));
        hipLaunchKernelGGL(kernel, dim3((unsigned)R), dim3(BP_BLOCK), lds, c->stream, m, n, c->p.nd, R,
                           (const T*)c->p.A_dense, c->p.lda, (const T*)c->Xt, (const T*)c->D_dev,
                           (const T*)c->scale_dev, (T*)c->r, c->kidx, (InstState<T>*)c->state, c->o.radius,
                           c->o.var_mask, steps, iters, trace, (T*)trace_t);
        DMMV_LAUNCH_CHECK();
        return DMMV_OK;
    };
    if (c->o.radius > 0) {
        if (span <= 4) return launch(k_descent_batched_pruned<T, 4, true>);
        return launch(k_descent_batched_pruned<T, 16, true>);
    }
    if (span <= 4) return launch(k_descent_batched_pruned<T, 4, false>);
    return launch(k_descent_batched_pruned<T, 16, false>);
}

}  // namespace

bool batched_pruned_applicable(const Ctx* c) {
    if (c->kind != KIND_BATCHED || !c->o.prune || c->o.keep_going || c->cmp_on) return false;
    const int64_t m = c->p.m, n = c->p.n;
    if (n <= 0 || c->p.R > INT32_MAX) return false;
    if (m > (int64_t)BP_BLOCK * BP_MAX_RPT) return false;
    const size_t lds = (size_t)(m + n) * c->esz + (size_t)n * 4;
    return lds <= BP_LDS_LIMIT;
}

dmmv_status batched_descent_pruned(Ctx* c, int32_t steps, int32_t iters, dmmv_move* trace, void* trace_t) {
    if (!batched_pruned_applicable(c)) return fail(DMMV_ERR_STATE, "pruned batched descent: not applicable to this handle");
    if (steps <= 0) return DMMV_OK;
    return c->p.dtype == DMMV_F64 ? descent_t<double>(c, steps, iters, trace, trace_t)
                                  : descent_t<float>(c, steps, iters, trace, trace_t);
}

}  // namespace dmmv
