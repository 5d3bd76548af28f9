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
//   3. takes candidates in ascending order of (lb, c), c = j nd + k - each wavefront among the
//      variables it screened, one per round - scores each one over all m rows (the same fma on
//      the same operands as the full evaluation, so the same bits), and stops when no wavefront's
//      next candidate has (lb, c) below the best (score, c) found: every candidate not scored
//      then has score >= lb >= that best score, and loses the tie on c;
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
constexpr int BP_UNROLL = 8;                     // independent global loads a thread issues before it uses them

template <class T>
struct BpShared {
    T top_r[BP_S];
    int32_t top_row[BP_S];
    T round_s[2][BP_WAVES];                      // score and candidate each wavefront scored in a round
    int64_t round_c[2][BP_WAVES];                //   (-1: it had none left that could win)
};

// does (s, c) beat the best (bs, bc)?  bc < 0: nothing found yet, only scores below bs = t count
template <class T>
__device__ __forceinline__ bool bp_better(T s, int64_t c, T bs, int64_t bc) {
    return c >= 0 && (s < bs || (s == bs && bc >= 0 && c < bc));
}

// KT: candidate values scored together per variable (register tile).  RAD: the neighbourhood is
// a radius around the current level (candidate levels differ from lane to lane); without it the
// levels are the same for every variable and their values of D are read once per tile.
// KI: type of a level index in LDS (8 bits when nd <= 256).
template <class T, int KT, bool RAD, class KI>
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
    KI* sh_k = reinterpret_cast<KI*>(sh_jmin + n);          // current level of every variable
    KI* sh_jarg = sh_k + n;                                // per variable: level of its next candidate

    const int64_t q = blockIdx.x;
    InstState<T> z = st[q];
    if (z.done || steps <= 0) return;                      // the same for the whole workgroup
    const int tid = threadIdx.x, lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    // the instance's column of r and of x: strided reads, eight in flight per thread
    for (int64_t i0 = tid; i0 < m; i0 += BP_BLOCK * BP_UNROLL) {
        T a[BP_UNROLL];
#pragma unroll
        for (int u = 0; u < BP_UNROLL; ++u) {
            const int64_t i = i0 + BP_BLOCK * u;
            a[u] = r[(i < m ? i : m - 1) * R + q];
        }
#pragma unroll
        for (int u = 0; u < BP_UNROLL; ++u) {
            const int64_t i = i0 + BP_BLOCK * u;
            if (i < m) sh_r[i] = a[u];
        }
    }
    for (int64_t j0 = tid; j0 < n; j0 += BP_BLOCK * BP_UNROLL) {
        int32_t a[BP_UNROLL];
#pragma unroll
        for (int u = 0; u < BP_UNROLL; ++u) {
            const int64_t j = j0 + BP_BLOCK * u;
            a[u] = kidx[(j < n ? j : n - 1) * R + q];
        }
#pragma unroll
        for (int u = 0; u < BP_UNROLL; ++u) {
            const int64_t j = j0 + BP_BLOCK * u;
            if (j < n) sh_k[j] = (KI)a[u];
        }
    }
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
            sh_jarg[j] = (KI)jk;
        }
        __syncthreads();

        // ---- 3. candidates in ascending (lb, c) until none can beat the best score ---------
        // Every wavefront walks the candidates of ITS variables (those its threads screened) in
        // ascending (lb, c) and scores one per round, as long as that candidate can still beat the
        // best (score, c) the workgroup knew when the round began; the rounds end when no
        // wavefront had such a candidate.  Then every candidate not scored has
        // (lb, c) >= (best score, its c), hence score >= lb >= best score, and loses the tie on c.
        T best_s = z.t;                                    // only scores below t count
        int64_t best_c = -1;
        for (int parity = 0;; parity ^= 1) {
            T s = Limits<T>::inf();
            int64_t c = -1;
            for (int64_t j = tid; j < n; j += BP_BLOCK) {
                const T v = sh_jmin[j];
                if (v < s) { s = v; c = j * (int64_t)nd + sh_jarg[j]; }   // j ascends: ties keep the lowest c
            }
            wave_argmin(s, c);
            const bool live = bp_better(s, c, best_s, best_c);   // the same for the whole wavefront
            T sfull = (T)0;
            if (live) {
                const int64_t j = c / nd;
                const int32_t k = (int32_t)(c % nd);
                const int32_t kc = sh_k[j];
                const T dcur = D[kc];
                const T delta = step_of(D[k], dcur, sc);
                // its score over all rows
                const T* __restrict__ col = X + ldx * j;
                // (eight loads in flight; a row past the end repeats row m - 1, which changes no maximum)
                T acc = (T)0;
                for (int64_t i0 = lane; i0 < m; i0 += 64 * BP_UNROLL) {
                    T a[BP_UNROLL];
#pragma unroll
                    for (int u = 0; u < BP_UNROLL; ++u) {
                        const int64_t i = i0 + 64 * u;
                        a[u] = col[i < m ? i : m - 1];
                    }
#pragma unroll
                    for (int u = 0; u < BP_UNROLL; ++u) {
                        const int64_t i = i0 + 64 * u;
                        acc = dmmv_max(acc, dmmv_abs(dmmv_fma(delta, a[u], sh_r[i < m ? i : m - 1])));
                    }
                }
                // this variable's next candidate: the smallest (lb, k) after (s, k); lanes take the levels
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
                    const bool after = ok && (lb > s || (lb == s && kk > k));
                    if (after && lb < bl) { bl = lb; bk = kk; }       // kk ascends per lane: ties keep the lowest
                }
                wave_argmin(bl, bk);
                if (lane == 0) {
                    sh_jmin[j] = bk >= 0 ? bl : Limits<T>::inf();
                    sh_jarg[j] = (KI)(bk >= 0 ? bk : 0);
                }
                sfull = wave_max(acc);
            }
            if (lane == 0) { F.round_s[parity][w] = sfull; F.round_c[parity][w] = live ? c : (int64_t)-1; }
            __syncthreads();
            bool any = false;
#pragma unroll
            for (int u = 0; u < BP_WAVES; ++u) {
                const T us = F.round_s[parity][u];
                const int64_t uc = F.round_c[parity][u];
                any = any || uc >= 0;
                if (bp_better(us, uc, best_s, best_c)) { best_s = us; best_c = uc; }
            }
            if (!any) break;                               // the same for the whole workgroup
            // the other pair of slots is written next: a wavefront gets there only after every
            // wavefront has passed this round's barrier, i.e. has read the slots of the round before
        }

        // ---- 4. decide and apply ---------------------------------------------------------
        z.best_s = best_s;
        if (best_c < 0) { z.done = 1; break; }
        {
            const int64_t j = best_c / nd;
            const int32_t k = (int32_t)(best_c % nd);
            const T delta = step_of(D[k], D[sh_k[j]], sc);
            const T* __restrict__ col = X + ldx * j;
            for (int64_t i0 = tid; i0 < m; i0 += BP_BLOCK * BP_UNROLL) {
                T a[BP_UNROLL];
#pragma unroll
                for (int u = 0; u < BP_UNROLL; ++u) {
                    const int64_t i = i0 + BP_BLOCK * u;
                    a[u] = col[i < m ? i : m - 1];
                }
#pragma unroll
                for (int u = 0; u < BP_UNROLL; ++u) {
                    const int64_t i = i0 + BP_BLOCK * u;
                    if (i < m) sh_r[i] = dmmv_fma(delta, a[u], sh_r[i]);
                }
            }
            __syncthreads();                               // everyone has read sh_k[j]
            if (tid == 0) {
                sh_k[j] = (KI)k;
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

static size_t bp_lds_bytes(int64_t m, int64_t n, int32_t nd, size_t esz) {
    return (size_t)(m + n) * esz + (size_t)n * 2 * (nd <= 256 ? 1 : 2);
}

template <class T>
dmmv_status descent_t(Ctx* c, int32_t steps, int32_t iters, dmmv_move* trace, void* trace_t) {
    const int64_t m = c->p.m, n = c->p.n, R = c->p.R;
    const size_t lds = bp_lds_bytes(m, n, c->p.nd, sizeof(T));
    const int32_t span = c->o.radius > 0 ? 2 * c->o.radius + 1 : c->p.nd;
    auto launch = [&](auto kernel) -> dmmv_status {
        DMMV_TRY(ensure_dynamic_lds(reinterpret_cast<const void*>(kernel), (int)BP_LDS_LIMIT));
        hipLaunchKernelGGL(kernel, dim3((unsigned)R), dim3(BP_BLOCK), lds, c->stream, m, n, c->p.nd, R,
                           (const T*)c->p.A_dense, c->p.lda, (const T*)c->Xt, (const T*)c->D_dev,
                           (const T*)c->scale_dev, (T*)c->r, c->kidx, (InstState<T>*)c->state, c->o.radius,
                           c->o.var_mask, steps, iters, trace, (T*)trace_t);
        DMMV_LAUNCH_CHECK();
        return DMMV_OK;
    };
    if (c->p.nd > 256) {
        if (c->o.radius > 0) return launch(k_descent_batched_pruned<T, 16, true, uint16_t>);
        return launch(k_descent_batched_pruned<T, 16, false, uint16_t>);
    }
    // the register tile that wastes least: 4 (a radius of 1, 2-bit codes), 8 (3-bit codes), 16
    if (c->o.radius > 0) {
        if (span <= 4) return launch(k_descent_batched_pruned<T, 4, true, uint8_t>);
        if (span <= 8) return launch(k_descent_batched_pruned<T, 8, true, uint8_t>);
        return launch(k_descent_batched_pruned<T, 16, true, uint8_t>);
    }
    if (span <= 4) return launch(k_descent_batched_pruned<T, 4, false, uint8_t>);
    if (span <= 8) return launch(k_descent_batched_pruned<T, 8, false, uint8_t>);
    return launch(k_descent_batched_pruned<T, 16, false, uint8_t>);
}

}  // namespace

bool batched_pruned_applicable(const Ctx* c) {
    // a batch, or a dense single instance (a batch of one: r [m][1], x [n][1], scale 1, with the
    // row-major copy of A that dmmv_create makes for options.prune)
    // - only a small one: one workgroup scores it, so a table of more than 2^24 pairs, or more than
    // 64 levels per variable (a thread walks the levels of its variable), is left to the chip-wide
    // full evaluation
    const bool small_dense = c->kind == KIND_DENSE && c->Xt != nullptr && c->p.nd <= 64 &&
                             c->p.m * c->p.n * (int64_t)c->p.nd <= ((int64_t)1 << 24);
    const bool kind_ok = c->kind == KIND_BATCHED || small_dense;
    if (!kind_ok || !c->o.prune || c->o.keep_going || c->cmp_on) return false;
    if (c->o.l2_rule == 1 || c->o.l2_rule == 2) return false;      // a bound on the score alone does not order (score, l2 change)
    const int64_t m = c->p.m, n = c->p.n;
    if (n <= 0 || c->p.R > INT32_MAX) return false;
    if (m > (int64_t)BP_BLOCK * BP_MAX_RPT) return false;
    return bp_lds_bytes(m, n, c->p.nd, c->esz) <= BP_LDS_LIMIT;
}

dmmv_status batched_descent_pruned(Ctx* c, int32_t steps, int32_t iters, dmmv_move* trace, void* trace_t) {
    if (!batched_pruned_applicable(c)) return fail(DMMV_ERR_STATE, "pruned batched descent: not applicable to this handle");
    if (steps <= 0) return DMMV_OK;
    return c->p.dtype == DMMV_F64 ? descent_t<double>(c, steps, iters, trace, trace_t)
                                  : descent_t<float>(c, steps, iters, trace, trace_t);
}

}  // namespace dmmv
