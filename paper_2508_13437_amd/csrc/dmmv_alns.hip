// ALNS outer loop of AMVM (Algorithm 1 of the paper) around the single-move descent:
// destroy (random / worst-remove, Appendix B.1-B.2), repair (random / greedy, B.1, B.3),
// local search, acceptance, adaptive operator weights (Appendix F.2).
//
// Everything is decided on the device; the host only enqueues a fixed sequence of kernels
// per outer iteration.  Whatever a floating-point value decides is decided on integers or by
// a fixed sequence of IEEE operations, so that an independent implementation can follow the
// run move by move:
//   - random numbers are a counter-based chain of SplitMix64 steps addressed by
//     (seed, instance, outer iteration, stream, counter);
//   - the impact score of the worst-remove operator is accumulated in fixed point
//     (a sum of integers does not depend on the order of its terms) and becomes an integer
//     sampling weight; exp is a fixed Horner polynomial after a fixed range reduction;
//   - variables are drawn against integer prefix sums, a repeated draw is skipped.
// This file holds what is independent of the matrix storage plus the dense kernels.
#include "dmmv_alns_common.h"

namespace dmmv {

// ----------------------------------------------------------------------------------------
// loop control.  R instances (R = 1 unless batched): instance q owns S[q], st[q], the slices
// q*n.. of weight / prefix / first, q*count.. of picked; x and r are instance-contiguous
// (kidx[j*R + q], r[i*R + q]) as everywhere in the batched path.
// ----------------------------------------------------------------------------------------
// Squared l2 norm of the residual of every instance, in double precision and in a fixed order:
// rows in blocks of 256, inside a block acc = fma(r_i, r_i, acc) by ascending row, then the
// block sums by ascending block.  Batch: one lane per instance walks all rows (coalesced over
// the instances).
template <class T>
__global__ void k_alns_sumsq_batched(int64_t m, int64_t R, const T* __restrict__ r, double* __restrict__ q2) {
    const int64_t q = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
    if (q >= R) return;
    double total = 0.0;
    for (int64_t i0 = 0; i0 < m; i0 += 256) {
        double acc = 0.0;
        const int64_t i1 = i0 + 256 < m ? i0 + 256 : m;
        for (int64_t i = i0; i < i1; ++i) {
            const double v = (double)r[i * R + q];
            acc = __builtin_fma(v, v, acc);
        }
        total += acc;
    }
    q2[q] = total;
}

// Single instance: one thread per block of 256 rows, then one thread adds the block sums.
template <class T>
__global__ __launch_bounds__(1024) void k_alns_sumsq_single(int64_t m, const T* __restrict__ r,
                                                            double* __restrict__ blocks, double* __restrict__ q2) {
    const int64_t nblk = (m + 255) / 256;
    for (int64_t bk = threadIdx.x; bk < nblk; bk += blockDim.x) {
        double acc = 0.0;
        const int64_t i0 = bk * 256, i1 = i0 + 256 < m ? i0 + 256 : m;
        for (int64_t i = i0; i < i1; ++i) {
            const double v = (double)r[i];
            acc = __builtin_fma(v, v, acc);
        }
        blocks[bk] = acc;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        double total = 0.0;
        for (int64_t bk = 0; bk < nblk; ++bk) total += blocks[bk];
        q2[0] = total;
    }
}

template <class T>
__global__ void k_alns_init(AlnsState* S, const InstState<T>* st, int64_t R, const double* q2) {
    const int64_t q = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
    if (q >= R) return;
    S[q].q2_cur = q2 ? q2[q] : 0.0;
    for (int u = 0; u < 4; ++u) S[q].w[u] = 1.0;
    S[q].t_cur = (double)st[q].t;
    S[q].t_best = (double)st[q].t;
    S[q].it = 0; S[q].d_op = 0; S[q].r_op = 0; S[q].accepted = 0; S[q].new_best = 0;
}

// operators of this outer iteration by roulette wheel
__global__ void k_alns_begin(AlnsState* S, int64_t R, uint64_t seed, int32_t it) {
    const int64_t q = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
    if (q >= R) return;
    const double ud = alns_unit(alns_rnd(seed, (uint64_t)q, (uint64_t)it, 0, 0));
    const double ur = alns_unit(alns_rnd(seed, (uint64_t)q, (uint64_t)it, 0, 1));
    S[q].it = it;
    S[q].d_op = (ud * (S[q].w[0] + S[q].w[1]) < S[q].w[0]) ? 0 : 1;
    S[q].r_op = (ur * (S[q].w[2] + S[q].w[3]) < S[q].w[2]) ? 0 : 1;
}

// Inclusive prefix sums of the weights (one workgroup per instance); only for worst-remove.
// The weights are integers, so the sums are the same in any order: a thread sums SC_E
// consecutive weights in registers, the wavefronts scan the threads' totals, and the total of a
// tile of 1024 * SC_E weights is carried into the next.
constexpr int SC_E = 8;
__global__ __launch_bounds__(1024) void k_alns_scan(int64_t n, const uint64_t* __restrict__ weight_all,
                                                    uint64_t* __restrict__ prefix_all, const AlnsState* S) {
    __shared__ uint64_t sh_w[16];
    const int64_t q = blockIdx.x;
    if (S[q].d_op != 1) return;
    const uint64_t* __restrict__ weight = weight_all + q * n;
    uint64_t* __restrict__ prefix = prefix_all + q * n;
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    uint64_t carry = 0;                                     // the same in every thread
    for (int64_t base = 0; base < n; base += 1024 * SC_E) {
        const int64_t j0 = base + (int64_t)threadIdx.x * SC_E;
        uint64_t v[SC_E];
#pragma unroll
        for (int u = 0; u < SC_E; ++u) v[u] = weight[j0 + u < n ? j0 + u : n - 1];   // clamped: the loads go out together
#pragma unroll
        for (int u = 0; u < SC_E; ++u) v[u] = j0 + u < n ? v[u] : 0;
#pragma unroll
        for (int u = 1; u < SC_E; ++u) v[u] += v[u - 1];
        const uint64_t tot = v[SC_E - 1];
        uint64_t inc = tot;                                 // inclusive over the wavefront's threads
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const uint64_t t = (uint64_t)__shfl_up((long long)inc, off, 64);
            if (lane >= off) inc += t;
        }
        if (lane == 63) sh_w[w] = inc;
        __syncthreads();
        uint64_t before = 0, all = 0;
#pragma unroll
        for (int k = 0; k < 16; ++k) {
            const uint64_t x = sh_w[k];
            if (k < w) before += x;
            all += x;
        }
        const uint64_t ex = carry + before + (inc - tot);   // everything ahead of this thread
#pragma unroll
        for (int u = 0; u < SC_E; ++u)
            if (j0 + u < n) prefix[j0 + u] = v[u] + ex;
        carry += all;
        __syncthreads();                                    // sh_w is written again
    }
}

// Draw `count` distinct variables (one workgroup per instance).  Draw c takes rnd(.., 1, c) mod
// total and the first variable whose prefix sum exceeds it (all weights 1 for the random
// operator); a variable drawn before is skipped.  blockDim.x draws are made at a time: a draw is
// the first of its variable exactly if it holds the largest stamp (iteration, -c) that
// variable has seen.
__global__ __launch_bounds__(1024) void k_alns_sample(int64_t n, int32_t count,
                                                      const uint64_t* __restrict__ prefix_all,
                                                      unsigned long long* first_all,
                                                      int32_t* __restrict__ picked_all, const AlnsState* S,
                                                      uint64_t seed) {
    __shared__ int32_t sh_cnt[16];
    __shared__ int32_t sh_have;
    const int64_t q = blockIdx.x;
    const uint64_t* __restrict__ prefix = prefix_all + q * n;
    unsigned long long* first = first_all + q * n;
    int32_t* __restrict__ picked = picked_all + q * (int64_t)count;
    const int32_t it = S[q].it;
    const bool weighted = S[q].d_op == 1;
    const uint64_t total = weighted ? prefix[n - 1] : (uint64_t)n;
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6, nw = blockDim.x >> 6;
    if (threadIdx.x == 0) sh_have = 0;
    __syncthreads();
    for (uint64_t base = 0;; base += blockDim.x) {
        const int32_t have = sh_have;
        if (have >= count) break;
        const uint64_t c = base + threadIdx.x;
        const uint64_t v = alns_rnd(seed, (uint64_t)q, (uint64_t)it, 1, c) % total;
        int64_t j;
        if (weighted) {
            int64_t lo = 0, hi = n - 1;
            while (lo < hi) {
                const int64_t mid = (lo + hi) / 2;
                if (prefix[mid] > v) hi = mid; else lo = mid + 1;
            }
            j = lo;
        } else {
            j = (int64_t)v;
        }
        const unsigned long long stamp = ((unsigned long long)(it + 1) << 32) | (0xFFFFFFFFull - (c & 0xFFFFFFFFull));
        atomicMax(&first[j], stamp);
        __syncthreads();
        const bool is_first = __hip_atomic_load(&first[j], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == stamp;
        const unsigned long long bal = __ballot(is_first);
        if (lane == 0) sh_cnt[w] = __popcll(bal);
        __syncthreads();
        int32_t before = 0, all = 0;
        for (int u = 0; u < nw; ++u) { if (u < w) before += sh_cnt[u]; all += sh_cnt[u]; }
        const int32_t pos = have + before + __popcll(bal & ((1ull << lane) - 1ull));
        if (is_first && pos < count) picked[pos] = (int32_t)j;
        __syncthreads();
        if (threadIdx.x == 0) sh_have = have + all;
        __syncthreads();
    }
}

// acceptance, best solution, weights, trace (one thread per instance)
template <class T>
__global__ void k_alns_end(AlnsState* S, InstState<T>* st, int64_t R, int32_t iters, double lambda,
                           double sigma1, double sigma2, double sigma3, const double* q2, int32_t* trace,
                           T* trace_t) {
    const int64_t q = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
    if (q >= R) return;
    const double t = (double)st[q].t;
    const int32_t it = S[q].it;
    // q2 != NULL: the l2 norm of the residual must not increase either
    const int accepted = t <= S[q].t_cur && (!q2 || q2[q] <= S[q].q2_cur);
    int new_best = 0;
    if (accepted) {
        if (q2) S[q].q2_cur = q2[q];
        double psi = sigma3;
        if (t < S[q].t_cur) psi = sigma2;
        if (t < S[q].t_best) { psi = sigma1; S[q].t_best = t; new_best = 1; }
        S[q].t_cur = t;
        const double keep = 1.0 - lambda;
        S[q].w[S[q].d_op] = keep * S[q].w[S[q].d_op] + lambda * psi;
        S[q].w[2 + S[q].r_op] = keep * S[q].w[2 + S[q].r_op] + lambda * psi;
    }
    S[q].accepted = accepted;
    S[q].new_best = new_best;
    const int64_t slot = q * (int64_t)iters + it;
    if (trace) {
        trace[slot * 4 + 0] = S[q].d_op; trace[slot * 4 + 1] = S[q].r_op;
        trace[slot * 4 + 2] = st[q].moves; trace[slot * 4 + 3] = accepted;
    }
    if (trace_t) { trace_t[slot * 2 + 0] = st[q].t; trace_t[slot * 2 + 1] = (T)S[q].t_best; }
    if (!accepted) st[q].t = (T)S[q].t_cur;          // the copy kernel restores x and r
}

// accepted: current <- working (and best <- working for a new best); rejected: working <- current
template <class T>
__global__ void k_alns_copy(int64_t m, int64_t n, int64_t R, const AlnsState* S, int32_t* kidx,
                            int32_t* kidx_cur, int32_t* kidx_best, T* r, T* r_cur) {
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    const int64_t t0 = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
    for (int64_t e = t0; e < n * R; e += stride) {
        const AlnsState& s = S[e % R];
        if (s.accepted) {
            const int32_t k = kidx[e];
            kidx_cur[e] = k;
            if (s.new_best) kidx_best[e] = k;
        } else {
            kidx[e] = kidx_cur[e];
        }
    }
    for (int64_t e = t0; e < m * R; e += stride) {
        if (S[e % R].accepted) r_cur[e] = r[e]; else r[e] = r_cur[e];
    }
}

template <class T>
__global__ void k_alns_snapshot(int64_t m, int64_t n, int64_t R, const int32_t* kidx, int32_t* kidx_cur,
                                int32_t* kidx_best, const T* r, T* r_cur, unsigned long long* first) {
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    const int64_t t0 = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
    for (int64_t e = t0; e < n * R; e += stride) { kidx_cur[e] = kidx[e]; kidx_best[e] = kidx[e]; first[e] = 0; }
    for (int64_t e = t0; e < m * R; e += stride) r_cur[e] = r[e];
}

template <class T>
__global__ void k_alns_export(const AlnsState* S, int64_t R, T* t_best_out) {
    const int64_t q = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
    if (q < R && t_best_out) t_best_out[q] = (T)S[q].t_best;
}

// ----------------------------------------------------------------------------------------
// dense matrix: impact weights and repair
// ----------------------------------------------------------------------------------------
// single instance: one workgroup per variable, the rows spread over its threads
template <class T>
__global__ __launch_bounds__(256) void k_alns_impact_dense(int64_t m, int64_t n, const T* __restrict__ A,
                                                           int64_t lda, const T* __restrict__ r,
                                                           const InstState<T>* st, double alpha,
                                                           uint64_t* __restrict__ weight, const AlnsState* S) {
    __shared__ uint64_t sh[4];
    if (S->d_op != 1) return;
    const int64_t j = blockIdx.x;
    const double t = (double)st[0].t;
    const double scale = alns_impact_scale(t);
    uint64_t sum = 0;
    if (scale != 0.0) {
        const T* __restrict__ col = A + lda * j;
        for (int64_t i = threadIdx.x; i < m; i += blockDim.x)
            sum += alns_impact_term(__builtin_fabs((double)col[i]), __builtin_fabs((double)r[i]), t, alpha, scale);
    }
    sum = block_sum_u64(sum, sh);
    if (threadIdx.x == 0) {
        int shift = alns_bits(m) + 24 + alns_bits(n) - 62;
        if (shift < 0) shift = 0;
        weight[j] = 1 + (sum >> shift);
    }
}

// batched: the instances whose destroy operator of this iteration is worst-remove, in ascending
// order (single workgroup); their number goes to flags[FLAG_WORST].  The impact kernel works on
// this list, so that its wavefronts are full of instances that need weights.
__global__ __launch_bounds__(1024) void k_alns_worst_list(int64_t R, const AlnsState* __restrict__ S,
                                                          int32_t* __restrict__ list, int32_t* flags) {
    __shared__ int32_t sh_cnt[16];
    __shared__ int32_t sh_base;
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    if (threadIdx.x == 0) sh_base = 0;
    __syncthreads();
    for (int64_t b0 = 0; b0 < R; b0 += 1024) {
        const int64_t q = b0 + threadIdx.x;
        const bool on = q < R && S[q].d_op == 1;
        const unsigned long long bal = __ballot(on);
        if (lane == 0) sh_cnt[w] = __popcll(bal);
        __syncthreads();
        int32_t before = 0, all = 0;
        for (int u = 0; u < 16; ++u) { if (u < w) before += sh_cnt[u]; all += sh_cnt[u]; }
        const int32_t base = sh_base;
        if (on) list[base + before + __popcll(bal & ((1ull << lane) - 1ull))] = (int32_t)q;
        __syncthreads();
        if (threadIdx.x == 0) sh_base = base + all;
        __syncthreads();
    }
    if (threadIdx.x == 0) flags[FLAG_WORST] = sh_base;
}

// batched: lane = listed instance (X through the scalar unit); grid.x = group of 64 of them
// instances, each of the 4 wavefronts takes the variables blockIdx.y*4 + w, +4*gridDim.y, ...
//
// Only a few per cent of the terms are not cut off by the shortcut of alns_impact_term (slack >
// a * 18 / alpha: the term truncates to 0), but they are scattered: almost every group of 64
// lanes holds one, so testing inside the loop would send every wavefront through the
// double-precision division and exponential for the sake of a lane or two.  The loop therefore
// only TESTS (one comparison in the working precision, with a margin of 1 %) and appends the
// terms that may count to a queue of
// the wavefront in LDS; whenever 64 are waiting, every lane computes one of them, for whichever
// instance it belongs to, and adds the integer to that instance's sum with an LDS atomic.  The
// sum is one of integers, so the order does not matter and the weights are the same bit for bit.
// A wavefront goes over the rows once for eight consecutive variables, so that an instance's
// residual (the only per-lane operand) is read once for all eight.
constexpr int IMQ_CAP = 128;                   // ring of waiting terms per wavefront (drained at 64)
constexpr int IMQ_ROWS = 1;                    // rows whose operands are fetched before they are tested (more rows in
                                               //   flight only make the unrolled loop longer: 14.9 ms with 4, 13.1 with 1)
constexpr int IMQ_VARS = 8;                    // consecutive variables a wavefront works on per pass over the rows
                                               //   (r is read once for all of them)

template <class T>
struct ImpactShared {
    T qx[4][IMQ_CAP], qr[4][IMQ_CAP];          // waiting terms: matrix entry, residual of the row,
    uint16_t qmeta[4][IMQ_CAP];                //   the lane (instance) they belong to, and in the
                                               //   high byte which of the pass's variables
    unsigned long long sum[4][IMQ_VARS][64];
    double sc[4][64], t[4][64], scale[4][64];  // per instance: scale factor, error, fixed-point scale
};

template <class T>
__global__ __launch_bounds__(256) void k_alns_impact_batched(int64_t m, int64_t n, int64_t R,
                                                             const T* __restrict__ Xt,
                                                             const T* __restrict__ scale_q,
                                                             const T* __restrict__ r,
                                                             const InstState<T>* st, double alpha,
                                                             uint64_t* __restrict__ weight,
                                                             const int32_t* __restrict__ list,
                                                             const int32_t* __restrict__ flags) {
    __shared__ ImpactShared<T> L;
    const int lane = threadIdx.x & 63;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t count = flags[FLAG_WORST];                // instances on the list (k_alns_worst_list)
    const int64_t slot = blockIdx.x * 64ll + lane;
    if (blockIdx.x * 64ll >= count) return;                 // the same for the whole workgroup
    const bool live = slot < count;
    const int64_t q = list[live ? slot : count - 1];
    const int64_t qc = q;
    const double t = (double)st[qc].t;
    const double scale = alns_impact_scale(t);
    const double sc = (double)scale_q[qc];
    int shift = alns_bits(m) + 24 + alns_bits(n) - 62;
    if (shift < 0) shift = 0;
    const bool counts = live && scale != 0.0;               // otherwise every weight of the instance is 1
    L.sc[w][lane] = sc;
    L.t[w][lane] = t;
    L.scale[w][lane] = scale;
    __builtin_amdgcn_wave_barrier();
    // May the term of matrix entry x and a row of slack t - |r_i| count?  The shortcut cuts it off
    // when slack > |sc x| * 18 / alpha, i.e. when |x| < slack * alpha / (18 sc).  The loop tests
    // |x| >= lim_i with lim_i = slack_i * cinv, cinv = alpha / (18 * 1.01 * sc), in the working
    // precision: the 1 % covers the roundings of cinv and of the product, so a term the test
    // leaves out is one the shortcut cuts off (the reverse need not hold: alns_impact_term
    // applies the exact shortcut again).  One comparison per term; lim_i is per row.
    const T tw = (T)t;                                      // exact: t is a value of type T
    T cinv = (T)(alpha / (18.0 * 1.01)) / (T)sc;
    if (!(cinv < Limits<T>::inf())) cinv = (T)0;            // a scale so small that this overflows: test nothing
    for (int64_t j0 = (blockIdx.y * 4ll + w) * IMQ_VARS; j0 < n; j0 += 4ll * IMQ_VARS * gridDim.y) {
#pragma unroll
        for (int v = 0; v < IMQ_VARS; ++v) L.sum[w][v][lane] = 0;
        int head = 0, waiting = 0;                          // the same in every lane
        // every lane computes one of the first `count` waiting terms, for the instance it belongs to
        auto drain = [&](int count) {
            __builtin_amdgcn_wave_barrier();
            if (lane < count) {
                const int e = (head + lane) & (IMQ_CAP - 1);
                const int meta = L.qmeta[w][e];
                const int owner = meta & 0xFF;
                const double a = __builtin_fabs(L.sc[w][owner] * (double)L.qx[w][e]);
                const uint64_t term = alns_impact_term(a, __builtin_fabs((double)L.qr[w][e]), L.t[w][owner], alpha,
                                                       L.scale[w][owner]);
                if (term) atomicAdd(&L.sum[w][meta >> 8][owner], (unsigned long long)term);
            }
            __builtin_amdgcn_wave_barrier();
            head = (head + count) & (IMQ_CAP - 1);
            waiting -= count;
        };
        for (int64_t i0 = 0; i0 < m; i0 += IMQ_ROWS) {
            T xs[IMQ_ROWS][IMQ_VARS], rs[IMQ_ROWS], lim[IMQ_ROWS];
#pragma unroll
            for (int u = 0; u < IMQ_ROWS; ++u) {
                const int64_t i = i0 + u < m ? i0 + u : m - 1;
                rs[u] = r[i * R + qc];
#pragma unroll
                for (int v = 0; v < IMQ_VARS; ++v) xs[u][v] = Xt[i * n + (j0 + v < n ? j0 + v : n - 1)];
            }
#pragma unroll
            for (int u = 0; u < IMQ_ROWS; ++u)              // a lane or a row that does not count takes nothing
                lim[u] = counts && i0 + u < m ? (tw - dmmv_abs(rs[u])) * cinv : Limits<T>::inf();
#pragma unroll
            for (int u = 0; u < IMQ_ROWS; ++u) {
#pragma unroll
                for (int v = 0; v < IMQ_VARS; ++v) {
                    if (j0 + v >= n) continue;               // the same for the whole wavefront
                    const bool take = dmmv_abs(xs[u][v]) >= lim[u];
                    const unsigned long long mask = __ballot(take);
                    if (mask) {                              // the same for the whole wavefront
                        if (take) {
                            const int before = __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32),
                                                                         __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0));
                            const int e = (head + waiting + before) & (IMQ_CAP - 1);
                            L.qx[w][e] = xs[u][v];
                            L.qr[w][e] = rs[u];
                            L.qmeta[w][e] = (uint16_t)(lane | (v << 8));
                        }
                        waiting += __builtin_popcountll(mask);
                        if (waiting >= 64) drain(64);
                    }
                }
            }
        }
        if (waiting > 0) drain(waiting);
        if (live) {
#pragma unroll
            for (int v = 0; v < IMQ_VARS; ++v)
                if (j0 + v < n) weight[q * n + j0 + v] = 1 + ((uint64_t)L.sum[w][v][lane] >> shift);
        }
        __builtin_amdgcn_wave_barrier();                    // the sums are cleared for the next pass
    }
}

// one workgroup per instance; thread i owns the rows i, i + blockDim.x, ...; the picked
// variables are reassigned one after the other, r follows each reassignment.  STAGE: the
// instance's r is copied to LDS first and written back at the end (in a batch its rows lie R
// elements apart in memory, and every picked variable would walk them again).
constexpr int RD_UNROLL = 8;                   // independent global loads a thread issues before it uses them
constexpr size_t RD_STAGE_BYTES = 48 * 1024;   // largest r that is staged

template <class T, bool STAGE>
__global__ __launch_bounds__(1024) void k_alns_repair_dense(int64_t m, int64_t R, int32_t nd,
                                                            const T* __restrict__ A, int64_t lda,
                                                            const T* __restrict__ D,
                                                            const T* __restrict__ scale_q, T* r,
                                                            int32_t* kidx, int32_t count,
                                                            const int32_t* __restrict__ picked_all,
                                                            InstState<T>* st, const AlnsState* S,
                                                            uint64_t seed) {
    extern __shared__ __align__(16) unsigned char repair_smem[];
    T* lr = reinterpret_cast<T*>(repair_smem);
    __shared__ T sh[16];
    const int64_t q = blockIdx.x;
    const int64_t nt = blockDim.x;
    const int32_t* __restrict__ picked = picked_all + q * (int64_t)count;
    const int32_t it = S[q].it;
    const bool greedy = S[q].r_op == 1;
    const T sc = scale_q[q];
    if (STAGE) {
        for (int64_t i0 = threadIdx.x; i0 < m; i0 += nt * RD_UNROLL) {
            T v[RD_UNROLL];
#pragma unroll
            for (int u = 0; u < RD_UNROLL; ++u) {
                const int64_t i = i0 + nt * u;
                v[u] = r[(i < m ? i : m - 1) * R + q];
            }
#pragma unroll
            for (int u = 0; u < RD_UNROLL; ++u) {
                const int64_t i = i0 + nt * u;
                if (i < m) lr[i] = v[u];
            }
        }
        __syncthreads();
    }
    // thread i touches only its own rows of r between barriers, staged or not
    auto rd = [&](int64_t i) -> T { return STAGE ? lr[i] : r[i * R + q]; };
    auto wr = [&](int64_t i, T v) { if (STAGE) lr[i] = v; else r[i * R + q] = v; };
    for (int32_t pos = 0; pos < count; ++pos) {
        const int64_t j = picked[pos];
        const int32_t kc = kidx[j * R + q];
        const bool has_lo = kc > 0, has_hi = kc < nd - 1;
        const T* __restrict__ col = A + lda * j;
        int32_t knew;
        if (has_lo && has_hi) {
            if (greedy) {
                const T dlo = step_of(D[kc - 1], D[kc], sc), dhi = step_of(D[kc + 1], D[kc], sc);
                T elo = (T)0, ehi = (T)0;
                for (int64_t i0 = threadIdx.x; i0 < m; i0 += nt * RD_UNROLL) {
                    T a[RD_UNROLL];
#pragma unroll
                    for (int u = 0; u < RD_UNROLL; ++u) {
                        const int64_t i = i0 + nt * u;
                        a[u] = col[i < m ? i : m - 1];
                    }
#pragma unroll
                    for (int u = 0; u < RD_UNROLL; ++u) {
                        const int64_t i = i0 + nt * u;
                        if (i < m) {
                            const T ri = rd(i);
                            elo = dmmv_max(elo, dmmv_abs(dmmv_fma(dlo, a[u], ri)));
                            ehi = dmmv_max(ehi, dmmv_abs(dmmv_fma(dhi, a[u], ri)));
                        }
                    }
                }
                elo = block_max(elo, sh);
                ehi = block_max(ehi, sh);
                knew = ehi < elo ? kc + 1 : kc - 1;
            } else {
                knew = (alns_rnd(seed, (uint64_t)q, (uint64_t)it, 2, (uint64_t)pos) & 1) ? kc + 1 : kc - 1;
            }
        } else {
            knew = has_lo ? kc - 1 : kc + 1;
        }
        const T delta = step_of(D[knew], D[kc], sc);
        for (int64_t i0 = threadIdx.x; i0 < m; i0 += nt * RD_UNROLL) {
            T a[RD_UNROLL];
#pragma unroll
            for (int u = 0; u < RD_UNROLL; ++u) {
                const int64_t i = i0 + nt * u;
                a[u] = col[i < m ? i : m - 1];
            }
#pragma unroll
            for (int u = 0; u < RD_UNROLL; ++u) {
                const int64_t i = i0 + nt * u;
                if (i < m) wr(i, dmmv_fma(delta, a[u], rd(i)));
            }
        }
        __syncthreads();                      // every thread has read kidx of this step
        if (threadIdx.x == 0) kidx[j * R + q] = knew;
    }
    T tmax = (T)0;
    for (int64_t i = threadIdx.x; i < m; i += nt) {
        const T v = rd(i);
        tmax = dmmv_max(tmax, dmmv_abs(v));
        if (STAGE) r[i * R + q] = v;
    }
    tmax = block_max(tmax, sh);
    if (threadIdx.x == 0) { st[q].t = tmax; st[q].done = 0; st[q].moves = 0; }
}

// ----------------------------------------------------------------------------------------
// host side: one outer iteration's kernels around the local search
// ----------------------------------------------------------------------------------------
static unsigned blocks_for(int64_t items, int per_block) {
    int64_t b = (items + per_block - 1) / per_block;
    return (unsigned)(b < 1 ? 1 : b);
}

template <class T>
static dmmv_status sumsq_t(Ctx* c) {
    const int64_t R = c->p.R;
    if (c->kind == KIND_BATCHED)
        hipLaunchKernelGGL(k_alns_sumsq_batched<T>, dim3(blocks_for(R, 64)), dim3(64), 0, c->stream, c->p.m, R,
                           (const T*)c->r, c->alns_q2);
    else
        hipLaunchKernelGGL(k_alns_sumsq_single<T>, dim3(1), dim3(1024), 0, c->stream, c->p.m, (const T*)c->r,
                           c->alns_q2_blocks, c->alns_q2);
    DMMV_LAUNCH_CHECK();
    return DMMV_OK;
}

template <class T>
static dmmv_status start_t(Ctx* c, bool l2_guard) {
    const int64_t R = c->p.R;
    if (l2_guard) DMMV_TRY(sumsq_t<T>(c));
    hipLaunchKernelGGL(k_alns_init<T>, dim3(blocks_for(R, 256)), dim3(256), 0, c->stream,
                       (AlnsState*)c->alns_state, (const InstState<T>*)c->state, R,
                       l2_guard ? (const double*)c->alns_q2 : nullptr);
    hipLaunchKernelGGL(k_alns_snapshot<T>, dim3(1024), dim3(256), 0, c->stream, c->p.m, c->p.n, R,
                       (const int32_t*)c->kidx, c->alns_kidx_cur, c->alns_kidx_best, (const T*)c->r,
                       (T*)c->alns_r_cur, (unsigned long long*)c->alns_first);
    DMMV_LAUNCH_CHECK();
    return DMMV_OK;
}

template <class T>
static dmmv_status destroy_repair_t(Ctx* c, const dmmv_alns_params& prm, int32_t it, int32_t count) {
    AlnsState* S = (AlnsState*)c->alns_state;
    const int64_t R = c->p.R;
    hipLaunchKernelGGL(k_alns_begin, dim3(blocks_for(R, 256)), dim3(256), 0, c->stream, S, R, prm.seed, it);
    if (c->kind == KIND_DENSE) {
        hipLaunchKernelGGL(k_alns_impact_dense<T>, dim3((unsigned)c->p.n), dim3(256), 0, c->stream, c->p.m,
                           c->p.n, (const T*)c->p.A_dense, c->p.lda, (const T*)c->r,
                           (const InstState<T>*)c->state, prm.alpha, c->alns_weight, (const AlnsState*)S);
    } else if (c->kind == KIND_BATCHED) {
        int64_t ny = (c->p.n + 4 * IMQ_VARS - 1) / (4 * IMQ_VARS);     // a wavefront takes IMQ_VARS variables per pass
        if (ny > 2048) ny = 2048;
        // (the list shares the buffer of the descent's list of running instances: never both at once)
        hipLaunchKernelGGL(k_alns_worst_list, dim3(1), dim3(1024), 0, c->stream, R, (const AlnsState*)S,
                           c->cmp_orig, c->flags);
        hipLaunchKernelGGL(k_alns_impact_batched<T>, dim3(blocks_for(R, 64), (unsigned)ny), dim3(256), 0,
                           c->stream, c->p.m, c->p.n, R, (const T*)c->Xt, (const T*)c->scale_dev,
                           (const T*)c->r, (const InstState<T>*)c->state, prm.alpha, c->alns_weight,
                           (const int32_t*)c->cmp_orig, (const int32_t*)c->flags);
    } else {
        DMMV_TRY(csc_alns_impact(c, prm.alpha));
    }
    hipLaunchKernelGGL(k_alns_scan, dim3((unsigned)R), dim3(1024), 0, c->stream, c->p.n,
                       (const uint64_t*)c->alns_weight, c->alns_prefix, (const AlnsState*)S);
    hipLaunchKernelGGL(k_alns_sample, dim3((unsigned)R), dim3(R > 1 ? 256 : 1024), 0, c->stream, c->p.n, count,
                       (const uint64_t*)c->alns_prefix, (unsigned long long*)c->alns_first, c->alns_picked,
                       (const AlnsState*)S, prm.seed);
    if (c->kind == KIND_CSC) {
        DMMV_TRY(csc_alns_repair(c, count, prm.seed));
    } else {
        const size_t rbytes = (size_t)c->p.m * sizeof(T);
        const bool stage = rbytes <= RD_STAGE_BYTES;
        auto repair = stage ? k_alns_repair_dense<T, true> : k_alns_repair_dense<T, false>;
        hipLaunchKernelGGL(repair, dim3((unsigned)R), dim3(R > 1 ? 256 : 1024), stage ? rbytes : 0, c->stream,
                           c->p.m, R, c->p.nd, (const T*)c->p.A_dense, c->p.lda, (const T*)c->D_dev,
                           (const T*)c->scale_dev, (T*)c->r, c->kidx, count, (const int32_t*)c->alns_picked,
                           (InstState<T>*)c->state, (const AlnsState*)S, prm.seed);
    }
    DMMV_LAUNCH_CHECK();
    return DMMV_OK;
}

template <class T>
static dmmv_status finish_iteration_t(Ctx* c, const dmmv_alns_params& prm, int32_t* trace, void* trace_t) {
    AlnsState* S = (AlnsState*)c->alns_state;
    const int64_t R = c->p.R;
    if (prm.l2_guard) DMMV_TRY(sumsq_t<T>(c));
    hipLaunchKernelGGL(k_alns_end<T>, dim3(blocks_for(R, 256)), dim3(256), 0, c->stream, S,
                       (InstState<T>*)c->state, R, prm.iters, prm.lambda, prm.sigma1, prm.sigma2, prm.sigma3,
                       prm.l2_guard ? (const double*)c->alns_q2 : nullptr, trace, (T*)trace_t);
    hipLaunchKernelGGL(k_alns_copy<T>, dim3(1024), dim3(256), 0, c->stream, c->p.m, c->p.n, R,
                       (const AlnsState*)S, c->kidx, c->alns_kidx_cur, c->alns_kidx_best, (T*)c->r,
                       (T*)c->alns_r_cur);
    DMMV_LAUNCH_CHECK();
    if (c->kind == KIND_CSC) DMMV_TRY(csc_alns_after_copy(c));
    return DMMV_OK;
}

template <class T>
static dmmv_status export_t(Ctx* c, void* t_best_out) {
    hipLaunchKernelGGL(k_alns_export<T>, dim3(blocks_for(c->p.R, 256)), dim3(256), 0, c->stream,
                       (const AlnsState*)c->alns_state, c->p.R, (T*)t_best_out);
    DMMV_LAUNCH_CHECK();
    return DMMV_OK;
}

dmmv_status alns_start(Ctx* c, bool l2_guard) {
    return c->p.dtype == DMMV_F64 ? start_t<double>(c, l2_guard) : start_t<float>(c, l2_guard);
}
dmmv_status alns_sumsq(Ctx* c) { return c->p.dtype == DMMV_F64 ? sumsq_t<double>(c) : sumsq_t<float>(c); }
dmmv_status alns_destroy_repair(Ctx* c, const dmmv_alns_params& prm, int32_t it, int32_t count) {
    return c->p.dtype == DMMV_F64 ? destroy_repair_t<double>(c, prm, it, count)
                                  : destroy_repair_t<float>(c, prm, it, count);
}
dmmv_status alns_finish_iteration(Ctx* c, const dmmv_alns_params& prm, int32_t* trace, void* trace_t) {
    return c->p.dtype == DMMV_F64 ? finish_iteration_t<double>(c, prm, trace, trace_t)
                                  : finish_iteration_t<float>(c, prm, trace, trace_t);
}
dmmv_status alns_export(Ctx* c, void* t_best_out) {
    return c->p.dtype == DMMV_F64 ? export_t<double>(c, t_best_out) : export_t<float>(c, t_best_out);
}

}  // namespace dmmv
