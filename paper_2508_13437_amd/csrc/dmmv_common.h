// Shared internals of libdmmv: context layout, error plumbing, wave64 reductions.
// gfx950 (CDNA4) only: 64-wide wavefronts, DPP row operations, LDS.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/dmmv.h"

namespace dmmv {

// ----------------------------------------------------------------------------------------
// error plumbing (host)
// ----------------------------------------------------------------------------------------
dmmv_status fail(dmmv_status st, const char* fmt, ...);

// Raise a kernel's dynamic-LDS limit on the CURRENT device, once per (device, kernel); thread-safe.
dmmv_status ensure_dynamic_lds(const void* kernel, int bytes);

#define DMMV_HIP_CHECK(expr)                                                              \
    do {                                                                                  \
        hipError_t e__ = (expr);                                                          \
        if (e__ != hipSuccess)                                                            \
            return ::dmmv::fail(DMMV_ERR_HIP, "%s failed: %s (%s:%d)", #expr,             \
                                hipGetErrorString(e__), __FILE__, __LINE__);              \
    } while (0)

#define DMMV_LAUNCH_CHECK() DMMV_HIP_CHECK(hipGetLastError())

#define DMMV_TRY(expr)                        \
    do {                                      \
        dmmv_status s__ = (expr);             \
        if (s__ != DMMV_OK) return s__;       \
    } while (0)

// ----------------------------------------------------------------------------------------
// context
// ----------------------------------------------------------------------------------------
enum Kind { KIND_DENSE = 0, KIND_CSC = 1, KIND_BATCHED = 2 };

// sparse path: reservoir of the rows of largest |r|
constexpr int RES_CAP = 128;      // capacity
constexpr int RES_MIN = 16;       // rebuild when fewer entries remain
constexpr int RES_FAST = 8;       // entries checked inline while streaming (one mask bit each)

// swap move: most rows of largest |r| the filter tries first
constexpr int SWAP_KMAX = 128;

// Per-instance loop state kept on the device.
template <class T>
struct alignas(16) InstState {
    T t;             // current max violation
    T best_s;        // score of the best move found by the last selection
    T delta;         // step of the move to apply
    int32_t apply_j; // variable of the move to apply, -1 = nothing to apply
    int32_t apply_k;
    int32_t done;    // 1: stopped (best move was not a strict improvement)
    int32_t moves;   // moves applied so far
};

// State of the ALNS outer loop kept on the device (single instance).
struct alignas(16) AlnsState {
    double w[4];        // operator weights: random destroy, worst-remove, random repair, greedy repair
    double t_cur;       // error of the current (last accepted) solution
    double t_best;      // error of the best solution so far
    double q2_cur;      // squared l2 norm of the residual of the current solution (l2 guard)
    int32_t it;         // outer iteration in progress
    int32_t d_op, r_op; // operators chosen for it
    int32_t accepted;   // verdict of the iteration just finished
    int32_t new_best;
};

// One partial arg-min record: score and flat candidate index (c < 0: empty).
template <class T>
struct alignas(16) Partial {
    T s;
    int64_t c;
};

// device flag slots
enum { FLAG_ERROR = 0, FLAG_ACTIVE = 1, FLAG_PLANES = 2, FLAG_MAXROW = 3, FLAG_MAXCOL = 4, FLAG_WORST = 5, FLAG_COUNT = 8 };
// error bits set by kernels
enum { ERRBIT_X_NOT_IN_D = 1, ERRBIT_CSR_RANGE = 2, ERRBIT_CSR_DUP = 4, ERRBIT_MOVE_RANGE = 8, ERRBIT_WAIT_LIMIT = 16 };

struct Ctx {
    dmmv_problem p;
    dmmv_options o;
    hipStream_t stream;
    Kind kind;
    size_t esz;
    bool x_set, r_valid;

    // ---- carved from the caller's workspace (device) ----
    void* D_dev;          // T[nd]
    void* scale_dev;      // T[R]
    int32_t* kidx;        // dense/sparse: [n]; batched: [n][R] (instances contiguous)
    void* r;              // dense/sparse: T[m]; batched: T[m][R]
    void* state;          // InstState<T>[R]
    void* partials;       // Partial<T>: single [n_partials]; batched [n_partials][R]
    int64_t n_partials;
    int32_t* flags;       // [FLAG_COUNT]
    void* persist_exchange; // dense single instance: arg-min records and arrival words of the one-launch descent
    void* red;            // T[red_elems] partial maxima of the max-|r| reduction
    int64_t red_elems;

    // sparse: rows cut into csc_P partitions of csc_mp rows; segment s = p*n + j
    int32_t csc_P, csc_mp, csc_gb;  // partitions, rows per partition, workgroups per partition
    bool csc_fused;       // the one-kernel evaluation (a workgroup walks every partition) scores the moves
    int64_t csc_nnzp;     // stored entries including segment padding (upper bound)
    int32_t* segptr;      // [P*n + 1] padded start of every segment
    uint16_t* row16;      // [nnzp] row offset inside the partition (pad = csc_mp)
    void* cval;           // T[nnzp]
    int32_t* fillpos;     // [P*n + 1] build scratch: end of the real entries of a segment
    uint16_t* row16_tmp;  // [nnzp] build scratch
    void* cval_tmp;       // T[nnzp] build scratch
    int32_t* blk_lo;      // [P][csc_gb + 1] first column of every evaluation workgroup
    void* part_scores;    // T[P][n*nd] per-partition maxima over the touched rows
    uint32_t* part_mask;  // [P][n] inline-checked reservoir rows met by the column
    void* res_val;        // T[RES_CAP] reservoir: largest |r|, sorted
    int32_t* res_row;     // [RES_CAP]
    int32_t* res_meta;    // [4] count, floor row
    void* res_floor;      // T[1] floor value
    int32_t csc_max_row;  // most stored entries in one row (slots of the pruned evaluation)
    int32_t csc_max_col;  // most entries of one column, the segments' padding included
    void* prune_part;     // Partial<T>[n] records of the pruned evaluation (options.prune)

    // batched
    void* Xt;             // T[m][n] row-major copy of X
    void* Bt;             // T[m][R]
    int32_t chunk_cols;   // columns per chunk of the fused evaluation (n_partials chunks)
    // ALNS outer loop (per instance; batched handles only with options.alns)
    void* alns_state;         // AlnsState[R]
    int32_t* alns_kidx_cur;   // [n] current (last accepted) solution
    int32_t* alns_kidx_best;  // [n] best solution
    void* alns_r_cur;         // T[m] residual of the current solution
    uint64_t* alns_weight;    // [n] integer sampling weights of the worst-remove operator
    uint64_t* alns_prefix;    // [n] their inclusive prefix sums
    uint64_t* alns_first;     // [n] stamp of the first draw of a variable in an iteration
    int32_t* alns_picked;     // [n] variables drawn, in the order of the draws
    uint8_t* alns_touched;    // [m] sparse repair: rows of the column being reassigned
    int32_t* alns_g_row;      // sparse repair: entries of the picked columns, global row (-1: padding)
    void* alns_g_val;         //   and value, a fixed stride per picked column (2^20 entries in all)
    double* alns_q2;          // [R] squared l2 norm of the working residual (l2 guard)
    double* alns_q2_blocks;   // [ceil(m / 256)] single instance: block sums of the above
    // batched descent: virtual batch of the instances still running
    bool cmp_on;              // the loop's arrays currently point at the virtual batch
    void* cmp_r;              // T[m][R'] / int32[n][R'] / InstState[R'] / T[R'] / int32[R'] (orig)
    int32_t* cmp_kidx;
    void* cmp_state;
    void* cmp_scale;
    int32_t* cmp_orig;
    void* cmp_full_r;         // the caller's batch while cmp_on
    int32_t* cmp_full_kidx;
    void* cmp_full_state;
    void* cmp_full_scale;
    int64_t cmp_full_R;
    void* search_part;        // dense, options.value_search: Partial<T>[n], one record per variable
    // swap move
    int32_t swap_nb;          // dense, batched: workgroups per instance of the evaluation
    int32_t* swap_rows;       // dense, batched: [R][SWAP_KMAX] rows of largest |r|, decreasing
    void* swap_part;          // Partial<T>[R][swap_nb]; sparse: one per evaluation workgroup
    int32_t* swap_skip;       // [R] 1: the last search of this ALNS iteration found no swap
    unsigned long long* swap_gbest;   // sparse: order bits of the best t' found so far by any workgroup
    // l2 change of every candidate (options.l2_rule)
    void* l2_g;           // T[n][R] g = A^T r of the current residual (instances contiguous)
    void* l2_c;           // T[n] squared column norms
    void* l2_scores;      // T[R][n*nd] score table the arg-min with the second criterion reads
    // batched evaluation on the matrix cores
    bool eval_mfma;       // the matrix-core kernel scores the moves
    void* rT;             // float[R][m64] instance-major copy of r, rows padded with zeros to a multiple of 64
    // batched residual on the matrix cores (options.residual_mfma)
    void* Xp;             // bf16[3][m][mfma_ldk] planes whose sum is X
    void* Qt;             // bf16[R][mfma_ldk] current codes D[k_j] per instance
    int64_t mfma_ldk;     // row stride of Xp and Qt: n rounded up to an odd number of K steps, zero-filled
    int32_t mfma_planes;  // bit s set: plane s of Xp is not all zero (bit 0 always)
};

}  // namespace dmmv

// the opaque handle of the C ABI is the context itself
struct dmmv_ctx : public dmmv::Ctx {};

namespace dmmv {

// Lays the device buffers out in a workspace starting at `base` (may be NULL: size only).
// Returns the bytes needed.  Fills the pointer fields of *c when c != NULL.
size_t workspace_layout(const dmmv_problem& p, const dmmv_options& o, Ctx* c, char* base);

static inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

// columns per workgroup of the sparse finalize kernel (one arg-min record each)
constexpr int CSC_FIN_BLOCK = 256;
// bytes of LDS a sparse evaluation workgroup may use for its partition of r
// (64 KiB: two workgroups share a compute unit's 160 KiB, so one can stage while the other
// streams)
constexpr int CSC_LDS_BYTES = 64 * 1024;
constexpr int CSC_MAX_PARTITIONS = 1024;

// ----------------------------------------------------------------------------------------
// per-path entry points (all enqueue on c->stream)
// ----------------------------------------------------------------------------------------
dmmv_status alns_start(Ctx* c, bool l2_guard);
dmmv_status alns_sumsq(Ctx* c);          // alns_q2 <- squared l2 norm of r, per instance
dmmv_status alns_destroy_repair(Ctx* c, const dmmv_alns_params& prm, int32_t it, int32_t count);
dmmv_status alns_finish_iteration(Ctx* c, const dmmv_alns_params& prm, int32_t* trace, void* trace_t);
dmmv_status alns_export(Ctx* c, void* t_best_out);
dmmv_status csc_alns_impact(Ctx* c, double alpha);
dmmv_status csc_alns_repair(Ctx* c, int32_t count, uint64_t seed);
dmmv_status csc_alns_after_copy(Ctx* c);
int64_t mfma_ldk(int64_t n);
dmmv_status batched_mfma_build(Ctx* c);
dmmv_status batched_mfma_residual(Ctx* c);
dmmv_status dense_residual(Ctx* c);
int64_t dense_num_partials(const dmmv_problem& p);    // arg-min records one evaluation writes
dmmv_status dense_eval(Ctx* c, void* scores_out, bool want_partials, bool honor_done);
bool dense_has_fused_select_apply(const Ctx* c);
dmmv_status dense_select_apply(Ctx* c, int32_t iters, dmmv_move* trace, void* trace_t);
dmmv_status dense_eval_search(Ctx* c, bool honor_done);   // one record per variable into search_part
dmmv_status dense_apply(Ctx* c, bool t_from_score, int32_t iters, dmmv_move* trace, void* trace_t);

int32_t swap_blocks_per_instance(const dmmv_problem& p);
dmmv_status swap_clear_skip(Ctx* c);
// best strictly improving swap of every instance (i = -1: none), carried out if apply != 0;
// use_skip: pass over instances marked by an earlier search and mark those without a swap
dmmv_status swap_move(Ctx* c, int32_t k_eps, int32_t apply, bool use_skip, dmmv_swap* best, void* best_t);
int64_t swap_csc_records(const dmmv_problem& p);
dmmv_status swap_move_csc(Ctx* c, int32_t apply, bool use_skip, dmmv_swap* best, void* best_t);

dmmv_status l2_build(Ctx* c);            // squared column norms, once per handle
dmmv_status l2_update_g(Ctx* c);         // g = A^T r for the current residual
dmmv_status l2_table(Ctx* c, void* dq_out);
// arg-min of a score table [R][n*nd] with the l2 change as second criterion (options.l2_rule 1, 2);
// stages the move in the loop state like the other selection kernels
dmmv_status l2_select(Ctx* c, const void* scores, int32_t keep_going, dmmv_move* best_out, void* best_score_out);
dmmv_status l2_after_apply_csc(Ctx* c, int32_t iters, dmmv_move* trace, void* trace_t);

dmmv_status csc_build(Ctx* c);
dmmv_status csc_residual(Ctx* c);
dmmv_status csc_reservoir(Ctx* c);      // rebuild the reservoir of largest |r| from r
dmmv_status csc_eval(Ctx* c, void* scores_out, bool want_partials, bool honor_done);
dmmv_status csc_apply(Ctx* c);          // staged move only; caller refreshes t and the reservoir
dmmv_status csc_select_apply(Ctx* c, int32_t iters, dmmv_move* trace, void* trace_t, bool pruned);
dmmv_status csc_eval_pruned(Ctx* c, bool honor_done);   // records of the columns of the worst row only

bool batched_eval_mfma_applicable(const dmmv_problem& p);
int64_t batched_eval_mfma_rt_elems(const dmmv_problem& p);
dmmv_status batched_eval_mfma_build(Ctx* c);
dmmv_status batched_eval_mfma(Ctx* c, void* scores_out, bool want_partials);
dmmv_status batched_build(Ctx* c);
dmmv_status batched_build_xt(Ctx* c);    // the row-major copy of X only
dmmv_status batched_residual(Ctx* c);
dmmv_status batched_eval(Ctx* c, void* scores_out, bool want_partials);
dmmv_status batched_apply(Ctx* c, bool t_from_score, int32_t iters, dmmv_move* trace, void* trace_t);
dmmv_status batched_set_x(Ctx* c, const void* x_values);
dmmv_status batched_get_x(Ctx* c, void* x_values);
dmmv_status batched_get_x_from(Ctx* c, const int32_t* kidx, void* x_values);
dmmv_status batched_set_r(Ctx* c, const void* r);
dmmv_status batched_get_r(Ctx* c, void* r);
dmmv_status batched_maxabs(Ctx* c);     // state[q].t = max_i |r[i][q]|
dmmv_status batched_compact(Ctx* c, int32_t* active_out);   // polling point of the descent
dmmv_status batched_compact_end(Ctx* c);
// dense single instance: all iterations of the descent in one launch (a fixed grid of workgroups
// that exchange one arg-min record per iteration); same moves as evaluation + selection + apply
size_t dense_persistent_exchange_bytes();
bool dense_persistent_fits(const dmmv_problem& p);
bool dense_persistent_applicable(const Ctx* c);
dmmv_status dense_descent_persistent(Ctx* c, int32_t iters, dmmv_move* trace, void* trace_t);

// options.prune on a batch: `steps` iterations of the descent for every instance in one launch,
// same moves as evaluation + selection + apply (an instance stops at its local optimum)
bool batched_pruned_applicable(const Ctx* c);
dmmv_status batched_descent_pruned(Ctx* c, int32_t steps, int32_t iters, dmmv_move* trace, void* trace_t);

// ----------------------------------------------------------------------------------------
// device helpers
// ----------------------------------------------------------------------------------------
#ifdef __HIPCC__

template <class T> struct Limits;
template <> struct Limits<float> {
    __device__ static float inf() { return __builtin_huge_valf(); }
};
template <> struct Limits<double> {
    __device__ static double inf() { return __builtin_huge_val(); }
};

__device__ __forceinline__ float dmmv_fma(float a, float b, float c) { return __builtin_fmaf(a, b, c); }
__device__ __forceinline__ double dmmv_fma(double a, double b, double c) { return __builtin_fma(a, b, c); }
__device__ __forceinline__ float dmmv_abs(float a) { return __builtin_fabsf(a); }
__device__ __forceinline__ double dmmv_abs(double a) { return __builtin_fabs(a); }
__device__ __forceinline__ float dmmv_max(float a, float b) { return __builtin_fmaxf(a, b); }
__device__ __forceinline__ double dmmv_max(double a, double b) { return __builtin_fmax(a, b); }

// step of the move (k_cur -> k): sc * (D[k] - D[k_cur]), two roundings
template <class T>
__device__ __forceinline__ T step_of(T dk, T dcur, T sc) {
    T diff = dk - dcur;
    return sc * diff;
}

// DPP controls (GFX9 encoding)
constexpr int DPP_QUAD_XOR1 = 0xB1;        // quad_perm [1,0,3,2]
constexpr int DPP_QUAD_XOR2 = 0x4E;        // quad_perm [2,3,0,1]
constexpr int DPP_ROW_HALF_MIRROR = 0x141;
constexpr int DPP_ROW_MIRROR = 0x140;

template <int CTRL>
__device__ __forceinline__ float dpp_mov(float v) {
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xF, 0xF, true));
}
template <int CTRL>
__device__ __forceinline__ double dpp_mov(double v) {
    int lo = __double2loint(v), hi = __double2hiint(v);
    lo = __builtin_amdgcn_update_dpp(0, lo, CTRL, 0xF, 0xF, true);
    hi = __builtin_amdgcn_update_dpp(0, hi, CTRL, 0xF, 0xF, true);
    return __hiloint2double(hi, lo);
}

// Maximum over the 64 lanes of a wavefront, result in every lane.  max is idempotent, so a
// butterfly of DPP permutations inside each row of 16 lanes (quad xor 1, quad xor 2, half-row
// mirror, row mirror) leaves every row with its maximum in all its lanes; the four row results
// are then read through the scalar unit (no trip through the LDS crossbar, whose latency a
// chain of reductions would pay once per exchange).  All 64 lanes must be active.
__device__ __forceinline__ float read_lane(float v, int l) {
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), l));
}
__device__ __forceinline__ double read_lane(double v, int l) {
    return __hiloint2double(__builtin_amdgcn_readlane(__double2hiint(v), l),
                            __builtin_amdgcn_readlane(__double2loint(v), l));
}
__device__ __forceinline__ int64_t read_lane(int64_t v, int l) {
    const uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)v, l);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)((uint64_t)v >> 32), l);
    return (int64_t)(((uint64_t)hi << 32) | lo);
}
template <class T>
__device__ __forceinline__ T wave_max(T v) {
    v = dmmv_max(v, dpp_mov<DPP_QUAD_XOR1>(v));
    v = dmmv_max(v, dpp_mov<DPP_QUAD_XOR2>(v));
    v = dmmv_max(v, dpp_mov<DPP_ROW_HALF_MIRROR>(v));
    v = dmmv_max(v, dpp_mov<DPP_ROW_MIRROR>(v));
    return dmmv_max(dmmv_max(read_lane(v, 0), read_lane(v, 16)), dmmv_max(read_lane(v, 32), read_lane(v, 48)));
}

// Lexicographic minimum of (score, index) over the wavefront, result in every lane.
// Records with c < 0 are empty and lose against everything.
template <class T>
__device__ __forceinline__ bool rec_less(T s1, int64_t c1, T s2, int64_t c2) {
    if (c1 < 0) return false;
    if (c2 < 0) return true;
    return (s1 < s2) || (s1 == s2 && c1 < c2);
}

// Row reductions run on DPP permutations (no LDS crossbar); the four row results are then read
// through the scalar unit.  All 64 lanes must be active.
__device__ __forceinline__ float dmmv_min(float a, float b) { return __builtin_fminf(a, b); }
__device__ __forceinline__ double dmmv_min(double a, double b) { return __builtin_fmin(a, b); }

template <int CTRL>
__device__ __forceinline__ int64_t dpp_mov(int64_t v) {
    const uint32_t lo = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)(uint32_t)v, CTRL, 0xF, 0xF, true);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)(uint32_t)((uint64_t)v >> 32), CTRL, 0xF, 0xF, true);
    return (int64_t)(((uint64_t)hi << 32) | lo);
}

// minimum over the wavefront, the same value in every lane
template <class T>
__device__ __forceinline__ T wave_min(T v) {
    v = dmmv_min(v, dpp_mov<DPP_QUAD_XOR1>(v));
    v = dmmv_min(v, dpp_mov<DPP_QUAD_XOR2>(v));
    v = dmmv_min(v, dpp_mov<DPP_ROW_HALF_MIRROR>(v));
    v = dmmv_min(v, dpp_mov<DPP_ROW_MIRROR>(v));
    return dmmv_min(dmmv_min(read_lane(v, 0), read_lane(v, 16)), dmmv_min(read_lane(v, 32), read_lane(v, 48)));
}
__device__ __forceinline__ int64_t wave_min(int64_t v) {
    int64_t o;
    o = dpp_mov<DPP_QUAD_XOR1>(v); v = o < v ? o : v;
    o = dpp_mov<DPP_QUAD_XOR2>(v); v = o < v ? o : v;
    o = dpp_mov<DPP_ROW_HALF_MIRROR>(v); v = o < v ? o : v;
    o = dpp_mov<DPP_ROW_MIRROR>(v); v = o < v ? o : v;
    const int64_t a = read_lane(v, 0), b = read_lane(v, 16), c = read_lane(v, 32), d = read_lane(v, 48);
    const int64_t ab = a < b ? a : b, cd = c < d ? c : d;
    return ab < cd ? ab : cd;
}

// (score, index) minimum in two passes: the smallest score, then the smallest index among the
// lanes that hold it.  Empty records take part as (+inf, INT64_MAX).
template <class T>
__device__ __forceinline__ void wave_argmin(T& s, int64_t& c) {
    const bool empty = c < 0;
    const T se = empty ? Limits<T>::inf() : s;
    const T smin = wave_min(se);
    const int64_t ce = (!empty && se == smin) ? c : INT64_MAX;
    const int64_t cmin = wave_min(ce);
    s = cmin == INT64_MAX ? (T)0 : smin;
    c = cmin == INT64_MAX ? (int64_t)-1 : cmin;
}

// Block-wide version; result valid in thread 0.  sh_s/sh_c hold blockDim.x/64 entries.
template <class T>
__device__ __forceinline__ void block_argmin(T& s, int64_t& c, T* sh_s, int64_t* sh_c) {
    wave_argmin(s, c);
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6, nw = (blockDim.x + 63) >> 6;
    if (lane == 0) { sh_s[w] = s; sh_c[w] = c; }
    __syncthreads();
    if (w == 0) {
        T ls = lane < nw ? sh_s[lane] : (T)0;
        int64_t lc = lane < nw ? sh_c[lane] : (int64_t)-1;
        wave_argmin(ls, lc);
        s = ls; c = lc;
    }
}

// Is candidate k of a variable currently at k_cur inside the neighbourhood?
__device__ __forceinline__ bool cand_allowed(int32_t kcur, int32_t k, int32_t radius, bool var_ok) {
    if (k == kcur) return true;
    if (!var_ok) return false;
    if (radius > 0) {
        int32_t d = k > kcur ? k - kcur : kcur - k;
        if (d > radius) return false;
    }
    return true;
}

#endif  // __HIPCC__

}  // namespace dmmv
