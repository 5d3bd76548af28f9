/*
 * libdmmv - GPU (gfx950) hot path of the AMVM heuristic for the Discrete Min-Max
 * Violation problem (arXiv 2508.13437):
 *
 *     choose x in D^n (D a finite set of reals) to minimise  t = max_i |A_i x - b_i| .
 *
 * The library keeps the residual r = A x - b on the device, scores every
 * single-coordinate move x_j -> D[k] as max_i |r_i + (D[k] - x_j) A_ij|, finds the best
 * move with a lowest-index tie-break, and applies it as a rank-1 residual update.  These
 * are the GPU-parallel boxes of the paper's Figure 1 (bulk candidate evaluation followed
 * by a global minimum reduction, section "GPU Acceleration"; greedy repair, Appendix B.3;
 * 1-OPT local search, section "Search Operators"), with the residual identity of
 * Appendix A restricted to one changed coordinate.
 *
 * Three storage kinds are supported by one handle type:
 *   dense    A column-major m x n                      (R = 1)
 *   sparse   A in CSR (a CSC copy is built at create)  (R = 1)
 *   batched  R independent instances sharing a dense A = X; instance q has its own
 *            target b_q, scale s_q and x_q; its variables take the values s_q * D[k]
 *            (one output row of a quantised linear layer, paper section
 *            "Quantization without outlier separation as DMMV").
 *
 * Conventions
 *   - Plain C ABI.  Pointers are DEVICE pointers unless marked HOST.  The caller owns every
 *     buffer it passes; the library borrows problem buffers until dmmv_destroy and never
 *     frees them.  The library allocates no device memory: its device state lives in the
 *     workspace the caller provides (size from dmmv_workspace_bytes, 256-byte aligned).
 *   - dtype selects float (DMMV_F32) or double (DMMV_F64) for A, b, D, scale, x, r and
 *     scores alike.
 *   - x is exchanged as VALUES of D (not indices), layout [R][n].  r is [R][m].  The score
 *     table is [R][n*nd]; flat candidate index c = j*nd + k (k = position in ascending D).
 *   - All work is enqueued on the stream given at create.  Calls return after enqueueing
 *     unless stated otherwise; results in device buffers are ordered on that stream.
 *   - Every call returns a dmmv_status; dmmv_last_error() gives a message for the last
 *     failure on the calling thread.  No exceptions or aborts cross the ABI.
 *   - Arithmetic contract (what makes results reproducible bit for bit):
 *       step      delta = s * (D[k] - D[k_j])                 (two roundings; s = 1 unscaled)
 *       pair      | fma(delta, A_ij, r_i) |                   (one fused multiply-add)
 *       residual  acc = 0; for j ascending (CSR: stored order): acc = fma(A_ij, D[k_j], acc);
 *                 r_i = fma(acc, s, -b_i)
 *     max and arg-min are exact.  Inputs must be finite.
 */
#ifndef DMMV_H
#define DMMV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct dmmv_ctx* dmmv_handle;

typedef enum { DMMV_F32 = 0, DMMV_F64 = 1 } dmmv_dtype;

typedef enum {
    DMMV_OK = 0,
    DMMV_ERR_NULL = -1,        /* a required pointer is NULL                               */
    DMMV_ERR_SHAPE = -2,       /* negative size, lda < m, CSR with duplicate / out-of-range  */
    DMMV_ERR_DTYPE = -3,       /* dtype not F32 / F64                                       */
    DMMV_ERR_DOMAIN = -4,      /* D not finite / not strictly ascending / nd < 2; x not in D */
    DMMV_ERR_WORKSPACE = -5,   /* workspace NULL, misaligned or too small                    */
    DMMV_ERR_HIP = -6,         /* a HIP runtime call failed                                  */
    DMMV_ERR_STATE = -7,       /* call order: x not set, residual not computed, ...          */
    DMMV_ERR_UNSUPPORTED = -8  /* combination not implemented (message says which)           */
} dmmv_status;

/* A move: variable j takes the value D[k].  j = -1 means "no move". */
typedef struct { int32_t j, k; } dmmv_move;

/* Problem description (paper, "Mathematical Problem Statement": A, b, value set V = D). */
typedef struct {
    int32_t dtype;               /* dmmv_dtype                                              */
    int32_t nd;                  /* |D|, 2 <= nd <= 65535                                   */
    int64_t m, n;                /* rows (constraints), variables                           */
    const void* D;               /* HOST [nd], strictly ascending, copied at create         */
    const void* A_dense;         /* column-major m x n with leading dimension lda, or NULL  */
    int64_t lda;
    const int64_t* csr_rowptr;   /* [m+1], or NULL.  Exactly one of A_dense / csr_* is set  */
    const int32_t* csr_col;      /* [nnz] column of each entry, any order inside a row      */
    const void* csr_val;         /* [nnz]                                                   */
    int64_t nnz;
    const void* b;               /* [R][m]                                                  */
    int64_t R;                   /* instances sharing A (R > 1 or scale != NULL => batched) */
    const void* scale;           /* HOST [R] positive scales, or NULL (all 1, R must be 1)  */
} dmmv_problem;

/* Neighbourhood and loop options. */
typedef struct {
    int32_t radius;          /* 0: every value of D is a candidate (default);
                                q > 0: only values at most q levels from the current one
                                (the paper's 1-OPT and greedy repair use q = 1)             */
    int32_t keep_going;      /* dmmv_solve: 0 = an instance stops at the first iteration whose
                                best move is not a strict improvement; 1 = keep scoring all
                                moves every iteration although nothing can be applied
                                (fixed-work mode for throughput measurement)                */
    int32_t poll_every;      /* dmmv_solve: every poll_every iterations the host waits for the
                                stream and stops enqueueing once every instance has stopped;
                                0 = never wait inside the loop.  A batch (without var_mask)
                                polls at least every 8 iterations and continues on the
                                instances that still run, packed densely                    */
    int32_t sparse_partition_rows; /* sparse matrices: rows per LDS-resident partition of r;
                                0 = automatic (as many as fit 64 KiB, at most 65535).  A tuning
                                and testing knob: results do not depend on it              */
    const uint8_t* var_mask; /* [R][n] nonzero = variable may move (greedy repair works on the
                                unassigned variables only); NULL = all                      */
    int32_t residual_mfma;   /* batched fp32 problems whose D is exact in bf16 (integer codes):
                                1 = dmmv_residual / dmmv_solve compute r = (X Q^T) diag(s) - B on the
                                matrix cores (X split into bf16 planes that sum to it exactly,
                                products exact, fp32 accumulation in the instruction's order), so r
                                agrees with the sequential-order kernel only to fp32 rounding of the
                                sum; 0 (default) = sequential order, bitwise reproducible.
                                dmmv_create fails with DMMV_ERR_UNSUPPORTED if 1 is not applicable */
    int32_t prune;           /* sparse matrices: 1 = the descent (dmmv_solve without keep_going, the
                                local search of dmmv_alns) scores only the moves of the variables
                                with an entry in the row of largest |r_i|: a move that leaves
                                that row alone cannot lower the maximum, so the moves applied are
                                the same as with the full evaluation and an iteration costs far
                                less.  Batches of instances: 1 = the descent bounds every move
                                from below by its score on 16 rows of large |r_i| (a maximum over
                                some rows never exceeds the maximum over all) and scores over all
                                rows only the moves, in ascending order of bound, that can still
                                beat the best score found; same moves again, all iterations of a
                                call in one launch (used when the instance's r and x fit in
                                96 KiB of LDS: (m + n) w + 2 n bytes, 4 n if nd > 256, and
                                m <= 16384; otherwise the full evaluation runs).  A dense single instance is
                                taken as a batch of one (one workgroup, all iterations in one launch)
                                when it is small - at most 64 levels and 2^24 (row, move) pairs per
                                table - so that a launch per step costs more than the step; larger
                                dense instances keep the chip-wide full evaluation.
                                dmmv_eval_moves and dmmv_argmin_move always score all             */
    int32_t alns;            /* batched problems: 1 = reserve the workspace dmmv_alns needs (current
                                and best solution, sampling weights and draws per instance, about
                                R*(36 n + m w) bytes).  Single-instance handles always have it    */
    int32_t value_search;    /* dense matrices: 1 = the descent (dmmv_solve without keep_going, the
                                local search of dmmv_alns) finds the best value of each variable
                                by bisection over D instead of scoring all nd values: the score of
                                a variable's values is quasi-convex in the value's index, also as
                                computed (D ascends and rounding is monotone), so about log2(nd)
                                values are scored per variable and the moves applied are the same
                                as with the full evaluation.  dmmv_eval_moves and
                                dmmv_argmin_move always score all                                */
    int32_t batched_eval;    /* batched problems: which kernel scores the moves.  0 or 1 = the
                                vector-unit kernel (default); 2 = the matrix-core kernel, for fp32
                                with nd <= 32 (dmmv_create fails with DMMV_ERR_UNSUPPORTED
                                otherwise; it needs R * m more floats of workspace).  It forms every
                                fused multiply-add as one element of an outer product with K = 1,
                                rounded once like the vector instruction, so both kernels give the
                                same bits; on MI355X it is the slower of the two (the maximum over
                                the rows stays on the vector unit and does not overlap)           */
    int32_t sparse_eval;     /* sparse matrices: which kernels score the moves.  0 = automatic;
                                1 = two kernels: workgroups own (row partition, column range) pairs and
                                write per-partition maxima, a second kernel combines them (residual
                                traffic independent of n: for matrices with very many rows);
                                2 = one kernel: a workgroup owns 256 columns and walks every row
                                partition, its maxima never leave the registers (every workgroup
                                reads all of r: taken automatically when (n / 256) m w bytes do not
                                exceed the matrix).  Same scores, records and moves either way    */
    int32_t l2_rule;         /* the change of the squared l2 norm of the residual, dq = ||r + delta a_j||^2 -
                                ||r||^2, beside the score (paper: the l-infinity and l2 changes of the
                                candidates are evaluated together; the quantisation use case keeps the
                                l2 norm from increasing).  0 = not used (default: lowest index among
                                equal scores).  1 = second criterion of every arg-min of the handle
                                (dmmv_argmin_move, dmmv_solve, the local search of dmmv_alns): smallest
                                score, then smallest dq, then lowest index.  2 = the same among the
                                candidates with dq <= 0 only, so that no move raises the l2 norm.
                                3 = reserve the workspace of dmmv_l2_changes only.  With 1 and 2 the
                                evaluation writes its whole score table every iteration (R n nd more
                                elements of workspace) and options.prune / value_search do not apply  */
    int32_t dense_loop;      /* one dense instance: how dmmv_solve iterates (paper: the iteration is not to
                                pay for host-side stepping and synchronisation).  1 = a launch of the
                                evaluation and one of selection + apply per iteration.  2 = all
                                iterations in ONE launch: a fixed grid of at most 256 workgroups shares
                                the moves, each keeps r, its columns of A, D and x in LDS, and they
                                exchange one arg-min record per iteration through memory (needs r, D, x
                                and one column to fit 156 KiB of LDS; dmmv_create fails with
                                DMMV_ERR_UNSUPPORTED otherwise).  0 = automatic: 2 when it fits and a model
                                of both loops says its iteration is the shorter one, else 1.  Same
                                scores, moves, traces and residual either way.  With 2 the workgroups
                                wait for one another, so all must be resident on the device at once;
                                if another kernel keeps some from starting, the wait ends after
                                wait_limit polls; x, r and the loop state are then untouched, and
                                dmmv_solve returns DMMV_ERR_STATE (dense_loop = 2) or runs the same
                                descent with launches (dense_loop = 0).  options.prune and value_search (without
                                keep_going) and l2_rule 1 / 2 keep their own loops                    */
    int32_t wait_limit;      /* dense_loop = 2: polls of another workgroup's arrival word before the
                                kernel gives up; 0 = default (2^22, a few seconds)                    */
} dmmv_options;

/* Bytes of device workspace dmmv_create needs for this problem (0 on invalid input, with
 * dmmv_last_error set).  HOST computation, no GPU call. */
size_t dmmv_workspace_bytes(const dmmv_problem* problem, const dmmv_options* options);

/* Validate, copy D and scale, build the internal layouts (CSC copy of a CSR matrix;
 * row-major copy of X and instance-interleaved copies of b for a batch).  `options` may be
 * NULL (defaults).  hip_stream is a hipStream_t (NULL = the default stream).  Waits for
 * the stream before returning so that layout errors (DMMV_ERR_SHAPE) can be reported. */
dmmv_status dmmv_create(dmmv_handle* out, const dmmv_problem* problem, const dmmv_options* options,
                        void* workspace, size_t workspace_bytes, void* hip_stream);

/* Releases the host-side handle.  Device buffers belong to the caller. */
dmmv_status dmmv_destroy(dmmv_handle h);

/* Set the current point from values x [R][n] (each must equal an entry of D exactly;
 * waits for the stream to report DMMV_ERR_DOMAIN).  Invalidates the residual. */
dmmv_status dmmv_set_x(dmmv_handle h, const void* x_values);

/* Overwrite the maintained residual with r [R][m] and recompute t = max |r|
 * (for starting from a residual computed elsewhere). */
dmmv_status dmmv_set_residual(dmmv_handle h, const void* r);

/* r = A x - b for the current x, in the fixed order of the arithmetic contract; also sets
 * t = max_i |r_i|.  r_out [R][m] may be NULL (internal state only).
 * Paper: residual s = Ax - b and objective t = ||s||_inf, "Materials and Methods". */
dmmv_status dmmv_residual(dmmv_handle h, void* r_out);

/* Score table of the current state: scores_out[q][j*nd + k] = max_i |fma(delta, A_ij, r_i)|.
 * The null move k = k_j scores exactly t.  Candidates outside the neighbourhood (radius,
 * var_mask) get +infinity.  Sparse matrices: the maximum still runs over all m rows (rows
 * without an entry in column j contribute |r_i|).
 * Paper: Appendix B.3 step 3, Appendix A component form, "evaluate all candidates in bulk". */
dmmv_status dmmv_eval_moves(dmmv_handle h, void* scores_out);

/* Best move per instance: smallest score, lowest flat index among equal scores.
 * scores [R][n*nd] is a table to reduce, or NULL to score the current state without
 * writing a table (fused evaluation + reduction).  best [R] and best_score [R] receive the
 * result (best.j = -1 only if n = 0).  The move is reported whether or not it improves.
 * Paper: "choose minima via global reductions", "tensor-wide argmin". */
dmmv_status dmmv_argmin_move(dmmv_handle h, const void* scores, dmmv_move* best, void* best_score);

/* Apply moves [R] (entries with j = -1 are skipped): x_j <- D[k],
 * r_i <- fma(delta, A_ij, r_i) for all rows (sparse: the rows of column j), t <- max |r|.
 * Paper: Appendix A boxed identity; Algorithm 2 residual update line. */
dmmv_status dmmv_apply_move(dmmv_handle h, const dmmv_move* moves);

/* Copy out the current x values [R][n], residual [R][m] and max violation [R]
 * (any may be NULL). */
dmmv_status dmmv_get_state(dmmv_handle h, void* x_values, void* r, void* max_violation);

/* The descent: set x = x0, compute r, then up to `iters` times { score all moves, take the
 * best, stop the instance unless it strictly lowers t, apply it }.
 *   x_out [R][n], max_violation_out [R], iters_done [R] (moves applied)   - any may be NULL
 *   trace [R][iters] applied moves in order (j = -1 past the end), trace_t [R][iters]
 *   the max violation after each                                            - may be NULL
 * x0 = NULL continues from the handle's current x.  r is recomputed from x at the start of
 * every call and maintained by rank-1 updates inside it, so calling dmmv_solve(h, NULL, k)
 * repeatedly is a descent whose residual is refreshed every k moves.
 * Waits for the stream before returning.
 * Paper: Algorithm 1 local-search step restricted to single-coordinate moves; strict
 * improvement as in Proposition 1 / Algorithm 2. */
dmmv_status dmmv_solve(dmmv_handle h, const void* x0, int32_t iters, void* x_out,
                       void* max_violation_out, int32_t* iters_done, dmmv_move* trace,
                       void* trace_t);

/* For callers that cannot allocate device memory (code under HIP graph capture around the call,
 * tight serving loops, harnesses that forbid hipMalloc): the whole of dmmv_create + dmmv_solve +
 * dmmv_destroy in one call that allocates nothing, on the device or on the heap.  The workspace is
 * an array of DMMV_STATIC_SCRATCH_BYTES inside the library's device image (every GPU the library
 * runs on holds its own copy until the process ends); the handle lives on the stack.  Arguments as
 * for dmmv_create (problem, options, hip_stream) and dmmv_solve (the rest); x0 must not be NULL.
 * The device of hip_stream must be the current device.  Fails with DMMV_ERR_WORKSPACE, before any
 * GPU work, when dmmv_workspace_bytes(problem, options) exceeds DMMV_STATIC_SCRATCH_BYTES.
 * Every call on a GPU uses that GPU's one array, so calls that overlap in time on one GPU race
 * (also from different streams or threads); what a call needs cleared it clears itself.  Waits for
 * the stream before returning. */
#define DMMV_STATIC_SCRATCH_BYTES (16u << 20)
dmmv_status dmmv_solve_static(const dmmv_problem* problem, const dmmv_options* options, const void* x0,
                              int32_t iters, void* x_out, void* max_violation_out, int32_t* iters_done,
                              dmmv_move* trace, void* trace_t, void* hip_stream);

/* Parameters of the ALNS outer loop (Algorithm 1 of the paper).  What the paper leaves open is
 * fixed as stated at each field. */
typedef struct {
    int32_t iters;           /* outer iterations: destroy, repair, local search, accept          */
    int32_t ls_moves;        /* local search: at most this many moves of the single-move descent
                                per outer iteration (it stops earlier at a local optimum)        */
    int32_t ls_radius;       /* neighbourhood of the local search, as dmmv_options.radius
                                (1 = the paper's 1-OPT move to a neighbouring level)              */
    int32_t destroy_count;   /* variables unassigned per iteration; 0 = 0.5 % of n, at least 1
                                (Appendix F)                                                     */
    double alpha;            /* coefficient of the impact score of the worst-remove operator
                                (Appendix B.2; Appendix F uses 0.3)                              */
    double lambda;           /* reaction factor of the operator weights (Appendix F.2 names the
                                roulette wheel, not its update): w <- (1-lambda) w + lambda psi,
                                only after an accepted iteration, as in Algorithm 1              */
    double sigma1, sigma2, sigma3; /* psi: new best / better than the current solution / accepted
                                without improvement                                              */
    uint64_t seed;           /* every random decision is a function of (seed, iteration, stream,
                                counter): two runs with the same seed are identical              */
    int32_t ls_swaps;        /* local search: after the descent, at most this many swap moves
                                (Algorithm 2; section "Search Operators": 1-OPT, then a swap),
                                each counted as one more move; it stops at the first search that
                                finds no improving swap                                           */
    int32_t k_eps;           /* rows of the swap filter (Corollary 1; Appendix F uses 100);
                                0 = 100                                                          */
    int32_t l2_guard;        /* 1 = an iteration is accepted only if the l2 norm of the residual
                                does not increase either (the check the paper applies at every
                                AMVM iteration of the quantisation use case, section "Experiment
                                setup and results").  The squared norm is summed in double
                                precision in a fixed order: rows in blocks of 256, inside a block
                                acc = fma(r_i, r_i, acc) by ascending row, then the block sums by
                                ascending block                                                  */
    int32_t reserved;        /* must be 0                                                        */
} dmmv_alns_params;

/* Algorithm 1 of the paper around the single-move descent, for every storage kind.
 * Per outer iteration: (1) one of two destroy operators and one of two
 * repair operators are chosen by roulette wheel on their weights (Appendix F.2); (2) destroy:
 * destroy_count distinct variables are drawn, uniformly (B.1) or with probability proportional
 * to the impact score d_j (B.2; R_j^k = (t - |s_k|) / |a_kj|, accumulated in fixed point);
 * (3) repair, in the order of the draws: each drawn variable moves to the level next below or
 * next above its old one, chosen at random (B.1) or as the one with the smaller worst-case
 * error, the lower on a tie (B.3), r following every reassignment; (4) local search;
 * (5) the result replaces the current solution if it is not worse, and the best solution if
 * it is strictly better; the weights of the two operators used are updated.
 * x0 (DEVICE, [n], NULL = keep the current x) is the starting point.  Outputs (DEVICE, any
 * may be NULL): x_best_out [n] values, t_best_out [1], trace [iters][4] int32 = destroy
 * operator (0 random, 1 worst-remove), repair operator (0 random, 1 greedy), moves the local
 * search made (swaps included), accepted; trace_t [iters][2] = error after the local search, best error so
 * far.  Afterwards the handle holds the current (last accepted) solution.  Waits for the
 * stream.  Batched handles (created with options.alns = 1): every instance runs its own loop
 * with its own random stream (the instance number is part of the counter); x0 and x_best_out
 * are [R][n], t_best_out [R], trace [R][iters][4], trace_t [R][iters][2]. */
dmmv_status dmmv_alns(dmmv_handle h, const void* x0, const dmmv_alns_params* params, void* x_best_out,
                      void* t_best_out, int32_t* trace, void* trace_t);

/* dq_out[q][j*nd + k] = change of the squared l2 norm of the residual under the move x_j -> D[k]
 * (handles created with options.l2_rule != 0), in the fixed arithmetic
 *     g_j = chain over the stored entries of column j by ascending row of fma(A_ij, r_i, .)
 *     c_j = the same chain of fma(A_ij, A_ij, .)         dq = delta * fma(delta, c_j, 2 g_j)
 * with delta the step of the score table.  For an fp32 batch G = X^T R_mat is computed on the matrix
 * cores with one row of the contraction per instruction, which keeps that chain bit for bit.
 * Needs a residual.
 * Paper: section "GPU Acceleration" (l-infinity and l2 changes of the candidates); Appendix A. */
dmmv_status dmmv_l2_changes(dmmv_handle h, void* dq_out);

/* A swap: variables i and j exchange their values (x_i > x_j before).  i = -1: none. */
typedef struct { int64_t i, j; } dmmv_swap;

/* Swap move of the local search, for every storage kind.  Over all pairs (i, j) with
 * x_i > x_j (both allowed by var_mask), with
 *     Delta = s * (D[k_i] - D[k_j]),   r'_k = fma(Delta, A_kj - A_ki, r_k),   t' = max_k |r'_k|,
 * the pair with the smallest t' is found, the lowest pair number i*n + j on a tie, and reported
 * if t' < t (strict improvement, Proposition 1); otherwise best.i = best.j = -1 and best_t = t.
 * apply != 0 carries the swap out: the two variables exchange their values, r <- r', t <- t'.
 * k_eps (0 = 100, at most 128) is the number of rows of largest |r_k| on which a pair is
 * tested first (the filter of Corollary 1, a necessary condition for an improvement): it
 * changes the time taken, never the result, which is that of the full enumeration.  Sparse
 * matrices ignore it: there the filter is the row of largest |r_k| itself (one of the two
 * variables must have an entry in it) and, for the rows stored in neither column, the
 * library's list of the rows of largest |r_k|.
 * best [R] and best_t [R] (DEVICE) may be NULL.  Needs a residual.
 * Paper: section "Search Operators", Proposition 1, Corollary 1; Appendix A (new residual);
 * Appendix B "Swap Move", Algorithm 2. */
dmmv_status dmmv_swap_move(dmmv_handle h, int32_t k_eps, int32_t apply, dmmv_swap* best, void* best_t);

/* Message of the last failure on this thread (static storage, HOST). */
const char* dmmv_last_error(void);

/* Library version string (HOST). */
const char* dmmv_version(void);

#ifdef __cplusplus
}
#endif
#endif /* DMMV_H */
