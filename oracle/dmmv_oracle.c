/*
 * CPU oracle for the single-move descent on the Discrete Min-Max Violation problem
 * (min over x in D^n of ||A x - b||_inf).
 *
 * TEST INFRASTRUCTURE ONLY: this library exists to check the GPU library and to be
 * timed as a baseline.  It shares no source, header or table with the GPU code and is
 * never called by it.  Plain scalar C, one fused multiply-add per (row, move) pair,
 * compiled without floating-point contraction so that only the explicit fma() calls
 * fuse.
 *
 * Pins (see tests): objective and best move against brute-force enumeration, the
 * score table against fresh recomputation of ||A x' - b||_inf, maintained residual
 * against recomputation, monotone objective, Chebyshev LP lower bound, the
 * Subset-Sum (m = 1, D = {0,1}) and A = I closed forms, sparse against dense.
 * The ALNS outer loop (alns_*.inc) has pins of its own: published SplitMix64 outputs, the
 * library exponential, the three bound equations of the worst-remove operator evaluated
 * literally, draw frequencies, greedy repair against fresh recomputation, and the loop's
 * invariants.
 * The swap move (swap_oracle_impl.inc) is pinned by fresh recomputation of ||A x' - b||_inf for
 * the exchanged x', by Proposition 1 and Corollary 1 evaluated in rational arithmetic, and by
 * the A = I closed form.
 * The l2 changes (l2_oracle_impl.inc) are pinned by fresh recomputation of ||A x' - b||_2^2 -
 * ||A x - b||_2^2 on integer data (exact), by numpy for real data, and the selection rule by
 * brute force over constructed ties.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#include "alns_common.inc"

#define REAL double
#define SFX(x) x##_f64
#define FMA fma
#define FABS fabs
#include "dmmv_oracle_impl.inc"
#include "swap_oracle_impl.inc"
#include "alns_oracle_impl.inc"
#include "l2_oracle_impl.inc"
#undef REAL
#undef SFX
#undef FMA
#undef FABS

#define REAL float
#define SFX(x) x##_f32
#define FMA fmaf
#define FABS fabsf
#include "dmmv_oracle_impl.inc"
#include "swap_oracle_impl.inc"
#include "alns_oracle_impl.inc"
#include "l2_oracle_impl.inc"
#undef REAL
#undef SFX
#undef FMA
#undef FABS

#ifdef _OPENMP
#include <omp.h>
int oracle_num_threads(void) { return omp_get_max_threads(); }
#else
int oracle_num_threads(void) { return 1; }
#endif
