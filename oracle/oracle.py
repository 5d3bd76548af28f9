"""numpy front end of the CPU oracle (ctypes over oracle/liboracle.so).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the benchmark's
cpu_baseline leg.  The GPU library never imports or calls anything here.

All functions take host numpy arrays.  x is passed as values of D and converted to the
index vector the C code uses; a value that is not in D raises ValueError.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import Optional

import numpy as np

from . import build as _build

_lib = None


def lib():
    global _lib
    if _lib is None:
        # DMMV_ORACLE_LIB: another build of this library (the mutation tests load deliberately
        # broken ones to see that the pins catch them)
        _lib = C.CDLL(os.environ.get("DMMV_ORACLE_LIB") or _build.build())
        _lib.oracle_num_threads.restype = C.c_int
        for s in ("f32", "f64"):
            real = C.c_float if s == "f32" else C.c_double
            getattr(_lib, f"oracle_max_abs_{s}").restype = real
            getattr(_lib, f"oracle_apply_move_dense_{s}").restype = real
            getattr(_lib, f"oracle_apply_move_csc_{s}").restype = real
            getattr(_lib, f"oracle_solve_dense_{s}").restype = C.c_int32
            getattr(_lib, f"oracle_solve_csr_{s}").restype = C.c_int32
    return _lib


def num_threads() -> int:
    return int(lib().oracle_num_threads())


def _sfx(dtype) -> str:
    dtype = np.dtype(dtype)
    if dtype == np.float32:
        return "f32"
    if dtype == np.float64:
        return "f64"
    raise TypeError(f"unsupported dtype {dtype}")


def _real(dtype):
    return C.c_float if np.dtype(dtype) == np.float32 else C.c_double


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _fn(name: str, dtype):
    return getattr(lib(), f"{name}_{_sfx(dtype)}")


def values_to_index(x: np.ndarray, D: np.ndarray) -> np.ndarray:
    """Index of every x value in the ascending set D (exact match required)."""
    D = np.asarray(D)
    x = np.asarray(x, dtype=D.dtype)
    if D.ndim != 1 or D.size < 2 or np.any(np.diff(D) <= 0) or not np.all(np.isfinite(D)):
        raise ValueError("D must be finite, strictly ascending, with at least two values")
    k = np.searchsorted(D, x)
    k = np.clip(k, 0, D.size - 1)
    if np.any(D[k] != x):
        raise ValueError("x has a value that is not in D")
    return np.ascontiguousarray(k.astype(np.int32))


def _dense(A: np.ndarray, dtype):
    A = np.asfortranarray(A, dtype=dtype)
    m, n = A.shape
    return A, m, n, max(m, 1)


def _mask(var_mask, n):
    if var_mask is None:
        return None
    vm = np.ascontiguousarray(var_mask, dtype=np.uint8)
    assert vm.shape == (n,)
    return vm


# ----------------------------------------------------------------------------- dense
def residual_dense(A, b, D, x, scale=1.0):
    dt = np.asarray(D).dtype
    A, m, n, lda = _dense(A, dt)
    D = np.ascontiguousarray(D)
    k = values_to_index(x, D)
    b = np.ascontiguousarray(b, dtype=dt)
    r = np.empty(m, dtype=dt)
    _fn("oracle_residual_dense", dt)(C.c_int64(m), C.c_int64(n), _p(A), C.c_int64(lda), _p(D),
                                     _p(k), _real(dt)(scale), _p(b), _p(r))
    return r


def max_abs(r):
    r = np.ascontiguousarray(r)
    return r.dtype.type(_fn("oracle_max_abs", r.dtype)(C.c_int64(r.size), _p(r)))


def eval_moves_dense(A, D, x, r, scale=1.0, radius=0, var_mask=None):
    dt = np.asarray(D).dtype
    A, m, n, lda = _dense(A, dt)
    D = np.ascontiguousarray(D)
    k = values_to_index(x, D)
    r = np.ascontiguousarray(r, dtype=dt)
    vm = _mask(var_mask, n)
    scores = np.empty(n * D.size, dtype=dt)
    _fn("oracle_eval_moves_dense", dt)(C.c_int64(m), C.c_int64(n), C.c_int32(D.size), _p(A),
                                       C.c_int64(lda), _p(D), _p(k), _real(dt)(scale), _p(r),
                                       C.c_int32(radius), _p(vm), _p(scores))
    return scores


def argmin_move(scores):
    scores = np.ascontiguousarray(scores)
    c = C.c_int64(-1)
    s = _real(scores.dtype)(0)
    _fn("oracle_argmin_move", scores.dtype)(C.c_int64(scores.size), _p(scores), C.byref(c),
                                            C.byref(s))
    return int(c.value), scores.dtype.type(s.value)


def apply_move_dense(A, D, x, r, j, k, scale=1.0):
    """Returns (x_new, r_new, t_new) after x_j <- D[k]."""
    dt = np.asarray(D).dtype
    A, m, n, lda = _dense(A, dt)
    D = np.ascontiguousarray(D)
    kidx = values_to_index(x, D)
    diff = dt.type(D[k] - D[kidx[j]])
    delta = dt.type(dt.type(scale) * diff)
    r = np.array(r, dtype=dt, copy=True)
    col = np.ascontiguousarray(A[:, j])
    t = _fn("oracle_apply_move_dense", dt)(C.c_int64(m), _p(col), _real(dt)(delta), _p(r))
    xn = np.array(x, dtype=dt, copy=True)
    xn[j] = D[k]
    return xn, r, dt.type(t)


@dataclass
class SolveResult:
    x: np.ndarray
    t: float
    iters_done: int
    r: Optional[np.ndarray]
    trace_j: np.ndarray
    trace_k: np.ndarray
    trace_t: np.ndarray


def solve_dense(A, b, D, x0, iters, scale=1.0, radius=0, var_mask=None) -> SolveResult:
    dt = np.asarray(D).dtype
    A, m, n, lda = _dense(A, dt)
    D = np.ascontiguousarray(D)
    k = values_to_index(x0, D)
    b = np.ascontiguousarray(b, dtype=dt)
    vm = _mask(var_mask, n)
    t = _real(dt)(0)
    r = np.empty(m, dtype=dt)
    tj = np.full(max(iters, 1), -1, dtype=np.int32)
    tk = np.full(max(iters, 1), -1, dtype=np.int32)
    tt = np.zeros(max(iters, 1), dtype=dt)
    done = _fn("oracle_solve_dense", dt)(
        C.c_int64(m), C.c_int64(n), C.c_int32(D.size), _p(A), C.c_int64(lda), _p(b), _p(D),
        _real(dt)(scale), _p(k), C.c_int32(iters), C.c_int32(radius), _p(vm), C.byref(t), _p(r),
        _p(tj), _p(tk), _p(tt))
    return SolveResult(D[k], dt.type(t.value), int(done), r, tj[:done], tk[:done], tt[:done])


# ----------------------------------------------------------------------------- sparse
def _csr(rowptr, col, val, dt):
    return (np.ascontiguousarray(rowptr, dtype=np.int64), np.ascontiguousarray(col, dtype=np.int32),
            np.ascontiguousarray(val, dtype=dt))


def csr_to_csc(m, n, rowptr, col, val):
    dt = np.asarray(val).dtype
    rowptr, col, val = _csr(rowptr, col, val, dt)
    nnz = int(rowptr[m])
    colptr = np.empty(n + 1, dtype=np.int64)
    rowidx = np.empty(max(nnz, 1), dtype=np.int32)
    cval = np.empty(max(nnz, 1), dtype=dt)
    _fn("oracle_csr_to_csc", dt)(C.c_int64(m), C.c_int64(n), _p(rowptr), _p(col), _p(val),
                                 _p(colptr), _p(rowidx), _p(cval))
    return colptr, rowidx[:nnz], cval[:nnz]


def residual_csr(m, rowptr, col, val, b, D, x):
    dt = np.asarray(D).dtype
    rowptr, col, val = _csr(rowptr, col, val, dt)
    D = np.ascontiguousarray(D)
    k = values_to_index(x, D)
    b = np.ascontiguousarray(b, dtype=dt)
    r = np.empty(m, dtype=dt)
    _fn("oracle_residual_csr", dt)(C.c_int64(m), _p(rowptr), _p(col), _p(val), _p(D), _p(k),
                                   _p(b), _p(r))
    return r


def eval_moves_csr(m, n, rowptr, col, val, D, x, r, radius=0, var_mask=None, method="sorted",
                   columns=None):
    """Score table of a CSR instance.  method="plain" scans all rows per column (the
    definition), "sorted" walks rows by decreasing |r|.  columns=(j0, j1) restricts the
    plain method to a column range (the rest of the table is NaN)."""
    dt = np.asarray(D).dtype
    colptr, rowidx, cval = csr_to_csc(m, n, rowptr, col, np.asarray(val, dtype=dt))
    rowidx = np.ascontiguousarray(rowidx)
    cval = np.ascontiguousarray(cval)
    D = np.ascontiguousarray(D)
    k = values_to_index(x, D)
    r = np.ascontiguousarray(r, dtype=dt)
    vm = _mask(var_mask, n)
    scores = np.full(n * D.size, np.nan, dtype=dt)
    if method == "plain":
        j0, j1 = (0, n) if columns is None else columns
        _fn("oracle_eval_moves_csc_plain", dt)(
            C.c_int64(m), C.c_int64(n), C.c_int32(D.size), _p(colptr), _p(rowidx), _p(cval),
            _p(D), _p(k), _p(r), C.c_int32(radius), _p(vm), C.c_int64(j0), C.c_int64(j1),
            _p(scores))
    else:
        _fn("oracle_eval_moves_csc_sorted", dt)(
            C.c_int64(m), C.c_int64(n), C.c_int32(D.size), _p(colptr), _p(rowidx), _p(cval),
            _p(D), _p(k), _p(r), C.c_int32(radius), _p(vm), _p(scores))
    return scores


def apply_move_csr(m, n, rowptr, col, val, D, x, r, j, k):
    dt = np.asarray(D).dtype
    colptr, rowidx, cval = csr_to_csc(m, n, rowptr, col, np.asarray(val, dtype=dt))
    rowidx = np.ascontiguousarray(rowidx)
    cval = np.ascontiguousarray(cval)
    D = np.ascontiguousarray(D)
    kidx = values_to_index(x, D)
    delta = dt.type(dt.type(1) * dt.type(D[k] - D[kidx[j]]))
    r = np.array(r, dtype=dt, copy=True)
    t = _fn("oracle_apply_move_csc", dt)(C.c_int64(m), _p(colptr), _p(rowidx), _p(cval),
                                         C.c_int64(j), _real(dt)(delta), _p(r))
    xn = np.array(x, dtype=dt, copy=True)
    xn[j] = D[k]
    return xn, r, dt.type(t)


def solve_csr(m, n, rowptr, col, val, b, D, x0, iters, radius=0, var_mask=None) -> SolveResult:
    dt = np.asarray(D).dtype
    rowptr, col, val = _csr(rowptr, col, val, dt)
    D = np.ascontiguousarray(D)
    k = values_to_index(x0, D)
    b = np.ascontiguousarray(b, dtype=dt)
    vm = _mask(var_mask, n)
    t = _real(dt)(0)
    r = np.empty(m, dtype=dt)
    tj = np.full(max(iters, 1), -1, dtype=np.int32)
    tk = np.full(max(iters, 1), -1, dtype=np.int32)
    tt = np.zeros(max(iters, 1), dtype=dt)
    done = _fn("oracle_solve_csr", dt)(
        C.c_int64(m), C.c_int64(n), C.c_int32(D.size), _p(rowptr), _p(col), _p(val), _p(b), _p(D),
        _p(k), C.c_int32(iters), C.c_int32(radius), _p(vm), C.byref(t), _p(r), _p(tj), _p(tk),
        _p(tt))
    return SolveResult(D[k], dt.type(t.value), int(done), r, tj[:done], tk[:done], tt[:done])


# ----------------------------------------------------------------------------- batched
@dataclass
class BatchedResult:
    x: np.ndarray            # [R][n]
    t: np.ndarray            # [R]
    iters_done: np.ndarray   # [R]
    trace_j: np.ndarray      # [R][iters] (-1 beyond iters_done)
    trace_k: np.ndarray
    trace_t: np.ndarray


def solve_batched(X, B, D, scale, x0, iters, radius=0) -> BatchedResult:
    dt = np.asarray(D).dtype
    X, m, n, ldx = _dense(X, dt)
    D = np.ascontiguousarray(D)
    B = np.ascontiguousarray(B, dtype=dt)
    R = B.shape[0]
    assert B.shape == (R, m)
    scale = np.ascontiguousarray(scale, dtype=dt)
    assert scale.shape == (R,)
    k = np.ascontiguousarray(
        np.stack([values_to_index(x0[q], D) for q in range(R)]) if R else
        np.zeros((0, n), np.int32))
    t = np.zeros(R, dtype=dt)
    done = np.zeros(R, dtype=np.int32)
    it = max(iters, 1)
    tj = np.full((R, it), -1, dtype=np.int32)
    tk = np.full((R, it), -1, dtype=np.int32)
    tt = np.zeros((R, it), dtype=dt)
    _fn("oracle_solve_batched", dt)(
        C.c_int64(m), C.c_int64(n), C.c_int32(D.size), C.c_int64(R), _p(X), C.c_int64(ldx),
        _p(B), _p(D), _p(scale), _p(k), C.c_int32(iters), C.c_int32(radius), _p(t), _p(done),
        _p(tj), _p(tk), _p(tt))
    return BatchedResult(D[k], t, done, tj, tk, tt)


# ------------------------------------------------------------------------------ ALNS outer loop
class AlnsParams(C.Structure):
    """Parameter block of the ALNS loop (Algorithm 1; Appendix F for alpha and the destroy rate)."""
    _fields_ = [("iters", C.c_int32), ("ls_moves", C.c_int32), ("ls_radius", C.c_int32),
                ("destroy_count", C.c_int32), ("alpha", C.c_double), ("lambda_", C.c_double),
                ("sigma1", C.c_double), ("sigma2", C.c_double), ("sigma3", C.c_double),
                ("seed", C.c_uint64), ("ls_swaps", C.c_int32), ("k_eps", C.c_int32),
                ("l2_guard", C.c_int32), ("reserved", C.c_int32)]


def alns_params(iters, ls_moves=8, ls_radius=1, destroy_count=0, alpha=0.3, lambda_=0.2,
                sigma1=3.0, sigma2=2.0, sigma3=1.0, seed=1, ls_swaps=0, k_eps=0, l2_guard=0) -> AlnsParams:
    return AlnsParams(int(iters), int(ls_moves), int(ls_radius), int(destroy_count), float(alpha),
                      float(lambda_), float(sigma1), float(sigma2), float(sigma3), int(seed),
                      int(ls_swaps), int(k_eps), int(l2_guard), 0)


@dataclass
class AlnsResult:
    x: np.ndarray            # best solution (values of D)
    t_best: float
    destroy: np.ndarray      # [iters] 0 random, 1 worst-remove
    repair: np.ndarray       # [iters] 0 random, 1 greedy
    moves: np.ndarray        # [iters] moves of the local search
    accepted: np.ndarray     # [iters]
    t: np.ndarray            # [iters] error after the local search
    best: np.ndarray         # [iters] best error so far
    weights: np.ndarray      # [4] final operator weights
    q2: Optional[np.ndarray] = None   # [iters] squared l2 norm of the residual after the local search


def alns_mix(z: int) -> int:
    lib().oracle_alns_mix.restype = C.c_uint64
    return int(lib().oracle_alns_mix(C.c_uint64(z & (2 ** 64 - 1))))


def alns_rnd(seed: int, inst: int, it: int, stream: int, c: int) -> int:
    lib().oracle_alns_rnd.restype = C.c_uint64
    return int(lib().oracle_alns_rnd(C.c_uint64(seed), C.c_uint64(inst), C.c_uint64(it),
                                     C.c_uint64(stream), C.c_uint64(c)))


def alns_expneg(y: float) -> float:
    lib().oracle_alns_expneg.restype = C.c_double
    return float(lib().oracle_alns_expneg(C.c_double(y)))


def full_csr(A):
    """A dense matrix as CSR with EVERY entry stored (zeros included), columns ascending."""
    A = np.asarray(A)
    m, n = A.shape
    rowptr = (np.arange(m + 1, dtype=np.int64) * n)
    col = np.tile(np.arange(n, dtype=np.int32), m)
    val = np.ascontiguousarray(A, dtype=A.dtype).reshape(-1).copy()
    return rowptr, col, val


def _csc_of(m, n, rowptr, col, val, dt):
    rowptr = np.ascontiguousarray(rowptr, dtype=np.int64)
    col = np.ascontiguousarray(col, dtype=np.int32)
    val = np.ascontiguousarray(val, dtype=dt)
    nnz = int(rowptr[m])
    colptr = np.empty(n + 1, dtype=np.int64)
    rowidx = np.empty(max(nnz, 1), dtype=np.int32)
    cval = np.empty(max(nnz, 1), dtype=dt)
    _fn("oracle_csr_to_csc", dt)(C.c_int64(m), C.c_int64(n), _p(rowptr), _p(col), _p(val),
                                 _p(colptr), _p(rowidx), _p(cval))
    return colptr, rowidx, cval


def alns_impact_weights(m, n, rowptr, col, val, r, alpha=0.3, scale=1.0) -> np.ndarray:
    dt = np.asarray(val).dtype
    rowptr = np.ascontiguousarray(rowptr, dtype=np.int64)
    col = np.ascontiguousarray(col, dtype=np.int32)
    val = np.ascontiguousarray(val)
    colptr, rowidx, cval = _csc_of(m, n, rowptr, col, val, dt)
    r = np.ascontiguousarray(r, dtype=dt)
    w = np.empty(max(n, 1), dtype=np.uint64)
    _fn("oracle_alns_impact_weights", dt)(C.c_int64(m), C.c_int64(n), _p(colptr), _p(rowidx), _p(cval),
                                          _real(dt)(scale), _p(r), C.c_double(alpha), _p(w))
    return w[:n]


def alns_sample(n, weight, count, seed, inst, it) -> np.ndarray:
    w = None if weight is None else np.ascontiguousarray(weight, dtype=np.uint64)
    picked = np.full(max(n, 1), -1, dtype=np.int32)
    lib().oracle_alns_sample(C.c_int64(n), _p(w), C.c_int64(count), C.c_uint64(seed), C.c_uint64(inst),
                             C.c_uint64(it), _p(picked))
    return picked[:min(count, n)]


def alns_repair(m, n, rowptr, col, val, D, x, r, picked, greedy, seed, inst, it, scale=1.0):
    """Returns (x, r) after reassigning the picked variables."""
    dt = np.asarray(D).dtype
    rowptr = np.ascontiguousarray(rowptr, dtype=np.int64)
    col = np.ascontiguousarray(col, dtype=np.int32)
    val = np.ascontiguousarray(val, dtype=dt)
    colptr, rowidx, cval = _csc_of(m, n, rowptr, col, val, dt)
    D = np.ascontiguousarray(D)
    k = values_to_index(x, D)
    r = np.ascontiguousarray(r, dtype=dt).copy()
    picked = np.ascontiguousarray(picked, dtype=np.int32)
    _fn("oracle_alns_repair", dt)(C.c_int64(m), C.c_int32(D.size), _p(colptr), _p(rowidx), _p(cval), _p(D),
                                  _real(dt)(scale), _p(k), _p(r), C.c_int64(picked.size), _p(picked),
                                  C.c_int32(int(greedy)), C.c_uint64(seed), C.c_uint64(inst), C.c_uint64(it))
    return D[k], r


def alns_csr(m, n, rowptr, col, val, b, D, x0, params: AlnsParams, inst=0, scale=1.0) -> AlnsResult:
    dt = np.asarray(D).dtype
    rowptr = np.ascontiguousarray(rowptr, dtype=np.int64)
    col = np.ascontiguousarray(col, dtype=np.int32)
    val = np.ascontiguousarray(val, dtype=dt)
    b = np.ascontiguousarray(b, dtype=dt)
    D = np.ascontiguousarray(D)
    k = values_to_index(x0, D)
    it = max(int(params.iters), 1)
    tr = [np.zeros(it, dtype=np.int32) for _ in range(4)]
    tr_t, tr_best = np.zeros(it, dtype=dt), np.zeros(it, dtype=dt)
    w = np.zeros(4, dtype=np.float64)
    tr_q2 = np.zeros(it, dtype=np.float64)
    f = _fn("oracle_alns", dt)
    f.restype = _real(dt)
    t_best = f(C.c_int64(m), C.c_int64(n), C.c_int32(D.size), _p(rowptr), _p(col), _p(val), _p(b), _p(D),
               _real(dt)(scale), _p(k), C.byref(params), C.c_uint64(inst), _p(tr[0]), _p(tr[1]), _p(tr[2]),
               _p(tr[3]), _p(tr_t), _p(tr_best), _p(w), _p(tr_q2))
    q = int(params.iters)
    return AlnsResult(D[k], float(t_best), tr[0][:q], tr[1][:q], tr[2][:q], tr[3][:q], tr_t[:q],
                      tr_best[:q], w, tr_q2[:q])


def sumsq(r) -> float:
    """Squared l2 norm in double precision, in the fixed order of the ALNS guard."""
    r = np.ascontiguousarray(r)
    f = _fn("oracle_sumsq", r.dtype)
    f.restype = C.c_double
    return float(f(C.c_int64(r.size), _p(r)))


def alns_dense(A, b, D, x0, params: AlnsParams, inst=0, scale=1.0) -> AlnsResult:
    """A dense matrix is the sparse case with every entry stored."""
    dt = np.asarray(D).dtype
    A = np.asarray(A, dtype=dt)
    rowptr, col, val = full_csr(A)
    return alns_csr(A.shape[0], A.shape[1], rowptr, col, val, b, D, x0, params, inst, scale)


# ------------------------------------------------------------------------------ swap move
def swap_table_csr(m, n, rowptr, col, val, D, x, r, scale=1.0, var_mask=None) -> np.ndarray:
    """t' of every ordered pair (i, j) with x_i > x_j, +inf elsewhere; shape [n, n]
    (Appendix B "Swap Move")."""
    dt = np.asarray(D).dtype
    D = np.ascontiguousarray(D)
    colptr, rowidx, cval = _csc_of(m, n, rowptr, col, val, dt)
    k = values_to_index(x, D)
    r = np.ascontiguousarray(r, dtype=dt)
    vm = _mask(var_mask, n)
    table = np.empty(n * n, dtype=dt)
    _fn("oracle_swap_table", dt)(C.c_int64(m), C.c_int64(n), _p(colptr), _p(rowidx), _p(cval), _p(D),
                                 _real(dt)(scale), _p(k), _p(r), _p(vm), _p(table))
    return table.reshape(n, n)


def best_swap_csr(m, n, rowptr, col, val, D, x, r, scale=1.0, var_mask=None):
    """Algorithm 2: (i, j, t') of the best strictly improving swap, or (-1, -1, t)."""
    dt = np.asarray(D).dtype
    D = np.ascontiguousarray(D)
    colptr, rowidx, cval = _csc_of(m, n, rowptr, col, val, dt)
    k = values_to_index(x, D)
    r = np.ascontiguousarray(r, dtype=dt)
    vm = _mask(var_mask, n)
    t_new = _real(dt)(0)
    f = _fn("oracle_best_swap", dt)
    f.restype = C.c_int64
    c = int(f(C.c_int64(m), C.c_int64(n), _p(colptr), _p(rowidx), _p(cval), _p(D), _real(dt)(scale),
              _p(k), _p(r), _p(vm), C.byref(t_new)))
    if c < 0:
        return -1, -1, dt.type(t_new.value)
    return c // n, c % n, dt.type(t_new.value)


def apply_swap_csr(m, n, rowptr, col, val, D, x, r, i, j, scale=1.0):
    """Exchange x_i and x_j; returns (x', r', t')."""
    dt = np.asarray(D).dtype
    D = np.ascontiguousarray(D)
    colptr, rowidx, cval = _csc_of(m, n, rowptr, col, val, dt)
    k = values_to_index(x, D)
    r = np.array(r, dtype=dt, copy=True)
    f = _fn("oracle_apply_swap", dt)
    f.restype = _real(dt)
    t = f(C.c_int64(m), _p(colptr), _p(rowidx), _p(cval), _p(D), _real(dt)(scale), _p(k), _p(r),
          C.c_int64(i), C.c_int64(j))
    return D[k], r, dt.type(t)


def swap_table_dense(A, D, x, r, scale=1.0, var_mask=None) -> np.ndarray:
    A = np.asarray(A, dtype=np.asarray(D).dtype)
    rowptr, col, val = full_csr(A)
    return swap_table_csr(A.shape[0], A.shape[1], rowptr, col, val, D, x, r, scale, var_mask)


def best_swap_dense(A, D, x, r, scale=1.0, var_mask=None):
    A = np.asarray(A, dtype=np.asarray(D).dtype)
    rowptr, col, val = full_csr(A)
    return best_swap_csr(A.shape[0], A.shape[1], rowptr, col, val, D, x, r, scale, var_mask)


def apply_swap_dense(A, D, x, r, i, j, scale=1.0):
    A = np.asarray(A, dtype=np.asarray(D).dtype)
    rowptr, col, val = full_csr(A)
    return apply_swap_csr(A.shape[0], A.shape[1], rowptr, col, val, D, x, r, i, j, scale)


# ------------------------------------------------------------------------------ l2 changes
def l2_column_sums(m, n, rowptr, col, val, r):
    """(g, c): g_j = a_j . r and c_j = ||a_j||^2, chains of fused multiply-adds by ascending row."""
    dt = np.asarray(val).dtype
    colptr, rowidx, cval = _csc_of(m, n, rowptr, col, val, dt)
    r = np.ascontiguousarray(r, dtype=dt)
    g = np.empty(max(n, 1), dtype=dt)
    c = np.empty(max(n, 1), dtype=dt)
    _fn("oracle_l2_column_sums", dt)(C.c_int64(n), _p(colptr), _p(rowidx), _p(cval), _p(r), _p(g), _p(c))
    return g[:n], c[:n]


def l2_changes_csr(m, n, rowptr, col, val, D, x, r, scale=1.0) -> np.ndarray:
    """dq[j*nd + k] = ||r + delta a_j||^2 - ||r||^2 for every single-coordinate move."""
    dt = np.asarray(D).dtype
    D = np.ascontiguousarray(D)
    colptr, rowidx, cval = _csc_of(m, n, rowptr, col, val, dt)
    k = values_to_index(x, D)
    r = np.ascontiguousarray(r, dtype=dt)
    dq = np.empty(max(n * D.size, 1), dtype=dt)
    _fn("oracle_l2_changes", dt)(C.c_int64(n), C.c_int32(D.size), _p(colptr), _p(rowidx), _p(cval), _p(D),
                                 _real(dt)(scale), _p(k), _p(r), _p(dq))
    return dq[:n * D.size]


def l2_changes_dense(A, D, x, r, scale=1.0) -> np.ndarray:
    A = np.asarray(A, dtype=np.asarray(D).dtype)
    rowptr, col, val = full_csr(A)
    return l2_changes_csr(A.shape[0], A.shape[1], rowptr, col, val, D, x, r, scale)


def argmin_move_l2(scores, dq, rule=1):
    """(flat index, score) of the best move: smallest score, then smallest dq, then lowest index;
    rule 2 considers only candidates with dq <= 0."""
    scores = np.ascontiguousarray(scores)
    dq = np.ascontiguousarray(dq, dtype=scores.dtype)
    c = C.c_int64(-1)
    s = _real(scores.dtype)(0)
    _fn("oracle_argmin_move_l2", scores.dtype)(C.c_int64(scores.size), _p(scores), _p(dq), C.c_int32(rule),
                                               C.byref(c), C.byref(s))
    return int(c.value), scores.dtype.type(s.value)


def solve_l2_csr(m, n, rowptr, col, val, b, D, x0, iters, rule=1, scale=1.0, radius=0) -> SolveResult:
    """The descent with the l2 change as second criterion (rule 1) or as a guard too (rule 2)."""
    dt = np.asarray(D).dtype
    rowptr = np.ascontiguousarray(rowptr, dtype=np.int64)
    col = np.ascontiguousarray(col, dtype=np.int32)
    val = np.ascontiguousarray(val, dtype=dt)
    b = np.ascontiguousarray(b, dtype=dt)
    D = np.ascontiguousarray(D)
    k = values_to_index(x0, D)
    it = max(int(iters), 1)
    tj, tk = np.full(it, -1, dtype=np.int32), np.full(it, -1, dtype=np.int32)
    tt = np.zeros(it, dtype=dt)
    t = _real(dt)(0)
    r = np.empty(max(m, 1), dtype=dt)
    f = _fn("oracle_solve_l2", dt)
    f.restype = C.c_int32
    done = int(f(C.c_int64(m), C.c_int64(n), C.c_int32(D.size), _p(rowptr), _p(col), _p(val), _p(b), _p(D),
                 _real(dt)(scale), _p(k), C.c_int32(iters), C.c_int32(radius), C.c_int32(rule), C.byref(t),
                 _p(r), _p(tj), _p(tk), _p(tt)))
    return SolveResult(D[k], dt.type(t.value), done, r[:m], tj[:done], tk[:done], tt[:done])


def solve_l2_dense(A, b, D, x0, iters, rule=1, scale=1.0, radius=0) -> SolveResult:
    A = np.asarray(A, dtype=np.asarray(D).dtype)
    rowptr, col, val = full_csr(A)
    return solve_l2_csr(A.shape[0], A.shape[1], rowptr, col, val, b, D, x0, iters, rule, scale, radius)
