"""ctypes binding of libdmmv.so: argument marshalling only.

Every step (residual, move scoring, arg-min, residual update, the descent loop, layout
conversions) runs in the library's HIP kernels.  PyTorch is used to own device memory and to
supply the HIP stream.  There is no CPU fallback: loading fails loudly when the library has
not been built (``python -m paper_2508_13437_amd.build``).
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import Optional, Sequence

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libdmmv.so")

DMMV_F32, DMMV_F64 = 0, 1
DMMV_OK = 0
STATUS_NAMES = {0: "DMMV_OK", -1: "DMMV_ERR_NULL", -2: "DMMV_ERR_SHAPE", -3: "DMMV_ERR_DTYPE",
                -4: "DMMV_ERR_DOMAIN", -5: "DMMV_ERR_WORKSPACE", -6: "DMMV_ERR_HIP",
                -7: "DMMV_ERR_STATE", -8: "DMMV_ERR_UNSUPPORTED"}

EXPORTS = ("dmmv_workspace_bytes", "dmmv_create", "dmmv_destroy", "dmmv_set_x",
           "dmmv_set_residual", "dmmv_residual", "dmmv_eval_moves", "dmmv_argmin_move",
           "dmmv_apply_move", "dmmv_get_state", "dmmv_solve", "dmmv_solve_static", "dmmv_alns", "dmmv_swap_move",
           "dmmv_l2_changes",
           "dmmv_time_eval", "dmmv_time_l2", "dmmv_loop_in_use",
           "dmmv_last_error",
           "dmmv_version")


class DmmvError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"{STATUS_NAMES.get(status, status)}: {message}")
        self.status = status


class Problem(C.Structure):
    _fields_ = [("dtype", C.c_int32), ("nd", C.c_int32), ("m", C.c_int64), ("n", C.c_int64),
                ("D", C.c_void_p), ("A_dense", C.c_void_p), ("lda", C.c_int64),
                ("csr_rowptr", C.c_void_p), ("csr_col", C.c_void_p), ("csr_val", C.c_void_p),
                ("nnz", C.c_int64), ("b", C.c_void_p), ("R", C.c_int64), ("scale", C.c_void_p)]


class Options(C.Structure):
    _fields_ = [("radius", C.c_int32), ("keep_going", C.c_int32), ("poll_every", C.c_int32),
                ("sparse_partition_rows", C.c_int32), ("var_mask", C.c_void_p),
                ("residual_mfma", C.c_int32), ("prune", C.c_int32), ("alns", C.c_int32),
                ("value_search", C.c_int32), ("batched_eval", C.c_int32), ("sparse_eval", C.c_int32),
                ("l2_rule", C.c_int32), ("dense_loop", C.c_int32), ("wait_limit", C.c_int32)]


class AlnsParams(C.Structure):
    _fields_ = [("iters", C.c_int32), ("ls_moves", C.c_int32), ("ls_radius", C.c_int32),
                ("destroy_count", C.c_int32), ("alpha", C.c_double), ("lambda_", C.c_double),
                ("sigma1", C.c_double), ("sigma2", C.c_double), ("sigma3", C.c_double),
                ("seed", C.c_uint64), ("ls_swaps", C.c_int32), ("k_eps", C.c_int32),
                ("l2_guard", C.c_int32), ("reserved", C.c_int32)]


_lib = None


def load() -> C.CDLL:
    """Load libdmmv.so (built in-tree).  Raises if it is missing: there is no fallback."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} not found: build it with "
                           "`python -m paper_2508_13437_amd.build` (needs hipcc)")
    lib = C.CDLL(LIB_PATH)
    lib.dmmv_workspace_bytes.restype = C.c_size_t
    lib.dmmv_workspace_bytes.argtypes = [C.POINTER(Problem), C.POINTER(Options)]
    lib.dmmv_create.restype = C.c_int
    lib.dmmv_create.argtypes = [C.POINTER(C.c_void_p), C.POINTER(Problem), C.POINTER(Options),
                                C.c_void_p, C.c_size_t, C.c_void_p]
    lib.dmmv_destroy.restype = C.c_int
    lib.dmmv_destroy.argtypes = [C.c_void_p]
    for name, nargs in (("dmmv_set_x", 2), ("dmmv_set_residual", 2), ("dmmv_residual", 2),
                        ("dmmv_eval_moves", 2), ("dmmv_argmin_move", 4), ("dmmv_apply_move", 2),
                        ("dmmv_get_state", 4), ("dmmv_l2_changes", 2)):
        fn = getattr(lib, name)
        fn.restype = C.c_int
        fn.argtypes = [C.c_void_p] * nargs
    lib.dmmv_solve.restype = C.c_int
    lib.dmmv_solve.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p,
                               C.c_void_p, C.c_void_p, C.c_void_p]
    lib.dmmv_solve_static.restype = C.c_int
    lib.dmmv_solve_static.argtypes = [C.POINTER(Problem), C.POINTER(Options), C.c_void_p, C.c_int32, C.c_void_p,
                                      C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
    lib.dmmv_alns.restype = C.c_int
    lib.dmmv_alns.argtypes = [C.c_void_p, C.c_void_p, C.POINTER(AlnsParams), C.c_void_p, C.c_void_p,
                              C.c_void_p, C.c_void_p]
    lib.dmmv_swap_move.restype = C.c_int
    lib.dmmv_swap_move.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p]
    lib.dmmv_loop_in_use.restype = C.c_int32
    lib.dmmv_loop_in_use.argtypes = [C.c_void_p]
    lib.dmmv_time_eval.restype = C.c_int
    lib.dmmv_time_eval.argtypes = [C.c_void_p, C.c_int32, C.POINTER(C.c_float)]
    lib.dmmv_time_l2.restype = C.c_int
    lib.dmmv_time_l2.argtypes = [C.c_void_p, C.c_int32, C.POINTER(C.c_float)]
    lib.dmmv_last_error.restype = C.c_char_p
    lib.dmmv_version.restype = C.c_char_p
    _lib = lib
    return lib


def _check(status: int):
    if status != DMMV_OK:
        raise DmmvError(status, load().dmmv_last_error().decode())


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else C.c_void_p(t.data_ptr())


def _np_dtype(dtype: torch.dtype):
    if dtype == torch.float32:
        return np.float32
    if dtype == torch.float64:
        return np.float64
    raise DmmvError(-3, f"unsupported dtype {dtype}")


@dataclass
class SolveResult:
    x: torch.Tensor            # [R][n] (or [n]) values of D
    max_violation: torch.Tensor  # [R]
    iters_done: torch.Tensor   # [R] int32, moves applied
    trace: Optional[torch.Tensor]    # [R][iters][2] int32 (j, k), -1 past the end
    trace_t: Optional[torch.Tensor]  # [R][iters]


class Handle:
    """Owns the library handle, its workspace and references to the borrowed tensors."""

    def __init__(self, *, D, b, A=None, csr=None, m=None, n=None, scale=None, radius: int = 0,
                 keep_going: bool = False, poll_every: int = 64, var_mask=None,
                 sparse_partition_rows: int = 0, residual_mfma: bool = False, prune: bool = False,
                 alns: bool = False, value_search: bool = False, batched_eval: int = 0, sparse_eval: int = 0,
                 l2_rule: int = 0, dense_loop: int = 0, wait_limit: int = 0,
                 stream: Optional[torch.cuda.Stream] = None, device=None, _create: bool = True):
        lib = load()
        self._h = C.c_void_p(None)
        dev = torch.device(device) if device is not None else (
            A.device if A is not None else csr[2].device)
        if dev.type != "cuda":
            raise DmmvError(-6, "tensors must live on the GPU")
        self.device = dev
        b = b.contiguous()
        self.dtype = b.dtype
        npdt = _np_dtype(self.dtype)
        self._D_host = np.ascontiguousarray(np.asarray(D, dtype=npdt))
        self.nd = int(self._D_host.shape[0])
        self._scale_host = None if scale is None else np.ascontiguousarray(np.asarray(scale, dtype=npdt))
        self.batched = scale is not None
        self.R = int(self._scale_host.shape[0]) if self.batched else 1
        p = Problem()
        p.dtype = DMMV_F64 if self.dtype == torch.float64 else DMMV_F32
        p.nd = self.nd
        p.D = self._D_host.ctypes.data_as(C.c_void_p)
        if A is not None:
            if A.dtype != self.dtype:
                raise DmmvError(-3, "A and b differ in dtype")
            if A.dim() != 2:
                raise DmmvError(-2, "A must be 2-D")
            if A.numel() > 0 and A.stride(0) != 1:
                A = A.t().contiguous().t()          # column-major copy
            self.m, self.n = int(A.shape[0]), int(A.shape[1])
            p.A_dense = A.data_ptr()
            p.lda = int(A.stride(1)) if (A.shape[1] > 1 and A.numel() > 0) else max(self.m, 1)
            self._A = A
        else:
            rowptr, col, val = csr
            rowptr = rowptr.to(torch.int64).contiguous()
            col = col.to(torch.int32).contiguous()
            val = val.contiguous()
            if val.dtype != self.dtype:
                raise DmmvError(-3, "csr values and b differ in dtype")
            self.m, self.n = int(m), int(n)
            p.csr_rowptr, p.csr_col, p.csr_val = rowptr.data_ptr(), col.data_ptr(), val.data_ptr()
            p.nnz = int(val.numel())
            self._csr = (rowptr, col, val)
        p.m, p.n = self.m, self.n
        if b.numel() != self.R * self.m:
            raise DmmvError(-2, f"b has {b.numel()} elements, expected R*m = {self.R * self.m}")
        p.b = b.data_ptr()
        self._b = b
        p.R = self.R
        p.scale = None if self._scale_host is None else self._scale_host.ctypes.data_as(C.c_void_p)
        o = Options()
        o.radius, o.keep_going, o.poll_every = int(radius), int(bool(keep_going)), int(poll_every)
        o.sparse_partition_rows = int(sparse_partition_rows)
        o.residual_mfma = int(bool(residual_mfma))
        o.prune = int(bool(prune))
        o.alns = int(bool(alns))
        o.batched_eval = int(batched_eval)
        o.sparse_eval = int(sparse_eval)
        o.l2_rule = int(l2_rule)
        o.dense_loop = int(dense_loop)
        o.wait_limit = int(wait_limit)
        o.value_search = int(bool(value_search))
        if var_mask is not None:
            var_mask = var_mask.to(torch.uint8).contiguous()
            if var_mask.numel() != self.R * self.n:
                raise DmmvError(-2, "var_mask must have R*n entries")
            o.var_mask = var_mask.data_ptr()
        self._var_mask = var_mask
        self._problem, self._options = p, o
        self.stream = stream if stream is not None else torch.cuda.current_stream(dev)
        if not _create:        # marshalled description only (dmmv_solve_static)
            return
        nbytes = lib.dmmv_workspace_bytes(C.byref(p), C.byref(o))
        if nbytes == 0:       # invalid problem: let dmmv_create name the status
            _check(lib.dmmv_create(C.byref(self._h), C.byref(p), C.byref(o), None, 0, None))
            raise DmmvError(-2, lib.dmmv_last_error().decode())
        self.workspace_bytes = int(nbytes)
        self._ws = torch.empty(self.workspace_bytes + 256, dtype=torch.uint8, device=dev)
        off = (-self._ws.data_ptr()) % 256
        with torch.cuda.device(dev):
            _check(lib.dmmv_create(C.byref(self._h), C.byref(p), C.byref(o),
                                   C.c_void_p(self._ws.data_ptr() + off), C.c_size_t(nbytes),
                                   C.c_void_p(self.stream.cuda_stream)))

    # -- lifetime ---------------------------------------------------------------------------
    def close(self):
        if getattr(self, "_h", None) is not None and self._h.value:
            load().dmmv_destroy(self._h)
            self._h = C.c_void_p(None)

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.close()

    # -- helpers ----------------------------------------------------------------------------
    def _new(self, *shape, dtype=None):
        return torch.empty(*shape, dtype=dtype or self.dtype, device=self.device)

    def _xshape(self):
        return (self.R, self.n) if self.batched else (self.n,)

    def _rshape(self):
        return (self.R, self.m) if self.batched else (self.m,)


def _arg(h: "Handle", t: torch.Tensor, dtype) -> torch.Tensor:
    """An input tensor in the layout the C call expects.  The call only enqueues work on the
    handle's stream; a converted temporary is therefore tied to that stream, so that the caching
    allocator does not hand its memory to another tensor before the work has run."""
    c = t.to(h.device, dtype).contiguous()
    if c.is_cuda:
        c.record_stream(h.stream)
    return c


# ---- the C entry points, same names -----------------------------------------------------------
def dmmv_create(**kw) -> Handle:
    return Handle(**kw)


def dmmv_destroy(h: Handle):
    h.close()


def dmmv_set_x(h: Handle, x: torch.Tensor):
    x = _arg(h, x, h.dtype)
    if x.numel() != h.R * h.n:
        raise DmmvError(-2, "x must have R*n entries")
    _check(load().dmmv_set_x(h._h, _ptr(x)))


def dmmv_set_residual(h: Handle, r: torch.Tensor):
    r = _arg(h, r, h.dtype)
    if r.numel() != h.R * h.m:
        raise DmmvError(-2, "r must have R*m entries")
    _check(load().dmmv_set_residual(h._h, _ptr(r)))


def dmmv_residual(h: Handle) -> torch.Tensor:
    r = h._new(h._rshape())
    _check(load().dmmv_residual(h._h, _ptr(r)))
    return r


def dmmv_eval_moves(h: Handle) -> torch.Tensor:
    shape = (h.R, h.n * h.nd) if h.batched else (h.n * h.nd,)
    scores = h._new(shape)
    _check(load().dmmv_eval_moves(h._h, _ptr(scores)))
    return scores


def dmmv_l2_changes(h: Handle) -> torch.Tensor:
    """Change of the squared l2 norm of the residual under every move, [R][n*nd] (handles created
    with l2_rule != 0)."""
    shape = (h.R, h.n * h.nd) if h.batched else (h.n * h.nd,)
    dq = h._new(shape)
    _check(load().dmmv_l2_changes(h._h, _ptr(dq)))
    return dq


def dmmv_argmin_move(h: Handle, scores: Optional[torch.Tensor] = None):
    """Returns (moves [R][2] int32 = (j, k), best_score [R])."""
    if scores is not None:
        scores = _arg(h, scores, h.dtype)
        if scores.numel() != h.R * h.n * h.nd:
            raise DmmvError(-2, "scores must have R*n*nd entries")
    best = h._new((h.R, 2), dtype=torch.int32)
    best_s = h._new((h.R,))
    _check(load().dmmv_argmin_move(h._h, _ptr(scores), _ptr(best), _ptr(best_s)))
    return best, best_s


def dmmv_apply_move(h: Handle, moves: torch.Tensor):
    moves = _arg(h, moves, torch.int32)
    if moves.numel() != 2 * h.R:
        raise DmmvError(-2, "moves must be [R][2] (j, k)")
    _check(load().dmmv_apply_move(h._h, _ptr(moves)))


def dmmv_get_state(h: Handle):
    """Returns (x, r, max_violation)."""
    x = h._new(h._xshape())
    r = h._new(h._rshape())
    t = h._new((h.R,))
    _check(load().dmmv_get_state(h._h, _ptr(x), _ptr(r), _ptr(t)))
    return x, r, t


def dmmv_get_x(h: Handle) -> torch.Tensor:
    x = h._new(h._xshape())
    _check(load().dmmv_get_state(h._h, _ptr(x), None, None))
    return x


def dmmv_solve(h: Handle, x0: Optional[torch.Tensor], iters: int, trace: bool = False) -> SolveResult:
    if x0 is not None:
        x0 = _arg(h, x0, h.dtype)
        if x0.numel() != h.R * h.n:
            raise DmmvError(-2, "x0 must have R*n entries")
    x = h._new(h._xshape())
    t = h._new((h.R,))
    done = h._new((h.R,), dtype=torch.int32)
    tr = h._new((h.R, max(iters, 1), 2), dtype=torch.int32) if trace else None
    tt = h._new((h.R, max(iters, 1))) if trace else None
    _check(load().dmmv_solve(h._h, _ptr(x0), C.c_int32(iters), _ptr(x), _ptr(t), _ptr(done),
                             _ptr(tr), _ptr(tt)))
    if trace and iters == 0:
        tr, tt = tr[:, :0], tt[:, :0]
    return SolveResult(x, t, done, tr, tt)


STATIC_SCRATCH_BYTES = 16 << 20


def dmmv_solve_static(x0: torch.Tensor, iters: int, trace: bool = False, **problem_and_options) -> SolveResult:
    """dmmv_create + dmmv_solve + dmmv_destroy in one C call that allocates nothing: the library's
    built-in scratch array is the workspace (problems that need more are refused).  Keyword
    arguments as for Handle (D, b, A or csr/m/n, scale, options)."""
    d = Handle(_create=False, **problem_and_options)       # argument marshalling only
    x0 = _arg(d, x0, d.dtype)
    if x0.numel() != d.R * d.n:
        raise DmmvError(-2, "x0 must have R*n entries")
    x = d._new(d._xshape())
    t = d._new((d.R,))
    done = d._new((d.R,), dtype=torch.int32)
    tr = d._new((d.R, max(iters, 1), 2), dtype=torch.int32) if trace else None
    tt = d._new((d.R, max(iters, 1))) if trace else None
    with torch.cuda.device(d.device):
        _check(load().dmmv_solve_static(C.byref(d._problem), C.byref(d._options), _ptr(x0), C.c_int32(iters),
                                        _ptr(x), _ptr(t), _ptr(done), _ptr(tr), _ptr(tt),
                                        C.c_void_p(d.stream.cuda_stream)))
    if trace and iters == 0:
        tr, tt = tr[:, :0], tt[:, :0]
    return SolveResult(x, t, done, tr, tt)


@dataclass
class AlnsResult:
    x_best: torch.Tensor       # [n] ([R][n] batched)
    t_best: torch.Tensor       # [1] ([R])
    trace: torch.Tensor        # [iters][4] int32: destroy op, repair op, local-search moves, accepted
    trace_t: torch.Tensor      # [iters][2]: error after the local search, best error so far
                               # (both with a leading [R] for batched handles)


def dmmv_alns(h: Handle, x0: Optional[torch.Tensor], iters: int, ls_moves: int = 8, ls_radius: int = 1,
              destroy_count: int = 0, alpha: float = 0.3, lambda_: float = 0.2, sigma1: float = 3.0,
              sigma2: float = 2.0, sigma3: float = 1.0, seed: int = 1, ls_swaps: int = 0,
              k_eps: int = 0, l2_guard: bool = False) -> AlnsResult:
    """The ALNS outer loop around the descent (and, with ls_swaps, the swap move)."""
    prm = AlnsParams(int(iters), int(ls_moves), int(ls_radius), int(destroy_count), float(alpha),
                     float(lambda_), float(sigma1), float(sigma2), float(sigma3), int(seed),
                     int(ls_swaps), int(k_eps), 1 if l2_guard else 0, 0)
    if x0 is not None:
        x0 = _arg(h, x0, h.dtype)
    x_best = h._new(h._xshape())
    t_best = h._new((h.R,))
    trace = torch.full((h.R, max(iters, 1), 4), -1, dtype=torch.int32, device=h.device)
    trace_t = h._new((h.R, max(iters, 1), 2))
    _check(load().dmmv_alns(h._h, _ptr(x0), C.byref(prm), _ptr(x_best), _ptr(t_best), _ptr(trace),
                            _ptr(trace_t)))
    if not h.batched:
        return AlnsResult(x_best, t_best, trace[0, :iters], trace_t[0, :iters])
    return AlnsResult(x_best, t_best, trace[:, :iters], trace_t[:, :iters])


@dataclass
class SwapResult:
    i: torch.Tensor          # [R] int64, -1 = no improving swap
    j: torch.Tensor          # [R] int64
    t: torch.Tensor          # [R] error after the swap (the current error when there is none)


def dmmv_swap_move(h: Handle, k_eps: int = 0, apply: bool = True) -> SwapResult:
    """Best strictly improving exchange of two variables' values (Algorithm 2)."""
    best = torch.empty((h.R, 2), dtype=torch.int64, device=h.device)
    best_t = h._new((h.R,))
    _check(load().dmmv_swap_move(h._h, C.c_int32(int(k_eps)), C.c_int32(1 if apply else 0), _ptr(best),
                                 _ptr(best_t)))
    return SwapResult(best[:, 0], best[:, 1], best_t)


def dmmv_loop_in_use(h: Handle) -> int:
    return int(load().dmmv_loop_in_use(h._h))


def dmmv_time_eval(h: Handle, reps: int) -> float:
    """Milliseconds for `reps` back-to-back launches of the fused evaluation kernel."""
    ms = C.c_float(0.0)
    _check(load().dmmv_time_eval(h._h, C.c_int32(reps), C.byref(ms)))
    return float(ms.value)


def dmmv_time_l2(h: Handle, reps: int) -> float:
    """Milliseconds for `reps` back-to-back launches of the contraction g = A^T r (l2 changes)."""
    ms = C.c_float(0.0)
    _check(load().dmmv_time_l2(h._h, C.c_int32(reps), C.byref(ms)))
    return float(ms.value)


def dmmv_version() -> str:
    return load().dmmv_version().decode()


# ---- one-shot convenience: (A, b, D, x0, iters) -> (x, max violation) --------------------------
def solve(A: torch.Tensor, b: torch.Tensor, D: Sequence[float], x0: torch.Tensor, iters: int,
          **options):
    with Handle(A=A, b=b, D=D, **options) as h:
        res = dmmv_solve(h, x0, iters)
        return res.x, res.max_violation


def from_instance(inst, device="cuda:0", **options) -> Handle:
    """Upload a workloads.Instance and create a handle for it."""
    dev = torch.device(device)
    b = torch.from_numpy(np.ascontiguousarray(inst.b)).to(dev)
    if inst.kind == "csr":
        csr = (torch.from_numpy(inst.csr_rowptr).to(dev), torch.from_numpy(inst.csr_col).to(dev),
               torch.from_numpy(inst.csr_val).to(dev))
        return Handle(D=inst.D, b=b, csr=csr, m=inst.m, n=inst.n, device=dev, **options)
    A = torch.from_numpy(np.ascontiguousarray(inst.A.T)).to(dev).t()    # column-major view
    scale = inst.scale if inst.kind == "batched" else None
    return Handle(D=inst.D, b=b, A=A, scale=scale, device=dev, **options)
