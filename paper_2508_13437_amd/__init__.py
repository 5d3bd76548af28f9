"""MI355X (gfx950) hot path of the AMVM heuristic for Discrete Min-Max Violation.

`paper_2508_13437_amd.dmmv` is the ctypes binding of libdmmv.so (HIP kernels + C ABI under
csrc/); `paper_2508_13437_amd.build` compiles it.
"""
from . import dmmv  # noqa: F401
from .dmmv import (  # noqa: F401
    DmmvError, Handle, SolveResult, dmmv_apply_move, dmmv_argmin_move, dmmv_create,
    dmmv_destroy, dmmv_eval_moves, dmmv_get_state, dmmv_get_x, dmmv_residual, dmmv_set_residual,
    dmmv_set_x, dmmv_solve, dmmv_time_eval, dmmv_version, from_instance, load, solve,
)
