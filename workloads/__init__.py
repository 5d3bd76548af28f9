"""Seeded synthetic DMMV instances shaped like the paper's three use cases.

This package only builds inputs (A, b, D, x0).  It contains none of the
method's arithmetic (no move scoring, arg-min or residual update) and is the
one piece of code that both the CPU oracle's tests and the HIP path's tests
and benchmark are allowed to share.
"""
from .configs import (  # noqa: F401
    Instance,
    make_config,
    dense_toy,
    fir_lowpass,
    tomography,
    llm_layer,
    random_dense,
    random_sparse,
    random_batched,
    CONFIG_NAMES,
)
