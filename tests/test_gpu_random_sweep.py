"""Seeded random sweep: shapes, dtypes, options and storage kinds drawn at random and pushed through
the same element-by-element checkers as the hand-picked cases (entry points step by step, whole
descents with their traces, the outer loop, the swap move), every result against the oracle, bitwise.
A configuration the library refuses by contract (an option that does not apply to the drawn shape)
must be refused with an error, never answered wrongly."""
import numpy as np
import pytest

import test_gpu_alns as ta
import test_gpu_parity as tp
import test_gpu_swap as ts
from workloads import random_batched, random_dense, random_sparse

pytestmark = pytest.mark.gpu


def attempt(name, fn):
    m = tp.dmmv()
    print("sweep case", name, flush=True)
    try:
        fn()
        return 1
    except m.DmmvError as e:
        assert e.status in (-8, -7, -5), (name, e)          # unsupported / state / workspace: contractual refusals
        return 0


def solve_check(inst, iters, **hopt):
    m = tp.dmmv()
    o = tp.oracle_solve(inst, iters, radius=hopt.get("radius", 0))
    with m.from_instance(inst, tp.DEV, **hopt) as h:
        res = m.dmmv_solve(h, tp.T(inst.x0), iters, trace=True)
        tp.check_single_trace(res, o, iters)


@pytest.mark.parametrize("seed", [11, 12])
def test_random_sweep_of_the_descent(seed):
    rng = np.random.default_rng(seed)
    ran = 0
    for _ in range(60):
        kind = int(rng.integers(0, 3))
        s = int(rng.integers(1, 1 << 30))
        dt = [np.float32, np.float64][int(rng.integers(0, 2))]
        integer = bool(rng.integers(0, 2))
        if kind == 0:
            mm, nn = int(rng.integers(1, 700)), int(rng.integers(1, 60))
            nd = int(rng.integers(2, 13 if integer else 40))
            radius = int(rng.choice([0, 0, 1, 2]))
            inst = random_dense(s, mm, nn, nd, dtype=dt, integer=integer)
            tag = f"dense {mm}x{nn} nd{nd} {dt.__name__} integer={integer} radius={radius}"
            ran += attempt(tag + " stepwise", lambda: tp.stepwise_check(inst, steps=3, radius=radius))
            for opts in ({}, {"dense_loop": 2}, {"dense_loop": 1}, {"prune": 1}, {"value_search": 1}):
                ran += attempt(f"{tag} solve {opts}", lambda: solve_check(inst, 25, radius=radius, **opts))
        elif kind == 1:
            mm, nn = int(rng.integers(1, 4000)), int(rng.integers(1, 300))
            nd = int(rng.integers(2, 9))
            dens = float(rng.choice([0.005, 0.02, 0.1, 0.5, 1.0]))
            dens = min(dens, 4e5 / (mm * nn))
            opt = {}
            part, mode = int(rng.choice([0, 0, 16, 100, 1000])), int(rng.choice([0, 1, 2]))
            if part:
                opt["sparse_partition_rows"] = part
            if mode:
                opt["sparse_eval"] = mode
            radius = int(rng.choice([0, 0, 1]))
            inst = random_sparse(s, mm, nn, nd, density=dens, dtype=dt, integer=integer,
                                 explicit_zeros=bool(rng.integers(0, 2)))
            tag = f"sparse {mm}x{nn} nd{nd} density={dens:.3f} {dt.__name__} integer={integer} {opt} radius={radius}"
            ran += attempt(tag + " stepwise", lambda: tp.stepwise_check(inst, steps=3, radius=radius, **dict(opt)))
            for extra in ({}, {"prune": 1}):
                ran += attempt(f"{tag} solve {extra}", lambda: solve_check(inst, 25, radius=radius, **opt, **extra))
        else:
            mm, nn, R = int(rng.integers(1, 200)), int(rng.integers(1, 90)), int(rng.integers(1, 300))
            nd = int(rng.integers(2, 13 if integer else 17))
            dtb = np.float32 if rng.integers(0, 4) else np.float64
            radius = int(rng.choice([0, 0, 1]))
            inst = random_batched(s, mm, nn, R, nd, dtype=dtb, integer=integer)
            for opts in ({}, {"prune": 1}, {"batched_eval": 2}, {"poll_every": 3}):
                if opts.get("batched_eval") and dtb != np.float32:
                    continue
                ran += attempt(f"batched {mm}x{nn} R={R} nd{nd} {dtb.__name__} integer={integer} radius={radius} {opts}",
                               lambda: tp.batched_check(inst, 12, radius=radius, **opts))
    assert ran >= 150          # refusals are the exception


@pytest.mark.parametrize("seed", [21])
def test_random_sweep_of_the_outer_loop_and_the_swap_move(seed):
    rng = np.random.default_rng(seed)
    ran = 0
    for _ in range(45):
        kind = int(rng.integers(0, 3))
        s = int(rng.integers(1, 1 << 30))
        dt = [np.float32, np.float64][int(rng.integers(0, 2))]
        integer = bool(rng.integers(0, 3) == 0)
        aseed = int(rng.integers(1, 1000))
        if kind == 0:
            mm, nn = int(rng.integers(1, 500)), int(rng.integers(1, 80))
            nd = int(rng.integers(2, 13 if integer else 20))
            inst = random_dense(s, mm, nn, nd, dtype=dt, integer=integer)
            kw = dict(ls_moves=int(rng.integers(1, 6)), destroy_count=int(rng.integers(1, max(2, nn // 4 + 1))), seed=aseed)
            if rng.integers(0, 2):
                kw["ls_swaps"] = int(rng.integers(1, 3))
            if rng.integers(0, 3) == 0:
                kw["l2_guard"] = 1
            if rng.integers(0, 3) == 0:
                kw["prune"] = 1
            k_eps, descend = int(rng.choice([0, 3, 100])), int(rng.integers(0, 8))
            ran += attempt(f"outer loop dense {kw}", lambda: ta.alns_check(inst, 12, **kw))
            ran += attempt("swap dense", lambda: ts.chain_check(inst, 4, k_eps=k_eps, descend=descend))
        elif kind == 1:
            mm, nn = int(rng.integers(1, 3000)), int(rng.integers(1, 200))
            nd = int(rng.integers(2, 7))
            dens = min(float(rng.choice([0.01, 0.05, 0.2, 0.6])), 2e5 / (mm * nn))
            inst = random_sparse(s, mm, nn, nd, density=dens, dtype=dt, integer=integer)
            kw = dict(ls_moves=int(rng.integers(1, 5)), destroy_count=int(rng.integers(1, max(2, nn // 5 + 1))), seed=aseed)
            if rng.integers(0, 3) == 0:
                kw["ls_swaps"] = 1
            if rng.integers(0, 3) == 0:
                kw["prune"] = 1
            part = int(rng.choice([0, 0, 64, 500]))
            if part:
                kw["sparse_partition_rows"] = part
            descend = int(rng.integers(0, 6))
            ran += attempt(f"outer loop sparse {kw}", lambda: ta.alns_check(inst, 10, **kw))
            if nn <= 120:
                ran += attempt("swap sparse", lambda: ts.chain_check(inst, 3, descend=descend))
        else:
            mm, nn, R = int(rng.integers(1, 120)), int(rng.integers(1, 60)), int(rng.integers(1, 70))
            nd = int(rng.integers(2, 13 if integer else 17))
            inst = random_batched(s, mm, nn, R, nd, integer=integer)
            kw = dict(ls_moves=int(rng.integers(1, 4)), destroy_count=int(rng.integers(1, max(2, nn // 4 + 1))), seed=aseed)
            if rng.integers(0, 3) == 0:
                kw["ls_swaps"] = 1
            if rng.integers(0, 3) == 0:
                kw["prune"] = 1
            descend = int(rng.integers(0, 5))
            ran += attempt(f"outer loop batched {kw}", lambda: ta.batched_alns_check(inst, 6, **kw))
            ran += attempt("swap batched", lambda: ts.chain_check(inst, 2, descend=descend))
    assert ran >= 60


@pytest.mark.parametrize("seed", [31])
def test_random_sweep_of_the_l2_changes_and_the_matrix_core_residual(seed):
    import test_gpu_l2 as tl

    rng = np.random.default_rng(seed)
    ran = 0
    for _ in range(90):
        kind = int(rng.integers(0, 3))
        s = int(rng.integers(1, 1 << 30))
        dt = [np.float32, np.float64][int(rng.integers(0, 2))]
        integer = bool(rng.integers(0, 2))
        rule = int(rng.choice([1, 2]))
        if kind == 0:
            mm, nn = int(rng.integers(1, 600)), int(rng.integers(1, 60))
            nd = int(rng.integers(2, 13 if integer else 30))
            radius = int(rng.choice([0, 1]))
            inst = random_dense(s, mm, nn, nd, dtype=dt, integer=integer)
            ran += attempt(f"l2 tables dense {mm}x{nn} nd{nd} {dt.__name__} integer={integer}", lambda: tl.check_tables(inst))
            ran += attempt(f"l2 descent dense rule {rule} radius {radius}", lambda: tl.check_descent(inst, 20, rule, radius=radius))
        elif kind == 1:
            mm, nn = int(rng.integers(1, 3000)), int(rng.integers(1, 200))
            nd = int(rng.integers(2, 7))
            dens = min(float(rng.choice([0.01, 0.05, 0.2, 0.6])), 2e5 / (mm * nn))
            inst = random_sparse(s, mm, nn, nd, density=dens, dtype=dt, integer=integer)
            opt = {}
            part = int(rng.choice([0, 0, 64, 500]))
            if part:
                opt["sparse_partition_rows"] = part
            ran += attempt(f"l2 tables sparse {mm}x{nn} nd{nd} density={dens:.3f} {dt.__name__} integer={integer}",
                           lambda: tl.check_tables(inst))
            ran += attempt(f"l2 descent sparse rule {rule} {opt}", lambda: tl.check_descent(inst, 20, rule, **opt))
        else:
            mm, nn, R = int(rng.integers(1, 300)), int(rng.integers(1, 200)), int(rng.integers(1, 150))
            nd = int(rng.integers(2, 13 if integer else 17))
            dtb = np.float32 if rng.integers(0, 4) else np.float64
            inst = random_batched(s, mm, nn, R, nd, dtype=dtb, integer=integer)
            ran += attempt(f"l2 tables batched {mm}x{nn} R={R} nd{nd} {dtb.__name__} integer={integer}",
                           lambda: tl.check_tables(inst, steps=1))
            if mm * nn * R < 4e5:
                ran += attempt(f"l2 descent batched rule {rule}", lambda: tl.check_descent(inst, 8, rule))
            if dtb == np.float32:
                ran += attempt(f"matrix-core residual {mm}x{nn} R={R}", lambda: tp.mfma_residual_check(inst))
    assert ran >= 150
