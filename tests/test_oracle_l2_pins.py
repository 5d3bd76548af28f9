"""Pins of the l2 part of the CPU oracle (change of the squared l2 norm of the residual per
candidate move, and its use as second criterion of the arg-min) against facts that do not come
from the oracle: fresh recomputation of ||A x' - b||^2 on integer data (exact), numpy on real
data, and brute force over tables with constructed ties."""
import itertools

import numpy as np
import pytest

from oracle import oracle as orc
from workloads import random_batched, random_dense, random_sparse


def fresh_tables(A, b, D, x, s=1.0, radius=0):
    """(scores, dq) straight from the definitions, in fp64: for every single-coordinate change x'
    of x the error max |s A x' - b| and the change of the squared l2 norm."""
    A = np.asarray(A, dtype=np.float64) * s
    b = np.asarray(b, dtype=np.float64)
    D = np.asarray(D, dtype=np.float64)
    x = np.asarray(x, dtype=np.float64)
    n, nd = A.shape[1], D.size
    r0 = A @ x - b
    q0 = float(r0 @ r0)
    scores = np.full(n * nd, np.inf)
    dq = np.zeros(n * nd)
    for j in range(n):
        kc = int(np.searchsorted(D, x[j]))
        for k in range(nd):
            y = x.copy(); y[j] = D[k]
            r1 = A @ y - b
            dq[j * nd + k] = float(r1 @ r1) - q0
            if k == kc or radius == 0 or abs(k - kc) <= radius:
                scores[j * nd + k] = np.abs(r1).max()
    return scores, dq


@pytest.mark.parametrize("dtype", [np.float64, np.float32])
@pytest.mark.parametrize("seed", range(3))
def test_l2_changes_equal_the_fresh_difference_of_squared_norms_on_integer_data(seed, dtype):
    inst = random_dense(800 + seed, 17, 7, 5, dtype=dtype, integer=True)
    r = orc.residual_dense(inst.A, inst.b, inst.D, inst.x0)
    got = orc.l2_changes_dense(inst.A, inst.D, inst.x0, r)
    _, want = fresh_tables(inst.A, inst.b, inst.D, inst.x0)
    assert np.array_equal(got.astype(np.float64), want)              # every operation is exact
    nd = inst.nd
    kc = np.searchsorted(inst.D, inst.x0)
    assert np.all(got[np.arange(inst.n) * nd + kc] == 0)              # null moves change nothing
    assert np.any(got < 0) and np.any(got > 0)


def test_l2_column_sums_against_numpy_and_their_fixed_order():
    inst = random_dense(810, 300, 9, 4)
    A = inst.A.astype(np.float64)
    rowptr, col, val = orc.full_csr(A)
    r = np.random.default_rng(1).normal(size=inst.m)
    g, c = orc.l2_column_sums(inst.m, inst.n, rowptr, col, val, r)
    assert np.allclose(g, A.T @ r, rtol=1e-12, atol=1e-12) and np.allclose(c, (A * A).sum(axis=0), rtol=1e-13)
    # the order is part of the definition: a chain of fused multiply-adds by ascending row
    import math
    acc = 0.0
    for i in range(inst.m):
        acc = math.fma(A[i, 3], r[i], acc) if hasattr(math, "fma") else float(np.float64(A[i, 3]) * r[i] + acc)
    if hasattr(math, "fma"):
        assert g[3] == acc
    # fp32: the same chain in single precision differs from the rounded fp64 sum, and is what is returned
    A32, r32 = A.astype(np.float32), r.astype(np.float32)
    g32, _ = orc.l2_column_sums(inst.m, inst.n, *orc.full_csr(A32), r32)
    assert g32.dtype == np.float32 and np.allclose(g32, A32.astype(np.float64).T @ r32, rtol=1e-4, atol=1e-3)


@pytest.mark.parametrize("s", [0.5, 4.0, 0.3])
def test_l2_changes_with_a_scale_are_those_of_the_scaled_matrix(s):
    """Instance q of a batch is the problem with matrix s X: the change of the squared norm under the
    move q_j -> D[k] is that of the fresh residuals of s X."""
    inst = random_dense(820, 15, 6, 5, integer=True)
    r = orc.residual_dense(inst.A, inst.b, inst.D, inst.x0, scale=s)
    got = orc.l2_changes_dense(inst.A, inst.D, inst.x0, r, scale=s)
    _, want = fresh_tables(inst.A, inst.b, inst.D, inst.x0, s=s)
    if s in (0.5, 4.0):
        assert np.array_equal(got, want)                               # power of two: still exact
    else:
        assert np.allclose(got, want, rtol=1e-12, atol=1e-9)
    assert not np.allclose(got, orc.l2_changes_dense(inst.A, inst.D, inst.x0, r, scale=1.0))


def test_l2_changes_sparse_equal_dense_and_ignore_explicit_zeros():
    inst = random_sparse(830, 40, 18, 4, density=0.3, dtype=np.float64, integer=True, explicit_zeros=True)
    A = np.zeros((inst.m, inst.n))
    for i in range(inst.m):
        A[i, inst.csr_col[inst.csr_rowptr[i]:inst.csr_rowptr[i + 1]]] = inst.csr_val[inst.csr_rowptr[i]:inst.csr_rowptr[i + 1]]
    r = orc.residual_csr(inst.m, inst.csr_rowptr, inst.csr_col, inst.csr_val, inst.b, inst.D, inst.x0)
    sp = orc.l2_changes_csr(inst.m, inst.n, inst.csr_rowptr, inst.csr_col, inst.csr_val, inst.D, inst.x0, r)
    assert np.array_equal(sp, orc.l2_changes_dense(A, inst.D, inst.x0, r))
    assert np.array_equal(sp, fresh_tables(A, inst.b, inst.D, inst.x0)[1])


def python_rule(scores, dq, rule):
    best = None
    for e, (s, q) in enumerate(zip(scores, dq)):
        if rule == 2 and not q <= 0:
            continue
        key = (s, q, e)
        if best is None or key < best:
            best = key
    return (-1, np.inf) if best is None else (best[2], best[0])


def test_argmin_with_the_l2_change_as_second_criterion():
    s = np.array([3.0, 1.0, 1.0, 1.0, 2.0, 1.0])
    q = np.array([0.0, 5.0, -2.0, -2.0, -9.0, 7.0])
    assert orc.argmin_move_l2(s, q, 1) == (2, 1.0)         # equal scores: smaller change, then lower index
    assert orc.argmin_move_l2(s, np.zeros(6), 1) == (1, 1.0)   # no difference in l2: the plain rule
    assert orc.argmin_move(s)[0] == 1
    # rule 2: candidates that increase the l2 norm are out, whatever their score
    s2 = np.array([1.0, 4.0, 2.0, 2.0])
    q2 = np.array([0.5, -1.0, 0.0, -3.0])
    assert orc.argmin_move_l2(s2, q2, 1) == (0, 1.0)
    assert orc.argmin_move_l2(s2, q2, 2) == (3, 2.0)
    assert orc.argmin_move_l2(s2, np.array([1.0, 1.0, 0.0, 1.0]), 2) == (2, 2.0)   # dq = 0 stays in
    rng = np.random.default_rng(5)
    for rule in (1, 2):
        for _ in range(200):
            ntab = int(rng.integers(1, 30))
            sc = rng.integers(0, 4, size=ntab).astype(np.float64)
            dq = rng.integers(-2, 3, size=ntab).astype(np.float64)
            want = python_rule(sc, dq, rule)
            got = orc.argmin_move_l2(sc, dq, rule)
            assert got[0] == want[0] and (want[0] < 0 or got[1] == want[1])


@pytest.mark.parametrize("rule", [1, 2])
@pytest.mark.parametrize("s", [1.0, 2.0])
def test_descent_with_the_l2_rule_replayed_from_fresh_tables(rule, s):
    """Every move of the oracle's descent is the lexicographic minimum of (error, change of the
    squared l2 norm, index) over tables recomputed from scratch (integer data: exact), it is taken
    only if the error drops strictly, and under rule 2 no move raises the l2 norm."""
    differs = 0
    for seed in range(6):
        inst = random_dense(840 + seed, 12, 8, 4, integer=True)
        res = orc.solve_l2_dense(inst.A, inst.b, inst.D, inst.x0, 30, rule=rule, scale=s)
        plain = orc.solve_dense(inst.A, inst.b, inst.D, inst.x0, 30, scale=s)
        x = inst.x0.astype(np.float64).copy()
        As = inst.A.astype(np.float64) * s
        t = np.abs(As @ x - inst.b).max()
        q = float(np.sum((As @ x - inst.b) ** 2))
        for it in range(res.iters_done + 1):
            scores, dq = fresh_tables(inst.A, inst.b, inst.D, x, s=s)
            c, sc = python_rule(scores, dq, rule)
            if not (c >= 0 and sc < t):
                assert it == res.iters_done                      # the oracle stopped here too
                break
            assert it < res.iters_done
            j, k = c // inst.nd, c % inst.nd
            assert (res.trace_j[it], res.trace_k[it]) == (j, k), (seed, it)
            x[j] = inst.D[k]
            t = sc
            assert res.trace_t[it] == t
            qn = float(np.sum((As @ x - inst.b) ** 2))
            if rule == 2:
                assert qn <= q
            q = qn
        assert np.array_equal(res.x, x) and res.t == t
        differs += int(res.iters_done != plain.iters_done or not np.array_equal(res.trace_j, plain.trace_j)
                       or not np.array_equal(res.trace_k, plain.trace_k))
    assert differs > 0            # the second criterion decided something the index rule decides otherwise


def test_rule_2_refuses_a_move_that_rule_1_takes():
    found = 0
    for seed in range(12):
        inst = random_dense(860 + seed, 10, 7, 4, integer=True)
        a = orc.solve_l2_dense(inst.A, inst.b, inst.D, inst.x0, 30, rule=1)
        b = orc.solve_l2_dense(inst.A, inst.b, inst.D, inst.x0, 30, rule=2)
        found += int(not np.array_equal(a.trace_j, b.trace_j) or not np.array_equal(a.trace_k, b.trace_k))
    assert found > 0


def test_descent_with_the_l2_rule_sparse_equals_dense_and_radius():
    inst = random_sparse(870, 30, 14, 5, density=0.35, dtype=np.float64, integer=True)
    A = np.zeros((inst.m, inst.n))
    for i in range(inst.m):
        A[i, inst.csr_col[inst.csr_rowptr[i]:inst.csr_rowptr[i + 1]]] = inst.csr_val[inst.csr_rowptr[i]:inst.csr_rowptr[i + 1]]
    for radius in (0, 1):
        a = orc.solve_l2_csr(inst.m, inst.n, inst.csr_rowptr, inst.csr_col, inst.csr_val, inst.b, inst.D, inst.x0, 40,
                             rule=1, radius=radius)
        b = orc.solve_l2_dense(A, inst.b, inst.D, inst.x0, 40, rule=1, radius=radius)
        assert a.iters_done == b.iters_done and np.array_equal(a.trace_j, b.trace_j) and np.array_equal(a.trace_t, b.trace_t)
        # first move against fresh tables with the neighbourhood applied
        scores, dq = fresh_tables(A, inst.b, inst.D, inst.x0, radius=radius)
        c, sc = python_rule(scores, dq, 1)
        if a.iters_done:
            assert (a.trace_j[0], a.trace_k[0]) == (c // inst.nd, c % inst.nd)
