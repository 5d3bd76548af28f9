"""Pins of the CPU oracle against things that are not the oracle.

Each test compares oracle output with what the paper's definitions and plain mathematics
fix: brute-force enumeration, a hand-worked example, closed forms of special cases, the
continuous Chebyshev LP bound, and numpy recomputation from scratch.  None of the
expected values is produced by the oracle or by the GPU library.
"""
import itertools
import json
import os

import numpy as np
import pytest

from oracle import oracle as orc
from workloads import random_batched, random_dense, random_sparse

GOLD = os.path.join(os.path.dirname(__file__), "golden")


# ------------------------------------------------------------------ numpy brute force
def fresh_objective(A, b, x):
    """||A x - b||_inf straight from the problem statement (fp64)."""
    return np.abs(np.asarray(A, np.float64) @ np.asarray(x, np.float64)
                  - np.asarray(b, np.float64)).max() if len(b) else 0.0


def brute_table(A, b, D, x):
    """Score of every single-coordinate change, each recomputed from scratch."""
    n, nd = A.shape[1], len(D)
    out = np.empty(n * nd)
    for j in range(n):
        for k in range(nd):
            y = np.array(x, np.float64)
            y[j] = D[k]
            out[j * nd + k] = fresh_objective(A, b, y)
    return out


def brute_argmin(scores):
    """Smallest score, lowest flat index among equals."""
    order = np.lexsort((np.arange(scores.size), scores))
    return int(order[0]), scores[order[0]]


def brute_global_optimum(A, b, D):
    n = A.shape[1]
    best = np.inf
    for combo in itertools.product(D, repeat=n):
        best = min(best, fresh_objective(A, b, np.array(combo)))
    return best


def chebyshev_lp_bound(A, b, lo, hi):
    from scipy.optimize import linprog

    m, n = A.shape
    c = np.zeros(n + 1)
    c[-1] = 1
    A_ub = np.block([[A, -np.ones((m, 1))], [-A, -np.ones((m, 1))]])
    res = linprog(c, A_ub=A_ub, b_ub=np.concatenate([b, -b]),
                  bounds=[(lo, hi)] * n + [(0, None)], method="highs")
    assert res.status == 0
    return res.x[-1]


def dense_of(inst):
    M = np.zeros((inst.m, inst.n), dtype=np.float64)
    for i in range(inst.m):
        for e in range(inst.csr_rowptr[i], inst.csr_rowptr[i + 1]):
            M[i, inst.csr_col[e]] = inst.csr_val[e]
    return M


# ------------------------------------------------------------------ hand-worked example
@pytest.mark.parametrize("dtype", [np.float64, np.float32])
def test_hand_example(dtype):
    g = json.load(open(os.path.join(GOLD, "hand_example.json")))
    A = np.array(g["A"], dtype)
    b = np.array(g["b"], dtype)
    D = np.array(g["D"], dtype)
    x0 = np.array(g["x0"], dtype)
    r0 = orc.residual_dense(A, b, D, x0)
    assert r0.tolist() == g["r0"]
    assert orc.eval_moves_dense(A, D, x0, r0).tolist() == g["scores0"]
    c, s = orc.argmin_move(orc.eval_moves_dense(A, D, x0, r0))
    assert (c, s) == (5, 4)
    x1, r1, t1 = orc.apply_move_dense(A, D, x0, r0, 1, 2)
    assert x1.tolist() == [2, 2] and r1.tolist() == [4, 3, 3] and t1 == 4
    assert orc.eval_moves_dense(A, D, x1, r1).tolist() == g["scores1"]
    res = orc.solve_dense(A, b, D, x0, iters=10)
    assert res.iters_done == 2
    assert res.trace_j.tolist() == g["trace_j"]
    assert res.trace_k.tolist() == g["trace_k"]
    assert res.trace_t.tolist() == g["trace_t"]
    assert res.x.tolist() == g["x_final"] and res.r.tolist() == g["r_final"]
    assert orc.eval_moves_dense(A, D, res.x, res.r).tolist() == g["scores2"]


# ------------------------------------------------------------------ brute force, integer data
@pytest.mark.parametrize("dtype", [np.float64, np.float32])
@pytest.mark.parametrize("seed", range(12))
def test_table_and_argmin_bruteforce_integer(seed, dtype):
    """Small-integer data: every operation is exact, so the rank-1 shortcut must equal the
    fresh recomputation bitwise, ties included."""
    rng = np.random.default_rng(seed)
    m, n, nd = int(rng.integers(1, 9)), int(rng.integers(1, 9)), int(rng.integers(2, 5))
    inst = random_dense(100 + seed, m, n, nd, dtype=dtype, integer=True)
    r = orc.residual_dense(inst.A, inst.b, inst.D, inst.x0)
    assert np.array_equal(r, inst.A.astype(np.float64) @ inst.x0 - inst.b)
    scores = orc.eval_moves_dense(inst.A, inst.D, inst.x0, r)
    want = brute_table(inst.A, inst.b, inst.D, inst.x0)
    assert np.array_equal(scores.astype(np.float64), want)
    c, s = orc.argmin_move(scores)
    cw, sw = brute_argmin(want)
    assert c == cw and s == sw
    # null moves carry the current objective exactly
    t = orc.max_abs(r)
    kidx = orc.values_to_index(inst.x0, inst.D)
    assert np.all(scores.reshape(n, nd)[np.arange(n), kidx] == t)


@pytest.mark.parametrize("seed", range(8))
def test_table_bruteforce_real(seed):
    """Real data, fp64: shortcut and fresh recomputation agree to rounding."""
    rng = np.random.default_rng(seed)
    m, n, nd = int(rng.integers(2, 30)), int(rng.integers(1, 9)), int(rng.integers(2, 5))
    inst = random_dense(200 + seed, m, n, nd, dtype=np.float64)
    r = orc.residual_dense(inst.A, inst.b, inst.D, inst.x0)
    np.testing.assert_allclose(r, inst.A @ inst.x0 - inst.b, rtol=0, atol=1e-13 * (1 + n))
    scores = orc.eval_moves_dense(inst.A, inst.D, inst.x0, r)
    np.testing.assert_allclose(scores, brute_table(inst.A, inst.b, inst.D, inst.x0),
                               rtol=1e-13, atol=1e-13)


# ------------------------------------------------------------------ the descent as a whole
@pytest.mark.parametrize("seed", range(10))
def test_descent_against_bruteforce_replay(seed):
    """Replay the oracle's trace with numpy: every step must be the brute-force best move,
    a strict improvement, and the maintained residual must equal a fresh A x - b."""
    rng = np.random.default_rng(seed)
    m, n, nd = int(rng.integers(2, 12)), int(rng.integers(2, 9)), int(rng.integers(2, 5))
    inst = random_dense(300 + seed, m, n, nd, dtype=np.float64, integer=True)
    res = orc.solve_dense(inst.A, inst.b, inst.D, inst.x0, iters=40)
    x = inst.x0.copy()
    t = fresh_objective(inst.A, inst.b, x)
    for it in range(res.iters_done):
        c, s = brute_argmin(brute_table(inst.A, inst.b, inst.D, x))
        assert s < t
        assert (res.trace_j[it], res.trace_k[it]) == (c // nd, c % nd)
        x[c // nd] = inst.D[c % nd]
        t = fresh_objective(inst.A, inst.b, x)
        assert res.trace_t[it] == t == s
    assert np.array_equal(res.x, x)
    assert np.array_equal(res.r, inst.A @ x - inst.b)           # rank-1 identity, exact here
    assert res.t == t
    # stopped for the right reason: either out of iterations or no strictly better move
    if res.iters_done < 40:
        _, s = brute_argmin(brute_table(inst.A, inst.b, inst.D, x))
        assert not (s < t)
    assert np.all(np.diff(np.concatenate([[fresh_objective(inst.A, inst.b, inst.x0)],
                                          res.trace_t])) < 0)


@pytest.mark.parametrize("seed", range(6))
def test_bounds_global_optimum_and_lp(seed):
    """final t >= global optimum over D^n (enumeration) >= continuous Chebyshev LP bound
    (MILP reformulation of the paper with x relaxed to the box [min D, max D])."""
    rng = np.random.default_rng(seed)
    m, n, nd = int(rng.integers(3, 10)), int(rng.integers(2, 7)), int(rng.integers(2, 5))
    inst = random_dense(400 + seed, m, n, nd, dtype=np.float64)
    res = orc.solve_dense(inst.A, inst.b, inst.D, inst.x0, iters=100)
    opt = brute_global_optimum(inst.A, inst.b, inst.D)
    lp = chebyshev_lp_bound(inst.A, inst.b, inst.D[0], inst.D[-1])
    assert res.t >= opt * (1 - 1e-12)
    assert opt >= lp - 1e-9
    assert abs(res.t - fresh_objective(inst.A, inst.b, res.x)) <= 1e-12 * (1 + res.t)


def test_residual_drift_bound():
    """Maintained residual after many moves stays within the rounding bound of a fresh one."""
    inst = random_dense(7, 300, 40, 16, dtype=np.float64)
    res = orc.solve_dense(inst.A, inst.b, inst.D, inst.x0, iters=200)
    fresh = inst.A @ res.x - inst.b
    u = np.finfo(np.float64).eps
    bound = (res.iters_done + inst.n) * u * (np.abs(inst.b) + np.abs(inst.A) @ np.abs(res.x)).max()
    assert np.abs(res.r - fresh).max() <= bound
    assert res.iters_done > 3


# ------------------------------------------------------------------ special cases
def test_subset_sum_closed_form():
    """NP-hardness reduction: m = 1, D = {0,1}, A = [a_1..a_n], b = S.
    score[j,k] = |r + (D[k] - x_j) a_j| with r = sum a_j x_j - S."""
    a = np.array([[3., 34., 4., 12., 5., 2.]])
    S = np.array([9.])
    D = np.array([0., 1.])
    x = np.array([1., 0., 0., 1., 0., 0.])
    r = orc.residual_dense(a, S, D, x)
    assert r[0] == 15 - 9
    scores = orc.eval_moves_dense(a, D, x, r).reshape(6, 2)
    for j in range(6):
        for k in range(2):
            assert scores[j, k] == abs(r[0] + (D[k] - x[j]) * a[0, j])
    res = orc.solve_dense(a, S, D, x, iters=10)
    # steepest single flips: 6 -> drop 12 (|-6|=6 no), flip +... verify only via the definition
    assert res.t == fresh_objective(a, S, res.x)
    assert res.t <= 6
    # 4 + 5 = 9 is a certificate; the descent need not find it, but t = 0 must be a fixed point
    xs = np.array([0., 0., 1., 0., 1., 0.])
    fixed = orc.solve_dense(a, S, D, xs, iters=10)
    assert fixed.iters_done == 0 and fixed.t == 0


@pytest.mark.parametrize("seed", range(5))
def test_identity_matrix_reaches_nearest_rounding(seed):
    """A = I: the objective separates, so the descent must end at
    t = max_j min_v |v - b_j| (nearest-value rounding), whatever the tie-breaks."""
    rng = np.random.default_rng(seed)
    n, nd = 9, 5
    D = np.sort(rng.uniform(-3, 3, nd))
    b = rng.uniform(-4, 4, n)
    x0 = rng.choice(D, n)
    res = orc.solve_dense(np.eye(n), b, D, x0, iters=200)
    want = max(min(abs(v - bj) for v in D) for bj in b)
    assert res.t == pytest.approx(want, rel=1e-15, abs=1e-15)
    assert res.iters_done < 200


# ------------------------------------------------------------------ options
@pytest.mark.parametrize("seed", range(4))
def test_radius_and_mask_equal_masked_full_table(seed):
    inst = random_dense(500 + seed, 12, 7, 5, dtype=np.float64)
    r = orc.residual_dense(inst.A, inst.b, inst.D, inst.x0)
    full = orc.eval_moves_dense(inst.A, inst.D, inst.x0, r).reshape(7, 5)
    kidx = orc.values_to_index(inst.x0, inst.D)
    rng = np.random.default_rng(seed)
    vm = (rng.uniform(size=7) < 0.6).astype(np.uint8)
    for radius in (0, 1, 2):
        got = orc.eval_moves_dense(inst.A, inst.D, inst.x0, r, radius=radius,
                                   var_mask=vm).reshape(7, 5)
        want = full.copy()
        for j in range(7):
            for k in range(5):
                if k == kidx[j]:
                    continue
                if not vm[j] or (radius > 0 and abs(k - kidx[j]) > radius):
                    want[j, k] = np.inf
        assert np.array_equal(got, want)


def test_x_outside_D_is_rejected():
    inst = random_dense(1, 4, 3, 3)
    bad = inst.x0.copy()
    bad[1] = 1234.5
    with pytest.raises(ValueError):
        orc.residual_dense(inst.A, inst.b, inst.D, bad)
    with pytest.raises(ValueError):
        orc.values_to_index(inst.x0, inst.D[::-1])


# ------------------------------------------------------------------ sparse == dense
@pytest.mark.parametrize("dtype", [np.float32, np.float64])
@pytest.mark.parametrize("seed", range(6))
def test_sparse_equals_dense(seed, dtype):
    """A CSR instance and the same matrix stored dense (zeros filled in) must give bitwise
    equal tables and traces: an absent entry is A_ij = 0 and fma(d, 0, r) = r.  The dense
    residual visits more columns but adds exact zeros, so r matches too on integer data."""
    inst = random_sparse(600 + seed, 17, 11, 3, density=0.3, dtype=dtype, integer=True,
                         explicit_zeros=(seed % 2 == 0))
    Ad = dense_of(inst).astype(dtype)
    args = (inst.m, inst.n, inst.csr_rowptr, inst.csr_col, inst.csr_val)
    r = orc.residual_csr(inst.m, inst.csr_rowptr, inst.csr_col, inst.csr_val, inst.b, inst.D,
                         inst.x0)
    assert np.array_equal(r, orc.residual_dense(Ad, inst.b, inst.D, inst.x0))
    want = orc.eval_moves_dense(Ad, inst.D, inst.x0, r)
    assert np.array_equal(orc.eval_moves_csr(*args, inst.D, inst.x0, r, method="plain"), want)
    assert np.array_equal(orc.eval_moves_csr(*args, inst.D, inst.x0, r, method="sorted"), want)
    assert np.array_equal(want.astype(np.float64),
                          brute_table(Ad, inst.b, inst.D, inst.x0))
    rs = orc.solve_csr(*args, inst.b, inst.D, inst.x0, iters=30)
    rd = orc.solve_dense(Ad, inst.b, inst.D, inst.x0, iters=30)
    assert rs.iters_done == rd.iters_done
    assert np.array_equal(rs.trace_j, rd.trace_j) and np.array_equal(rs.trace_k, rd.trace_k)
    assert np.array_equal(rs.trace_t, rd.trace_t)
    assert np.array_equal(rs.x, rd.x) and np.array_equal(rs.r, rd.r)


@pytest.mark.parametrize("seed", range(4))
def test_sparse_real_data_equals_dense(seed):
    """Real-valued entries: the table depends only on r, so given the same r the sparse
    and dense tables are bitwise equal; columns that hold every large-|r| row exercise the
    'rows outside the column' branch."""
    inst = random_sparse(700 + seed, 40, 25, 4, density=0.15, dtype=np.float32)
    Ad = dense_of(inst).astype(np.float32)
    args = (inst.m, inst.n, inst.csr_rowptr, inst.csr_col, inst.csr_val)
    r = orc.residual_csr(inst.m, inst.csr_rowptr, inst.csr_col, inst.csr_val, inst.b, inst.D,
                         inst.x0)
    want = orc.eval_moves_dense(Ad, inst.D, inst.x0, r)
    assert np.array_equal(orc.eval_moves_csr(*args, inst.D, inst.x0, r, method="plain"), want)
    assert np.array_equal(orc.eval_moves_csr(*args, inst.D, inst.x0, r, method="sorted"), want)
    xn, rn, tn = orc.apply_move_csr(*args, inst.D, inst.x0, r, 3, 1)
    xd, rd, td = orc.apply_move_dense(Ad, inst.D, inst.x0, r, 3, 1)
    assert np.array_equal(rn, rd) and tn == td and np.array_equal(xn, xd)


def test_sparse_empty_column_and_full_column():
    """A column with no entries scores max|r| for every value; a column holding every row
    has no outside rows at all."""
    rowptr = np.array([0, 1, 2, 3], dtype=np.int64)
    col = np.array([0, 0, 0], dtype=np.int32)           # column 0 full, column 1 empty
    val = np.array([1., -2., 3.], dtype=np.float32)
    D = np.array([0., 1., 2.], dtype=np.float32)
    b = np.array([1., 1., 1.], dtype=np.float32)
    x = np.array([1., 0.], dtype=np.float32)
    r = orc.residual_csr(3, rowptr, col, val, b, D, x)
    assert r.tolist() == [0., -3., 2.]
    for method in ("plain", "sorted"):
        s = orc.eval_moves_csr(3, 2, rowptr, col, val, D, x, r, method=method).reshape(2, 3)
        assert s[1].tolist() == [3., 3., 3.]
        assert s[0].tolist() == [1., 3., 5.]            # r - a, r, r + a -> max |.|


# ------------------------------------------------------------------ batched
@pytest.mark.parametrize("seed", range(3))
def test_batched_power_of_two_scale_equals_scaled_value_set(seed):
    """With a power-of-two scale s every product by s is exact, so the instance
    (X, s, D) must behave bitwise like (X, 1, s*D): this pins where the scale enters the
    residual and the step size."""
    inst = random_batched(800 + seed, 14, 6, 5, 4, dtype=np.float32, integer=True)
    res = orc.solve_batched(inst.A, inst.b, inst.D, inst.scale, inst.x0, iters=20)
    for q in range(inst.R):
        s = inst.scale[q]
        single = orc.solve_dense(inst.A, inst.b[q], inst.D * s, inst.x0[q] * s, iters=20)
        assert res.iters_done[q] == single.iters_done
        d = single.iters_done
        assert np.array_equal(res.trace_j[q, :d], single.trace_j)
        assert np.array_equal(res.trace_k[q, :d], single.trace_k)
        assert np.array_equal(res.trace_t[q, :d], single.trace_t)
        assert np.array_equal(res.x[q] * s, single.x)
        assert res.t[q] == single.t == fresh_objective(inst.A, inst.b[q], single.x)


def test_batched_real_scale_objective_matches_fresh():
    inst = random_batched(900, 50, 12, 7, 8, dtype=np.float32)
    res = orc.solve_batched(inst.A, inst.b, inst.D, inst.scale, inst.x0, iters=30)
    for q in range(inst.R):
        fresh = fresh_objective(inst.A, inst.b[q],
                                inst.scale[q].astype(np.float64) * res.x[q])
        assert abs(res.t[q] - fresh) <= 1e-5 * max(fresh, 1e-30)
        d = res.iters_done[q]
        assert np.all(np.diff(res.trace_t[q, :d]) < 0)
        assert np.all(np.isin(res.x[q], inst.D))


# ------------------------------------------------------------------ precision cross-check
@pytest.mark.parametrize("seed", range(4))
def test_f32_equals_f64_on_integer_data(seed):
    i64 = random_dense(1000 + seed, 9, 6, 4, dtype=np.float64, integer=True)
    r64 = orc.solve_dense(i64.A, i64.b, i64.D, i64.x0, iters=30)
    r32 = orc.solve_dense(i64.A.astype(np.float32), i64.b.astype(np.float32),
                          i64.D.astype(np.float32), i64.x0.astype(np.float32), iters=30)
    assert np.array_equal(r64.trace_j, r32.trace_j) and np.array_equal(r64.trace_k, r32.trace_k)
    assert np.array_equal(r64.trace_t, r32.trace_t.astype(np.float64))


# ------------------------------------------------------------------ planted mistakes are caught
def test_pins_catch_a_wrong_sign_and_a_transpose():
    """Sanity of the pins themselves: a numpy model of the table with a flipped sign of the
    step, or with A transposed, disagrees with the brute-force table on a generic case."""
    inst = random_dense(42, 6, 6, 3, dtype=np.float64, integer=True)
    A, b, D, x = inst.A, inst.b, inst.D, inst.x0
    r = A @ x - b
    kidx = orc.values_to_index(x, D)
    want = brute_table(A, b, D, x).reshape(6, 3)

    def model(sign, M):
        out = np.empty((6, 3))
        for j in range(6):
            for k in range(3):
                out[j, k] = np.abs(r + sign * (D[k] - D[kidx[j]]) * M[:, j]).max()
        return out

    assert np.array_equal(model(+1, A), want)
    assert not np.array_equal(model(-1, A), want)
    assert not np.array_equal(model(+1, A.T.copy()), want)
