"""Pins of the swap-move oracle (Algorithm 2, Proposition 1, Corollary 1) against facts that do
not come from the oracle: fresh recomputation of ||A x' - b||_inf for the exchanged x', the
inequalities of Proposition 1 and Corollary 1 in rational arithmetic, the A = I closed form."""
from fractions import Fraction

import numpy as np
import pytest
import scipy.sparse as sp

from oracle import oracle


def _int_instance(seed, m, n, nd, dtype=np.float64, density=1.0):
    """Integer data: every product and sum is exact, so bitwise equality with exact arithmetic holds."""
    rng = np.random.default_rng(seed)
    A = rng.integers(-4, 5, size=(m, n)).astype(dtype)
    if density < 1.0:
        A *= rng.random((m, n)) < density
    D = np.arange(nd, dtype=dtype) - nd // 2
    x = rng.choice(D, size=n)
    b = rng.integers(-6, 7, size=m).astype(dtype)
    return A, b, D, x


def _fresh_t(A, b, x):
    return np.max(np.abs(A.astype(np.float64) @ x.astype(np.float64) - b.astype(np.float64)))


@pytest.mark.parametrize("dtype", [np.float64, np.float32])
@pytest.mark.parametrize("seed", [0, 1, 2])
def test_table_is_the_error_of_the_exchanged_solution(seed, dtype):
    A, b, D, x = _int_instance(seed, 9, 7, 5, dtype)
    r = oracle.residual_dense(A, b, D, x)
    tab = oracle.swap_table_dense(A, D, x, r)
    n = x.size
    for i in range(n):
        for j in range(n):
            if x[i] > x[j]:
                y = x.copy(); y[i], y[j] = x[j], x[i]
                assert tab[i, j] == _fresh_t(A, b, y), (i, j)
            else:
                assert np.isinf(tab[i, j])


@pytest.mark.parametrize("seed", range(6))
def test_improving_pairs_are_those_of_proposition_1(seed):
    """t' < t  iff  (-t - s_k)/Delta < a_kj - a_ki < (t - s_k)/Delta for every row k."""
    A, b, D, x = _int_instance(10 + seed, 8, 8, 4)
    r = oracle.residual_dense(A, b, D, x)
    t = Fraction(int(np.max(np.abs(r))))
    tab = oracle.swap_table_dense(A, D, x, r)
    n, m = x.size, b.size
    found = 0
    for i in range(n):
        for j in range(n):
            if not x[i] > x[j]:
                continue
            Delta = Fraction(int(x[i] - x[j]))
            ok = all((-t - int(r[k])) / Delta < int(A[k, j] - A[k, i]) < (t - int(r[k])) / Delta
                     for k in range(m))
            assert ok == (tab[i, j] < float(t)), (i, j)
            found += ok
    i, j, tn = oracle.best_swap_dense(A, D, x, r)
    assert (i >= 0) == (found > 0)


@pytest.mark.parametrize("seed", range(4))
def test_improving_pairs_pass_the_filter_of_corollary_1(seed):
    """The condition on the k_eps rows of largest |s_k| is necessary for an improvement."""
    A, b, D, x = _int_instance(30 + seed, 12, 9, 5)
    r = oracle.residual_dense(A, b, D, x)
    t = Fraction(int(np.max(np.abs(r))))
    tab = oracle.swap_table_dense(A, D, x, r)
    rows = np.argsort(-np.abs(r), kind="stable")[:4]
    n = x.size
    seen = 0
    for i in range(n):
        for j in range(n):
            if not (x[i] > x[j] and tab[i, j] < float(t)):
                continue
            seen += 1
            Delta = Fraction(int(x[i] - x[j]))
            for k in rows:
                eps = t - abs(int(r[k]))
                diff = int(A[k, j] - A[k, i])
                if r[k] > 0:
                    assert diff < eps / Delta
                elif r[k] < 0:
                    assert diff > -eps / Delta
    assert seed != 0 or seen > 0


def test_best_swap_is_the_lowest_pair_among_the_smallest_errors():
    A, b, D, x = _int_instance(4, 10, 10, 3)
    r = oracle.residual_dense(A, b, D, x)
    tab = oracle.swap_table_dense(A, D, x, r)
    t = np.max(np.abs(r))
    i, j, tn = oracle.best_swap_dense(A, D, x, r)
    flat = tab.reshape(-1)
    if flat.min() < t:
        c = int(np.flatnonzero(flat == flat.min())[0])
        assert (i, j) == (c // x.size, c % x.size) and tn == flat.min()
    else:
        assert (i, j) == (-1, -1) and tn == t


def test_a_swap_that_leaves_the_error_unchanged_is_not_taken():
    """Two equal columns at different levels: exchanging them changes nothing, t' = t, and only
    t' < t counts (Algorithm 2)."""
    A = np.array([[1.0, 1.0], [-2.0, -2.0], [0.5, 0.5]])
    D = np.array([-1.0, 0.0, 1.0])
    x = np.array([1.0, -1.0])
    b = np.array([0.25, 0.5, -0.75])
    r = oracle.residual_dense(A, b, D, x)
    assert oracle.swap_table_dense(A, D, x, r)[0, 1] == np.max(np.abs(r))
    assert oracle.best_swap_dense(A, D, x, r) == (-1, -1, np.max(np.abs(r)))


def test_equal_improvements_go_to_the_lowest_pair():
    """Columns 1 and 2 are both zero and both at the lowest level: exchanging column 0 with either
    gives the same t' = 0 < t; the pair with the lower index i * n + j is the one returned."""
    A = np.array([[1.0, 0.0, 0.0]])
    D = np.array([-1.0, 0.0, 1.0])
    x = np.array([1.0, -1.0, -1.0])
    b = np.array([-1.0])
    r = oracle.residual_dense(A, b, D, x)
    tab = oracle.swap_table_dense(A, D, x, r)
    assert tab[0, 1] == 0.0 and tab[0, 2] == 0.0 and np.max(np.abs(r)) == 2.0
    assert oracle.best_swap_dense(A, D, x, r) == (0, 1, 0.0)


def test_identity_matrix_closed_form():
    """A = I: only rows i and j change, s'_i = x_j - b_i and s'_j = x_i - b_j."""
    rng = np.random.default_rng(5)
    n = 7
    A = np.eye(n)
    D = np.array([-2.0, -0.5, 0.25, 1.0, 3.0])
    x = rng.choice(D, n)
    b = rng.normal(size=n)
    r = x - b
    tab = oracle.swap_table_dense(A, D, x, r)
    for i in range(n):
        for j in range(n):
            if x[i] > x[j]:
                rest = max([abs(r[k]) for k in range(n) if k not in (i, j)], default=0.0)
                # r_i - Delta and r_j + Delta, each one rounding like the fma
                Delta = x[i] - x[j]
                want = max(rest, abs(r[i] - Delta), abs(r[j] + Delta))
                assert tab[i, j] == want


def test_apply_keeps_the_value_multiset_and_the_residual():
    A, b, D, x = _int_instance(6, 11, 9, 6)
    r = oracle.residual_dense(A, b, D, x)
    i, j, tn = oracle.best_swap_dense(A, D, x, r)
    assert i >= 0
    rowptr, col, val = oracle.full_csr(A)
    y, r2, t2 = oracle.apply_swap_dense(A, D, x, r, i, j)
    assert sorted(y) == sorted(x) and y[i] == x[j] and y[j] == x[i]
    assert np.array_equal(r2, A @ y - b) and t2 == tn == np.max(np.abs(A @ y - b))


def test_scale_and_mask():
    A, b, D, x = _int_instance(7, 8, 8, 4)
    sc = 0.5
    r = oracle.residual_dense(A, b, D, x, scale=sc)
    tab = oracle.swap_table_dense(A, D, x, r, scale=sc)
    for i in range(8):
        for j in range(8):
            if x[i] > x[j]:
                y = x.copy(); y[i], y[j] = x[j], x[i]
                assert tab[i, j] == _fresh_t(A, b, sc * y)
    vm = np.ones(8, dtype=np.uint8); vm[2] = 0
    tm = oracle.swap_table_dense(A, D, x, r, scale=sc, var_mask=vm)
    assert np.all(np.isinf(tm[2, :])) and np.all(np.isinf(tm[:, 2]))
    keep = np.ones((8, 8), bool); keep[2, :] = False; keep[:, 2] = False
    assert np.array_equal(tm[keep], tab[keep])


def test_sparse_matrix_equals_its_dense_form():
    A, b, D, x = _int_instance(8, 14, 10, 3, density=0.3)
    r = oracle.residual_dense(A, b, D, x)
    S = sp.csr_matrix(A)
    tab_s = oracle.swap_table_csr(14, 10, S.indptr, S.indices, S.data, D, x, r)
    assert np.array_equal(tab_s, oracle.swap_table_dense(A, D, x, r))


def test_alns_with_swaps_never_ends_worse_and_counts_swaps():
    rng = np.random.default_rng(9)
    A = rng.normal(size=(24, 12)); D = np.arange(-3.0, 4.0)
    xs = rng.choice(D, 12); b = A @ xs + rng.uniform(-0.4, 0.4, 24)
    x0 = rng.choice(D, 12)
    base = oracle.alns_dense(A, b, D, x0, oracle.alns_params(12, ls_moves=4, seed=3))
    sw = oracle.alns_dense(A, b, D, x0, oracle.alns_params(12, ls_moves=4, seed=3, ls_swaps=2))
    t0 = np.max(np.abs(A @ x0 - b))
    assert sw.t_best <= t0 and np.all(np.diff(sw.best) <= 0)
    assert np.isclose(np.max(np.abs(A @ sw.x - b)), sw.t_best)
    # with no swap allowed the loop is the one without the field
    assert np.array_equal(base.t, oracle.alns_dense(A, b, D, x0, oracle.alns_params(12, ls_moves=4, seed=3, ls_swaps=0)).t)
    assert np.any(sw.moves > 4) or np.array_equal(sw.t, base.t)
