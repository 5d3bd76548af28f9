"""Pins of the ALNS part of the CPU oracle (Algorithm 1; Appendix B operators) against facts
that do not come from the oracle: published generator outputs, the library exponential, the
paper's bound equations evaluated literally, brute force, and invariants of the loop."""
import itertools
import json
import math
import os

import numpy as np
import pytest

from oracle import oracle as orc
from workloads import random_dense, random_sparse

HERE = os.path.dirname(os.path.abspath(__file__))
M64 = 2 ** 64 - 1
GOLDEN = 0x9E3779B97F4A7C15


def test_mix_reproduces_published_splitmix64_outputs():
    g = json.load(open(os.path.join(HERE, "golden", "splitmix64_seed1234567.json")))
    state = g["seed"]
    for want in g["outputs"]:
        state = (state + GOLDEN) & M64
        assert orc.alns_mix(state) == int(want)


def test_rnd_is_a_chain_of_generator_steps_and_streams_differ():
    # first link = first SplitMix64 output of the seed (instance 0)
    seed = 1234567
    z = orc.alns_mix((seed + GOLDEN) & M64)
    for ctr in (3, 0, 5):                       # it, stream, c
        z = orc.alns_mix((z + GOLDEN * (ctr + 1)) & M64)
    assert orc.alns_rnd(seed, 0, 3, 0, 5) == z
    vals = {orc.alns_rnd(9, q, it, s, c) for q in range(3) for it in range(3) for s in range(3) for c in range(3)}
    assert len(vals) == 81


def test_expneg_matches_the_library_exponential():
    rng = np.random.default_rng(1)
    ys = np.concatenate([np.linspace(0, 50, 2001), rng.uniform(0, 699.9, 2000), [0.0, 1e-300, 1e-12, 699.99]])
    for y in ys:
        got, want = orc.alns_expneg(float(y)), math.exp(-float(y))
        assert abs(got - want) <= 4e-16 * want, (y, got, want)
    assert orc.alns_expneg(0.0) == 1.0
    assert orc.alns_expneg(700.0) == 0.0 and orc.alns_expneg(float("inf")) == 0.0
    assert orc.alns_expneg(float("nan")) == 0.0


def literal_impact(A, b, x, alpha):
    """Appendix B.2 as printed: LB, UB, R, then the numerator of d_j and sum |s_k|."""
    A = np.asarray(A, dtype=np.float64); b = np.asarray(b, dtype=np.float64); x = np.asarray(x, dtype=np.float64)
    s = A @ x - b
    t = np.abs(s).max()
    m, n = A.shape
    num = np.zeros(n)
    Rs = np.zeros((m, n))
    for j in range(n):
        for k in range(m):
            rest = A[k] @ x - A[k, j] * x[j]             # sum_{i != j} a_ki x_i
            lb = (-t + b[k] - rest) / A[k, j]
            ub = (t + b[k] - rest) / A[k, j]
            R = min(ub - x[j], x[j] - lb) if A[k, j] > 0 else min(lb - x[j], x[j] - ub)
            Rs[k, j] = R
            num[j] += abs(s[k]) * math.exp(-alpha * R)
    return s, t, Rs, num


@pytest.mark.parametrize("seed", range(3))
def test_impact_weights_follow_the_bound_equations(seed):
    inst = random_dense(100 + seed, 14, 6, 5)
    A = inst.A.astype(np.float64)
    assert np.all(A != 0)
    s, t, Rs, num = literal_impact(A, inst.b, inst.x0, 0.3)
    # the collapse used by the oracle: R = (t - |s_k|) / |a_kj| >= 0
    assert np.allclose(Rs, (t - np.abs(s))[:, None] / np.abs(A), rtol=1e-9, atol=1e-9)
    rowptr, col, val = orc.full_csr(A)
    r = orc.residual_dense(A, inst.b, inst.D, inst.x0)
    w = orc.alns_impact_weights(inst.m, inst.n, rowptr, col, val, r, alpha=0.3).astype(np.float64)
    e = math.frexp(t)[1]
    scale = 2.0 ** (24 - e)
    # fixed point with truncation: each of the m terms loses less than 1
    assert np.all(np.abs((w - 1) - num * scale) <= inst.m + 1e-6 * num * scale)
    # proportions are those of the paper's d_j
    assert np.allclose((w - 1) / (w - 1).sum(), num / num.sum(), atol=1e-5)


def test_impact_weight_ignores_rows_with_zero_coefficient_and_handles_zero_residual():
    A = np.array([[1.0, 0.0], [0.0, 2.0], [1.0, 1.0]])
    D = np.array([0.0, 1.0, 2.0]); x = np.array([1.0, 1.0]); b = A @ x
    rowptr, col, val = orc.full_csr(A)
    w = orc.alns_impact_weights(3, 2, rowptr, col, val, np.zeros(3), alpha=0.3)
    assert np.array_equal(w, [1, 1])                       # t = 0: nothing to weigh
    r = np.array([0.5, -0.25, 0.125])
    w_full = orc.alns_impact_weights(3, 2, rowptr, col, val, r, alpha=0.3)
    # dropping the explicit zeros from the storage changes nothing
    keep = val != 0
    rp = np.concatenate([[0], np.cumsum([keep[i * 2:(i + 1) * 2].sum() for i in range(3)])]).astype(np.int64)
    w_sparse = orc.alns_impact_weights(3, 2, rp, col[keep], val[keep], r, alpha=0.3)
    assert np.array_equal(w_full, w_sparse)


def test_sample_takes_the_variable_whose_interval_of_the_prefix_sums_holds_the_draw():
    """Draw c of an iteration is v = rnd(seed, inst, it, 1, c) mod total; it names the first
    variable whose inclusive prefix sum exceeds v, and a variable already taken is drawn again."""
    w = np.array([5, 1, 10, 4], dtype=np.uint64)
    prefix = np.cumsum(w.astype(np.int64))
    on_a_boundary = 0
    for it in range(60):
        v = orc.alns_rnd(11, 2, it, 1, 0) % 20
        on_a_boundary += int(v in (5, 6, 16))
        want = int(np.searchsorted(prefix, v, side="right"))
        assert orc.alns_sample(4, w, 1, 11, 2, it)[0] == want
    assert on_a_boundary > 0                               # v equal to a prefix sum was among them
    # equal weights: variable = v mod n, repeats skipped, in draw order
    n = 9
    for it in range(10):
        want, c = [], 0
        while len(want) < 4:
            j = int(orc.alns_rnd(8, 1, it, 1, c) % n)
            c += 1
            if j not in want:
                want.append(j)
        assert orc.alns_sample(n, None, 4, 8, 1, it).tolist() == want
        assert orc.alns_sample(n, np.ones(n, dtype=np.uint64), 4, 8, 1, it).tolist() == want


def test_sample_distinct_ordered_and_proportional():
    n = 50
    p = orc.alns_sample(n, None, n, 3, 0, 0)
    assert sorted(p.tolist()) == list(range(n))            # all of them: a permutation
    p = orc.alns_sample(n, None, 7, 3, 0, 1)
    assert len(set(p.tolist())) == 7 and p.min() >= 0 and p.max() < n
    # frequencies of single draws follow the weights
    w = np.array([5, 1, 10, 4], dtype=np.uint64)
    counts = np.zeros(4)
    N = 6000
    for it in range(N):
        counts[orc.alns_sample(4, w, 1, 5, 0, it)[0]] += 1
    expect = N * w.astype(np.float64) / 20
    chi2 = ((counts - expect) ** 2 / expect).sum()
    assert chi2 < 16.3                                     # 99.9 % point of chi-square with 3 dof


def test_greedy_repair_moves_down_when_both_neighbours_score_the_same():
    """A column of zeros: either neighbour leaves the residual as it is, so the errors tie and
    the lower level is taken; at the lowest level only the upper neighbour exists."""
    A = np.array([[1.0, 0.0, 0.0], [2.0, 0.0, 0.0]])
    rowptr, col, val = orc.full_csr(A)
    D = np.array([-1.0, 0.0, 1.0, 2.0])
    x = np.array([1.0, 1.0, -1.0])
    b = np.array([0.5, 0.25])
    r = orc.residual_dense(A, b, D, x)
    x_new, r_new = orc.alns_repair(2, 3, rowptr, col, val, D, x, r, np.array([1, 2], dtype=np.int32), True, 1, 0, 0)
    assert x_new.tolist() == [1.0, 0.0, 0.0]
    assert np.array_equal(r_new, r)


def test_greedy_repair_is_the_better_of_the_two_neighbour_levels():
    inst = random_dense(321, 18, 7, 6)
    A = inst.A.astype(np.float64)
    rowptr, col, val = orc.full_csr(A)
    D = inst.D
    x = inst.x0.copy()
    x[0], x[1] = D[0], D[-1]                               # two variables at the ends of D
    r = orc.residual_dense(A, inst.b, D, x)
    picked = np.array([3, 0, 1, 5], dtype=np.int32)
    x_new, r_new = orc.alns_repair(inst.m, inst.n, rowptr, col, val, D, x, r, picked, True, 1, 0, 0)
    xs = x.copy()
    for j in picked:
        k = int(np.searchsorted(D, xs[j]))
        cands = [kk for kk in (k - 1, k + 1) if 0 <= kk < D.size]
        errs = []
        for kk in cands:
            y = xs.copy(); y[j] = D[kk]
            errs.append(np.abs(A @ y - inst.b).max())
        best = cands[int(np.argmin(errs))]                 # argmin takes the lower level on a tie
        assert abs(errs[0] - errs[-1]) > 1e-9 or len(cands) == 1
        xs[j] = D[best]
    assert np.array_equal(x_new, xs)
    assert np.allclose(r_new, A @ xs - inst.b, atol=1e-9)


def test_random_repair_follows_the_generator_bit():
    inst = random_dense(322, 10, 6, 5)
    rowptr, col, val = orc.full_csr(inst.A)
    D = inst.D
    x = np.full(inst.n, D[2])
    x[4] = D[0]
    r = orc.residual_dense(inst.A, inst.b, D, x)
    picked = np.array([2, 4, 0], dtype=np.int32)
    x_new, r_new = orc.alns_repair(inst.m, inst.n, rowptr, col, val, D, x, r, picked, False, 77, 3, 9)
    for pos, j in enumerate(picked):
        up = orc.alns_rnd(77, 3, 9, 2, pos) & 1
        k = int(np.searchsorted(D, x[j]))
        want = k + 1 if (up or k == 0) else k - 1
        assert x_new[j] == D[want]
    assert np.allclose(r_new, inst.A @ x_new - inst.b, atol=1e-9)


@pytest.mark.parametrize("kind,dtype", [("dense", np.float64), ("dense", np.float32), ("sparse", np.float32)])
def test_alns_loop_invariants(kind, dtype):
    if kind == "dense":
        inst = random_dense(500, 40, 16, 5, dtype=dtype, integer=True)
        rowptr, col, val = orc.full_csr(inst.A)
        A = inst.A.astype(np.float64)
    else:
        inst = random_sparse(501, 60, 24, 4, 0.3, dtype=dtype, integer=True)
        rowptr, col, val = inst.csr_rowptr, inst.csr_col, inst.csr_val
        A = np.zeros((inst.m, inst.n))
        for i in range(inst.m):
            A[i, col[rowptr[i]:rowptr[i + 1]]] = val[rowptr[i]:rowptr[i + 1]]
    prm = orc.alns_params(40, ls_moves=6, ls_radius=1, destroy_count=3, seed=5)
    res = orc.alns_csr(inst.m, inst.n, rowptr, col, val, inst.b, inst.D, inst.x0, prm)
    t0 = np.abs(A @ inst.x0.astype(np.float64) - inst.b).max()
    # best error: never increases, starts no worse than x0, and belongs to the returned x
    assert np.all(np.diff(res.best) <= 0) and res.best[0] <= t0
    assert res.t_best == res.best[-1]
    assert np.abs(A @ res.x.astype(np.float64) - inst.b).max() == res.t_best      # integer data: exact
    assert np.all(np.isin(res.x, inst.D))
    # acceptance: not worse than the current solution, whose error is the last accepted one
    cur = t0
    for it in range(40):
        assert bool(res.accepted[it]) == (res.t[it] <= cur)
        if res.accepted[it]:
            cur = res.t[it]
        assert 0 <= res.moves[it] <= 6 and res.destroy[it] in (0, 1) and res.repair[it] in (0, 1)
    assert set(res.destroy.tolist()) == {0, 1} and set(res.repair.tolist()) == {0, 1}
    assert np.all(res.weights > 0)
    # same seed, same run; another seed, another run
    again = orc.alns_csr(inst.m, inst.n, rowptr, col, val, inst.b, inst.D, inst.x0, prm)
    assert np.array_equal(again.t, res.t) and np.array_equal(again.x, res.x)
    other = orc.alns_csr(inst.m, inst.n, rowptr, col, val, inst.b, inst.D, inst.x0,
                         orc.alns_params(40, ls_moves=6, ls_radius=1, destroy_count=3, seed=6))
    assert not np.array_equal(other.t, res.t)


def test_operator_choice_and_weights_replayed_from_the_trace():
    """Roulette wheel and weight update of the appendix on parameter setting, replayed outside the
    oracle from its trace: operator 0 of a pair is taken when u (w0 + w1) < w0 with u =
    (rnd >> 11) 2^-53 of stream 0, and an accepted iteration moves the two chosen weights to
    (1 - lambda) w + lambda psi, psi = sigma1 for a new best and sigma3 otherwise (with this
    acceptance rule the current solution is always a best one, so sigma2 never applies)."""
    inst = random_dense(507, 30, 12, 5, integer=True)
    rowptr, col, val = orc.full_csr(inst.A)
    lam, s1, s2, s3 = 0.35, 5.0, 2.5, 0.25
    iters = 60
    prm = orc.alns_params(iters, ls_moves=4, ls_radius=1, destroy_count=2, lambda_=lam, sigma1=s1, sigma2=s2,
                          sigma3=s3, seed=9)
    res = orc.alns_csr(inst.m, inst.n, rowptr, col, val, inst.b, inst.D, inst.x0, prm, inst=4)
    w = [1.0, 1.0, 1.0, 1.0]
    best = np.abs(inst.A.astype(np.float64) @ inst.x0 - inst.b).max()
    seen = set()
    for it in range(iters):
        ud = (orc.alns_rnd(9, 4, it, 0, 0) >> 11) * 2.0 ** -53
        ur = (orc.alns_rnd(9, 4, it, 0, 1) >> 11) * 2.0 ** -53
        d_op = 0 if ud * (w[0] + w[1]) < w[0] else 1
        r_op = 0 if ur * (w[2] + w[3]) < w[2] else 1
        assert (res.destroy[it], res.repair[it]) == (d_op, r_op)
        if res.accepted[it]:
            psi = s1 if res.t[it] < best else s3
            seen.add(psi)
            best = min(best, res.t[it])
            w[d_op] = (1 - lam) * w[d_op] + lam * psi
            w[2 + r_op] = (1 - lam) * w[2 + r_op] + lam * psi
        assert res.best[it] == best
    assert seen == {s1, s3}
    assert np.allclose(res.weights, w, rtol=1e-14, atol=0)
    # far from 1/2 the choice is that of u alone: u < 1/2 takes operator 0 at the first iteration
    for seed in range(12):
        one = orc.alns_csr(inst.m, inst.n, rowptr, col, val, inst.b, inst.D, inst.x0,
                           orc.alns_params(1, ls_moves=1, destroy_count=1, seed=seed))
        u = (orc.alns_rnd(seed, 0, 0, 0, 0) >> 11) * 2.0 ** -53
        assert one.destroy[0] == (0 if u < 0.5 else 1)


def test_the_returned_solution_is_the_first_one_that_reached_the_best_error():
    """Algorithm 1 replaces the best solution only by a strictly better one: iterations that are
    accepted with an equal error move the current solution, not the returned one."""
    inst = random_dense(508, 24, 10, 4, integer=True)
    rowptr, col, val = orc.full_csr(inst.A)
    found = 0
    for seed in range(6):
        full = orc.alns_csr(inst.m, inst.n, rowptr, col, val, inst.b, inst.D, inst.x0,
                            orc.alns_params(50, ls_moves=3, destroy_count=2, seed=seed))
        t0 = np.abs(inst.A.astype(np.float64) @ inst.x0 - inst.b).max()
        improving = [it for it in range(50) if full.best[it] < (full.best[it - 1] if it else t0)]
        last = improving[-1] + 1 if improving else 0
        later_equal = [it for it in range(last, 50) if full.accepted[it]]
        short = orc.alns_csr(inst.m, inst.n, rowptr, col, val, inst.b, inst.D, inst.x0,
                             orc.alns_params(last, ls_moves=3, destroy_count=2, seed=seed))
        assert np.array_equal(full.x, short.x)
        found += len(later_equal) > 0
    assert found > 0                                       # some run did accept equal errors afterwards


def test_greedy_repair_counts_the_rows_outside_the_column():
    """The error of a candidate level is the maximum over ALL rows.  Here a row the variable does
    not appear in dominates both candidates, they tie, and the lower level is taken - although
    the upper level is better on the variable's own row."""
    rowptr = np.array([0, 1, 2], dtype=np.int64)           # A = identity, stored sparse
    col = np.array([0, 1], dtype=np.int32)
    val = np.array([1.0, 1.0])
    D = np.array([-1.0, 0.0, 1.0])
    x = np.array([0.0, 1.0])
    b = np.array([1.0, -9.0])                              # r = (-1, 10)
    r = x - b
    x_new, r_new = orc.alns_repair(2, 2, rowptr, col, val, D, x, r, np.array([0], dtype=np.int32), True, 1, 0, 0)
    assert x_new.tolist() == [-1.0, 1.0] and r_new.tolist() == [-2.0, 10.0]
    # without the dominating row the upper level wins
    b2 = np.array([1.0, 1.0])
    x_new, _ = orc.alns_repair(2, 2, rowptr, col, val, D, x, x - b2, np.array([0], dtype=np.int32), True, 1, 0, 0)
    assert x_new.tolist() == [1.0, 1.0]


def test_impact_weights_of_a_huge_matrix_are_shifted_to_keep_their_total_below_2_to_the_62():
    """m = 2^20 rows and n = 2^19 columns: 21 + 24 + 20 bits could reach 2^65, so every weight is
    1 + (sum >> 3).  Entries on rows that attain the largest violation have slack 0 and add
    trunc(t 2^24 / 2^e) each."""
    m, n = 1 << 20, 1 << 19
    r = np.zeros(m)
    t = 12582913 / 2.0 ** 24                               # 0.75 + 2^-24: frexp exponent 0
    r[5] = t
    r[77] = -t
    rows = np.array([5, 5, 77], dtype=np.int64)
    cols = np.array([3, 9, 9], dtype=np.int32)
    rowptr = np.zeros(m + 1, dtype=np.int64)
    np.add.at(rowptr, rows + 1, 1)
    rowptr = np.cumsum(rowptr)
    w = orc.alns_impact_weights(m, n, rowptr, cols, np.array([2.0, -1.0, 0.5]), r, alpha=0.3)
    assert w[3] == 1 + (12582913 >> 3) and w[9] == 1 + ((2 * 12582913) >> 3)
    assert w[0] == 1 and int(w.sum()) == n + (12582913 >> 3) + ((2 * 12582913) >> 3)


def test_alns_zero_iterations_and_lower_bound_by_enumeration():
    inst = random_dense(502, 9, 5, 3, integer=True)
    rowptr, col, val = orc.full_csr(inst.A)
    res0 = orc.alns_csr(inst.m, inst.n, rowptr, col, val, inst.b, inst.D, inst.x0, orc.alns_params(0))
    assert np.array_equal(res0.x, inst.x0)
    assert res0.t_best == np.abs(inst.A @ inst.x0 - inst.b).max()
    opt = min(np.abs(inst.A @ np.array(x) - inst.b).max() for x in itertools.product(inst.D, repeat=inst.n))
    res = orc.alns_csr(inst.m, inst.n, rowptr, col, val, inst.b, inst.D, inst.x0,
                       orc.alns_params(60, ls_moves=10, ls_radius=0, destroy_count=2, seed=3))
    assert res.t_best >= opt
    assert res.t_best <= res0.t_best


def test_alns_dense_entry_equals_full_storage_sparse_entry():
    inst = random_dense(503, 25, 10, 4, dtype=np.float32)
    prm = orc.alns_params(15, seed=21)
    a = orc.alns_dense(inst.A, inst.b, inst.D, inst.x0, prm)
    rowptr, col, val = orc.full_csr(inst.A)
    b = orc.alns_csr(inst.m, inst.n, rowptr, col, val, inst.b, inst.D, inst.x0, prm)
    assert np.array_equal(a.t, b.t) and np.array_equal(a.x, b.x)
    # the first local search of a run that destroys nothing would be the plain descent:
    # with the repaired variable moved, the descent still reaches a local optimum of the same kind
    assert a.t_best <= np.abs(inst.A.astype(np.float64) @ inst.x0 - inst.b).max() * (1 + 1e-6)


# ---- l2 guard of the acceptance step -----------------------------------------------------------
def test_sumsq_against_numpy_and_exact_on_integers():
    rng = np.random.default_rng(21)
    for m in (0, 1, 255, 256, 257, 1000, 5000):
        r = rng.normal(size=m)
        assert np.isclose(orc.sumsq(r), float(np.dot(r, r)), rtol=1e-13, atol=0)
        ri = rng.integers(-1000, 1000, size=m).astype(np.float32)
        assert orc.sumsq(ri) == float(np.sum(ri.astype(np.int64) ** 2))      # every partial sum is exact
    # fp32 residuals are squared in double precision: no fp32 rounding of the squares
    r32 = np.array([1.0 + 2.0 ** -20, 3.0], dtype=np.float32)
    assert orc.sumsq(r32) == (1.0 + 2.0 ** -20) ** 2 + 9.0


def test_l2_guard_keeps_both_norms_from_increasing():
    rng = np.random.default_rng(22)
    A = rng.normal(size=(40, 18)); D = np.arange(-3.0, 4.0)
    b = A @ rng.choice(D, 18) + rng.uniform(-0.4, 0.4, 40)
    x0 = rng.choice(D, 18)
    free = orc.alns_dense(A, b, D, x0, orc.alns_params(40, ls_moves=2, seed=5))
    guard = orc.alns_dense(A, b, D, x0, orc.alns_params(40, ls_moves=2, seed=5, l2_guard=1))
    r0 = A @ x0 - b
    for res, guarded in ((free, False), (guard, True)):
        q_cur, t_cur = float(r0 @ r0), np.abs(r0).max()
        for it in range(40):
            ok = res.t[it] <= t_cur and (not guarded or res.q2[it] <= q_cur)
            assert bool(res.accepted[it]) == ok, (guarded, it)
            if ok:
                if guarded:
                    assert res.q2[it] <= q_cur
                q_cur, t_cur = res.q2[it], res.t[it]
    # the guard rejected something the plain rule accepts (else the test shows nothing)
    assert guard.accepted.sum() < free.accepted.sum() or not np.array_equal(guard.t, free.t)
    # the best solution's residual has the recorded error
    assert np.isclose(np.abs(A @ guard.x - b).max(), guard.t_best)


# ---- per-instance scale (batched instances: variables take the values s * D[k]) ------------------
def _scaled_csr(inst_A, s):
    """CSR of s * A with every entry stored (s a power of two: the products are exact)."""
    rowptr, col, val = orc.full_csr(np.asarray(inst_A) * s)
    return rowptr, col, val


@pytest.mark.parametrize("dtype", [np.float64, np.float32])
@pytest.mark.parametrize("s", [0.25, 8.0])
def test_power_of_two_scale_is_the_same_run_as_the_scale_folded_into_the_matrix(dtype, s):
    """Instance q of a batch is the problem with matrix s_q X (section "Quantization without
    outlier separation as DMMV": A = X s_row).  With s a power of two, s X_ij is exact and every
    rounding of the scaled run (residual, steps, pairs, slacks of the impact score) meets the same
    real number as the run on the matrix s X with scale 1: the whole outer loop must agree bit for
    bit - operators, draws, repairs, local-search moves, errors, weights and the solution."""
    inst = random_dense(610, 36, 14, 5, dtype=dtype)
    prm = orc.alns_params(30, ls_moves=5, ls_radius=1, destroy_count=3, seed=17, ls_swaps=1, l2_guard=1)
    a = orc.alns_dense(inst.A, inst.b, inst.D, inst.x0, prm, inst=3, scale=s)
    b = orc.alns_dense((inst.A.astype(np.float64) * s).astype(dtype), inst.b, inst.D, inst.x0, prm, inst=3, scale=1.0)
    for f in ("destroy", "repair", "moves", "accepted", "t", "best", "weights", "q2", "x"):
        assert np.array_equal(getattr(a, f), getattr(b, f)), f
    assert a.t_best == b.t_best
    # the scale is not a no-op: the unscaled problem runs differently
    c = orc.alns_dense(inst.A, inst.b, inst.D, inst.x0, prm, inst=3, scale=1.0)
    assert not np.array_equal(a.t, c.t)
    # and both destroy operators and the local search took part
    assert set(a.destroy.tolist()) == {0, 1} and a.moves.sum() > 0


@pytest.mark.parametrize("s", [0.5, 4.0, 0.37])
def test_impact_weights_with_a_scale_follow_the_bound_equations_of_the_scaled_matrix(s):
    inst = random_dense(611, 14, 6, 5)
    A = inst.A.astype(np.float64)
    r = orc.residual_dense(A, inst.b, inst.D, inst.x0, scale=s)
    # Appendix B.2 evaluated literally for the matrix s A
    sres, t, Rs, num = literal_impact(A * s, inst.b, inst.x0, 0.3)
    assert np.allclose(sres, r, rtol=1e-12, atol=1e-12)
    rowptr, col, val = orc.full_csr(A)
    w = orc.alns_impact_weights(inst.m, inst.n, rowptr, col, val, r, alpha=0.3, scale=s).astype(np.float64)
    scale = 2.0 ** (24 - math.frexp(t)[1])
    assert np.all(np.abs((w - 1) - num * scale) <= inst.m + 1e-6 * num * scale)
    # without the scale the slacks are divided by other coefficients: other weights
    w1 = orc.alns_impact_weights(inst.m, inst.n, rowptr, col, val, r, alpha=0.3, scale=1.0).astype(np.float64)
    assert not np.allclose(w1, w, rtol=1e-3)
    if s in (0.5, 4.0):                                    # power of two: same bits as the folded matrix
        rp, cc, vv = _scaled_csr(A, s)
        w2 = orc.alns_impact_weights(inst.m, inst.n, rp, cc, vv, r, alpha=0.3, scale=1.0)
        assert np.array_equal(w2.astype(np.float64), w)


@pytest.mark.parametrize("s", [0.5, 2.0, 1.7])
def test_repair_with_a_scale_is_the_repair_of_the_scaled_matrix(s):
    inst = random_dense(612, 18, 7, 6)
    A = inst.A.astype(np.float64)
    rowptr, col, val = orc.full_csr(A)
    D = inst.D
    x = inst.x0.copy()
    r = orc.residual_dense(A, inst.b, D, x, scale=s)
    assert np.allclose(r, (A * s) @ x - inst.b, atol=1e-12)     # starting residual carries the scale
    picked = np.array([3, 0, 6, 5], dtype=np.int32)
    for greedy in (True, False):
        x_new, r_new = orc.alns_repair(inst.m, inst.n, rowptr, col, val, D, x, r, picked, greedy, 5, 2, 7, scale=s)
        xs = x.copy()
        for pos, j in enumerate(picked):
            k = int(np.searchsorted(D, xs[j]))
            cands = [kk for kk in (k - 1, k + 1) if 0 <= kk < D.size]
            if greedy:
                errs = []
                for kk in cands:
                    y = xs.copy(); y[j] = D[kk]
                    errs.append(np.abs((A * s) @ y - inst.b).max())
                assert len(cands) == 1 or abs(errs[0] - errs[1]) > 1e-9
                best = cands[int(np.argmin(errs))]
            else:
                up = orc.alns_rnd(5, 2, 7, 2, pos) & 1
                best = k + 1 if (up or k == 0) and k + 1 < D.size else k - 1
            xs[j] = D[best]
        assert np.array_equal(x_new, xs), greedy
        assert np.allclose(r_new, (A * s) @ xs - inst.b, atol=1e-9)
    if s in (0.5, 2.0):
        rp, cc, vv = _scaled_csr(A, s)
        xa, ra = orc.alns_repair(inst.m, inst.n, rowptr, col, val, D, x, r, picked, True, 5, 2, 7, scale=s)
        xb, rb = orc.alns_repair(inst.m, inst.n, rp, cc, vv, D, x, r, picked, True, 5, 2, 7, scale=1.0)
        assert np.array_equal(xa, xb) and np.array_equal(ra, rb)


# ---- the loop replayed outside the oracle ---------------------------------------------------------
def _replay_alns(A, b, D, x0, res, iters, ls_moves, ls_radius, count, seed, inst, alpha=0.3, s=1.0):
    """Algorithm 1 replayed from the oracle's trace on small-integer data (every operation exact).
    The draws and the repair come from the oracle's own routines, which have pins of their own; the
    local search is written out here from its definition: while moves are left, the error of every
    single-coordinate change (within ls_radius levels) is recomputed FRESH as max |A x' - b|, the
    smallest wins (lowest flat index on a tie) and is taken only if it is strictly below the
    current error.  Returns how many local searches stopped on a plateau (best score == error)
    with moves to spare."""
    As = np.asarray(A, dtype=np.float64) * s
    b = np.asarray(b, dtype=np.float64)
    D = np.asarray(D, dtype=np.float64)
    m, n = As.shape
    nd = D.size
    rowptr, col, val = orc.full_csr(np.asarray(A, dtype=np.float64))
    x_cur = np.asarray(x0, dtype=np.float64).copy()
    t_cur = np.abs(As @ x_cur - b).max()
    plateaus = 0
    for it in range(iters):
        x = x_cur.copy()
        r = As @ x - b
        if res.destroy[it] == 1:
            w = orc.alns_impact_weights(m, n, rowptr, col, val, r, alpha=alpha, scale=s)
            picked = orc.alns_sample(n, w, count, seed, inst, it)
        else:
            picked = orc.alns_sample(n, None, count, seed, inst, it)
        assert len(picked) == min(count, n)
        x, r = orc.alns_repair(m, n, rowptr, col, val, D, x, r, picked, bool(res.repair[it]), seed, inst, it, scale=s)
        assert np.array_equal(r, As @ x - b)
        t = np.abs(r).max()
        moves = 0
        while moves < ls_moves:
            best = (np.inf, -1, -1)
            for j in range(n):
                kc = int(np.searchsorted(D, x[j]))
                for k in range(nd):
                    if k != kc and ls_radius > 0 and abs(k - kc) > ls_radius:
                        continue
                    y = x.copy(); y[j] = D[k]
                    sc = np.abs(As @ y - b).max()
                    if sc < best[0]:
                        best = (sc, j, k)
            if not best[0] < t:
                plateaus += int(best[0] == t)
                break
            x[best[1]] = D[best[2]]
            t = best[0]
            moves += 1
        assert res.moves[it] == moves, (it, res.moves[it], moves)
        assert res.t[it] == t, (it, res.t[it], t)
        ok = t <= t_cur
        assert bool(res.accepted[it]) == ok
        if ok:
            x_cur, t_cur = x, t
    return plateaus


@pytest.mark.parametrize("radius", [1, 0])
def test_local_search_of_the_loop_is_the_strict_best_improvement_descent(radius):
    inst = random_dense(620, 16, 9, 5, integer=True)
    iters, ls_moves, count, seed = 40, 6, 2, 4
    prm = orc.alns_params(iters, ls_moves=ls_moves, ls_radius=radius, destroy_count=count, seed=seed)
    res = orc.alns_dense(inst.A, inst.b, inst.D, inst.x0, prm, inst=1)
    plateaus = _replay_alns(inst.A, inst.b, inst.D, inst.x0, res, iters, ls_moves, radius, count, seed, 1)
    # the case that tells '<' from '<=': a best move that only EQUALS the current error was refused
    assert plateaus > 0
    assert 0 < res.moves.sum() and res.moves.max() <= ls_moves


def test_neighbourhood_radius_of_the_local_search_changes_the_run():
    """ls_radius = 1 tries the two neighbouring levels only (the paper's 1-OPT), 0 every level:
    on this instance a jump of more than one level is the best move somewhere, so the runs part."""
    inst = random_dense(620, 16, 9, 5, integer=True)
    near = orc.alns_dense(inst.A, inst.b, inst.D, inst.x0, orc.alns_params(40, ls_moves=6, ls_radius=1, destroy_count=2, seed=4), inst=1)
    far = orc.alns_dense(inst.A, inst.b, inst.D, inst.x0, orc.alns_params(40, ls_moves=6, ls_radius=0, destroy_count=2, seed=4), inst=1)
    assert not (np.array_equal(near.t, far.t) and np.array_equal(near.moves, far.moves))


def test_loop_with_a_scale_replays_on_the_scaled_matrix():
    inst = random_dense(621, 14, 8, 4, integer=True)
    iters, ls_moves, count, seed, s = 25, 4, 2, 12, 0.5
    prm = orc.alns_params(iters, ls_moves=ls_moves, ls_radius=1, destroy_count=count, seed=seed)
    res = orc.alns_dense(inst.A, inst.b, inst.D, inst.x0, prm, inst=6, scale=s)
    _replay_alns(inst.A, inst.b, inst.D, inst.x0, res, iters, ls_moves, 1, count, seed, 6, s=s)
    assert res.t_best == np.abs((inst.A * s) @ res.x - inst.b).max()


@pytest.mark.parametrize("n,count", [(199, 1), (200, 1), (201, 2), (1000, 5), (7, 1)])
def test_default_destroy_count_is_half_a_percent_rounded_up(n, count):
    """Appendix F: 0.5 % of the variables are unassigned; read as ceil(0.005 n), at least one.
    With no local search the error after the first iteration is that of x0 with exactly that many
    variables reassigned, which the replay checks (the replay asserts the number of draws)."""
    assert count == max(1, math.ceil(n * 5 / 1000))
    inst = random_dense(630 + n, 6, n, 4, integer=True)
    prm = orc.alns_params(3, ls_moves=0, ls_radius=1, destroy_count=0, seed=2)
    res = orc.alns_dense(inst.A, inst.b, inst.D, inst.x0, prm)
    _replay_alns(inst.A, inst.b, inst.D, inst.x0, res, 3, 0, 1, count, 2, 0)
    if count > 1:
        # one draw fewer gives another error after the first iteration: the count is visible
        with pytest.raises(AssertionError):
            _replay_alns(inst.A, inst.b, inst.D, inst.x0, res, 3, 0, 1, count - 1, 2, 0)


def test_impact_weights_of_a_vanishing_error():
    """Reading (the paper does not treat it): when the largest violation is below 2^-900 the
    fixed-point scale 2^24 / 2^e would leave the double range, and every variable gets weight 1
    (uniform draws).  From 2^-899 on the formula applies: an entry on a row that attains the
    error has slack 0 and adds trunc(t 2^24 / 2^e) = 2^23."""
    A = np.array([[1.0, 0.0], [0.0, 2.0], [1.0, 1.0]])
    rowptr, col, val = orc.full_csr(A)
    for e, uniform in ((-901, True), (-950, True), (-1074, True), (-899, False), (-850, False)):
        r = np.array([2.0 ** e, 0.0, 0.0])
        w = orc.alns_impact_weights(3, 2, rowptr, col, val, r, alpha=0.3)
        if uniform:
            assert w.tolist() == [1, 1], e
        else:
            assert w.tolist() == [1 + 2 ** 23, 1], e
