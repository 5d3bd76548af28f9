"""The l2 change of every candidate move and the arg-min with it as second criterion
(options.l2_rule), HIP library against the CPU oracle, bit for bit: the chains g_j = a_j . r and
c_j = ||a_j||^2 are fixed in order, and on fp32 batches the matrix-core kernel (one row of the
contraction per instruction) must keep them."""
import numpy as np
import pytest
import torch

from oracle import oracle as orc
from workloads import make_config, random_batched, random_dense, random_sparse

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


def dmmv():
    from paper_2508_13437_amd import dmmv as mod
    return mod


def T(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def N(t):
    return t.detach().cpu().numpy()


def oracle_dq(inst, x, r, q=None):
    if inst.kind == "csr":
        return orc.l2_changes_csr(inst.m, inst.n, inst.csr_rowptr, inst.csr_col, inst.csr_val, inst.D, x, r)
    if inst.kind == "batched":
        return orc.l2_changes_dense(inst.A, inst.D, x, r, scale=float(inst.scale[q]))
    return orc.l2_changes_dense(inst.A, inst.D, x, r)


def oracle_solve(inst, iters, rule, q=None, radius=0):
    if inst.kind == "csr":
        return orc.solve_l2_csr(inst.m, inst.n, inst.csr_rowptr, inst.csr_col, inst.csr_val, inst.b, inst.D, inst.x0,
                                iters, rule=rule, radius=radius)
    if inst.kind == "batched":
        return orc.solve_l2_dense(inst.A, inst.b[q], inst.D, inst.x0[q], iters, rule=rule, scale=float(inst.scale[q]),
                                  radius=radius)
    return orc.solve_l2_dense(inst.A, inst.b, inst.D, inst.x0, iters, rule=rule, radius=radius)


def check_tables(inst, steps=2):
    """dmmv_l2_changes against the oracle at the start and after a few moves of the plain descent."""
    m = dmmv()
    with m.from_instance(inst, DEV, l2_rule=3) as h:
        m.dmmv_set_x(h, T(inst.x0))
        m.dmmv_residual(h)
        for step in range(steps + 1):
            x, r, t = (N(a) for a in m.dmmv_get_state(h))
            got = N(m.dmmv_l2_changes(h))
            if inst.kind == "batched":
                for q in range(inst.R):
                    assert np.array_equal(got[q], oracle_dq(inst, x[q], r[q], q)), (inst.name, step, q)
            else:
                assert np.array_equal(got, oracle_dq(inst, x, r)), (inst.name, step)
            mv, _ = m.dmmv_argmin_move(h, None)          # l2_rule = 3: the plain arg-min
            m.dmmv_apply_move(h, mv)


def check_descent(inst, iters, rule, **opt):
    m = dmmv()
    radius = opt.get("radius", 0)
    with m.from_instance(inst, DEV, l2_rule=rule, **opt) as h:
        res = m.dmmv_solve(h, T(inst.x0), iters, trace=True)
        x, r, t = (N(a) for a in m.dmmv_get_state(h))
    tr, tt, done = N(res.trace), N(res.trace_t), N(res.iters_done)
    moved = 0
    for q in range(inst.R):
        o = oracle_solve(inst, iters, rule, q if inst.kind == "batched" else None, radius)
        d = int(done[q])
        assert d == o.iters_done, (inst.name, rule, q, d, o.iters_done)
        assert np.array_equal(tr[q, :d, 0], o.trace_j) and np.array_equal(tr[q, :d, 1], o.trace_k), (inst.name, rule, q)
        assert np.array_equal(tt[q, :d], o.trace_t) and np.all(tr[q, d:] == -1)
        xq = x[q] if inst.kind == "batched" else x
        rq = r[q] if inst.kind == "batched" else r
        assert np.array_equal(xq, o.x) and np.array_equal(rq, o.r) and t[q] == o.t
        moved += d
    return moved


@pytest.mark.parametrize("dtype", [np.float64, np.float32])
def test_l2_tables_dense_and_sparse(dtype):
    for shape in [(1, 1, 2), (37, 11, 5), (300, 40, 16), (1000, 6, 37)]:
        check_tables(random_dense(3000 + shape[0], *shape, dtype=dtype))
    check_tables(random_dense(3010, 40, 9, 4, dtype=dtype, integer=True))
    for mm, nn, nd, dens in [(1, 1, 2, 1.0), (70, 40, 4, 0.1), (200, 150, 3, 0.05), (2100, 64, 3, 0.02)]:
        check_tables(random_sparse(3020 + mm, mm, nn, nd, density=dens, dtype=dtype))
    inst = random_sparse(3030, 150, 60, 4, density=0.2, dtype=dtype)
    m = dmmv()
    with m.from_instance(inst, DEV, l2_rule=3, sparse_partition_rows=64) as h:       # several partitions
        m.dmmv_set_x(h, T(inst.x0))
        r = N(m.dmmv_residual(h))
        assert np.array_equal(N(m.dmmv_l2_changes(h)), oracle_dq(inst, inst.x0, r))


@pytest.mark.parametrize("shape", [(1, 1, 1, 2), (17, 5, 3, 3), (64, 64, 64, 4), (100, 33, 65, 8), (130, 70, 130, 16),
                                   (257, 129, 200, 16), (300, 200, 129, 8), (70, 300, 40, 4)])
def test_l2_tables_batched_matrix_cores_keep_the_chain(shape):
    """fp32 batches: G = X^T R on the matrix cores, one row of the contraction per instruction."""
    mm, nn, R, nd = shape
    print("l2 batched", shape, flush=True)
    check_tables(random_batched(3100 + mm + nn, mm, nn, R, nd), steps=1)


def test_l2_tables_batched_f64_and_integer():
    check_tables(random_batched(3200, 60, 24, 20, 5, dtype=np.float64), steps=1)
    check_tables(random_batched(3201, 40, 16, 70, 5, integer=True), steps=2)


@pytest.mark.parametrize("rule", [1, 2])
def test_l2_descent_dense(rule):
    moved = 0
    for seed in range(4):                                   # integer data: exact ties, the second criterion decides
        moved += check_descent(random_dense(3300 + seed, 37, 11, 5, dtype=[np.float64, np.float32][seed % 2], integer=True), 40, rule)
    moved += check_descent(random_dense(3310, 300, 40, 16, dtype=np.float64), 30, rule)
    moved += check_descent(random_dense(3311, 700, 20, 6, dtype=np.float32), 30, rule, radius=1)
    assert moved > 20


@pytest.mark.parametrize("rule", [1, 2])
def test_l2_descent_sparse(rule):
    moved = 0
    moved += check_descent(random_sparse(3400, 120, 90, 3, density=0.1), 60, rule)
    moved += check_descent(random_sparse(3401, 60, 50, 4, density=0.15, dtype=np.float64, integer=True), 40, rule)
    moved += check_descent(random_sparse(3402, 600, 200, 3, density=0.03), 50, rule, sparse_partition_rows=100)
    moved += check_descent(make_config(3, "small"), 40, rule)
    for mode in (1, 2):
        moved += check_descent(random_sparse(3403, 300, 120, 4, density=0.08), 30, rule, sparse_eval=mode)
    assert moved > 20


@pytest.mark.parametrize("rule", [1, 2])
def test_l2_descent_batched(rule):
    moved = 0
    moved += check_descent(random_batched(3500, 40, 16, 20, 5, integer=True), 25, rule)
    moved += check_descent(random_batched(3501, 100, 33, 65, 8), 12, rule)
    moved += check_descent(random_batched(3502, 30, 12, 9, 4, dtype=np.float64), 12, rule)
    moved += check_descent(make_config(4, "small"), 10, rule)
    assert moved > 20


def test_l2_rule_changes_the_descent_and_standalone_argmin_agrees():
    """On integer data the plain rule (lowest index) and the second criterion part ways; the
    standalone arg-min of a handle with the rule names the move the loop takes first."""
    m = dmmv()
    differs = 0
    for seed in range(6):
        inst = random_dense(3600 + seed, 12, 8, 4, integer=True)
        plain = orc.solve_dense(inst.A, inst.b, inst.D, inst.x0, 30)
        o = orc.solve_l2_dense(inst.A, inst.b, inst.D, inst.x0, 30, rule=1)
        differs += int(not np.array_equal(plain.trace_j, o.trace_j) or not np.array_equal(plain.trace_k, o.trace_k))
        with m.from_instance(inst, DEV, l2_rule=1) as h:
            m.dmmv_set_x(h, T(inst.x0))
            r = N(m.dmmv_residual(h))
            scores = m.dmmv_eval_moves(h)
            want_c, want_s = orc.argmin_move_l2(N(scores), orc.l2_changes_dense(inst.A, inst.D, inst.x0, r), 1)
            for given in (scores, None):
                mv, ms = m.dmmv_argmin_move(h, given)
                assert tuple(N(mv)[0]) == (want_c // inst.nd, want_c % inst.nd) and N(ms)[0] == want_s
            if o.iters_done:
                assert (o.trace_j[0], o.trace_k[0]) == (want_c // inst.nd, want_c % inst.nd)
    assert differs > 0


def test_l2_errors():
    m = dmmv()
    inst = random_dense(3700, 10, 4, 3)
    with m.from_instance(inst, DEV) as h:
        m.dmmv_set_x(h, T(inst.x0))
        m.dmmv_residual(h)
        with pytest.raises(m.DmmvError) as e:
            m.dmmv_l2_changes(h)
        assert e.value.status == -7
    with pytest.raises(m.DmmvError) as e:
        m.from_instance(inst, DEV, l2_rule=4)
    assert e.value.status == -2
    with m.from_instance(inst, DEV, l2_rule=1) as h:
        m.dmmv_set_x(h, T(inst.x0))
        with pytest.raises(m.DmmvError) as e:
            m.dmmv_l2_changes(h)                          # no residual yet
        assert e.value.status == -7


@pytest.mark.timeout(600)
def test_l2_full_size_layer_sampled_instances():
    """G = X^T R for the whole full-size layer on the matrix cores; a seeded sample of instances
    against the oracle's chains, and a few iterations of the descent with the second criterion."""
    m = dmmv()
    inst = make_config(4)
    sel = np.sort(np.random.default_rng(600).choice(inst.R, size=6, replace=False))
    with m.from_instance(inst, DEV, l2_rule=1) as h:
        m.dmmv_set_x(h, T(inst.x0))
        r = N(m.dmmv_residual(h))
        dq = m.dmmv_l2_changes(h)
        for q in sel:
            assert np.array_equal(N(dq[q]), orc.l2_changes_dense(inst.A, inst.D, inst.x0[q], r[q], scale=float(inst.scale[q]))), q
        del dq
        iters = 3
        res = m.dmmv_solve(h, T(inst.x0), iters, trace=True)
        tr, tt, done = N(res.trace), N(res.trace_t), N(res.iters_done)
    for q in sel[:3]:
        o = orc.solve_l2_dense(inst.A, inst.b[q], inst.D, inst.x0[q], iters, rule=1, scale=float(inst.scale[q]))
        d = int(done[q])
        assert d == o.iters_done and np.array_equal(tr[q, :d, 0], o.trace_j) and np.array_equal(tr[q, :d, 1], o.trace_k)
        assert np.array_equal(tt[q, :d], o.trace_t)
