"""Parity of the HIP library (through its C ABI) against the CPU oracle, element by element.

Bar: the arithmetic contract fixes every rounding (one fma per pair, fixed residual order),
so score tables, move traces, final x and max violation must be bitwise equal, fp32 and fp64.
"""
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


def oracle_solve(inst, iters, x0=None, **opt):
    x0 = inst.x0 if x0 is None else x0
    if inst.kind == "dense":
        return orc.solve_dense(inst.A, inst.b, inst.D, x0, iters, **opt)
    if inst.kind == "csr":
        return orc.solve_csr(inst.m, inst.n, inst.csr_rowptr, inst.csr_col, inst.csr_val, inst.b,
                             inst.D, x0, iters, **opt)
    return orc.solve_batched(inst.A, inst.b, inst.D, inst.scale, x0, iters, **opt)


def oracle_residual(inst, x):
    if inst.kind == "dense":
        return orc.residual_dense(inst.A, inst.b, inst.D, x)
    return orc.residual_csr(inst.m, inst.csr_rowptr, inst.csr_col, inst.csr_val, inst.b, inst.D, x)


def oracle_table(inst, x, r, **opt):
    if inst.kind == "dense":
        return orc.eval_moves_dense(inst.A, inst.D, x, r, **opt)
    return orc.eval_moves_csr(inst.m, inst.n, inst.csr_rowptr, inst.csr_col, inst.csr_val, inst.D,
                              x, r, method="plain", **opt)


def check_single_trace(res, o, iters):
    d = int(res.iters_done[0])
    assert d == o.iters_done
    tr = N(res.trace)[0]
    assert np.array_equal(tr[:d, 0], o.trace_j) and np.array_equal(tr[:d, 1], o.trace_k)
    assert np.all(tr[d:] == -1)
    assert np.array_equal(N(res.trace_t)[0, :d], o.trace_t)
    assert np.array_equal(N(res.x).reshape(-1), o.x)
    assert N(res.max_violation)[0] == o.t


def stepwise_check(inst, steps=4, **opt):
    """Every entry point against the oracle, a few moves deep."""
    m = dmmv()
    vm = opt.get("var_mask")
    hopt = dict(radius=opt.pop("radius", 0))
    opt["radius"] = hopt["radius"]
    for key in ("sparse_partition_rows", "sparse_eval"):
        if key in opt:
            hopt[key] = opt.pop(key)
    if vm is not None:
        hopt["var_mask"] = T(vm)
    with m.from_instance(inst, DEV, **hopt) as h:
        x = inst.x0.copy()
        m.dmmv_set_x(h, T(x))
        r_gpu = N(m.dmmv_residual(h))
        r = oracle_residual(inst, x)
        assert np.array_equal(r_gpu, r)
        for _ in range(steps):
            want = oracle_table(inst, x, r, **opt)
            got = N(m.dmmv_eval_moves(h))
            assert np.array_equal(got, want)
            c, s = orc.argmin_move(want)
            mv, ms = m.dmmv_argmin_move(h, T(want))
            assert tuple(N(mv)[0]) == (c // inst.nd, c % inst.nd) and N(ms)[0] == s
            mv2, ms2 = m.dmmv_argmin_move(h, None)          # fused evaluation + reduction
            assert tuple(N(mv2)[0]) == (c // inst.nd, c % inst.nd) and N(ms2)[0] == s
            xs, rs, ts = m.dmmv_get_state(h)
            assert np.array_equal(N(xs), x) and np.array_equal(N(rs), r)
            assert N(ts)[0] == orc.max_abs(r)
            j, k = c // inst.nd, c % inst.nd
            m.dmmv_apply_move(h, mv)
            if inst.kind == "dense":
                x, r, t = orc.apply_move_dense(inst.A, inst.D, x, r, j, k)
            else:
                x, r, t = orc.apply_move_csr(inst.m, inst.n, inst.csr_rowptr, inst.csr_col,
                                             inst.csr_val, inst.D, x, r, j, k)
            xs, rs, ts = m.dmmv_get_state(h)
            assert np.array_equal(N(xs), x) and np.array_equal(N(rs), r) and N(ts)[0] == t


# ------------------------------------------------------------------------------ dense
@pytest.mark.parametrize("dtype", [np.float64, np.float32])
@pytest.mark.parametrize("shape", [(1, 1, 2), (5, 3, 2), (63, 7, 3), (64, 9, 4), (65, 5, 5),
                                   (257, 13, 9), (300, 40, 16), (1000, 6, 37), (130, 4, 200)])
def test_dense_stepwise(shape, dtype):
    mm, nn, nd = shape
    stepwise_check(random_dense(10 + mm, mm, nn, nd, dtype=dtype), steps=3)


@pytest.mark.parametrize("dtype", [np.float64, np.float32])
@pytest.mark.parametrize("seed", range(4))
def test_dense_integer_ties(seed, dtype):
    """Small-integer data: exact ties are frequent, the lowest-index rule decides."""
    inst = random_dense(50 + seed, 37, 11, 5, dtype=dtype, integer=True)
    stepwise_check(inst, steps=4)
    with dmmv().from_instance(inst, DEV) as h:
        res = dmmv().dmmv_solve(h, T(inst.x0), 40, trace=True)
    check_single_trace(res, oracle_solve(inst, 40), 40)


@pytest.mark.parametrize("dtype", [np.float64, np.float32])
def test_dense_solve_long_trace(dtype):
    inst = random_dense(77, 700, 48, 16, dtype=dtype)
    with dmmv().from_instance(inst, DEV, poll_every=7) as h:
        res = dmmv().dmmv_solve(h, T(inst.x0), 150, trace=True)
        o = oracle_solve(inst, 150)
        assert o.iters_done >= 15
        check_single_trace(res, o, 150)
        x, r, t = dmmv().dmmv_get_state(h)
        assert np.array_equal(N(r), o.r)
        # the maintained t equals a fresh max |r| of the maintained residual
        assert N(t)[0] == np.abs(o.r).max()
        # resuming from the result does nothing more
        assert o.iters_done < 150
        res2 = dmmv().dmmv_solve(h, res.x, 10, trace=True)
        assert int(res2.iters_done[0]) == 0 and N(res2.max_violation)[0] == o.t


@pytest.mark.parametrize("dtype", [np.float64, np.float32])
def test_dense_tall_matrix_several_row_chunks(dtype):
    """More rows than one staged chunk and than the fused select+apply handles."""
    inst = random_dense(31, 40001, 3, 5, dtype=dtype)
    stepwise_check(inst, steps=2)
    with dmmv().from_instance(inst, DEV) as h:
        res = dmmv().dmmv_solve(h, T(inst.x0), 12, trace=True)
    check_single_trace(res, oracle_solve(inst, 12), 12)
    inst = random_dense(32, 9000, 2, 70, dtype=dtype)      # several value tiles, two chunks (f64)
    stepwise_check(inst, steps=2)


def test_dense_radius_and_mask():
    inst = random_dense(91, 90, 17, 9, dtype=np.float64)
    rng = np.random.default_rng(3)
    vm = (rng.uniform(size=inst.n) < 0.5).astype(np.uint8)
    for radius in (1, 2):
        stepwise_check(inst, steps=2, radius=radius, var_mask=vm)
        with dmmv().from_instance(inst, DEV, radius=radius, var_mask=T(vm)) as h:
            res = dmmv().dmmv_solve(h, T(inst.x0), 30, trace=True)
        check_single_trace(res, oracle_solve(inst, 30, radius=radius, var_mask=vm), 30)


def test_dense_keep_going_reports_same_result():
    inst = random_dense(5, 120, 10, 4, dtype=np.float64)
    o = oracle_solve(inst, 60)
    assert o.iters_done < 60
    with dmmv().from_instance(inst, DEV, keep_going=True) as h:
        res = dmmv().dmmv_solve(h, T(inst.x0), 60, trace=True)
    check_single_trace(res, o, 60)


def test_deterministic_repeat():
    inst = random_dense(123, 500, 33, 16, dtype=np.float32)
    outs = []
    for _ in range(2):
        with dmmv().from_instance(inst, DEV) as h:
            res = dmmv().dmmv_solve(h, T(inst.x0), 50, trace=True)
            outs.append((N(res.trace).copy(), N(res.trace_t).copy(), N(res.x).copy()))
    for a, b in zip(outs[0], outs[1]):
        assert np.array_equal(a, b)


# ------------------------------------------------------------------------------ sparse
@pytest.mark.parametrize("dtype", [np.float32, np.float64])
@pytest.mark.parametrize("shape", [(1, 1, 2, 1.0), (20, 9, 3, 0.3), (33, 12, 3, 0.9),
                                   (70, 40, 4, 0.1), (200, 150, 3, 0.05), (129, 31, 11, 0.2),
                                   (2100, 64, 3, 0.02)])
def test_sparse_stepwise(shape, dtype):
    mm, nn, nd, dens = shape
    stepwise_check(random_sparse(20 + mm, mm, nn, nd, density=dens, dtype=dtype), steps=3)


@pytest.mark.parametrize("rows", [1, 7, 64, 1000])
def test_sparse_row_partitions(rows):
    """Several LDS partitions of r (forced small): results must not depend on the cut."""
    inst = random_sparse(555, 150, 60, 4, density=0.2, dtype=np.float32)
    stepwise_check(inst, steps=3, sparse_partition_rows=rows)
    inst = random_sparse(556, 90, 25, 3, density=0.5, dtype=np.float64, integer=True)
    stepwise_check(inst, steps=3, sparse_partition_rows=rows)
    with dmmv().from_instance(inst, DEV, sparse_partition_rows=rows) as h:
        res = dmmv().dmmv_solve(h, T(inst.x0), 30, trace=True)
    check_single_trace(res, oracle_solve(inst, 30), 30)


def test_sparse_long_columns_and_many_groups():
    """Columns longer than two wavefront loads, and more rows than one top-K group."""
    inst = random_sparse(557, 5000, 20, 3, density=0.3, dtype=np.float32)
    stepwise_check(inst, steps=2)
    stepwise_check(inst, steps=2, sparse_partition_rows=700)
    # more than 32 groups: the candidate list needs a reduction pass before the merge
    inst = random_sparse(558, 70000, 12, 3, density=0.01, dtype=np.float32)
    stepwise_check(inst, steps=2)


@pytest.mark.parametrize("seed", range(3))
def test_sparse_integer_ties_and_full_columns(seed):
    """Dense-ish columns over few rows: columns that contain every listed top row force the
    exact outside-the-column scan; integer data gives exact ties."""
    inst = random_sparse(300 + seed, 45, 14, 3, density=0.85, dtype=np.float32, integer=True,
                         explicit_zeros=True)
    stepwise_check(inst, steps=4)
    with dmmv().from_instance(inst, DEV) as h:
        res = dmmv().dmmv_solve(h, T(inst.x0), 40, trace=True)
    check_single_trace(res, oracle_solve(inst, 40), 40)


def test_sparse_all_rows_in_one_column_beyond_list():
    """m > list length and one column holding every row: no outside rows at all."""
    mm, nn = 80, 3
    rows = np.arange(mm)
    rowptr = np.arange(mm + 1, dtype=np.int64)
    col = np.zeros(mm, dtype=np.int32)
    rng = np.random.default_rng(0)
    inst = random_sparse(1, mm, nn, 3, density=0.0, dtype=np.float32)
    inst.csr_rowptr, inst.csr_col = rowptr, col
    inst.csr_val = rng.standard_normal(mm).astype(np.float32)
    assert rows.size == inst.csr_val.size
    stepwise_check(inst, steps=2)


@pytest.mark.parametrize("density,nn", [(1.0, 5), (1.0, 100), (0.97, 70)])
def test_sparse_columns_holding_all_large_rows(density, nn):
    """More rows than the reservoir holds and columns that contain every reservoir row: the
    outside maximum needs the walk past the inline list and the exact scan; with 100 such
    columns the per-workgroup list of deferred columns overflows into the rescan path."""
    inst = random_sparse(900 + nn, 333, nn, 3, density=density, dtype=np.float32)
    stepwise_check(inst, steps=2)
    stepwise_check(inst, steps=2, sparse_partition_rows=100)
    with dmmv().from_instance(inst, DEV) as h:
        res = dmmv().dmmv_solve(h, T(inst.x0), 25, trace=True)
    check_single_trace(res, oracle_solve(inst, 25), 25)


def test_sparse_long_descent_reservoir_maintenance():
    """A few hundred moves on a matrix with far more rows than the reservoir: the sorted
    reservoir is updated incrementally after every move, drained, rebuilt and truncated."""
    inst = random_sparse(977, 6000, 400, 5, density=0.02, dtype=np.float32)
    rng = np.random.default_rng(5)
    x0 = rng.choice(inst.D, size=inst.n).astype(np.float32)
    for rows in (0, 2500):
        with dmmv().from_instance(inst, DEV, sparse_partition_rows=rows) as h:
            res = dmmv().dmmv_solve(h, T(x0), 400, trace=True)
            o = oracle_solve(inst, 400, x0=x0)
            assert o.iters_done > 100
            check_single_trace(res, o, 400)
            x, r, t = dmmv().dmmv_get_state(h)
            assert np.array_equal(N(r), o.r)
            # the table of the final state still matches (reservoir consistent with r)
            assert np.array_equal(N(dmmv().dmmv_eval_moves(h)), oracle_table(inst, o.x, o.r))


@pytest.mark.parametrize("mode", [1, 2])
def test_sparse_both_evaluation_kernels(mode):
    """options.sparse_eval forces the two-kernel path (1: per-partition maxima + combine) or the
    one-kernel path (2: a workgroup walks every partition): each must give the oracle's tables,
    arg-min records and traces on its own, whatever the automatic choice would be - ragged shapes,
    forced and misaligned partition sizes, several value tiles, long columns, columns that hold
    every large row, masks and radius, both precisions."""
    m = dmmv()
    for mm, nn, nd, dens, dtype in [(1, 1, 2, 1.0, np.float32), (20, 9, 3, 0.3, np.float64), (33, 12, 3, 0.9, np.float32),
                                    (200, 150, 3, 0.05, np.float32), (129, 31, 11, 0.2, np.float64),
                                    (2100, 300, 3, 0.02, np.float32), (300, 700, 20, 0.03, np.float32)]:
        stepwise_check(random_sparse(20 + mm, mm, nn, nd, density=dens, dtype=dtype), steps=2, sparse_eval=mode)
    # the one-kernel path takes at most 16 partitions; 10 and 13 rows also give partitions that
    # do not start on 16 bytes
    for rows in ((1, 7, 64, 1000) if mode == 1 else (10, 13, 64, 1000)):
        inst = random_sparse(555, 150, 60, 4, density=0.2, dtype=np.float32)
        stepwise_check(inst, steps=2, sparse_partition_rows=rows, sparse_eval=mode)
        inst = random_sparse(556, 90, 25, 3, density=0.5, dtype=np.float64, integer=True)
        stepwise_check(inst, steps=2, sparse_partition_rows=rows, sparse_eval=mode)
        with m.from_instance(inst, DEV, sparse_partition_rows=rows, sparse_eval=mode) as h:
            res = m.dmmv_solve(h, T(inst.x0), 30, trace=True)
        check_single_trace(res, oracle_solve(inst, 30), 30)
    inst = random_sparse(557, 5000, 20, 3, density=0.3, dtype=np.float32)          # long columns
    stepwise_check(inst, steps=2, sparse_eval=mode)
    stepwise_check(inst, steps=2, sparse_partition_rows=700, sparse_eval=mode)
    stepwise_check(random_sparse(558, 70000, 12, 3, density=0.01, dtype=np.float32), steps=2, sparse_eval=mode)
    for seed in range(2):                                                           # ties, full columns
        inst = random_sparse(300 + seed, 45, 14, 3, density=0.85, dtype=np.float32, integer=True, explicit_zeros=True)
        stepwise_check(inst, steps=3, sparse_eval=mode)
    for density, nn in [(1.0, 5), (1.0, 100), (0.97, 70)]:                          # columns holding all large rows
        inst = random_sparse(900 + nn, 333, nn, 3, density=density, dtype=np.float32)
        stepwise_check(inst, steps=2, sparse_eval=mode)
        stepwise_check(inst, steps=2, sparse_partition_rows=100, sparse_eval=mode)
    inst = random_sparse(910, 260, 90, 9, density=0.1, dtype=np.float32)            # mask and radius
    vm = (np.random.default_rng(3).uniform(size=inst.n) < 0.6).astype(np.uint8)
    stepwise_check(inst, steps=2, radius=1, var_mask=vm, sparse_eval=mode)
    inst = random_sparse(977, 6000, 400, 5, density=0.02, dtype=np.float32)         # long descent
    x0 = np.random.default_rng(5).choice(inst.D, size=inst.n).astype(np.float32)
    o = oracle_solve(inst, 400, x0=x0)
    for rows, keep in ((0, False), (2500, True)):
        with m.from_instance(inst, DEV, sparse_partition_rows=rows, sparse_eval=mode, keep_going=keep) as h:
            res = m.dmmv_solve(h, T(x0), 400, trace=True)
            check_single_trace(res, o, 400)
            assert np.array_equal(N(m.dmmv_eval_moves(h)), oracle_table(inst, o.x, o.r))
    inst = make_config(3, "small")
    with m.from_instance(inst, DEV, sparse_eval=mode) as h:
        res = m.dmmv_solve(h, T(inst.x0), inst.iters, trace=True)
    check_single_trace(res, oracle_solve(inst, inst.iters), inst.iters)
    if mode == 2:
        with pytest.raises(m.DmmvError) as e:                 # 150 partitions: refused, not mis-run
            m.from_instance(random_sparse(555, 150, 60, 4, density=0.2), DEV, sparse_partition_rows=1, sparse_eval=2)
        assert e.value.status == -8


def test_sparse_solve_small_tomography():
    inst = make_config(3, "small")
    with dmmv().from_instance(inst, DEV) as h:
        res = dmmv().dmmv_solve(h, T(inst.x0), inst.iters, trace=True)
    o = oracle_solve(inst, inst.iters)
    assert o.iters_done >= 10
    check_single_trace(res, o, inst.iters)


def test_sparse_unsorted_rows_and_errors():
    m = dmmv()
    inst = random_sparse(9, 30, 12, 3, density=0.4, dtype=np.float32)
    # shuffle the entries inside each row: the result must not change (scores do not depend
    # on the order; the residual follows the stored order, so compare tables for a given r)
    rng = np.random.default_rng(1)
    col, val = inst.csr_col.copy(), inst.csr_val.copy()
    for i in range(inst.m):
        a, b = inst.csr_rowptr[i], inst.csr_rowptr[i + 1]
        p = rng.permutation(b - a)
        col[a:b], val[a:b] = col[a:b][p], val[a:b][p]
    r = oracle_residual(inst, inst.x0)
    want = oracle_table(inst, inst.x0, r)
    with m.Handle(D=inst.D, b=T(inst.b), csr=(T(inst.csr_rowptr), T(col), T(val)), m=inst.m,
                  n=inst.n) as h:
        m.dmmv_set_x(h, T(inst.x0))
        m.dmmv_set_residual(h, T(r))
        assert np.array_equal(N(m.dmmv_eval_moves(h)), want)
    # duplicate entry
    col2 = inst.csr_col.copy()
    a, b = inst.csr_rowptr[0], inst.csr_rowptr[1]
    row0 = next(i for i in range(inst.m) if inst.csr_rowptr[i + 1] - inst.csr_rowptr[i] >= 2)
    a = inst.csr_rowptr[row0]
    col2[a + 1] = col2[a]
    with pytest.raises(m.DmmvError) as e:
        m.Handle(D=inst.D, b=T(inst.b), csr=(T(inst.csr_rowptr), T(col2), T(inst.csr_val)),
                 m=inst.m, n=inst.n)
    assert e.value.status == -2
    # column out of range
    col3 = inst.csr_col.copy()
    col3[0] = inst.n
    with pytest.raises(m.DmmvError) as e:
        m.Handle(D=inst.D, b=T(inst.b), csr=(T(inst.csr_rowptr), T(col3), T(inst.csr_val)),
                 m=inst.m, n=inst.n)
    assert e.value.status == -2


# ------------------------------------------------------------------------------ batched
def batched_check(inst, iters, **hopt):
    m = dmmv()
    o = oracle_solve(inst, iters, radius=hopt.get("radius", 0))
    with m.from_instance(inst, DEV, **hopt) as h:
        res = m.dmmv_solve(h, T(inst.x0), iters, trace=True)
        assert np.array_equal(N(res.iters_done), o.iters_done)
        tr = N(res.trace)
        assert np.array_equal(tr[:, :, 0], o.trace_j) and np.array_equal(tr[:, :, 1], o.trace_k)
        assert np.array_equal(N(res.trace_t), o.trace_t)
        assert np.array_equal(N(res.x), o.x)
        assert np.array_equal(N(res.max_violation), o.t)
        # maintained residual vs fresh fp64 recomputation, and t == max |r|
        x, r, t = m.dmmv_get_state(h)
        r = N(r)
        assert np.array_equal(np.abs(r).max(axis=1), N(t))
        fresh = (inst.scale.astype(np.float64)[:, None] * o.x) @ inst.A.astype(np.float64).T - inst.b
        scale_mag = np.abs(inst.b).max() + 1.0
        assert np.abs(r - fresh).max() <= 1e-4 * scale_mag
    return o


@pytest.mark.parametrize("shape", [(1, 1, 1, 2), (17, 5, 3, 3), (64, 8, 64, 4), (100, 33, 65, 8),
                                   (130, 70, 130, 16), (50, 19, 7, 21)])
def test_batched_random(shape):
    mm, nn, R, nd = shape
    batched_check(random_batched(40 + mm, mm, nn, R, nd, dtype=np.float32), 12)


def test_batched_f64_and_integer_ties():
    batched_check(random_batched(8, 40, 12, 9, 5, dtype=np.float64), 10)
    batched_check(random_batched(9, 30, 10, 70, 4, dtype=np.float32, integer=True), 15)


@pytest.mark.parametrize("shape,dtype", [((8200, 7, 515, 5), np.float32), ((8195, 37, 600, 9), np.float32),
                                         ((8200, 6, 512, 4), np.float64), ((2100, 33, 600, 8), np.float32)])
def test_batched_residual_kernels_for_large_batches(shape, dtype):
    """Enough instances and rows for the residual kernels that large batches take (the LDS-tiled
    one from 256 instances and 512 workgroups on, the 32-rows-per-lane one below that): every
    element equals the oracle's sequential-order sum bit for bit, ragged edges included."""
    m = dmmv()
    mm, nn, R, nd = shape
    inst = random_batched(3000 + nn, mm, nn, R, nd, dtype=dtype)
    with m.from_instance(inst, DEV) as h:
        m.dmmv_set_x(h, T(inst.x0))
        r = N(m.dmmv_residual(h))
        x, r2, t = m.dmmv_get_state(h)
        assert np.array_equal(np.abs(r).max(axis=1), N(t))
    for q in list(range(0, R, 41)) + [R - 1]:
        rq = orc.residual_dense(inst.A, inst.b[q], inst.D, inst.x0[q], scale=inst.scale[q])
        assert np.array_equal(r[q], rq), q


def test_batched_stepwise_tables():
    m = dmmv()
    inst = random_batched(66, 75, 21, 67, 16, dtype=np.float32)
    with m.from_instance(inst, DEV) as h:
        m.dmmv_set_x(h, T(inst.x0))
        r = N(m.dmmv_residual(h))
        tab = N(m.dmmv_eval_moves(h))
        mv, ms = m.dmmv_argmin_move(h, None)
        mv_t, ms_t = m.dmmv_argmin_move(h, T(tab))
        assert np.array_equal(N(mv), N(mv_t)) and np.array_equal(N(ms), N(ms_t))
        for q in range(inst.R):
            rq = orc.residual_dense(inst.A, inst.b[q], inst.D, inst.x0[q], scale=inst.scale[q])
            assert np.array_equal(r[q], rq)
            want = orc.eval_moves_dense(inst.A, inst.D, inst.x0[q], rq, scale=inst.scale[q])
            assert np.array_equal(tab[q], want)
            c, s = orc.argmin_move(want)
            assert tuple(N(mv)[q]) == (c // inst.nd, c % inst.nd) and N(ms)[q] == s
        # apply a different move per instance, some skipped
        moves = N(mv).copy()
        moves[::3, 0] = -1
        m.dmmv_apply_move(h, T(moves))
        x2, r2, t2 = m.dmmv_get_state(h)
        for q in range(inst.R):
            if moves[q, 0] < 0:
                assert np.array_equal(N(r2)[q], r[q])
                continue
            xq, rq, tq = orc.apply_move_dense(inst.A, inst.D, inst.x0[q], r[q], moves[q, 0],
                                              moves[q, 1], scale=inst.scale[q])
            assert np.array_equal(N(r2)[q], rq) and N(t2)[q] == tq and np.array_equal(N(x2)[q], xq)


def test_batched_radius():
    batched_check(random_batched(12, 60, 14, 20, 8, dtype=np.float32), 10, radius=1)


@pytest.mark.parametrize("idx", [4, 5])
def test_batched_small_llm_configs(idx):
    inst = make_config(idx, "small")
    o = batched_check(inst, inst.iters)
    assert o.iters_done.sum() > inst.R


# ------------------------------------------------------------------------------ configs
def test_config1_dense_toy_full():
    inst = make_config(1)
    with dmmv().from_instance(inst, DEV) as h:
        res = dmmv().dmmv_solve(h, T(inst.x0), inst.iters, trace=True)
        check_single_trace(res, oracle_solve(inst, inst.iters), inst.iters)
        # a cold start gives a long trace on the same instance
        rng = np.random.default_rng(0)
        x0 = rng.choice(inst.D, size=inst.n)
        res = dmmv().dmmv_solve(h, T(x0), inst.iters, trace=True)
        o = oracle_solve(inst, inst.iters, x0=x0)
        assert o.iters_done >= 10
        check_single_trace(res, o, inst.iters)


def test_config2_fir_small_and_full_prefix():
    small = make_config(2, "small")
    rng = np.random.default_rng(0)
    x0 = rng.choice(small.D, size=small.n)
    with dmmv().from_instance(small, DEV) as h:
        res = dmmv().dmmv_solve(h, T(x0), small.iters, trace=True)
    check_single_trace(res, oracle_solve(small, small.iters, x0=x0), small.iters)
    inst = make_config(2)
    with dmmv().from_instance(inst, DEV) as h:
        res = dmmv().dmmv_solve(h, T(inst.x0), inst.iters, trace=True)
        check_single_trace(res, oracle_solve(inst, inst.iters), inst.iters)
        x0 = np.clip(inst.x0 + rng.integers(-40, 41, size=inst.n), inst.D[0], inst.D[-1])
        res = dmmv().dmmv_solve(h, T(x0), 12, trace=True)
        check_single_trace(res, oracle_solve(inst, 12, x0=x0), 12)


# ------------------------------------------------------------------------------ edges / errors
def test_empty_inputs():
    m = dmmv()
    D = np.array([0.0, 1.0])
    # no variables
    A = torch.zeros((5, 0), dtype=torch.float64, device=DEV)
    b = T(np.arange(5, dtype=np.float64))
    with m.Handle(A=A, b=b, D=D) as h:
        res = m.dmmv_solve(h, torch.zeros(0, dtype=torch.float64, device=DEV), 5, trace=True)
        assert int(res.iters_done[0]) == 0 and float(res.max_violation[0]) == 4.0
        mv, ms = m.dmmv_argmin_move(h, None)
        assert N(mv)[0, 0] == -1 and np.isinf(N(ms)[0])
    # no rows
    A = torch.zeros((0, 4), dtype=torch.float64, device=DEV)
    with m.Handle(A=A, b=torch.zeros(0, dtype=torch.float64, device=DEV), D=D) as h:
        x0 = T(np.array([0.0, 1.0, 1.0, 0.0]))
        res = m.dmmv_solve(h, x0, 5, trace=True)
        assert int(res.iters_done[0]) == 0 and float(res.max_violation[0]) == 0.0
        m.dmmv_set_x(h, x0)
        m.dmmv_residual(h)
        assert np.all(N(m.dmmv_eval_moves(h)) == 0.0)
    # zero iterations
    inst = random_dense(1, 10, 4, 3)
    with m.from_instance(inst, DEV) as h:
        res = m.dmmv_solve(h, T(inst.x0), 0, trace=True)
        assert int(res.iters_done[0]) == 0
        assert float(res.max_violation[0]) == np.abs(oracle_residual(inst, inst.x0)).max()


def test_error_paths():
    m = dmmv()
    inst = random_dense(2, 10, 4, 3)
    with pytest.raises(m.DmmvError) as e:
        m.Handle(A=T(inst.A), b=T(inst.b), D=inst.D[::-1].copy())
    assert e.value.status == -4
    with pytest.raises(m.DmmvError) as e:
        m.Handle(A=T(inst.A), b=T(inst.b), D=inst.D[:1])
    assert e.value.status == -4
    with m.from_instance(inst, DEV) as h:
        bad = inst.x0.copy()
        bad[2] = 99.0
        with pytest.raises(m.DmmvError) as e:
            m.dmmv_set_x(h, T(bad))
        assert e.value.status == -4
        with pytest.raises(m.DmmvError) as e:
            m.dmmv_eval_moves(h)            # no residual yet
        assert e.value.status == -7
        m.dmmv_set_x(h, T(inst.x0))
        m.dmmv_residual(h)
        with pytest.raises(m.DmmvError) as e:
            m.dmmv_apply_move(h, T(np.array([[inst.n, 0]], dtype=np.int32)))
        assert e.value.status == -2
        # still usable afterwards
        assert np.array_equal(N(m.dmmv_eval_moves(h)),
                              oracle_table(inst, inst.x0, oracle_residual(inst, inst.x0)))


# ------------------------------------------------------------------------------ full-size configs
def test_config3_tomography_full_prefix_and_sampled_scores():
    """Full 65 340 x 65 536 projection matrix: the first moves of the descent, and sampled
    columns of the score table against the definition (max over ALL rows)."""
    m = dmmv()
    inst = make_config(3)
    iters = 40
    with m.from_instance(inst, DEV) as h:
        res = m.dmmv_solve(h, T(inst.x0), iters, trace=True)
        o = oracle_solve(inst, iters)
        assert o.iters_done == iters
        check_single_trace(res, o, iters)
        x, r, t = m.dmmv_get_state(h)
        assert np.array_equal(N(r), o.r) and N(t)[0] == o.t
        tab = N(m.dmmv_eval_moves(h)).reshape(inst.n, inst.nd)
        # columns of the last moves (they hold the largest rows) plus a seeded sample
        rng = np.random.default_rng(7)
        cols = np.unique(np.concatenate([o.trace_j[-10:], rng.integers(0, inst.n, size=150)]))
        for j in cols:
            want = orc.eval_moves_csr(inst.m, inst.n, inst.csr_rowptr, inst.csr_col, inst.csr_val,
                                      inst.D, o.x, o.r, method="plain",
                                      columns=(int(j), int(j) + 1)).reshape(inst.n, inst.nd)[j]
            assert np.array_equal(tab[j], want), j
        # properties that hold for the whole table: null moves score t, nothing scores below
        # the largest |r| over the rows a column cannot touch (at least the 2nd largest overall)
        kidx = orc.values_to_index(o.x, inst.D)
        assert np.all(tab[np.arange(inst.n), kidx] == o.t)
        assert tab.min() >= 0


@pytest.mark.parametrize("prune", [False, True])
@pytest.mark.parametrize("idx,iters,sample", [(4, 3, 16), (5, 2, 8)])
def test_llm_configs_full_sampled_instances(idx, iters, sample, prune):
    """Full-size batched layer: every instance runs on the GPU (full evaluation, and the descent
    with exact pruning); a seeded sample of instances is replayed by the oracle and must match
    bitwise; all instances pass cheap checks."""
    m = dmmv()
    inst = make_config(idx)
    print("full-size batched case", idx, iters, sample, prune, flush=True)
    with m.from_instance(inst, DEV, prune=prune) as h:
        res = m.dmmv_solve(h, T(inst.x0), iters, trace=True)
        x = N(res.x)
        t = N(res.max_violation)
        done = N(res.iters_done)
        tr = N(res.trace)
        tt = N(res.trace_t)
        xs, r, ts = m.dmmv_get_state(h)
        r = N(r)
    rng = np.random.default_rng(idx)
    sel = np.sort(rng.choice(inst.R, size=sample, replace=False))
    o = orc.solve_batched(inst.A, inst.b[sel], inst.D, inst.scale[sel], inst.x0[sel], iters)
    assert np.array_equal(done[sel], o.iters_done)
    assert np.array_equal(tr[sel][:, :, 0], o.trace_j) and np.array_equal(tr[sel][:, :, 1], o.trace_k)
    assert np.array_equal(tt[sel], o.trace_t)
    assert np.array_equal(x[sel], o.x) and np.array_equal(t[sel], o.t)
    # every instance: x in D, t == max |maintained r|, traces strictly decreasing
    assert np.all(np.isin(x, inst.D))
    assert np.array_equal(np.abs(r).max(axis=1), t)
    for q in range(0, inst.R, 97):
        d = done[q]
        assert np.all(np.diff(tt[q, :d]) < 0)
        assert np.all(tr[q, d:] == -1)
    # sampled instances: maintained residual against a fresh fp64 recomputation
    X64 = inst.A.astype(np.float64)
    for q in sel[:4]:
        fresh = X64 @ (inst.scale[q].astype(np.float64) * x[q]) - inst.b[q]
        assert np.abs(r[q] - fresh).max() <= 1e-5 * max(1.0, np.abs(inst.b[q]).max())
        assert abs(t[q] - np.abs(fresh).max()) <= 1e-5 * np.abs(fresh).max()


# ------------------------------------------------------------- batched residual on the matrix cores
def mfma_residual_check(inst):
    """r from the matrix-core path against the fp64 definition, element by element.  The
    path's products are exact (bf16 planes of X times bf16-exact codes), so the error is
    that of an fp32 accumulation of n terms in some order plus the final fma."""
    m = dmmv()
    X64 = inst.A.astype(np.float64)
    with m.from_instance(inst, DEV, residual_mfma=True) as h:
        m.dmmv_set_x(h, T(inst.x0))
        r = N(m.dmmv_residual(h))
        _, r_state, t = m.dmmv_get_state(h)
        assert np.array_equal(N(r_state), r)
        assert np.array_equal(np.abs(r).max(axis=1) if inst.m else np.zeros(inst.R, r.dtype), N(t))
    ref = np.stack([orc.residual_dense(X64, inst.b[q].astype(np.float64), inst.D.astype(np.float64),
                                       inst.x0[q].astype(np.float64), scale=float(inst.scale[q]))
                    for q in range(inst.R)]) if inst.R else np.zeros((0, inst.m))
    mag = (np.abs(inst.scale.astype(np.float64))[:, None] * np.abs(inst.x0.astype(np.float64))) @ np.abs(X64).T \
        + np.abs(inst.b.astype(np.float64))
    tol = (inst.n + 2) * 2.0 ** -24 * mag + 1e-30
    err = np.abs(r.astype(np.float64) - ref)
    assert np.all(err <= tol), float((err / tol).max())
    return r


@pytest.mark.parametrize("shape", [(1, 1, 1, 2), (17, 5, 3, 3), (64, 64, 64, 4), (100, 33, 65, 8),
                                   (130, 70, 130, 16), (257, 129, 200, 16), (300, 200, 129, 8),
                                   # several 256 x 256 tiles: a ragged band of row tiles, more tiles than XCDs
                                   (520, 100, 515, 4), (1100, 70, 300, 3), (256, 64, 2305, 2)])
def test_batched_mfma_residual_random(shape):
    mm, nn, R, nd = shape
    print("mfma residual", shape, flush=True)
    mfma_residual_check(random_batched(4000 + mm + nn, mm, nn, R, nd))


def test_batched_mfma_residual_integer_data_is_exact():
    # small integers: every partial sum is exact in fp32, so any summation order gives the
    # sequential kernel's bits
    inst = random_batched(4100, 96, 40, 70, 5, integer=True)
    r = mfma_residual_check(inst)
    m = dmmv()
    with m.from_instance(inst, DEV) as h:
        m.dmmv_set_x(h, T(inst.x0))
        assert np.array_equal(N(m.dmmv_residual(h)), r)


@pytest.mark.parametrize("idx", [4, 5])
def test_batched_mfma_residual_small_llm_configs(idx):
    # cfg 5 has bf16-valued X (one plane), cfg 4 needs all three
    mfma_residual_check(make_config(idx, "small"))


def test_batched_mfma_solve_is_consistent():
    m = dmmv()
    inst = make_config(4, "small")
    iters = 12
    with m.from_instance(inst, DEV, residual_mfma=True) as h:
        res = m.dmmv_solve(h, T(inst.x0), iters, trace=True)
        x, r, t = m.dmmv_get_state(h)
        x, r, t = N(x), N(r), N(t)
        assert np.array_equal(np.abs(r).max(axis=1), t)
        assert np.array_equal(N(res.max_violation), t)
        tt = N(res.trace_t)
        for q in range(inst.R):
            d = int(res.iters_done[q])
            assert np.all(np.diff(tt[q, :d]) < 0)
        fresh = (inst.scale.astype(np.float64)[:, None] * x) @ inst.A.astype(np.float64).T - inst.b
        assert np.abs(r - fresh).max() <= 1e-4 * (np.abs(inst.b).max() + 1.0)
    # the sequential-order path ends within 1e-5 relative of it (same descent up to near-ties)
    with m.from_instance(inst, DEV) as h:
        res0 = m.dmmv_solve(h, T(inst.x0), iters)
        t0 = N(res0.max_violation)
    assert np.median(np.abs(t - t0) / t0) <= 1e-5


def test_batched_mfma_not_applicable_is_an_error():
    m = dmmv()
    inst = random_batched(4200, 20, 6, 4, 3)
    D_bad = inst.D.copy()
    D_bad[0] = np.float32(-1.0009765625) * 3                       # needs more than 8 significand bits
    with pytest.raises(m.DmmvError) as e:
        m.Handle(D=np.sort(D_bad), b=T(inst.b), A=T(inst.A.T).t(), scale=inst.scale, residual_mfma=True)
    assert e.value.status == -8
    d = random_dense(4201, 20, 6, 3, dtype=np.float32)
    with pytest.raises(m.DmmvError) as e:
        m.Handle(D=d.D, b=T(d.b), A=T(d.A.T).t(), residual_mfma=True)
    assert e.value.status == -8
    b64 = random_batched(4202, 20, 6, 4, 3, dtype=np.float64)
    with pytest.raises(m.DmmvError) as e:
        m.Handle(D=b64.D, b=T(b64.b), A=T(b64.A.T).t(), scale=b64.scale, residual_mfma=True)
    assert e.value.status == -8


# ------------------------------------------------------------- pruned descent on sparse matrices
@pytest.mark.parametrize("case", ["ties", "full_columns", "long", "tomography", "tiny", "one_column", "long_columns"])
def test_sparse_pruned_descent_applies_the_same_moves(case):
    """options.prune scores only the columns that touch the row of largest |r|; whenever an
    improving move exists it is among them, so the whole trace must equal the oracle's."""
    m = dmmv()
    x0 = None
    if case == "ties":
        inst, iters, kw = random_sparse(301, 45, 14, 3, density=0.85, dtype=np.float32, integer=True,
                                        explicit_zeros=True), 40, {}
    elif case == "full_columns":
        inst, iters, kw = random_sparse(970, 333, 70, 3, density=0.97, dtype=np.float32), 25, dict(sparse_partition_rows=100)
    elif case == "long":
        inst, iters, kw = random_sparse(977, 6000, 400, 5, density=0.02, dtype=np.float32), 400, dict(sparse_partition_rows=2500)
        x0 = np.random.default_rng(5).choice(inst.D, size=inst.n).astype(np.float32)
    elif case == "tomography":
        inst = make_config(3, "small")
        iters, kw = inst.iters, {}
    elif case == "long_columns":
        # columns of more entries than a wavefront keeps in registers: the other kernel variant
        inst, iters, kw = random_sparse(978, 900, 30, 4, density=0.8, dtype=np.float32), 30, dict(sparse_partition_rows=300)
    elif case == "tiny":
        inst, iters, kw = random_sparse(12, 1, 1, 2, density=1.0, dtype=np.float64), 5, {}
    else:
        inst, iters, kw = random_sparse(13, 80, 3, 4, density=0.5, dtype=np.float64), 30, dict(radius=1)
    print("pruned case", case, inst.name, flush=True)
    hopt = dict(kw)
    radius = hopt.get("radius", 0)
    o = oracle_solve(inst, iters, x0=x0, radius=radius)
    with m.from_instance(inst, DEV, prune=True, **hopt) as h:
        res = m.dmmv_solve(h, T(inst.x0 if x0 is None else x0), iters, trace=True)
        check_single_trace(res, o, iters)
        x, r, t = m.dmmv_get_state(h)
        assert np.array_equal(N(r), o.r)
        # the full table is still available on a pruning handle
        assert np.array_equal(N(m.dmmv_eval_moves(h)), oracle_table(inst, o.x, o.r, radius=radius))


def test_sparse_pruned_descent_full_size_tomography_prefix():
    m = dmmv()
    inst = make_config(3)
    iters = 60
    o = oracle_solve(inst, iters)
    with m.from_instance(inst, DEV, prune=True) as h:
        res = m.dmmv_solve(h, T(inst.x0), iters, trace=True)
    check_single_trace(res, o, iters)


# ------------------------------------------------------------- layout options of the boundary
def test_padded_leading_dimension_dense_and_batched():
    """A column-major matrix whose columns are lda > m apart (a view into a taller allocation)."""
    m = dmmv()
    inst = random_dense(61, 37, 9, 5, dtype=np.float32)
    lda = 48
    big = torch.full((inst.n, lda), 1.0e30, dtype=torch.float32, device=DEV)     # poison past row m
    big[:, :inst.m] = T(np.ascontiguousarray(inst.A.T))
    A = big.t()[:inst.m]
    assert A.stride() == (1, lda)
    with m.Handle(A=A, b=T(inst.b), D=inst.D) as h:
        assert h._problem.lda == lda
        res = m.dmmv_solve(h, T(inst.x0), 30, trace=True)
    check_single_trace(res, oracle_solve(inst, 30), 30)
    bi = random_batched(62, 37, 9, 70, 4)
    big = torch.full((bi.n, lda), 1.0e30, dtype=torch.float32, device=DEV)
    big[:, :bi.m] = T(np.ascontiguousarray(bi.A.T))
    with m.Handle(A=big.t()[:bi.m], b=T(bi.b), D=bi.D, scale=bi.scale, alns=True) as h:
        assert h._problem.lda == lda
        res = m.dmmv_solve(h, T(bi.x0), 12, trace=True)
        o = oracle_solve(bi, 12)
        assert np.array_equal(N(res.trace)[:, :, 0], o.trace_j) and np.array_equal(N(res.trace_t), o.trace_t)
        assert np.array_equal(N(res.x), o.x)
        a = m.dmmv_alns(h, T(bi.x0), 4, ls_moves=2, destroy_count=2, seed=5)
        oa = orc.alns_dense(bi.A, bi.b[3], bi.D, bi.x0[3], orc.alns_params(4, ls_moves=2, destroy_count=2, seed=5),
                            inst=3, scale=float(bi.scale[3]))
        assert np.array_equal(N(a.trace_t)[3, :, 0], oa.t) and np.array_equal(N(a.x_best)[3], oa.x)


def test_batched_var_mask():
    m = dmmv()
    inst = random_batched(63, 40, 12, 66, 5)
    rng = np.random.default_rng(8)
    vm = (rng.uniform(size=(inst.R, inst.n)) < 0.6).astype(np.uint8)
    with m.from_instance(inst, DEV, var_mask=T(vm), radius=2) as h:
        res = m.dmmv_solve(h, T(inst.x0), 10, trace=True)
    for q in (0, 1, 33, 65):
        o = orc.solve_dense(inst.A, inst.b[q], inst.D, inst.x0[q], 10, radius=2, var_mask=vm[q],
                            scale=float(inst.scale[q]))
        d = o.iters_done
        assert int(res.iters_done[q]) == d
        assert np.array_equal(N(res.trace)[q, :d, 0], o.trace_j) and np.array_equal(N(res.trace_t)[q, :d], o.trace_t)
        assert np.array_equal(N(res.x)[q], o.x)


# ------------------------------------------------------------- batched descent drops stopped instances
@pytest.mark.parametrize("poll", [1, 2, 3, 8])
def test_batched_descent_continues_on_the_running_instances_only(poll):
    """At its polling points a batch gathers the instances that still run into a dense batch of
    their own; traces, move counts and results must not notice."""
    inst = random_batched(8100 + poll, 90, 24, 200, 6, iters=40)
    batched_check(inst, 40, poll_every=poll)
    # integer data: many instances stop at once, some never move
    batched_check(random_batched(8200 + poll, 30, 10, 130, 4, integer=True), 25, poll_every=poll)


def test_batched_descent_small_llm_config_with_polling():
    o = batched_check(make_config(4, "small"), 60, poll_every=4)
    assert o.iters_done.min() < o.iters_done.max()


# ---- batched evaluation with the multiply-adds on the matrix cores (options.batched_eval = 2) --
@pytest.mark.parametrize("shape", [(1, 1, 1, 2), (17, 5, 3, 3), (64, 8, 64, 4), (100, 33, 65, 8),
                                   (130, 70, 130, 16), (50, 19, 7, 21), (70, 40, 9, 32)])
def test_batched_matrix_core_evaluation_random(shape):
    mm, nn, R, nd = shape
    batched_check(random_batched(40 + mm, mm, nn, R, nd, dtype=np.float32), 12, batched_eval=2)


def test_batched_matrix_core_evaluation_ties_radius_and_tables():
    m = dmmv()
    batched_check(random_batched(9, 30, 10, 70, 4, dtype=np.float32, integer=True), 15, batched_eval=2)
    batched_check(random_batched(12, 60, 14, 20, 8, dtype=np.float32), 10, radius=1, batched_eval=2)
    # the full score table, bit for bit that of the vector-unit kernel and of the oracle
    inst = random_batched(66, 75, 21, 67, 16, dtype=np.float32)
    tabs = []
    for mode in (1, 2):
        with m.from_instance(inst, DEV, batched_eval=mode) as h:
            m.dmmv_set_x(h, T(inst.x0))
            r = N(m.dmmv_residual(h))
            tabs.append(N(m.dmmv_eval_moves(h)))
    assert np.array_equal(tabs[0], tabs[1])
    for q in (0, 33, 66):
        want = orc.eval_moves_dense(inst.A, inst.D, inst.x0[q], r[q], scale=inst.scale[q])
        assert np.array_equal(tabs[1][q], want)


@pytest.mark.parametrize("idx", [4, 5])
def test_batched_matrix_core_evaluation_small_llm_configs(idx):
    inst = make_config(idx, "small")
    batched_check(inst, inst.iters, batched_eval=2)


def test_batched_matrix_core_evaluation_not_applicable_is_an_error():
    m = dmmv()
    for inst in (random_batched(8, 40, 12, 9, 5, dtype=np.float64), random_batched(9, 20, 6, 5, 40, dtype=np.float32),
                 random_dense(10, 20, 6, 4, dtype=np.float32)):
        with pytest.raises(m.DmmvError) as e:
            m.from_instance(inst, DEV, batched_eval=2)
        assert e.value.status == -8


# ---- dense descent with the best value of a variable found by bisection (options.value_search)
def search_check(inst, iters, **hopt):
    print("value search case", inst.name, iters, hopt, flush=True)
    oopt = {k: v for k, v in hopt.items() if k in ("radius",)}
    vm = hopt.pop("var_mask_np", None)
    if vm is not None:
        oopt["var_mask"] = vm
        hopt["var_mask"] = T(vm)
    o = oracle_solve(inst, iters, **oopt)
    with dmmv().from_instance(inst, DEV, value_search=True, **hopt) as h:
        res = dmmv().dmmv_solve(h, T(inst.x0), iters, trace=True)
        check_single_trace(res, o, iters)
        x, r, t = dmmv().dmmv_get_state(h)
        assert np.array_equal(N(r), o.r) and N(t)[0] == (np.abs(o.r).max() if inst.m else 0)
    return o


@pytest.mark.parametrize("dtype", [np.float64, np.float32])
@pytest.mark.parametrize("shape", [(1, 1, 2), (7, 3, 3), (40, 17, 4), (130, 33, 16), (300, 20, 65), (520, 12, 257),
                                   (90, 9, 1024)])
def test_value_search_dense_random(shape, dtype):
    mm, nn, nd = shape
    o = search_check(random_dense(9700 + mm, mm, nn, nd, dtype=dtype), 40)
    assert mm < 40 or o.iters_done > 0


@pytest.mark.parametrize("dtype", [np.float64, np.float32])
@pytest.mark.parametrize("seed", range(4))
def test_value_search_integer_ties_and_plateaus(seed, dtype):
    # small integers: equal scores on neighbouring values are frequent; the lowest value must win
    search_check(random_dense(9800 + seed, 37, 11, 13, dtype=dtype, integer=True), 40)
    # columns of zeros and ones: long runs of values with the same score
    inst = random_dense(9810 + seed, 25, 9, 13, dtype=dtype, integer=True)
    inst.A[:, ::2] = np.sign(inst.A[:, ::2])
    inst.A[:, 3] = 0
    search_check(inst, 40)


def test_value_search_radius_mask_and_tall_matrix():
    inst = random_dense(9820, 90, 17, 40, dtype=np.float64)
    vm = (np.random.default_rng(3).uniform(size=inst.n) < 0.5).astype(np.uint8)
    for radius in (1, 3, 0):
        search_check(inst, 30, radius=radius, var_mask_np=vm)
    # more rows than a thread keeps in registers: rows are read from memory at every step
    search_check(random_dense(9821, 5000, 4, 50, dtype=np.float32), 12)
    search_check(random_dense(9822, 40001, 3, 9, dtype=np.float64), 6)


def test_value_search_fir_configs_and_alns():
    search_check(make_config(2, "small"), 80)
    search_check(make_config(2), 500)
    search_check(make_config(1), 200)
    # inside the ALNS loop the local search takes the same moves
    m = dmmv()
    inst = make_config(2, "small")
    prm = orc.alns_params(15, ls_moves=4, seed=4)
    o = orc.alns_dense(inst.A, inst.b, inst.D, inst.x0, prm)
    with m.from_instance(inst, DEV, value_search=True) as h:
        res = m.dmmv_alns(h, T(inst.x0), 15, ls_moves=4, seed=4)
    assert np.array_equal(N(res.trace_t)[:, 0], o.t) and np.array_equal(N(res.trace)[:, 2], o.moves)
    assert np.array_equal(N(res.x_best), o.x)


def test_value_search_many_small_shapes():
    rng = np.random.default_rng(4343)
    for case in range(40):
        mm, nn, nd = int(rng.integers(0, 120)), int(rng.integers(1, 30)), int(rng.integers(2, 80))
        dtype = [np.float32, np.float64][case % 2]
        inst = random_dense(21000 + case, mm, nn, min(nd, 13) if case % 3 == 0 else nd, dtype=dtype,
                            integer=bool(case % 3 == 0))
        search_check(inst, 25, radius=int(rng.integers(0, 4)))
