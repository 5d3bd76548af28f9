"""Parity of the swap move (dmmv_swap_move, through the C ABI) against the CPU oracle, which
enumerates every pair.  The pair found, its error, and the state after carrying it out must be
bitwise equal, whatever k_eps and whichever staging the kernel uses for the sizes at hand."""
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


def chain_check(inst, max_swaps, k_eps=0, var_mask=None, descend=0, **hopt):
    """Swap after swap from x0 (after `descend` moves of the descent) until none improves."""
    m = dmmv()
    print("swap case", inst.name, max_swaps, k_eps, descend, flush=True)
    R = inst.R
    b = inst.b.reshape(R, inst.m)
    x0 = inst.x0.reshape(R, inst.n)
    scale = inst.scale if inst.scale is not None else np.ones(R, dtype=inst.dtype)
    opts = dict(hopt)
    if var_mask is not None:
        opts["var_mask"] = T(var_mask)
    with m.from_instance(inst, DEV, **opts) as h:
        m.dmmv_solve(h, T(inst.x0), descend)
        x, r, t = (N(a).reshape(R, -1) for a in m.dmmv_get_state(h))
        xs = [x[q].copy() for q in range(R)]
        rs = [r[q].copy() for q in range(R)]
        live = [True] * R
        n_found = 0
        for step in range(max_swaps + 1):
            probe = m.dmmv_swap_move(h, k_eps=k_eps, apply=False)         # reports, changes nothing
            res = m.dmmv_swap_move(h, k_eps=k_eps, apply=True)
            gi, gj, gt = N(res.i), N(res.j), N(res.t)
            assert np.array_equal(N(probe.i), gi) and np.array_equal(N(probe.j), gj) and np.array_equal(N(probe.t), gt)
            x, r, t = (N(a).reshape(R, -1) for a in m.dmmv_get_state(h))
            for q in range(R):
                vm = None if var_mask is None else np.asarray(var_mask).reshape(R, inst.n)[q]
                if inst.kind == "csr":
                    oi, oj, ot = orc.best_swap_csr(inst.m, inst.n, inst.csr_rowptr, inst.csr_col, inst.csr_val,
                                                   inst.D, xs[q], rs[q], var_mask=vm)
                else:
                    oi, oj, ot = orc.best_swap_dense(inst.A, inst.D, xs[q], rs[q], scale=float(scale[q]), var_mask=vm)
                assert (gi[q], gj[q]) == (oi, oj), (step, q, gi[q], gj[q], oi, oj, gt[q], ot)
                assert gt[q] == ot
                if oi >= 0:
                    n_found += 1
                    if inst.kind == "csr":
                        xs[q], rs[q], tq = orc.apply_swap_csr(inst.m, inst.n, inst.csr_rowptr, inst.csr_col,
                                                              inst.csr_val, inst.D, xs[q], rs[q], oi, oj)
                    else:
                        xs[q], rs[q], tq = orc.apply_swap_dense(inst.A, inst.D, xs[q], rs[q], oi, oj, scale=float(scale[q]))
                    assert tq == ot
                else:
                    live[q] = False
                assert np.array_equal(x[q], xs[q]), (step, q)
                assert np.array_equal(r[q], rs[q]), (step, q)
                assert t[q, 0] == (np.abs(rs[q]).max() if inst.m else 0)
            if not any(live):
                break
    return n_found


@pytest.mark.parametrize("dtype", [np.float64, np.float32])
@pytest.mark.parametrize("shape", [(1, 1, 2), (1, 2, 2), (7, 3, 3), (40, 17, 4), (130, 65, 16), (300, 130, 5),
                                   (520, 257, 8)])
def test_swap_dense_random(shape, dtype):
    mm, nn, nd = shape
    found = chain_check(random_dense(8100 + mm, mm, nn, nd, dtype=dtype), 3)
    assert mm < 40 or found > 0


@pytest.mark.parametrize("dtype", [np.float64, np.float32])
def test_swap_dense_integer_ties(dtype):
    # small integers: every operation exact, equal errors frequent -> the lowest pair number decides
    found = chain_check(random_dense(8200, 24, 40, 5, dtype=dtype, integer=True), 6)
    assert found > 0
    chain_check(random_dense(8201, 9, 70, 3, dtype=dtype, integer=True), 6)


@pytest.mark.parametrize("k_eps", [1, 2, 7, 64, 100, 128, 1000])
def test_swap_result_does_not_depend_on_k_eps(k_eps):
    chain_check(random_dense(8300, 150, 90, 6), 2, k_eps=k_eps)
    chain_check(random_batched(8301, 70, 40, 6, 4), 2, k_eps=k_eps)


def test_swap_after_the_descent():
    # at a local optimum of the single moves an improving swap may or may not exist; both are checked
    chain_check(random_dense(8400, 60, 30, 4), 4, descend=200)
    chain_check(random_dense(8401, 200, 24, 8, dtype=np.float32), 4, descend=200)
    chain_check(make_config(1), 2, descend=200)


def test_swap_fir_config():
    chain_check(make_config(2), 1, descend=0)
    chain_check(make_config(2), 1, descend=500)


@pytest.mark.parametrize("shape", [(1, 1, 1, 2), (17, 5, 3, 3), (64, 24, 64, 4), (100, 33, 65, 8), (130, 70, 130, 16)])
def test_swap_batched_random(shape):
    mm, nn, R, nd = shape
    chain_check(random_batched(8500 + mm, mm, nn, R, nd), 2)


def test_swap_batched_integer_and_f64():
    chain_check(random_batched(8600, 40, 16, 20, 5, integer=True), 4)
    chain_check(random_batched(8601, 33, 20, 9, 4, dtype=np.float64), 3)


def test_swap_var_mask():
    inst = random_dense(8700, 50, 40, 5)
    vm = (np.random.default_rng(1).random(40) < 0.6).astype(np.uint8)
    chain_check(inst, 3, var_mask=vm)
    inst = random_batched(8701, 30, 20, 7, 4)
    vm = (np.random.default_rng(2).random((7, 20)) < 0.7).astype(np.uint8)
    chain_check(inst, 2, var_mask=vm)
    # nothing may move: no swap
    m = dmmv()
    inst = random_dense(8702, 20, 10, 3)
    with m.from_instance(inst, DEV, var_mask=T(np.zeros(10, dtype=np.uint8))) as h:
        m.dmmv_solve(h, T(inst.x0), 0)
        res = m.dmmv_swap_move(h)
        assert N(res.i)[0] == -1 and N(res.j)[0] == -1


def test_swap_many_rows_residual_not_staged():
    # m beyond what the kernel keeps in LDS: the residual is read from memory
    chain_check(random_dense(8800, 20000, 24, 4, dtype=np.float32), 2)
    chain_check(random_dense(8801, 9000, 12, 3, dtype=np.float64), 2)


def test_swap_many_variables_values_not_staged():
    # n beyond what the kernel keeps in LDS: D[k_j] is read from memory, no filter row is staged
    chain_check(random_dense(8900, 3, 8000, 3, dtype=np.float64), 1)


def test_swap_all_values_equal_and_empty():
    m = dmmv()
    inst = random_dense(9000, 12, 9, 3)
    inst.x0[:] = inst.D[1]
    with m.from_instance(inst, DEV) as h:
        m.dmmv_solve(h, T(inst.x0), 0)
        res = m.dmmv_swap_move(h)
        assert N(res.i)[0] == -1 and N(res.t)[0] == N(m.dmmv_get_state(h)[2])[0]
    chain_check(random_dense(9001, 0, 6, 3), 1)
    chain_check(random_dense(9002, 5, 0, 3), 1)
    chain_check(random_sparse(9003, 6, 0, 3), 1)
    chain_check(random_sparse(9004, 0, 5, 3), 1)


def test_swap_errors():
    m = dmmv()
    inst = random_dense(9101, 10, 5, 3)
    with m.from_instance(inst, DEV) as h:
        with pytest.raises(m.DmmvError) as e:
            m.dmmv_swap_move(h)
        assert e.value.status == -7
        m.dmmv_solve(h, T(inst.x0), 0)
        with pytest.raises(m.DmmvError) as e:
            m.dmmv_swap_move(h, k_eps=-1)
        assert e.value.status == -2


# ---- sparse matrices --------------------------------------------------------------------------
@pytest.mark.parametrize("dtype", [np.float32, np.float64])
@pytest.mark.parametrize("shape", [(1, 1, 2, 1.0), (5, 3, 2, 0.6), (40, 30, 3, 0.2), (150, 100, 4, 0.08),
                                   (300, 260, 3, 0.03), (90, 500, 5, 0.05)])
def test_swap_sparse_random(shape, dtype):
    mm, nn, nd, dens = shape
    chain_check(random_sparse(9200 + mm, mm, nn, nd, density=dens, dtype=dtype), 3)


def test_swap_sparse_integer_ties_and_explicit_zeros():
    found = chain_check(random_sparse(9300, 40, 60, 3, density=0.15, integer=True), 5)
    assert found > 0
    chain_check(random_sparse(9301, 30, 50, 4, density=0.2, integer=True, explicit_zeros=True, dtype=np.float64), 5)


def test_swap_sparse_several_partitions_and_empty_columns():
    # rows cut into partitions of 16: columns span several segments, some are empty
    chain_check(random_sparse(9400, 100, 80, 3, density=0.05), 3, sparse_partition_rows=16)
    chain_check(random_sparse(9401, 70, 40, 4, density=0.02), 2, sparse_partition_rows=8)


def test_swap_sparse_columns_cover_the_reservoir():
    # few rows: every row sits in the reservoir, and dense columns store most of them, so the
    # residual that stays is taken from deep in the reservoir, or is zero
    chain_check(random_sparse(9500, 12, 20, 3, density=0.9), 3)
    chain_check(random_sparse(9501, 6, 9, 4, density=1.0, dtype=np.float64), 3)
    # more rows than the reservoir holds, columns that store almost all of them: full scan
    chain_check(random_sparse(9502, 200, 12, 3, density=0.97), 2)


def test_swap_sparse_after_descent_and_mask():
    chain_check(random_sparse(9600, 120, 90, 3, density=0.1), 3, descend=300)
    inst = random_sparse(9601, 60, 50, 4, density=0.15)
    vm = (np.random.default_rng(3).random(50) < 0.7).astype(np.uint8)
    chain_check(inst, 3, var_mask=vm)


def test_swap_sparse_tomography_small():
    chain_check(make_config(3, "small"), 1, descend=0)
    chain_check(make_config(3, "small"), 1, descend=2000)


@pytest.mark.parametrize("descend", [0, 100000])
def test_swap_full_size_tomography_sampled(descend):
    """Full-size sparse instance (65536 variables): the oracle carries out the reported swap and
    must get the reported error and residual, and searches the pairs inside random subsets of the
    variables that contain the reported pair, where that pair must again be the best."""
    import scipy.sparse as sp
    m = dmmv()
    inst = make_config(3)
    print("swap full size", inst.name, descend, flush=True)
    rng = np.random.default_rng(78 + descend)
    with m.from_instance(inst, DEV) as h:
        m.dmmv_solve(h, T(inst.x0), descend)
        x0, r0, t0 = (N(a) for a in m.dmmv_get_state(h))
        res = m.dmmv_swap_move(h, apply=True)
        gi, gj, gt = int(N(res.i)[0]), int(N(res.j)[0]), N(res.t)[0]
        x1, r1, t1 = (N(a) for a in m.dmmv_get_state(h))
        # the descent goes on from the state the swap left
        after = m.dmmv_solve(h, None, 50)
        assert N(after.max_violation)[0] <= gt
    assert gi >= 0 and gt < t0[0] and t1[0] == gt
    M = sp.csr_matrix((inst.csr_val, inst.csr_col, inst.csr_rowptr), shape=(inst.m, inst.n))
    kstar = int(np.argmax(np.abs(r0)))
    in_row = M.indices[M.indptr[kstar]:M.indptr[kstar + 1]]
    assert gi in in_row or gj in in_row
    for rep in range(3):
        S = np.unique(np.concatenate([rng.choice(inst.n, size=300, replace=False),
                                      rng.choice(in_row, size=min(10, in_row.size), replace=False), [gi, gj]]))
        sub = M[:, S].tocsr()
        sub.sort_indices()
        oi, oj, ot = orc.best_swap_csr(inst.m, S.size, sub.indptr.astype(np.int64), sub.indices.astype(np.int32),
                                       sub.data, inst.D, x0[S], r0)
        assert ot == gt and (S[oi], S[oj]) == (gi, gj), (rep, ot, gt, S[oi], S[oj], gi, gj)
        if rep == 0:
            xs, rs, ts = orc.apply_swap_csr(inst.m, S.size, sub.indptr.astype(np.int64), sub.indices.astype(np.int32),
                                            sub.data, inst.D, x0[S], r0, oi, oj)
            assert ts == gt and np.array_equal(rs, r1)
    xe = x0.copy(); xe[gi], xe[gj] = x0[gj], x0[gi]
    assert np.array_equal(x1, xe)


def test_swap_many_small_shapes():
    """A sweep of odd small shapes (seeded), every storage kind and both precisions."""
    rng = np.random.default_rng(4242)
    for case in range(60):
        mm, nn, nd = int(rng.integers(0, 90)), int(rng.integers(1, 75)), int(rng.integers(2, 10))
        dtype = [np.float32, np.float64][case % 2]
        kind = case % 3
        if kind == 0:
            inst = random_dense(20000 + case, mm, nn, nd, dtype=dtype, integer=bool(case % 4 == 0))
        elif kind == 1:
            inst = random_batched(20000 + case, max(mm, 1), nn, int(rng.integers(1, 12)), nd, dtype=dtype,
                                  integer=bool(case % 4 == 1))
        else:
            inst = random_sparse(20000 + case, max(mm, 1), nn, nd, density=float(rng.uniform(0.05, 0.6)), dtype=dtype,
                                 integer=bool(case % 4 == 2))
        chain_check(inst, 2, k_eps=int(rng.integers(0, 9)))
