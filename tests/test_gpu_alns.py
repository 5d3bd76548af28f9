"""Parity of the ALNS outer loop (dmmv_alns, through the C ABI) against the CPU oracle.

Every random decision is a function of (seed, iteration, stream, counter) and every decision a
floating-point value takes is taken on integers or by a fixed sequence of IEEE operations, so
operator choices, local-search move counts, acceptance flags, errors, the best solution and its
error must all be bitwise equal."""
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


def alns_check(inst, iters, **kw):
    m = dmmv()
    hopt = {}
    for key in ("sparse_partition_rows", "prune"):
        if key in kw:
            hopt[key] = kw.pop(key)
    print("alns case", inst.name, iters, kw, hopt, flush=True)
    prm = orc.alns_params(iters, **kw)
    if inst.kind == "csr":
        o = orc.alns_csr(inst.m, inst.n, inst.csr_rowptr, inst.csr_col, inst.csr_val, inst.b, inst.D,
                         inst.x0, prm)
    else:
        o = orc.alns_dense(inst.A, inst.b, inst.D, inst.x0, prm)
    with m.from_instance(inst, DEV, **hopt) as h:
        res = m.dmmv_alns(h, T(inst.x0), iters, **kw)
        tr, tt = N(res.trace), N(res.trace_t)
        assert np.array_equal(tr[:, 0], o.destroy), (tr[:, 0], o.destroy)
        assert np.array_equal(tr[:, 1], o.repair)
        assert np.array_equal(tt[:, 0], o.t), (tt[:, 0], o.t)
        assert np.array_equal(tr[:, 2], o.moves)
        assert np.array_equal(tr[:, 3], o.accepted)
        assert np.array_equal(tt[:, 1], o.best)
        assert np.array_equal(N(res.x_best), o.x)
        assert N(res.t_best)[0] == o.t_best
        # the handle holds the current solution: its r is the residual of its x, t = max |r|
        x, r, t = m.dmmv_get_state(h)
        x, r, t = N(x), N(r), N(t)
        if inst.m:
            assert np.abs(r).max() == t[0]
        acc = np.nonzero(o.accepted)[0]
        want_cur = o.t[acc[-1]] if acc.size else None
        if want_cur is not None:
            assert t[0] == want_cur
    return o


@pytest.mark.parametrize("dtype", [np.float64, np.float32])
@pytest.mark.parametrize("shape", [(5, 3, 2), (40, 16, 5), (130, 70, 4), (300, 33, 9), (1100, 12, 16)])
def test_alns_dense(shape, dtype):
    mm, nn, nd = shape
    alns_check(random_dense(7000 + mm, mm, nn, nd, dtype=dtype), 25, ls_moves=4, destroy_count=max(1, nn // 8), seed=mm)


@pytest.mark.parametrize("seed", range(3))
def test_alns_dense_integer_ties(seed):
    o = alns_check(random_dense(7100 + seed, 30, 20, 4, dtype=np.float32, integer=True), 40, ls_moves=5,
                   destroy_count=3, seed=seed, ls_radius=0)
    assert set(o.destroy.tolist()) == {0, 1} and set(o.repair.tolist()) == {0, 1}


@pytest.mark.parametrize("dtype", [np.float32, np.float64])
@pytest.mark.parametrize("shape", [(20, 9, 3, 0.4), (200, 150, 3, 0.1), (700, 300, 4, 0.05), (64, 40, 5, 1.0)])
def test_alns_sparse(shape, dtype):
    mm, nn, nd, dens = shape
    alns_check(random_sparse(7200 + mm, mm, nn, nd, dens, dtype=dtype), 20, ls_moves=4,
               destroy_count=max(1, nn // 10), seed=mm + 1)


def test_alns_sparse_with_pruned_local_search():
    alns_check(random_sparse(7250, 700, 300, 4, 0.05, dtype=np.float32), 20, ls_moves=4, destroy_count=12, seed=8,
               prune=True)
    alns_check(make_config(3, "small"), 12, ls_moves=6, seed=3, prune=True)


@pytest.mark.parametrize("rows", [7, 64, 1000])
def test_alns_sparse_row_partitions(rows):
    alns_check(random_sparse(7300, 300, 120, 3, 0.15, dtype=np.float32, integer=True), 20, ls_moves=3,
               destroy_count=9, seed=4, sparse_partition_rows=rows)


def test_alns_edge_parameters():
    inst = random_dense(7400, 25, 10, 4)
    alns_check(inst, 0)
    alns_check(inst, 8, ls_moves=0, destroy_count=2, seed=2)
    alns_check(inst, 8, ls_moves=3, destroy_count=10, seed=3)       # every variable unassigned
    alns_check(inst, 8, ls_moves=3, destroy_count=500, seed=3)      # clipped to n
    alns_check(inst, 8, ls_moves=3, destroy_count=0, seed=5)        # default rate: one variable
    two = random_dense(7401, 12, 6, 2)                              # |D| = 2: one neighbour level only
    alns_check(two, 12, ls_moves=3, destroy_count=2, seed=9)


@pytest.mark.parametrize("idx", [1, 2, 3])
def test_alns_small_configs(idx):
    inst = make_config(idx, "small") if idx != 1 else make_config(1)
    alns_check(inst, 12, ls_moves=6, seed=idx)


def test_alns_same_seed_same_run_and_batched_is_refused():
    m = dmmv()
    inst = random_dense(7500, 60, 24, 5, dtype=np.float32)
    with m.from_instance(inst, DEV) as h:
        a = m.dmmv_alns(h, T(inst.x0), 15, seed=11)
        b = m.dmmv_alns(h, T(inst.x0), 15, seed=11)
        c = m.dmmv_alns(h, T(inst.x0), 15, seed=12)
        assert torch.equal(a.trace, b.trace) and torch.equal(a.trace_t, b.trace_t) and torch.equal(a.x_best, b.x_best)
        assert not torch.equal(a.trace_t, c.trace_t)
    bi = random_batched(7501, 20, 6, 4, 3)
    with m.from_instance(bi, DEV) as h:                     # created without options.alns
        with pytest.raises(m.DmmvError) as e:
            m.dmmv_alns(h, T(bi.x0), 3)
        assert e.value.status == -7


def batched_alns_check(inst, iters, **kw):
    m = dmmv()
    print("alns batched case", inst.name, iters, kw, flush=True)
    hopt = {key: kw.pop(key) for key in ("batched_eval", "prune") if key in kw}
    prm = orc.alns_params(iters, **kw)
    with m.from_instance(inst, DEV, alns=True, **hopt) as h:
        res = m.dmmv_alns(h, T(inst.x0), iters, **kw)
        tr, tt = N(res.trace), N(res.trace_t)
        xb, tb = N(res.x_best), N(res.t_best)
        x, r, t = m.dmmv_get_state(h)
        r, t = N(r), N(t)
    for q in range(inst.R):
        o = orc.alns_dense(inst.A, inst.b[q], inst.D, inst.x0[q], prm, inst=q, scale=float(inst.scale[q]))
        assert np.array_equal(tr[q, :, 0], o.destroy), q
        assert np.array_equal(tr[q, :, 1], o.repair), q
        assert np.array_equal(tt[q, :, 0], o.t), (q, tt[q, :, 0], o.t)
        assert np.array_equal(tr[q, :, 2], o.moves), q
        assert np.array_equal(tr[q, :, 3], o.accepted), q
        assert np.array_equal(tt[q, :, 1], o.best), q
        assert np.array_equal(xb[q], o.x), q
        assert tb[q] == o.t_best
        assert np.abs(r[q]).max() == t[q]


@pytest.mark.parametrize("shape", [(1, 1, 1, 2), (17, 5, 3, 3), (64, 24, 64, 4), (100, 33, 65, 8), (130, 70, 130, 16)])
def test_alns_batched_random(shape):
    mm, nn, R, nd = shape
    batched_alns_check(random_batched(7600 + mm, mm, nn, R, nd), 10, ls_moves=3, destroy_count=max(1, nn // 8), seed=mm)


def test_alns_batched_integer_ties_and_f64():
    batched_alns_check(random_batched(7700, 40, 16, 20, 5, integer=True), 20, ls_moves=4, destroy_count=3, seed=4,
                       ls_radius=0)
    batched_alns_check(random_batched(7701, 30, 12, 9, 4, dtype=np.float64), 12, ls_moves=3, destroy_count=2, seed=6)


@pytest.mark.parametrize("idx", [4, 5])
def test_alns_batched_small_llm_configs(idx):
    batched_alns_check(make_config(idx, "small"), 6, ls_moves=4, seed=idx)


@pytest.mark.parametrize("idx,iters,ls", [(2, 40, 4), (3, 4, 3)])
def test_alns_full_size_configs(idx, iters, ls):
    """Full-size FIR and tomography workloads, a few outer iterations (what the oracle manages
    in seconds), default destroy rate (0.5 % of n: 1 and 328 variables)."""
    inst = make_config(idx)
    alns_check(inst, iters, ls_moves=ls, seed=100 + idx)


# ---- the swap move inside the local search (dense and batched) -----------------------------
@pytest.mark.parametrize("dtype", [np.float64, np.float32])
def test_alns_dense_with_swaps(dtype):
    alns_check(random_dense(7900, 60, 30, 5, dtype=dtype), 12, ls_moves=3, ls_swaps=2, destroy_count=4, seed=5)
    alns_check(random_dense(7901, 33, 50, 3, dtype=dtype, integer=True), 10, ls_moves=2, ls_swaps=3, seed=6)


def test_alns_dense_toy_with_swaps():
    alns_check(make_config(1), 6, ls_moves=20, ls_swaps=2, seed=11, k_eps=16)


def test_alns_batched_with_swaps():
    batched_alns_check(random_batched(7910, 40, 24, 20, 4), 8, ls_moves=3, ls_swaps=2, destroy_count=3, seed=2)
    batched_alns_check(random_batched(7911, 30, 16, 70, 5, integer=True), 8, ls_moves=2, ls_swaps=2, seed=3)


def test_alns_sparse_with_swaps():
    alns_check(random_sparse(7920, 80, 60, 3, density=0.12), 10, ls_moves=3, ls_swaps=2, destroy_count=4, seed=8)
    alns_check(random_sparse(7921, 50, 70, 4, density=0.1, integer=True), 8, ls_moves=2, ls_swaps=2, seed=9, prune=1)


# ---- l2 guard of the acceptance step ----------------------------------------------------------
@pytest.mark.parametrize("dtype", [np.float64, np.float32])
def test_alns_l2_guard_dense(dtype):
    alns_check(random_dense(7930, 300, 30, 5, dtype=dtype), 30, ls_moves=2, destroy_count=4, seed=5, l2_guard=1)
    alns_check(random_dense(7931, 700, 20, 4, dtype=dtype), 20, ls_moves=1, ls_swaps=1, seed=6, l2_guard=1)


def test_alns_l2_guard_changes_the_run():
    # the guard must actually reject something here, else the cases above show nothing
    inst = random_dense(7930, 300, 30, 5)
    a = orc.alns_dense(inst.A, inst.b, inst.D, inst.x0, orc.alns_params(30, ls_moves=2, destroy_count=4, seed=5))
    b = orc.alns_dense(inst.A, inst.b, inst.D, inst.x0, orc.alns_params(30, ls_moves=2, destroy_count=4, seed=5, l2_guard=1))
    assert not np.array_equal(a.accepted, b.accepted)


def test_alns_l2_guard_sparse_and_batched():
    alns_check(random_sparse(7932, 600, 80, 3, density=0.1), 15, ls_moves=2, destroy_count=5, seed=7, l2_guard=1)
    batched_alns_check(random_batched(7933, 300, 24, 70, 4), 10, ls_moves=2, destroy_count=3, seed=2, l2_guard=1)
    batched_alns_check(random_batched(7934, 40, 16, 9, 5, dtype=np.float64), 10, ls_moves=2, seed=3, l2_guard=1)


def test_alns_batched_with_the_matrix_core_evaluation():
    batched_alns_check(random_batched(7940, 70, 24, 20, 4), 8, ls_moves=3, ls_swaps=1, destroy_count=3, seed=2,
                       batched_eval=2)


@pytest.mark.parametrize("dtype", [np.float32, np.float64])
def test_alns_sparse_gathered_repair_paths(dtype):
    # the gathered repair kernel beyond its common case: columns touching more chunks of rows than
    # one pass of its look takes (several hundred entries spread over 12007 rows, a row count that
    # ends inside a chunk), more levels than it keeps in LDS, and a row count that needs the second
    # round of its scan over the chunk maxima (fp32; in fp64 that many rows go to the general kernel)
    alns_check(random_sparse(7960, 12007, 30, 3, density=0.05, dtype=dtype), 8, ls_moves=2, destroy_count=6, seed=6)
    alns_check(random_sparse(7961, 900, 40, 1500, density=0.1, dtype=dtype), 8, ls_moves=2, destroy_count=5, seed=7)
    alns_check(random_sparse(7962, 70001, 24, 4, density=0.003, dtype=dtype), 6, ls_moves=2, destroy_count=6, seed=8)


def test_alns_sparse_general_repair_kernel():
    # a column longer than the gathered kernel takes (1024 entries), and more rows than its tables
    # hold (131072 in fp32): both fall back to the general repair kernel
    alns_check(random_sparse(7950, 1400, 20, 3, density=0.9), 8, ls_moves=2, destroy_count=5, seed=4)
    alns_check(random_sparse(7951, 140000, 24, 4, density=0.002), 6, ls_moves=2, destroy_count=6, seed=5)


def test_alns_dense_all_options_together():
    # value search in the local search, swaps after it, the l2 guard in the acceptance step
    m = dmmv()
    inst = random_dense(7960, 200, 24, 40, dtype=np.float64)
    kw = dict(ls_moves=3, ls_swaps=2, destroy_count=4, seed=12, l2_guard=1, k_eps=8)
    o = orc.alns_dense(inst.A, inst.b, inst.D, inst.x0, orc.alns_params(25, **kw))
    with m.from_instance(inst, DEV, value_search=True) as h:
        res = m.dmmv_alns(h, T(inst.x0), 25, **kw)
    tr, tt = N(res.trace), N(res.trace_t)
    assert np.array_equal(tr[:, 0], o.destroy) and np.array_equal(tr[:, 1], o.repair)
    assert np.array_equal(tr[:, 2], o.moves) and np.array_equal(tr[:, 3], o.accepted)
    assert np.array_equal(tt[:, 0], o.t) and np.array_equal(tt[:, 1], o.best)
    assert np.array_equal(N(res.x_best), o.x) and N(res.t_best)[0] == o.t_best
