"""options.prune on a batch of instances: the descent screens every candidate on the 16 rows of
largest |r| and scores only those that can still win.  It must make exactly the moves of the
full evaluation, i.e. the oracle's (bitwise: traces, x, t, residual)."""
import numpy as np
import pytest
import torch

from oracle import oracle as orc
from workloads import make_config, random_batched

from test_gpu_parity import DEV, N, T, batched_check, dmmv
from test_gpu_alns import batched_alns_check

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("shape", [(1, 1, 1, 2), (3, 2, 2, 3), (17, 5, 3, 3), (64, 8, 64, 4), (100, 33, 65, 8),
                                   (130, 70, 130, 16), (300, 300, 7, 16), (50, 19, 7, 21), (1030, 40, 5, 40)])
def test_pruned_batched_random(shape):
    mm, nn, R, nd = shape
    print("pruned batched case", shape, flush=True)
    batched_check(random_batched(9000 + mm, mm, nn, R, nd, dtype=np.float32), 14, prune=True)


def test_pruned_batched_many_levels_and_instances_too_large_for_lds():
    # more than 256 levels: 16-bit level indices in LDS
    batched_check(random_batched(9050, 40, 6, 5, 300, dtype=np.float32), 10, prune=True)
    batched_check(random_batched(9051, 33, 5, 3, 700, dtype=np.float64), 8, radius=40, prune=True)
    # (m + n) w + 2 n bytes exceed the LDS a workgroup may take: the full evaluation runs instead
    batched_check(random_batched(9052, 8, 21000, 3, 3, dtype=np.float32), 4, prune=True)
    # more rows than a thread's 64-bit row mask covers: the full evaluation again
    batched_check(random_batched(9053, 16400, 5, 3, 3, dtype=np.float32), 4, prune=True)
    # the largest m that is pruned
    batched_check(random_batched(9054, 16384, 6, 2, 3, dtype=np.float32), 6, prune=True)


def test_pruned_batched_f64_and_integer_ties():
    batched_check(random_batched(9100, 40, 12, 9, 5, dtype=np.float64), 10, prune=True)
    batched_check(random_batched(9101, 30, 10, 70, 4, dtype=np.float32, integer=True), 15, prune=True)
    batched_check(random_batched(9102, 70, 40, 33, 9, dtype=np.float64, integer=True), 25, prune=True)
    batched_check(random_batched(9103, 5, 300, 12, 6, dtype=np.float32, integer=True), 25, prune=True)


@pytest.mark.parametrize("radius", [1, 2, 7])
def test_pruned_batched_radius(radius):
    batched_check(random_batched(9200 + radius, 60, 14, 20, 8, dtype=np.float32), 12, radius=radius, prune=True)
    batched_check(random_batched(9210 + radius, 45, 300, 6, 12, dtype=np.float32, integer=True), 12, radius=radius, prune=True)


def test_pruned_batched_var_mask():
    m = dmmv()
    inst = random_batched(9300, 40, 12, 66, 5)
    rng = np.random.default_rng(8)
    vm = (rng.uniform(size=(inst.R, inst.n)) < 0.6).astype(np.uint8)
    with m.from_instance(inst, DEV, var_mask=T(vm), radius=2, prune=True) as h:
        res = m.dmmv_solve(h, T(inst.x0), 10, trace=True)
    for q in (0, 1, 33, 65):
        o = orc.solve_dense(inst.A, inst.b[q], inst.D, inst.x0[q], 10, radius=2, var_mask=vm[q],
                            scale=float(inst.scale[q]))
        d = o.iters_done
        assert int(res.iters_done[q]) == d
        assert np.array_equal(N(res.trace)[q, :d, 0], o.trace_j) and np.array_equal(N(res.trace_t)[q, :d], o.trace_t)
        assert np.array_equal(N(res.x)[q], o.x)


@pytest.mark.parametrize("idx", [4, 5])
def test_pruned_batched_small_llm_configs(idx):
    inst = make_config(idx, "small")
    batched_check(inst, inst.iters, prune=True)


def test_pruned_batched_continues_where_the_last_call_stopped():
    """Two calls of 4 and 30 iterations make the moves of one call of 34 (the second call starts
    from a freshly computed residual, so its t may differ from the maintained one by rounding)."""
    m = dmmv()
    inst = random_batched(9400, 80, 30, 40, 6)
    o = orc.solve_batched(inst.A, inst.b, inst.D, inst.scale, inst.x0, 34)
    with m.from_instance(inst, DEV, prune=True) as h:
        first = m.dmmv_solve(h, T(inst.x0), 4)
        second = m.dmmv_solve(h, T(N(first.x)), 30)
    assert np.array_equal(N(second.x), o.x) and np.allclose(N(second.max_violation), o.t, rtol=1e-5, atol=0)
    assert np.array_equal(N(first.iters_done) + N(second.iters_done), o.iters_done)


def test_pruned_and_full_descent_agree_on_a_larger_batch():
    m = dmmv()
    inst = random_batched(9500, 700, 520, 300, 16, iters=60)
    out = []
    for prune in (False, True):
        with m.from_instance(inst, DEV, prune=prune) as h:
            res = m.dmmv_solve(h, T(inst.x0), 60, trace=True)
            out.append((N(res.x), N(res.max_violation), N(res.iters_done), N(res.trace), N(res.trace_t)))
    for a, b in zip(out[0], out[1]):
        assert np.array_equal(a, b)
    assert out[0][2].max() > 5


def test_alns_batched_with_pruned_local_search():
    batched_alns_check(random_batched(9600, 64, 24, 64, 4), 10, ls_moves=3, destroy_count=3, seed=5, prune=True)
    batched_alns_check(random_batched(9601, 40, 16, 20, 5, integer=True), 20, ls_moves=4, destroy_count=3, seed=4,
                       ls_radius=2, prune=True)
    batched_alns_check(random_batched(9602, 30, 12, 9, 4, dtype=np.float64), 12, ls_moves=3, destroy_count=2, seed=6,
                       ls_swaps=1, l2_guard=1, prune=True)
    batched_alns_check(make_config(4, "small"), 6, ls_moves=4, seed=4, prune=True)


def test_pruned_and_full_descent_agree_on_the_full_size_layer():
    """Config 4 at full size, 12 iterations: all 4096 instances make the same moves either way."""
    m = dmmv()
    inst = make_config(4)
    out = []
    for prune in (False, True):
        print("full-size layer, prune =", prune, flush=True)
        with m.from_instance(inst, DEV, prune=prune) as h:
            res = m.dmmv_solve(h, T(inst.x0), 12, trace=True)
            out.append((N(res.x), N(res.max_violation), N(res.iters_done), N(res.trace), N(res.trace_t)))
    for a, b in zip(out[0], out[1]):
        assert np.array_equal(a, b)


def test_pruned_descent_of_the_full_size_layer_follows_the_oracle_to_the_local_optimum():
    """Config 4 at full size with pruning, up to 100 iterations (every instance but a few reaches
    its local optimum); four seeded instances are replayed by the oracle's full enumeration and
    must show the same moves, errors and solutions."""
    m = dmmv()
    inst = make_config(4)
    iters = 100
    with m.from_instance(inst, DEV, prune=True) as h:
        res = m.dmmv_solve(h, T(inst.x0), iters, trace=True)
        x, t, done = N(res.x), N(res.max_violation), N(res.iters_done)
        tr, tt = N(res.trace), N(res.trace_t)
    sel = np.sort(np.random.default_rng(44).choice(inst.R, size=4, replace=False))
    print("oracle replay of instances", sel, flush=True)
    o = orc.solve_batched(inst.A, inst.b[sel], inst.D, inst.scale[sel], inst.x0[sel], iters)
    assert np.array_equal(done[sel], o.iters_done)
    assert np.array_equal(tr[sel][:, :, 0], o.trace_j) and np.array_equal(tr[sel][:, :, 1], o.trace_k)
    assert np.array_equal(tt[sel], o.trace_t)
    assert np.array_equal(x[sel], o.x) and np.array_equal(t[sel], o.t)
    assert o.iters_done.min() >= 10


# ---- a dense single instance as a batch of one ----------------------------------------------------
def dense_pruned_check(inst, iters, **opt):
    """dmmv_solve with options.prune on a dense single instance (one workgroup, all iterations in one
    launch) against the oracle's full enumeration: traces, x, residual, error, bit for bit."""
    from test_gpu_parity import check_single_trace, oracle_solve
    m = dmmv()
    hopt = dict(opt)
    if "var_mask" in hopt:
        hopt["var_mask"] = T(hopt["var_mask"])
    with m.from_instance(inst, DEV, prune=True, **hopt) as h:
        res = m.dmmv_solve(h, T(inst.x0), iters, trace=True)
        x, r, t = m.dmmv_get_state(h)
        o = oracle_solve(inst, iters, **opt)
        check_single_trace(res, o, iters)
        assert np.array_equal(N(r), o.r) and N(t)[0] == o.t
        # the handle still serves the other entry points (full table, standalone arg-min)
        want = orc.eval_moves_dense(inst.A, inst.D, o.x, o.r, **{k: v for k, v in opt.items() if k in ("radius", "var_mask")})
        assert np.array_equal(N(m.dmmv_eval_moves(h)), want)
    return o.iters_done


@pytest.mark.parametrize("dtype", [np.float64, np.float32])
def test_pruned_dense_single_instance(dtype):
    from workloads import random_dense
    moved = 0
    for shape in [(1, 1, 2), (5, 3, 2), (65, 5, 5), (257, 13, 9), (300, 40, 16), (1000, 6, 37), (130, 4, 300), (700, 48, 16)]:
        print("pruned dense case", shape, dtype, flush=True)
        moved += dense_pruned_check(random_dense(9600 + shape[0], *shape, dtype=dtype), 60)
    for seed in range(3):
        moved += dense_pruned_check(random_dense(9650 + seed, 37, 11, 5, dtype=dtype, integer=True), 40)
    inst = random_dense(9660, 90, 17, 9, dtype=dtype)
    vm = (np.random.default_rng(3).uniform(size=inst.n) < 0.5).astype(np.uint8)
    for radius in (1, 2):
        moved += dense_pruned_check(inst, 30, radius=radius, var_mask=vm)
    assert moved > 100


def test_pruned_dense_configs_and_outer_loop():
    from test_gpu_alns import alns_check
    from workloads import random_dense
    dense_pruned_check(make_config(1), 50)
    dense_pruned_check(make_config(2, "small"), 80)
    dense_pruned_check(make_config(2), 20)
    # from a poor starting point the toy workload has a long descent
    inst = make_config(1)
    inst.x0 = np.random.default_rng(11).choice(inst.D, size=inst.n)
    assert dense_pruned_check(inst, 200) > 30
    # the local search of the outer loop in one launch per outer iteration
    alns_check(random_dense(9670, 60, 30, 5), 12, ls_moves=4, destroy_count=4, seed=5, prune=1)
    alns_check(make_config(1), 10, ls_moves=8, seed=6, prune=1)
