"""The dense descent as one launch (options.dense_loop = 2) against the CPU oracle and against
the launch-per-step loop (dense_loop = 1): traces, x, r and the error bit for bit.

Paper, section "GPU Acceleration": the iteration is to run without host-side stepping and
synchronisation; the moves are those of the single-move descent (Algorithm 2's local search).
"""
import numpy as np
import pytest
import torch

from oracle import oracle as orc
from workloads import make_config, random_dense

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


def dmmv():
    from paper_2508_13437_amd import dmmv as mod
    return mod


def T(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def N(t):
    return t.detach().cpu().numpy()


def check(inst, iters, x0=None, keep_going=False, **opt):
    """dense_loop 2 and 1 against the oracle: trace, x, error, stored r and t."""
    m = dmmv()
    x0 = inst.x0 if x0 is None else x0
    oopt = {k: v for k, v in opt.items() if k in ("radius", "var_mask")}
    o = orc.solve_dense(inst.A, inst.b, inst.D, x0, iters, **oopt)
    hopt = dict(opt)
    if "var_mask" in hopt:
        hopt["var_mask"] = T(hopt["var_mask"])
    for loop in (2, 1):
        with m.from_instance(inst, DEV, dense_loop=loop, keep_going=keep_going, **hopt) as h:
            res = m.dmmv_solve(h, T(x0), iters, trace=True)
            d = int(res.iters_done[0])
            assert d == o.iters_done, (loop, d, o.iters_done)
            tr = N(res.trace)[0]
            assert np.array_equal(tr[:d, 0], o.trace_j) and np.array_equal(tr[:d, 1], o.trace_k), loop
            assert np.all(tr[d:] == -1)
            assert np.array_equal(N(res.trace_t)[0, :d], o.trace_t)
            assert np.array_equal(N(res.x).reshape(-1), o.x)
            assert N(res.max_violation)[0] == o.t
            x, r, t = m.dmmv_get_state(h)
            assert np.array_equal(N(x).reshape(-1), o.x) and np.array_equal(N(r), o.r) and N(t)[0] == o.t
            # the handle goes on from there: a second call finds the same local optimum state
            res2 = m.dmmv_solve(h, None, 3, trace=True)
            o2 = orc.solve_dense(inst.A, inst.b, inst.D, o.x, 3, **oopt)
            assert int(res2.iters_done[0]) == o2.iters_done and N(res2.max_violation)[0] == o2.t
    return o


@pytest.mark.parametrize("dtype", [np.float64, np.float32])
@pytest.mark.parametrize("shape", [(1, 1, 2), (5, 3, 2), (63, 7, 3), (64, 9, 16), (65, 5, 17), (257, 13, 9),
                                   (300, 40, 16), (1000, 6, 37), (130, 4, 200), (700, 48, 16), (90, 300, 3),
                                   (2000, 3, 1000)])
def test_one_launch_descent_random(shape, dtype):
    mm, nn, nd = shape
    print("one-launch descent", shape, dtype.__name__, flush=True)
    inst = random_dense(900 + mm + nn, mm, nn, nd, dtype=dtype)
    rng = np.random.default_rng(mm)
    x0 = rng.choice(inst.D, size=inst.n)
    o = check(inst, 60, x0=x0)
    assert mm < 5 or o.iters_done >= 1


@pytest.mark.parametrize("dtype", [np.float64, np.float32])
@pytest.mark.parametrize("seed", range(3))
def test_one_launch_descent_integer_ties(seed, dtype):
    """Small-integer data: exact ties between workgroups' records, the lowest index wins."""
    inst = random_dense(950 + seed, 37, 70, 5, dtype=dtype, integer=True)
    check(inst, 50)


def test_one_launch_descent_radius_mask_and_fixed_work():
    inst = random_dense(91, 90, 17, 9, dtype=np.float64)
    rng = np.random.default_rng(3)
    vm = (rng.uniform(size=inst.n) < 0.5).astype(np.uint8)
    for radius in (1, 2):
        check(inst, 30, radius=radius, var_mask=vm)
    # fixed-work mode: all iterations run, the result is that of the descent
    o = check(inst, 40, keep_going=True)
    assert o.iters_done < 40


def test_one_launch_descent_iteration_cap_and_zero_iterations():
    inst = random_dense(17, 200, 30, 8, dtype=np.float32)
    rng = np.random.default_rng(1)
    x0 = rng.choice(inst.D, size=inst.n)
    o = check(inst, 5, x0=x0)
    assert o.iters_done == 5                      # cut short by the cap, not by a local optimum
    check(inst, 0, x0=x0)


def test_one_launch_descent_on_the_dense_workloads():
    m = dmmv()
    toy = make_config(1)
    rng = np.random.default_rng(0)
    check(toy, toy.iters)
    o = check(toy, toy.iters, x0=rng.choice(toy.D, size=toy.n))
    assert o.iters_done >= 10
    fir = make_config(2)
    x0 = np.clip(fir.x0 + rng.integers(-40, 41, size=fir.n), fir.D[0], fir.D[-1])
    o = check(fir, 40, x0=x0)
    assert o.iters_done >= 10


def test_one_launch_descent_refused_when_it_does_not_fit():
    m = dmmv()
    inst = random_dense(5, 30000, 3, 4, dtype=np.float64)          # r alone exceeds the LDS
    with pytest.raises(m.DmmvError) as e:
        m.from_instance(inst, DEV, dense_loop=2)
    assert e.value.status == -8                                     # DMMV_ERR_UNSUPPORTED
    with m.from_instance(inst, DEV) as h:                            # automatic: the launch loop
        res = m.dmmv_solve(h, T(inst.x0), 3, trace=True)
    o = orc.solve_dense(inst.A, inst.b, inst.D, inst.x0, 3)
    assert int(res.iters_done[0]) == o.iters_done and N(res.max_violation)[0] == o.t


def test_one_launch_descent_bounded_wait_reports_instead_of_hanging():
    """A wait limit of one poll: a workgroup that finds another one not yet arrived gives up, every
    workgroup leaves, dmmv_solve reports the state error and the handle is still at its starting
    point.  (With so short a limit the wait may also simply succeed; then the result is checked.)"""
    m = dmmv()
    inst = random_dense(33, 256, 64, 16, dtype=np.float64)
    rng = np.random.default_rng(2)
    x0 = rng.choice(inst.D, size=inst.n)
    o = orc.solve_dense(inst.A, inst.b, inst.D, x0, 50)
    with m.from_instance(inst, DEV, dense_loop=2, wait_limit=1) as h:
        try:
            res = m.dmmv_solve(h, T(x0), 50, trace=True)
        except m.DmmvError as e:
            print("bounded wait: gave up as intended:", e, flush=True)
            assert e.status == -7                                   # DMMV_ERR_STATE
            x, r, t = m.dmmv_get_state(h)
            assert np.array_equal(N(x).reshape(-1), x0)
            assert np.array_equal(N(r), orc.residual_dense(inst.A, inst.b, inst.D, x0))
        else:
            print("bounded wait: every arrival was already there", flush=True)
            assert int(res.iters_done[0]) == o.iters_done and N(res.max_violation)[0] == o.t
    # the automatic choice falls back to the loop of launches instead of failing
    with m.from_instance(inst, DEV, wait_limit=1) as h:
        assert m.dmmv_loop_in_use(h) == 2
        res = m.dmmv_solve(h, T(x0), 50, trace=True)
        d = int(res.iters_done[0])
        assert d == o.iters_done and N(res.max_violation)[0] == o.t
        tr = N(res.trace)[0]
        assert np.array_equal(tr[:d, 0], o.trace_j) and np.array_equal(tr[:d, 1], o.trace_k) and np.all(tr[d:] == -1)
        assert np.array_equal(N(res.trace_t)[0, :d], o.trace_t)
    # the default limit on the same problem
    with m.from_instance(inst, DEV, dense_loop=2) as h:
        res = m.dmmv_solve(h, T(x0), 50, trace=True)
        assert int(res.iters_done[0]) == o.iters_done and N(res.max_violation)[0] == o.t
