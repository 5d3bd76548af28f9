"""Acceptance at full size and full length on the three large workloads, and oracle checks of the
full-size paths the benchmark times.

The descent runs free on the GPU for the configured number of iterations (to its local optimum);
the oracle runs the same descent in full on the sparse instance and on a seeded sample of the
instances of each batch (32 rows of the layer, 16 rows of the MLP layer), and every move, every
error after a move and the final point must agree bit for bit - for the path that scores every
move and for the exactly pruned one.  Every instance of a batch gets the checks that need no
oracle: the reported error against a fresh fp64 recomputation of ||X (s q) - b||_inf, a strictly
decreasing trace, q in D.
"""
import functools
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import pytest
import torch

from oracle import oracle as orc
from workloads import make_config

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


def dmmv():
    from paper_2508_13437_amd import dmmv as mod
    return mod


def T(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def N(t):
    return t.detach().cpu().numpy()


@functools.lru_cache(maxsize=3)
def config(idx):
    return make_config(idx)


# ------------------------------------------------------------------------------ tomography
@functools.lru_cache(maxsize=1)
def tomography_oracle():
    inst = config(3)
    print("oracle: full descent of the tomography instance", flush=True)
    return orc.solve_csr(inst.m, inst.n, inst.csr_rowptr, inst.csr_col, inst.csr_val, inst.b, inst.D,
                         inst.x0, inst.iters)


@pytest.mark.timeout(400)
@pytest.mark.parametrize("prune", [False, True])
def test_tomography_whole_descent(prune):
    """All moves of the configured 2000-iteration descent (it stops at its local optimum after a
    few hundred), free-running, against the oracle's full enumeration."""
    m = dmmv()
    inst = config(3)
    o = tomography_oracle()
    assert 100 < o.iters_done < inst.iters            # a real local optimum, well past any prefix
    with m.from_instance(inst, DEV, prune=prune) as h:
        res = m.dmmv_solve(h, T(inst.x0), inst.iters, trace=True)
        x, r, t = m.dmmv_get_state(h)
    d = int(res.iters_done[0])
    assert d == o.iters_done
    tr = N(res.trace)[0]
    assert np.array_equal(tr[:d, 0], o.trace_j) and np.array_equal(tr[:d, 1], o.trace_k)
    assert np.all(tr[d:] == -1)
    assert np.array_equal(N(res.trace_t)[0, :d], o.trace_t)
    assert np.array_equal(N(res.x), o.x) and N(res.max_violation)[0] == o.t
    assert np.array_equal(N(r), o.r) and N(t)[0] == o.t
    assert np.all(np.diff(o.trace_t) < 0)


# ------------------------------------------------------------------------------ batches
SAMPLE = {4: 32, 5: 16}


def sample_of(idx):
    inst = config(idx)
    return np.sort(np.random.default_rng(100 + idx).choice(inst.R, size=SAMPLE[idx], replace=False))


@functools.lru_cache(maxsize=2)
def batch_oracle(idx):
    inst = config(idx)
    sel = sample_of(idx)
    print(f"oracle: {sel.size} instances of workload {idx}, {inst.iters} iterations", flush=True)
    return orc.solve_batched(inst.A, inst.b[sel], inst.D, inst.scale[sel], inst.x0[sel], inst.iters)


@pytest.mark.timeout(600)
@pytest.mark.parametrize("prune", [False, True])
@pytest.mark.parametrize("idx", [4, 5])
def test_llm_batches_whole_descent(idx, prune):
    m = dmmv()
    inst = config(idx)
    sel = sample_of(idx)
    o = batch_oracle(idx)
    print("whole descent of batch", idx, "prune", prune, flush=True)
    with m.from_instance(inst, DEV, prune=prune) as h:
        res = m.dmmv_solve(h, T(inst.x0), inst.iters, trace=True)
        x, t, done = N(res.x), N(res.max_violation), N(res.iters_done)
        tr, tt = N(res.trace), N(res.trace_t)
        r = N(m.dmmv_get_state(h)[1])
    # sampled instances: the oracle's descent, move by move
    assert np.array_equal(done[sel], o.iters_done)
    assert np.array_equal(tr[sel][:, :, 0], o.trace_j) and np.array_equal(tr[sel][:, :, 1], o.trace_k)
    assert np.array_equal(tt[sel], o.trace_t)
    assert np.array_equal(x[sel], o.x) and np.array_equal(t[sel], o.t)
    assert o.iters_done.max() > 40 and o.iters_done.min() < inst.iters
    # every instance: values in D, error == max |maintained r| == fresh fp64 error to 1e-5,
    # a strictly decreasing trace that ends where the move count says
    assert np.all(np.isin(x, inst.D))
    assert np.array_equal(np.abs(r).max(axis=1), t)
    it = np.arange(inst.iters)[None, :]
    live = it < done[:, None]
    assert np.all(tr[:, :, 0][~live] == -1) and np.all(tr[:, :, 0][live] >= 0)
    dec = np.diff(tt, axis=1) < 0
    assert np.all(dec[live[:, 1:]])
    last = np.where(done > 0, tt[np.arange(inst.R), np.maximum(done - 1, 0)], t)
    assert np.array_equal(last, t)
    # The maintained fp32 residual against a fresh fp64 one.  Each r_i is an fp32 sum of n products
    # followed by one fused multiply-add per move, so it may differ from the exact value by
    # (n + 2 + moves) 2^-24 (|s| sum_j |X_ij| |q_j| + |b_i|) and the reported error by the largest of
    # these (checked on every 8th instance); in practice the two agree to a few 1e-6 relative,
    # and every instance must stay within 1e-4.
    X64 = inst.A.astype(np.float64)
    aX = np.abs(X64)
    worst = 0.0
    for q0 in range(0, inst.R, 1024):
        q1 = min(inst.R, q0 + 1024)
        sx = inst.scale[q0:q1, None].astype(np.float64) * x[q0:q1]
        fresh = sx @ X64.T - inst.b[q0:q1]
        ft = np.abs(fresh).max(axis=1)
        rel = np.abs(t[q0:q1] - ft) / ft
        worst = max(worst, float(rel.max()))
        assert np.all(rel <= 1e-4)
        sub = slice(q0, q1, 8)
        mag = np.abs(sx[::8]) @ aX.T + np.abs(inst.b[sub]).astype(np.float64)
        bound = (inst.n + 2 + done[sub, None]) * 2.0 ** -24 * mag
        assert np.all(np.abs(r[sub].astype(np.float64) - fresh[::8]) <= bound)
    print("largest |t - fresh fp64 error| / error over all instances:", worst, flush=True)


# ------------------------------------------------------------------------------ swap move
@pytest.mark.timeout(600)
@pytest.mark.parametrize("idx,count", [(4, 3), (5, 2)])
def test_swap_move_full_size_batch_against_the_full_enumeration(idx, count):
    """The swap search at the local optimum of the descent (the state the benchmark times), on the
    whole batch; for a few seeded instances the oracle enumerates all n (n - 1) ordered pairs over
    all rows and must name the same pair and error."""
    m = dmmv()
    inst = config(idx)
    sel = np.sort(np.random.default_rng(200 + idx).choice(inst.R, size=count, replace=False))
    with m.from_instance(inst, DEV, prune=True) as h:
        m.dmmv_solve(h, T(inst.x0), inst.iters)
        x, r, t = (N(a) for a in m.dmmv_get_state(h))
        sw = m.dmmv_swap_move(h, apply=True)
        gi, gj, gt = N(sw.i), N(sw.j), N(sw.t)
        x1, r1, t1 = (N(a) for a in m.dmmv_get_state(h))
    print("oracle: swap enumeration for instances", sel, flush=True)

    def one(q):
        return orc.best_swap_dense(inst.A, inst.D, x[q], r[q], scale=float(inst.scale[q]))

    with ThreadPoolExecutor(max_workers=count) as ex:
        want = list(ex.map(one, sel))
    for q, (oi, oj, ot) in zip(sel, want):
        assert (int(gi[q]), int(gj[q])) == (oi, oj) and gt[q] == ot, (q, gi[q], gj[q], gt[q], oi, oj, ot)
        if oi >= 0:
            xs, rs, ts = orc.apply_swap_dense(inst.A, inst.D, x[q], r[q], oi, oj, scale=float(inst.scale[q]))
            assert np.array_equal(x1[q], xs) and np.array_equal(r1[q], rs) and t1[q] == ts
    # every instance: a reported swap exchanges two different levels, lowers the error strictly and
    # leaves t = max |r|; an instance without one keeps its state
    has = gi >= 0
    assert has.sum() > inst.R // 2
    assert np.all(gt[has] < t[has]) and np.array_equal(gt[~has], t[~has])
    assert np.array_equal(np.abs(r1).max(axis=1), t1) and np.array_equal(t1, gt)
    qs = np.nonzero(has)[0]
    assert np.all(x[qs, gi[qs]] > x[qs, gj[qs]])
    xe = x.copy()
    xe[qs, gi[qs]], xe[qs, gj[qs]] = x[qs, gj[qs]], x[qs, gi[qs]]
    assert np.array_equal(x1, xe)


# ------------------------------------------------------------------------------ outer loop
@pytest.mark.timeout(600)
@pytest.mark.parametrize("prune", [True, False])
def test_alns_full_size_batch_sampled_instances(prune):
    """Two outer iterations of Algorithm 1 on every instance of the full-size layer (default destroy
    rate: 21 variables), a handful of instances replayed by the oracle: operators, local-search
    moves, acceptance, errors and the best point must agree bit for bit."""
    m = dmmv()
    inst = config(4)
    iters, kw = 2, dict(ls_moves=4, seed=31)
    sel = np.sort(np.random.default_rng(300).choice(inst.R, size=8, replace=False))
    with m.from_instance(inst, DEV, alns=True, prune=prune) as h:
        res = m.dmmv_alns(h, T(inst.x0), iters, **kw)
        tr, tt, xb, tb = N(res.trace), N(res.trace_t), N(res.x_best), N(res.t_best)
        x, r, t = (N(a) for a in m.dmmv_get_state(h))
    print("oracle: outer loop for instances", sel, flush=True)

    def one(q):
        return orc.alns_dense(inst.A, inst.b[q], inst.D, inst.x0[q], orc.alns_params(iters, **kw), inst=int(q),
                              scale=float(inst.scale[q]))

    with ThreadPoolExecutor(max_workers=8) as ex:
        want = list(ex.map(one, sel))
    used = set()
    for q, o in zip(sel, want):
        assert np.array_equal(tr[q, :, 0], o.destroy) and np.array_equal(tr[q, :, 1], o.repair), q
        assert np.array_equal(tr[q, :, 2], o.moves) and np.array_equal(tr[q, :, 3], o.accepted), q
        assert np.array_equal(tt[q, :, 0], o.t) and np.array_equal(tt[q, :, 1], o.best), q
        assert np.array_equal(xb[q], o.x) and tb[q] == o.t_best, q
        used |= set(zip(o.destroy.tolist(), o.repair.tolist()))
    assert len(used) >= 3                         # worst-remove and greedy repair among them
    assert np.array_equal(np.abs(r).max(axis=1), t) and np.all(np.isin(xb, inst.D))
    assert np.all(tb <= tt[:, 0, 1]) and np.all(tt[:, 1, 1] <= tt[:, 0, 1])


# ------------------------------------------------------------------------------ matrix cores
@pytest.mark.timeout(600)
@pytest.mark.parametrize("idx", [4, 5])
def test_matrix_core_residual_full_size_against_the_fp64_definition(idx):
    """r = (X Q^T) diag(s) - B from the matrix cores at full size: every element within the bound
    of an fp32 accumulation of n exact products in some order plus the final fused multiply-add,
    (n + 2) 2^-24 (|s| sum_j |X_ij| |q_j| + |b_i|); a sample of instances also against the
    oracle's residual in fp64."""
    m = dmmv()
    inst = config(idx)
    with m.from_instance(inst, DEV, residual_mfma=True) as h:
        m.dmmv_set_x(h, T(inst.x0))
        r = N(m.dmmv_residual(h))
        _, r_state, t = m.dmmv_get_state(h)
        assert np.array_equal(N(r_state), r) and np.array_equal(np.abs(r).max(axis=1), N(t))
    X64 = inst.A.astype(np.float64)
    aX = np.abs(X64)
    worst = 0.0
    for q0 in range(0, inst.R, 1024):
        q1 = min(inst.R, q0 + 1024)
        sx = inst.scale[q0:q1, None].astype(np.float64) * inst.x0[q0:q1]
        ref = sx @ X64.T - inst.b[q0:q1]
        tol = (inst.n + 2) * 2.0 ** -24 * (np.abs(sx) @ aX.T + np.abs(inst.b[q0:q1]).astype(np.float64)) + 1e-30
        err = np.abs(r[q0:q1].astype(np.float64) - ref)
        assert np.all(err <= tol), (q0, float((err / tol).max()))
        worst = max(worst, float((err / tol).max()))
    print("matrix-core residual: largest error / bound =", worst, flush=True)
    for q in np.random.default_rng(400 + idx).choice(inst.R, size=4, replace=False):
        ref = orc.residual_dense(X64, inst.b[q].astype(np.float64), inst.D.astype(np.float64),
                                 inst.x0[q].astype(np.float64), scale=float(inst.scale[q]))
        mag = np.abs(float(inst.scale[q]) * inst.x0[q].astype(np.float64)) @ aX.T + np.abs(inst.b[q])
        assert np.all(np.abs(r[q] - ref) <= (inst.n + 2) * 2.0 ** -24 * mag + 1e-30)


@pytest.mark.timeout(600)
def test_matrix_core_evaluation_full_size_equals_the_vector_unit_evaluation():
    """options.batched_eval = 2 on the full-size layer: the whole score table and the fused arg-min
    must carry the bits of the vector-unit kernel; two seeded instances also against the oracle."""
    m = dmmv()
    inst = config(4)
    x0 = T(inst.x0)
    tabs, best = [], []
    for mode in (1, 2):
        with m.from_instance(inst, DEV, batched_eval=mode) as h:
            m.dmmv_set_x(h, x0)
            r = m.dmmv_residual(h)
            tabs.append(m.dmmv_eval_moves(h))
            best.append(m.dmmv_argmin_move(h, None))
    assert torch.equal(tabs[0], tabs[1])
    assert torch.equal(best[0][0], best[1][0]) and torch.equal(best[0][1], best[1][1])
    r = N(r)
    for q in np.random.default_rng(500).choice(inst.R, size=2, replace=False):
        want = orc.eval_moves_dense(inst.A, inst.D, inst.x0[q], r[q], scale=float(inst.scale[q]))
        assert np.array_equal(N(tabs[1][q]), want), q
        c, s = orc.argmin_move(want)
        assert tuple(N(best[1][0])[q]) == (c // inst.nd, c % inst.nd) and N(best[1][1])[q] == s
