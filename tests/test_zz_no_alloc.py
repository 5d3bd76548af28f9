"""dmmv_solve_static: the one-shot descent whose workspace is the library's built-in scratch array
(for callers that cannot allocate) against dmmv_create + dmmv_solve with a caller workspace.
Two calls in a row, the second with a smaller input, must both agree bit for bit."""
import numpy as np
import pytest
import torch

from paper_2508_13437_amd import dmmv
from workloads import make_config, random_batched, random_dense, random_sparse

pytestmark = pytest.mark.gpu


def _kwargs(inst, dev):
    b = torch.from_numpy(np.ascontiguousarray(inst.b)).to(dev)
    if inst.kind == "csr":
        csr = (torch.from_numpy(inst.csr_rowptr).to(dev), torch.from_numpy(inst.csr_col).to(dev),
               torch.from_numpy(inst.csr_val).to(dev))
        return dict(D=inst.D, b=b, csr=csr, m=inst.m, n=inst.n, device=dev)
    A = torch.from_numpy(np.ascontiguousarray(inst.A.T)).to(dev).t()
    return dict(D=inst.D, b=b, A=A, scale=inst.scale if inst.kind == "batched" else None, device=dev)


def _both(inst, dev, iters, **opt):
    x0 = torch.from_numpy(np.ascontiguousarray(inst.x0)).to(dev)
    got = dmmv.dmmv_solve_static(x0, iters, trace=True, **_kwargs(inst, dev), **opt)
    with dmmv.Handle(**_kwargs(inst, dev), **opt) as h:
        assert h.workspace_bytes <= dmmv.STATIC_SCRATCH_BYTES
        want = dmmv.dmmv_solve(h, x0, iters, trace=True)
    for f in ("x", "max_violation", "iters_done", "trace", "trace_t"):
        assert torch.equal(getattr(got, f), getattr(want, f)), (inst.name, f)
    return int(want.iters_done.sum())


def test_static_scratch_descent_equals_the_descent_with_a_caller_workspace(gpu_device):
    dev = gpu_device
    moved = 0
    # larger first, then smaller: the second call finds the first one's leftovers in the scratch
    moved += _both(random_dense(41, 700, 90, 16, dtype=np.float64), dev, 60)
    moved += _both(random_dense(42, 130, 17, 5, dtype=np.float64), dev, 30)
    moved += _both(random_sparse(43, 900, 400, 4, 0.05, dtype=np.float32), dev, 50)
    moved += _both(random_sparse(44, 200, 90, 3, 0.1, dtype=np.float32), dev, 25, prune=True)
    moved += _both(random_batched(45, 150, 60, 70, 8), dev, 20)
    moved += _both(random_batched(46, 70, 33, 9, 4), dev, 12, prune=True)
    moved += _both(make_config(1), dev, 20)
    assert moved > 100


def test_static_scratch_refuses_what_does_not_fit(gpu_device):
    inst = make_config(3, "small")
    huge = random_batched(48, 600, 300, 4000, 8)               # needs 42 MB of workspace
    with pytest.raises(dmmv.DmmvError) as e:
        dmmv.dmmv_solve_static(torch.from_numpy(huge.x0).to(gpu_device), 3, **_kwargs(huge, gpu_device))
    assert e.value.status == -5 and "scratch" in str(e.value)
    # and the scratch still works afterwards
    _both(inst, gpu_device, 10)
