"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every symbol the
header declares, sizes workspaces and rejects invalid problems before touching the device."""
import ctypes as C
import os
import re

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def mod():
    from paper_2508_13437_amd import dmmv
    if not os.path.exists(dmmv.LIB_PATH):
        from paper_2508_13437_amd import build
        build.build(force=True)
    return dmmv


def declared_functions():
    names = set()
    inc = os.path.join(ROOT, "include")
    for f in sorted(os.listdir(inc)):
        if f.endswith(".h"):
            text = re.sub(r"/\*.*?\*/", "", open(os.path.join(inc, f)).read(), flags=re.S)
            names |= set(re.findall(r"\b(dmmv_[a-z0-9_]+)\s*\(", text))
    return sorted(names)


def test_every_declared_symbol_is_exported(mod):
    lib = mod.load()
    names = declared_functions()
    assert {"dmmv_residual", "dmmv_eval_moves", "dmmv_argmin_move", "dmmv_apply_move",
            "dmmv_solve"} <= set(names)
    for name in names:
        assert hasattr(lib, name), name
    assert set(names) == set(mod.EXPORTS)


def _problem(mod, dtype=np.float64, m=10, n=5, D=(0.0, 1.0, 2.0), R=1, scale=None, sparse=False):
    p = mod.Problem()
    p.dtype = mod.DMMV_F64 if dtype == np.float64 else mod.DMMV_F32
    Dh = np.asarray(D, dtype=dtype)
    p.nd, p.m, p.n, p.R = len(Dh), m, n, R
    p.D = Dh.ctypes.data_as(C.c_void_p)
    p.b = 4096
    if sparse:
        p.csr_rowptr, p.csr_col, p.csr_val, p.nnz = 4096, 4096, 4096, 3 * m
    else:
        p.A_dense, p.lda = 4096, max(m, 1)
    keep = [Dh]
    if scale is not None:
        sh = np.asarray(scale, dtype=dtype)
        p.scale = sh.ctypes.data_as(C.c_void_p)
        keep.append(sh)
    return p, keep


def test_workspace_sizes_and_validation(mod):
    lib = mod.load()
    o = mod.Options()
    p, keep = _problem(mod)
    base = lib.dmmv_workspace_bytes(C.byref(p), C.byref(o))
    assert base > 0 and base % 256 == 0
    p2, keep2 = _problem(mod, m=1000, n=500)
    assert lib.dmmv_workspace_bytes(C.byref(p2), C.byref(o)) > base
    ps, keeps = _problem(mod, dtype=np.float32, m=1000, n=500, sparse=True)
    pb, keepb = _problem(mod, dtype=np.float32, m=100, n=50, R=3, scale=(1.0, 2.0, 0.5))
    assert lib.dmmv_workspace_bytes(C.byref(ps), C.byref(o)) > 3000 * 8
    assert lib.dmmv_workspace_bytes(C.byref(pb), C.byref(o)) >= 100 * 50 * 4 + 3 * 100 * 4
    cases = [
        (dict(D=(0.0,)), b"nd"), (dict(D=(0.0, 0.0)), b"ascending"),
        (dict(D=(0.0, np.inf)), b"finite"), (dict(m=-1), b"m >= 0"),
        (dict(R=2), b"scale"), (dict(R=2, scale=(1.0, -1.0)), b"positive"),
    ]
    for kw, needle in cases:
        q, k = _problem(mod, **kw)
        assert lib.dmmv_workspace_bytes(C.byref(q), C.byref(o)) == 0
        assert needle in lib.dmmv_last_error(), (kw, lib.dmmv_last_error())
    q, k = _problem(mod)
    q.dtype = 7
    assert lib.dmmv_workspace_bytes(C.byref(q), C.byref(o)) == 0
    q, k = _problem(mod)
    q.lda = 3
    assert lib.dmmv_workspace_bytes(C.byref(q), C.byref(o)) == 0


def test_create_rejects_bad_workspace_without_gpu(mod):
    lib = mod.load()
    o = mod.Options()
    p, keep = _problem(mod)
    h = C.c_void_p(None)
    assert lib.dmmv_create(C.byref(h), C.byref(p), C.byref(o), None, 0, None) == -5
    assert lib.dmmv_create(C.byref(h), C.byref(p), C.byref(o), C.c_void_p(4097), 1 << 20, None) == -5
    assert lib.dmmv_create(C.byref(h), C.byref(p), C.byref(o), C.c_void_p(4096), 16, None) == -5
    assert b"too small" in lib.dmmv_last_error()
    assert lib.dmmv_create(None, C.byref(p), C.byref(o), C.c_void_p(4096), 1 << 20, None) == -1
    assert lib.dmmv_destroy(None) == -1
    assert lib.dmmv_solve(None, None, 1, None, None, None, None, None) == -1
    assert mod.dmmv_version().startswith("libdmmv")


def test_binding_fails_loudly_without_library(mod, monkeypatch):
    monkeypatch.setattr(mod, "_lib", None)
    monkeypatch.setattr(mod, "LIB_PATH", "/nonexistent/libdmmv.so")
    with pytest.raises(RuntimeError):
        mod.load()


def test_product_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_2508_13437_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h")):
                text = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in text.lower(), os.path.join(dirpath, f)


def test_bench_refuses_more_than_one_gpu():
    import subprocess
    import sys
    p = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert p.returncode == 2
    assert "one GPU" in p.stderr and p.stdout.strip() == ""


def test_alns_parameter_blocks_of_binding_and_oracle_have_the_layout_of_the_header(mod):
    # include/dmmv.h: four int32, five doubles, one uint64, four int32 -> 4*4 + 5*8 + 8 + 4*4 bytes, no padding
    import ctypes as C
    from oracle import oracle as orc
    assert C.sizeof(mod.AlnsParams) == 80 == C.sizeof(orc.AlnsParams)
    assert [f[0].rstrip("_") for f in mod.AlnsParams._fields_] == [f[0].rstrip("_") for f in orc.AlnsParams._fields_]
    hdr = open(os.path.join(ROOT, "include", "dmmv.h")).read()
    body = hdr[hdr.index("typedef struct {\n    int32_t iters;"):hdr.index("} dmmv_alns_params;")]
    import re
    names = []
    for decl in re.findall(r"^\s+(?:int32_t|double|uint64_t)\s+([a-z0-9_, ]+);", body, flags=re.M):
        names += [v.strip() for v in decl.split(",")]
    assert names == ["iters", "ls_moves", "ls_radius", "destroy_count", "alpha", "lambda", "sigma1", "sigma2", "sigma3", "seed", "ls_swaps", "k_eps", "l2_guard", "reserved"]


def test_options_block_of_the_binding_has_the_layout_of_the_header(mod):
    import re
    hdr = open(os.path.join(ROOT, "include", "dmmv.h")).read()
    body = hdr[hdr.index("typedef struct {\n    int32_t radius;"):hdr.index("} dmmv_options;")]
    names = []
    for decl in re.findall(r"^\s+(?:const\s+)?(?:int32_t|uint8_t\*)\s+\*?([a-z0-9_]+);", body, flags=re.M):
        names.append(decl)
    assert names == [f[0] for f in mod.Options._fields_], (names, [f[0] for f in mod.Options._fields_])
    # four int32, one pointer (8-byte aligned already), nine int32 -> padded to the pointer's alignment
    assert C.sizeof(mod.Options) == 64


def test_workspace_grows_with_the_options_that_need_buffers(mod):
    lib = mod.load()
    pd, keep = _problem(mod, m=300, n=40)
    o = mod.Options()
    base = lib.dmmv_workspace_bytes(C.byref(pd), C.byref(o))
    o.value_search = 1
    assert lib.dmmv_workspace_bytes(C.byref(pd), C.byref(o)) >= base + 40 * 16
    pb, keepb = _problem(mod, dtype=np.float32, m=100, n=50, R=3, scale=(1.0, 2.0, 0.5))
    o = mod.Options()
    base = lib.dmmv_workspace_bytes(C.byref(pb), C.byref(o))
    o.batched_eval = 2
    with_rt = lib.dmmv_workspace_bytes(C.byref(pb), C.byref(o))
    assert with_rt >= base + 3 * 128 * 4                     # rows padded to a multiple of 64
    o = mod.Options()
    o.alns = 1
    assert lib.dmmv_workspace_bytes(C.byref(pb), C.byref(o)) > base


def test_sparse_matrix_that_needs_too_many_partitions_is_refused_before_any_gpu_work(mod):
    """The partition count the layout will use (rows / sparse_partition_rows) is checked on the host:
    more than 1024 partitions, or padded segments that overflow 32-bit offsets, fail in
    dmmv_workspace_bytes, dmmv_create and dmmv_solve_static alike, with no GPU call made."""
    lib = mod.load()
    ps, keep = _problem(mod, dtype=np.float32, m=5000, n=50, sparse=True)
    o = mod.Options()
    assert lib.dmmv_workspace_bytes(C.byref(ps), C.byref(o)) > 0
    o.sparse_partition_rows = 4                            # 1250 partitions
    assert lib.dmmv_workspace_bytes(C.byref(ps), C.byref(o)) == 0
    assert b"partitions" in lib.dmmv_last_error()
    h = C.c_void_p(None)
    assert lib.dmmv_create(C.byref(h), C.byref(ps), C.byref(o), C.c_void_p(4096), 1 << 30, None) == -8
    assert lib.dmmv_solve_static(C.byref(ps), C.byref(o), C.c_void_p(4096), 1, None, None, None, None, None, None) == -8
    # fp64 partitions hold 8192 rows: 2^27 rows would need 16384 partitions
    pl, keepl = _problem(mod, dtype=np.float64, m=1 << 27, n=8, sparse=True)
    assert lib.dmmv_workspace_bytes(C.byref(pl), C.byref(mod.Options())) == 0
    # 4 * partitions * n pads beyond 2^31 entries
    pw, keepw = _problem(mod, dtype=np.float32, m=16 * 16384, n=40_000_000, sparse=True)
    assert lib.dmmv_workspace_bytes(C.byref(pw), C.byref(mod.Options())) == 0
    assert b"32-bit" in lib.dmmv_last_error()


def test_one_launch_dense_descent_is_refused_on_the_host_when_it_cannot_fit(mod):
    """options.dense_loop = 2 needs r, D, x and one column of A in 156 KiB of LDS, and one dense
    instance; anything else fails in dmmv_workspace_bytes / dmmv_create with no GPU call made."""
    lib = mod.load()
    small, keep = _problem(mod, dtype=np.float64, m=300, n=40)
    o = mod.Options()
    o.dense_loop = 2
    assert lib.dmmv_workspace_bytes(C.byref(small), C.byref(o)) > 0
    tall, keept = _problem(mod, dtype=np.float64, m=30000, n=4)       # r alone: 234 KiB
    assert lib.dmmv_workspace_bytes(C.byref(tall), C.byref(o)) == 0
    assert b"dense_loop" in lib.dmmv_last_error()
    h = C.c_void_p(None)
    assert lib.dmmv_create(C.byref(h), C.byref(tall), C.byref(o), C.c_void_p(4096), 1 << 30, None) == -8
    sp, keeps = _problem(mod, dtype=np.float32, m=500, n=50, sparse=True)
    assert lib.dmmv_workspace_bytes(C.byref(sp), C.byref(o)) == 0
    pb, keepb = _problem(mod, dtype=np.float32, m=100, n=50, R=3, scale=(1.0, 2.0, 0.5))
    assert lib.dmmv_workspace_bytes(C.byref(pb), C.byref(o)) == 0
    o.dense_loop = 3
    assert lib.dmmv_workspace_bytes(C.byref(small), C.byref(o)) == 0
    o.dense_loop = 0
    o.wait_limit = -1
    assert lib.dmmv_workspace_bytes(C.byref(small), C.byref(o)) == 0


def test_static_scratch_entry_point_refuses_large_problems_on_the_host(mod):
    lib = mod.load()
    p, keep = _problem(mod, dtype=np.float32, m=600, n=300, R=4000, scale=np.ones(4000))
    need = lib.dmmv_workspace_bytes(C.byref(p), None)
    assert need > mod.STATIC_SCRATCH_BYTES
    hdr = open(os.path.join(ROOT, "include", "dmmv.h")).read()
    assert re.search(r"#define DMMV_STATIC_SCRATCH_BYTES \((\d+)u << 20\)", hdr).group(1) == str(mod.STATIC_SCRATCH_BYTES >> 20)
    assert lib.dmmv_solve_static(C.byref(p), None, C.c_void_p(4096), 3, None, None, None, None, None, None) == -5
    assert b"scratch" in lib.dmmv_last_error()
    assert lib.dmmv_solve_static(C.byref(p), None, None, 3, None, None, None, None, None, None) == -1
    assert lib.dmmv_solve_static(C.byref(p), None, C.c_void_p(4096), -1, None, None, None, None, None, None) == -2
