"""Compile the HIP sources under csrc/ into paper_2508_13437_amd/libdmmv.so for gfx950."""
from __future__ import annotations

import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libdmmv.so")
SOURCES = ["dmmv_api.hip", "dmmv_dense.hip", "dmmv_dense_search.hip", "dmmv_sparse.hip", "dmmv_sparse_eval.hip",
           "dmmv_batched.hip", "dmmv_batched_pruned.hip", "dmmv_batched_mfma.hip", "dmmv_batched_eval_mfma.hip", "dmmv_alns.hip", "dmmv_swap.hip", "dmmv_swap_sparse.hip", "dmmv_l2.hip", "dmmv_dense_persistent.hip"]
HEADERS = [os.path.join(CSRC, "dmmv_common.h"), os.path.join(CSRC, "dmmv_sparse_common.h"),
           os.path.join(CSRC, "dmmv_alns_common.h"),
           os.path.join(os.path.dirname(HERE), "include", "dmmv.h"),
           os.path.join(os.path.dirname(HERE), "include", "dmmv_bench.h")]

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    "-ffp-contract=off",                                   # only explicit fma() fuses
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-fno-gpu-rdc", "-Wall", "-Wno-unused-function",
]


def needs_build() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    deps = [os.path.join(CSRC, s) for s in SOURCES] + HEADERS
    return any(os.path.getmtime(d) > t for d in deps)


def _compile(src: str) -> str:
    obj = os.path.join(OBJ, src.replace(".hip", ".o"))
    cmd = [HIPCC, *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError(f"hipcc failed for {src}:\n{res.stdout}\n{res.stderr}")
    return obj


def build(force: bool = True, extra_flags=()) -> str:
    """Compile every HIP source and link the shared library.  Always recompiles when force."""
    if not force and not needs_build():
        return LIB
    os.makedirs(OBJ, exist_ok=True)
    if extra_flags:
        FLAGS.extend(extra_flags)
    with ThreadPoolExecutor(max_workers=4) as ex:
        objs = list(ex.map(_compile, SOURCES))
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError(f"link failed:\n{res.stdout}\n{res.stderr}")
    return LIB


if __name__ == "__main__":
    print(build(force=True))
