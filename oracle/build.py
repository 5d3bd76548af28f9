"""Compile the CPU oracle (plain C) into oracle/liboracle.so.  Test infrastructure only."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
LIB = os.path.join(HERE, "liboracle.so")
SOURCES = [os.path.join(HERE, f) for f in ("dmmv_oracle.c", "dmmv_oracle_impl.inc", "alns_common.inc",
                                           "alns_oracle_impl.inc", "swap_oracle_impl.inc", "l2_oracle_impl.inc")]


def _cpu_has_fma() -> bool:
    try:
        with open("/proc/cpuinfo") as f:
            for line in f:
                if line.startswith("flags"):
                    return " fma " in line + " "
    except OSError:
        pass
    return False


def needs_build() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    return any(os.path.getmtime(s) > t for s in SOURCES)


def build(force: bool = False) -> str:
    if not force and not needs_build():
        return LIB
    cmd = ["gcc", "-std=c11", "-O2", "-ffp-contract=off", "-fno-fast-math", "-fopenmp",
           "-fPIC", "-shared", "-Wall", "-Wextra", "-o", LIB, SOURCES[0], "-lm"]
    if _cpu_has_fma():
        cmd.insert(1, "-mfma")          # inline the explicit fma() calls; same results as libm's
    subprocess.check_call(cmd, cwd=HERE)
    return LIB


if __name__ == "__main__":
    print(build(force=True))
