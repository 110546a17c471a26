"""Compile the C oracle (test infrastructure) with gcc.

Two libraries come from the one source file ``spmm_oracle.c``: the serial
build that parity tests use, and a row-parallel OpenMP build of the same
source whose only use is the benchmark's CPU-baseline timing.
"""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "spmm_oracle.c")
LIB_SERIAL = os.path.join(HERE, "liboracle_spmm.so")
LIB_OMP = os.path.join(HERE, "liboracle_spmm_omp.so")

_COMMON = ["gcc", "-O2", "-ffp-contract=off", "-fPIC", "-shared", "-std=c11",
           "-Wall", "-Wextra", "-Werror"]


def build(force=True):
    """Build both libraries; with force=False only what is missing or stale."""
    for lib, extra in ((LIB_SERIAL, []), (LIB_OMP, ["-fopenmp"])):
        fresh = (os.path.exists(lib)
                 and os.path.getmtime(lib) >= os.path.getmtime(SRC))
        if force or not fresh:
            subprocess.run(_COMMON + extra + [SRC, "-o", lib, "-lm"], check=True)
    return LIB_SERIAL, LIB_OMP


if __name__ == "__main__":
    print(build())
