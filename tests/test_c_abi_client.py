"""The C ABI is usable from plain C: the header compiles as C99 with -pedantic and
a small client links against the shared library (no Python, no torch in between)."""
import os
import shutil
import subprocess

import pytest

import paper_2506_15174_amd as spmm

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)


@pytest.mark.skipif(shutil.which("gcc") is None, reason="needs gcc")
def test_plain_c_client_builds_and_runs(tmp_path):
    assert os.path.exists(spmm.LIB_PATH), "build the library first (python -m paper_2506_15174_amd.build)"
    lib_dir = os.path.dirname(spmm.LIB_PATH)
    rocm_lib = os.path.join(os.environ.get("ROCM_PATH", "/opt/rocm"), "lib")
    exe = str(tmp_path / "client")
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-Werror", "-pedantic", "-I", os.path.join(ROOT, "include"),
                    os.path.join(HERE, "c_abi_client.c"), "-L", lib_dir, "-lspmm_cdna4",
                    "-Wl,-rpath," + lib_dir, "-Wl,-rpath," + rocm_lib, "-o", exe], check=True)
    res = subprocess.run([exe], capture_output=True, text=True, timeout=60)
    assert res.returncode == 0, res.stdout + res.stderr
    assert "M=3 K=4 nnz=3" in res.stdout and "groups=3 blocks=1" in res.stdout
    assert "execute on host-only plan: invalid argument" in res.stdout
