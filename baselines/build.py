"""Build the comparison-system shim used by bench.py (hipSPARSE CSR SpMM and
rocBLAS SGEMM behind two C calls).  Not part of the product library."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
LIB = os.path.join(HERE, "libhip_baselines.so")
ROCM = os.environ.get("ROCM_PATH", "/opt/rocm")


def build():
    cmd = [os.path.join(ROCM, "bin", "hipcc"), "-x", "c++", "-O2", "-std=c++17", "-fPIC", "-shared",
           "-D__HIP_PLATFORM_AMD__=1", "-I", os.path.join(ROCM, "include"),
           os.path.join(HERE, "hip_baselines.cpp"), "-o", LIB,
           "-L", os.path.join(ROCM, "lib"), "-lhipsparse", "-lrocblas", "-lamdhip64"]
    subprocess.run(cmd, check=True)
    return LIB


MICROBENCH = os.path.join(HERE, "microbench_paths")


def build_microbench():
    """Compile the memory-path microbenchmark (a gfx950 executable; run it on the GPU machine)."""
    cmd = [os.path.join(ROCM, "bin", "hipcc"), "--offload-arch=gfx950", "-O3",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           os.path.join(HERE, "microbench_paths.hip"), "-o", MICROBENCH]
    subprocess.run(cmd, check=True, stdout=subprocess.DEVNULL, stderr=subprocess.DEVNULL)
    return MICROBENCH


if __name__ == "__main__":
    print(build())
    print(build_microbench())
