"""Build the gfx950 shared library in-tree with hipcc.

    python -m paper_2506_15174_amd.build

Output: paper_2506_15174_amd/lib/libspmm_cdna4.so (C ABI of include/spmm.h).
"""
import os
import shutil
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB_DIR = os.path.join(HERE, "lib")
LIB_PATH = os.path.join(LIB_DIR, "libspmm_cdna4.so")

SOURCES = ["spmm_kernels.hip", "spmm_plan.cpp", "spmm_api.cpp"]
HEADERS = ["spmm_format.h", "spmm_kernels.h", "spmm_plan.h"]


ROCM = os.environ.get("ROCM_PATH", "/opt/rocm")


def _hipcc():
    exe = shutil.which("hipcc") or os.path.join(ROCM, "bin", "hipcc")
    if not os.path.exists(exe):
        raise RuntimeError("hipcc not found; the library targets gfx950 only")
    return exe


def is_stale():
    if not os.path.exists(LIB_PATH):
        return True
    t = os.path.getmtime(LIB_PATH)
    deps = [os.path.join(CSRC, f) for f in SOURCES + HEADERS]
    deps.append(os.path.join(os.path.dirname(HERE), "include", "spmm.h"))
    return any(os.path.getmtime(d) > t for d in deps)


def _run(cmd, verbose):
    res = subprocess.run(cmd, capture_output=True, text=True)
    noise = ("is not a recognized feature for this target", "-Rpass-analysis=kernel-resource-usage")
    import re
    err = "\n".join(ln for ln in res.stderr.splitlines()
                    if not any(n in ln for n in noise) and not re.match(r"^\s*(\d+)?\s*\|", ln))
    if verbose and err:
        print(err)
    if res.returncode != 0:
        raise RuntimeError("%s failed:\n%s" % (cmd[0], err))
    return res.stderr


def check_no_spills(remarks):
    """The kernels issue their loads of B rows from inline assembly and await them later
    (an explicit s_waitcnt): a register the compiler spills or copies in between would
    carry stale data.  No instance may therefore use scratch memory at all: the compiler's
    resource remarks (-Rpass-analysis=kernel-resource-usage) must report zero spilled
    VGPRs and SGPRs and a zero scratch size for every kernel.  Returns the number of
    kernels checked; raises with the offenders otherwise."""
    import re
    name, bad, seen = None, [], 0
    for ln in remarks.splitlines():
        m = re.search(r"Function Name: (\S+)", ln)
        if m:
            name = m.group(1)
            seen += 1
            continue
        m = re.search(r"(VGPRs Spill|SGPRs Spill|ScratchSize \[bytes/lane\]): (\d+)", ln)
        if m and name and int(m.group(2)) != 0:
            bad.append("%s: %s = %s" % (name, m.group(1), m.group(2)))
    if seen == 0:
        raise RuntimeError("the compiler printed no resource remarks: the spill check did not run")
    if bad:
        raise RuntimeError("kernel instances use scratch memory (give them a larger register budget "
                           "or a shallower pipeline):\n  " + "\n  ".join(bad))
    return seen


def build(verbose=False):
    """Compile every source for gfx950 and link the shared library.

    The device translation unit goes through hipcc on its own (its fat binary
    is embedded in its object file); host-only units are plain C++; the link is
    an ordinary shared-library link against the HIP runtime."""
    os.makedirs(LIB_DIR, exist_ok=True)
    obj_dir = os.path.join(LIB_DIR, "obj")
    os.makedirs(obj_dir, exist_ok=True)
    hipcc = _hipcc()
    common = ["-O3", "-std=c++17", "-fPIC", "-Wall", "-Wextra", "-Wno-unused-parameter",
              "-I", CSRC, "-I", os.path.join(ROCM, "include"), "-D__HIP_PLATFORM_AMD__=1"]
    objects = []
    for s in SOURCES:
        obj = os.path.join(obj_dir, os.path.splitext(s)[0] + ".o")
        if s.endswith(".hip"):
            cmd = [hipcc, "--offload-arch=gfx950",
                   # packed-fp32 forms are kept out of the generated code on purpose
                   "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
                   "-Rpass-analysis=kernel-resource-usage"]
        else:
            cmd = [hipcc, "-x", "c++"]
        remarks = _run(cmd + common + ["-c", os.path.join(CSRC, s), "-o", obj], verbose)
        if s.endswith(".hip"):
            n = check_no_spills(remarks)
            if verbose:
                print("%s: %d kernel instances, none uses scratch memory" % (s, n))
        objects.append(obj)
    _run([hipcc, "-shared", "-fPIC"] + objects +
         ["-L", os.path.join(ROCM, "lib"), "-lamdhip64", "-pthread", "-o", LIB_PATH], verbose)
    return LIB_PATH


if __name__ == "__main__":
    print(build(verbose=True))
