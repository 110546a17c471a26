"""Host-side checks of bench.py: the byte model, the kernel label it prints against the
launch table of the kernels' source, and the refusal of more than one GPU."""
import os
import re
import subprocess
import sys

import bench

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_algorithmic_bytes_model():
    # int32 row_ptr and col_idx, fp32 values, B read once, C written once
    M, K, nnz, N = 512, 2048, 209715, 128
    assert bench.bytes_min(M, K, nnz, N) == 4 * (M + 1) + 8 * nnz + 4 * K * N + 4 * M * N == 2990492


def test_kernel_label_follows_the_launch_table():
    src = open(os.path.join(ROOT, "paper_2506_15174_amd", "csrc", "spmm_kernels.hip")).read()
    table = {int(u): (int(d2), int(d4), int(d8))
             for u, d2, d4, d8 in re.findall(r"case (\d): launch_slices<\d, (\d), (\d), (\d)>\(", src)}
    assert sorted(table) == [1, 2, 4, 8]
    for ufi, (d2, d4, d8) in table.items():
        assert bench.kernel_shape(128, ufi) == "S=2,VW=4,D=%d" % d2
        assert bench.kernel_shape(64, ufi) == "S=4,VW=4,D=%d" % d4
        assert bench.kernel_shape(32, ufi) == "S=8,VW=4,D=%d" % d8
        # 128 columns of a 16384-row B exceed one L2, 64 fit: tiles of 64
        assert bench.kernel_shape(128, ufi, 16384).startswith("S=4,VW=4,D=%d" % d4)
    # plans made for narrow B: chunks of 16 / 32 / 64 columns on 8 / 16 / 32 or 64 slices, depth by height
    narrow = {int(u): int(d) for u, d in re.findall(r"case (\d): ok = launch_narrow<\d, (\d)>\(", src)}
    assert sorted(narrow) == [1, 2, 4, 8]
    for ufi, d in narrow.items():
        assert bench.kernel_shape(32, ufi, ufk=16) == "S=8,VW=4,D=%d,UFK=16" % d
        assert bench.kernel_shape(16, ufi, ufk=32) == "S=16,VW=4,D=%d,UFK=32" % d
        assert bench.kernel_shape(8, ufi, ufk=64) == "S=32,VW=4,D=%d,UFK=64" % d
        assert bench.kernel_shape(4, ufi, ufk=64) == "S=64,VW=4,D=%d,UFK=64" % d
    assert bench.tiles_of_64(128, 16384) and not bench.tiles_of_64(128, 8192)
    assert not bench.tiles_of_64(64, 16384) and not bench.tiles_of_64(128, 16385)
    # the executor's own condition, as written in its source
    api = open(os.path.join(ROOT, "paper_2506_15174_amd", "csrc", "spmm_api.cpp")).read()
    assert "h.K * 512 > ((int64_t)4 << 20) && (int64_t)h.K * 256 <= ((int64_t)4 << 20)" in api


def test_counter_figures_are_passed_on_only_for_the_profiled_sources(monkeypatch):
    """Traffic and counter figures come from the committed counter summaries, which carry
    the hash of the library sources they were taken on: they are withheld once the sources
    differ, and a plan cut into column ranges is labelled as such."""
    now = bench.kernel_source_hash()
    traffic, prov = bench.measured_traffic("stress", 128)
    assert prov is not None and prov["file"].startswith("profiles/") and prov["source_hash_now"] == now
    assert (traffic is not None) == prov["current"] == (prov["source_hash_at_profile"] == now)
    counters = bench.measured_counters("stress", 128)
    assert (counters is not None) == prov["current"]
    if counters:
        assert set(counters) == {"l2_hit", "valu_busy", "l1_busy"} and all(0 < v <= 100 for v in counters.values())
    monkeypatch.setattr(bench, "kernel_source_hash", lambda: "0" * 16)
    traffic, prov = bench.measured_traffic("stress", 128)
    assert traffic is None and not prov["current"] and prov["withheld_bytes"] > 0
    assert bench.measured_counters("stress", 128) is None
    assert bench.kernel_shape(128, 8, 16384, k_slices=4) == "S=2,VW=4,D=2, 4 column ranges"


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True,
                       text=True, timeout=120)
    assert r.returncode != 0
    assert "one GPU" in (r.stdout + r.stderr)


def test_build_refuses_kernel_instances_that_spill():
    """The build parses the compiler's resource remarks and fails when any kernel instance
    uses scratch memory (a spilled register could be an in-flight load destination)."""
    import pytest
    from paper_2506_15174_amd import build
    ok = ("remark: k.hip:1:1: Function Name: kernel_a [-Rpass-analysis=kernel-resource-usage]\n"
          "remark: k.hip:1:1:     VGPRs: 64 [-Rpass-analysis=kernel-resource-usage]\n"
          "remark: k.hip:1:1:     ScratchSize [bytes/lane]: 0 [-Rpass-analysis=kernel-resource-usage]\n"
          "remark: k.hip:1:1:     SGPRs Spill: 0 [-Rpass-analysis=kernel-resource-usage]\n"
          "remark: k.hip:1:1:     VGPRs Spill: 0 [-Rpass-analysis=kernel-resource-usage]\n")
    assert build.check_no_spills(ok) == 1
    with pytest.raises(RuntimeError, match="kernel_a: VGPRs Spill = 3"):
        build.check_no_spills(ok.replace("VGPRs Spill: 0", "VGPRs Spill: 3"))
    with pytest.raises(RuntimeError, match="ScratchSize"):
        build.check_no_spills(ok.replace("lane]: 0", "lane]: 16"))
    with pytest.raises(RuntimeError, match="no resource remarks"):
        build.check_no_spills("")
