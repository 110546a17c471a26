#!/usr/bin/env python3
"""Benchmark of the hot path: fp32 CSR SpMM C = A x B on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload conv|stress|ffn|ffn-all|matrix|sweep|narrow|sparsity|ablation|tune]

A step is one pass of the whole hot path (spmm_execute, every kernel it
launches) over the workload's column counts, with the plan and all operands
resident in HBM before the timed region.  Plan creation is timed separately
(it is amortised over inferences) and never part of a step.

Prints ONE JSON line:
  value         GFLOP/s = 2 nnz sum(bCols) / step time
  roofline      dominant kernel (the widest column count of the workload):
                algorithmic bytes 4(M+1) + 8 nnz + 4 K N + 4 M N per launch over
                the kernel's average duration, measured with HIP events on the
                launch stream inside the timed region, against 8 TB/s
                (hot: the same operands every call, the paper's protocol);
                roofline.gather: wave-wide loads of B rows per second against the
                measured gather ceiling; per_bcols[N].cold: the same launch with
                plan, B and C rotated over more copies than the caches hold
  cpu_baseline  the CPU oracle timed on the host cores for the same products
  baselines     hipSPARSE CSR SpMM (fastest of its CSR algorithms) and rocBLAS
                SGEMM on the densified matrix, same inputs, timed with HIP events
                inside a small C shim (baselines/)

Other workloads print one JSON line of their own: `sweep` (48 matrices x 3 column
counts against the two libraries), `narrow` (the same for 4 / 8 / 16 columns), `ffn-all` (the same for the eight
feed-forward matrices), `sparsity` (the same for a 512 x 512 matrix from 50 to 99 % pruned at 64 and 4 columns,
the sweep of the paper's Figure 9), `ablation` (the method's ingredients switched
on one by one, the ladder of the paper's Figure 7) and `tune` (every panel height
and three group budgets forced per matrix: what the closed schedule rule loses
against the best candidate, and the plan's size against CSR and dense).
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
# 256 CUs x 4 SIMDs x 16 lanes x 2 flop x 2.4 GHz, no packed-fp32 forms
FP32_VALU_PEAK_TFLOPS = 78.6


def bytes_min(M, K, nnz, N):
    return 4 * (M + 1) + 8 * nnz + 4 * K * N + 4 * M * N


def build_workload(name, args=None):
    from workloads import generators as gen
    if name == "matrix":
        # one matrix of the sweep's recipe, for counter runs: --shape MxK --sparsity s --bcols N
        M, K = (int(x) for x in args.shape.lower().split("x"))
        return ("magnitude-pruned N(0,1) %dx%d @%g%% (sweep recipe, seed %d), bCols %d"
                % (M, K, 100 * args.sparsity, args.seed, args.bcols),
                gen.magnitude_pruned(M, K, args.sparsity, args.seed), (args.bcols,))
    if name == "conv":
        return ("conv1x1 512x2048 @80% magnitude-pruned N(0,1), bCols 32/64/128 (configs[1])",
                gen.conv_layer(), (32, 64, 128))
    if name == "stress":
        return ("stress 16384x16384 @95% Zipf(1.5) rows, 5% empty, bCols 128 (configs[3])",
                gen.stress(), (128,))
    if name == "ffn":
        return ("ffn 4096x1024 @70% lognormal rows, bCols 32/64/128 (configs[2])",
                gen.ffn(0, 0), (32, 64, 128))
    raise SystemExit("unknown workload %r" % name)


_BASE = None
# Every per-launch figure (this library, hipSPARSE, rocBLAS) is the median over SAMPLES
# HIP-event intervals of INNER back-to-back calls issued from one C loop on the default
# stream (baselines/hip_baselines.cpp): at 4-7 us per kernel an interpreter between two
# launches (3.4 us per ctypes call) would pace them.
SAMPLES, INNER = 10, 20


def _baseline_lib():
    """The comparison-system shim (hipSPARSE CSR SpMM with every algorithm the
    header offers, rocBLAS SGEMM); built on demand, loaded after torch so that it
    shares torch's HIP runtime."""
    global _BASE
    if _BASE is None:
        import ctypes
        from baselines import build as bbuild
        if not os.path.exists(bbuild.LIB):
            bbuild.build()
        lib = ctypes.CDLL(bbuild.LIB)
        vp, ci = ctypes.c_void_p, ctypes.c_int
        lib.baseline_hipsparse_spmm.argtypes = [ci, ci, ci, ci, vp, vp, vp, vp, vp, ci, ci, vp]
        lib.baseline_rocblas_sgemm.argtypes = [ci, ci, ci, vp, vp, vp, ci, ci, vp]
        lib.baseline_time_spmm_execute.argtypes = [vp, vp, vp, ci, vp, ci, ci, vp]
        lib.baseline_time_spmm_execute_rotating.argtypes = [vp, vp, vp, vp, ci, ci, ci, ci, vp]
        _BASE = lib
    return _BASE


def measure_baselines(torch, np, csr, cols, Bs, dense_limit=1 << 28):
    """hipSPARSE CSR SpMM (best of its algorithms) and rocBLAS SGEMM on the same
    device-resident inputs; times in microseconds, rates with the same numerator
    2 nnz N as the library's own figure."""
    import ctypes
    out = {}
    try:
        lib = _baseline_lib()
        nnz = int(csr.row_ptr[-1])
        d_rp = torch.from_numpy(csr.row_ptr.astype(np.int32)).cuda()
        d_ci = torch.from_numpy(csr.col_idx.astype(np.int32)).cuda()
        d_v = torch.from_numpy(csr.vals).cuda()
        A_dn = None
        if csr.M * csr.K <= dense_limit:
            A_dn = torch.zeros((csr.M, csr.K), dtype=torch.float32, device="cuda")
            rows = torch.repeat_interleave(torch.arange(csr.M, device="cuda"),
                                           torch.from_numpy(np.diff(csr.row_ptr).astype(np.int64)).cuda())
            A_dn.index_put_((rows, d_ci.long()), d_v, accumulate=True)
        for N in cols:
            C = torch.empty((csr.M, N), dtype=torch.float32, device="cuda")
            torch.cuda.synchronize()
            ms = (ctypes.c_float * 4)(-1, -1, -1, -1)
            entry = {}
            if nnz > 0:
                rc = lib.baseline_hipsparse_spmm(csr.M, csr.K, N, nnz, d_rp.data_ptr(), d_ci.data_ptr(),
                                                 d_v.data_ptr(), Bs[N].data_ptr(), C.data_ptr(), SAMPLES, INNER, ms)
                good = [m for m in ms if m > 0]
                if rc == 0 and good:
                    best = min(good)
                    entry["hipsparse_us_by_alg"] = [round(m * 1e3, 2) for m in ms]
                    entry["hipsparse_best_us"] = round(best * 1e3, 3)
                    entry["hipsparse_gflops"] = round(2.0 * nnz * N / (best * 1e-3) / 1e9, 1)
            if A_dn is not None:
                one = ctypes.c_float(-1)
                rc = lib.baseline_rocblas_sgemm(csr.M, csr.K, N, A_dn.data_ptr(), Bs[N].data_ptr(), C.data_ptr(),
                                                SAMPLES, INNER, ctypes.byref(one))
                if rc == 0 and one.value > 0:
                    entry["rocblas_sgemm_us"] = round(one.value * 1e3, 3)
                    entry["rocblas_effective_gflops"] = round(2.0 * nnz * N / (one.value * 1e-3) / 1e9, 1)
            out[str(N)] = entry
    except Exception as exc:  # comparison systems are context, never a reason to fail the bench
        out["error"] = repr(exc)
    return out


def kernel_source_hash():
    """First 16 hex digits of the SHA-256 over the library's sources (kernels, format,
    inspector, C ABI): counter summaries under profiles/ record the hash they were taken
    at, so that a figure measured on other code is never passed on as this code's."""
    import hashlib
    h = hashlib.sha256()
    csrc = os.path.join(ROOT, "paper_2506_15174_amd", "csrc")
    for name in sorted(os.listdir(csrc)):
        if name.endswith((".hip", ".cpp", ".h")):
            with open(os.path.join(csrc, name), "rb") as f:
                h.update(name.encode() + b"\0" + f.read())
    return h.hexdigest()[:16]


def measured_traffic(workload, N):
    """HBM bytes per launch (scaled FETCH_SIZE + WRITE_SIZE) from the committed rocprofv3
    counter summaries: lines `traffic_bytes_per_launch <workload> <bCols> <bytes> <source hash>`.
    Counters cannot be read from inside this process, so the figure is the last profiled
    one; it is passed on only when the summary was taken on the library sources that are
    in the tree now (kernel_source_hash), else the bytes are withheld.
    Returns (bytes or None, provenance dict or None)."""
    import glob
    now = kernel_source_hash()
    for path in sorted(glob.glob(os.path.join(ROOT, "profiles", "*.md"))):
        with open(path) as f:
            for line in f:
                parts = line.split()
                if len(parts) >= 4 and parts[0] == "traffic_bytes_per_launch" \
                        and parts[1] == workload and parts[2] == str(N):
                    taken_at = parts[4] if len(parts) > 4 else None
                    prov = {"file": "profiles/" + os.path.basename(path), "source_hash_at_profile": taken_at,
                            "source_hash_now": now, "current": taken_at == now}
                    if taken_at != now:
                        prov["withheld_bytes"] = int(parts[3])
                        return None, prov
                    return int(parts[3]), prov
    return None, None


def measured_counters(workload, N):
    """L2 hit rate, VALU busy and vector-L1 busy (per cent) of the product's main kernel from
    the same committed counter run as measured_traffic: lines `counters_per_launch <workload>
    <bCols> l2_hit=.. valu_busy=.. l1_busy=.. <source hash>`; passed on under the same
    condition (taken on the library sources that are in the tree now)."""
    import glob
    now = kernel_source_hash()
    for path in sorted(glob.glob(os.path.join(ROOT, "profiles", "*.md"))):
        with open(path) as f:
            for line in f:
                parts = line.split()
                if len(parts) >= 5 and parts[0] == "counters_per_launch" and parts[1] == workload \
                        and parts[2] == str(N) and parts[-1] == now:
                    return {k: float(v) for k, v in (x.split("=") for x in parts[3:-1])}
    return None


def tiles_of_64(N, K):
    """True when spmm_execute runs more than 64 columns as tiles of 64: 128 columns of B
    exceed one 4 MiB L2 and 64 columns fit (8192 < K <= 16384)."""
    return N > 64 and K * 512 > 4 << 20 and K * 256 <= 4 << 20


def kernel_shape(N, ufi, K=0, ufk=8, k_slices=1):
    """Template arguments of the instance spmm_execute launches for a tile of N columns
    (N a multiple of 4, at most 128) of a plan with panels of `ufi` rows and chunks of
    `ufk` columns: slices per wave, floats per lane, pipeline depth (the tables of
    spmm_launch_chunks).  When 128 columns of B exceed one L2 and 64 fit
    (8192 < K <= 16384) the product runs as two tiles of 64 columns, unless the plan is cut
    into column ranges (k_slices > 1), which runs full tiles.  Plans made for narrow B (ufk
    16 / 32 / 64) run on 8 / 16 / 32 or 64 slices."""
    if ufk != 8:
        S = {16: 8, 32: 16}.get(ufk, 64 if N <= 4 else 32)
        depth = {8: 4, 4: 3, 2: 4, 1: 4}[ufi]
        return "S=%d,VW=4,D=%d,UFK=%d" % (S, depth, ufk)
    depth = {8: (2, 3, 4), 4: (2, 3, 4), 2: (2, 2, 6), 1: (2, 2, 8)}[ufi]
    if k_slices == 1 and tiles_of_64(N, K):
        return "S=4,VW=4,D=%d, tiles of 64 columns" % depth[1]
    if N > 64:
        return "S=2,VW=4,D=%d%s" % (depth[0], ", %d column ranges" % k_slices if k_slices > 1 else "")
    if N > 32:
        return "S=4,VW=4,D=%d" % depth[1]
    return "S=8,VW=4,D=%d" % depth[2]


SPARSITY_SWEEP = (0.5, 0.6, 0.7, 0.8, 0.85, 0.9, 0.95, 0.98, 0.99)


def _measure_points(torch, np, spmm, gen, entries, cols, make_matrix, keep=None, with_baselines=True):
    """Per (matrix, bCols): one hinted plan, the per-launch time of spmm_execute and of the
    two comparison libraries on the same device-resident inputs.  With `keep` (a list) the
    plan, B and C of every point stay alive and are appended to it as
    (plan, B, C, N, nnz); otherwise they are released matrix by matrix."""
    rows_out = []
    for entry in entries:
        csr = make_matrix(entry)
        nnz = int(csr.row_ptr[-1])
        # one plan per column count: the schedule constants are chosen per bCols
        plans = {N: spmm.plan_create(csr.M, csr.K, csr.row_ptr, csr.col_idx, csr.vals, n_hint=N) for N in cols}
        Bs = {N: torch.from_numpy(gen.activations_for(csr, N)).cuda() for N in cols}
        Cs = {N: torch.empty((csr.M, N), dtype=torch.float32, device="cuda") for N in cols}
        base = measure_baselines(torch, np, csr, cols, Bs) if with_baselines else {}
        for N in cols:
            plan, info = plans[N], plans[N].describe()
            _, med = time_execute(torch, plan, Bs[N], Cs[N], N)
            b = base.get(str(N), {})
            rows_out.append({"index": entry["index"], "M": csr.M, "K": csr.K, "sparsity": entry["sparsity"],
                             "nnz": nnz, "N": N, "ufi": info["ufi"], "group_nnz": info["group_nnz"],
                             "n_blocks": info["n_blocks"], "us": round(med * 1e3, 3),
                             "gflops": round(2.0 * nnz * N / (med * 1e-3) / 1e9, 1),
                             "hbm_model_gbs": round(bytes_min(csr.M, csr.K, nnz, N) / (med * 1e-3) / 1e9, 1),
                             "hipsparse_us": b.get("hipsparse_best_us"), "rocblas_us": b.get("rocblas_sgemm_us")})
            print(json.dumps(rows_out[-1]), file=sys.stderr, flush=True)
            if keep is not None:
                keep.append((plan, Bs[N], Cs[N], N, nnz))
        if keep is None:
            for plan in plans.values():
                plan.destroy()
        del plans, Bs, Cs
    return rows_out


def _summarise(rows_out, cols):
    """Geometric-mean speedups over the two libraries and the share of points faster, per
    column count and over all points (the shape of the paper's Table 1)."""
    import math
    summary = {}
    for N in tuple(cols) + ("all",):
        sel = [r for r in rows_out if N == "all" or r["N"] == N]
        for key in ("hipsparse_us", "rocblas_us"):
            sp = [r[key] / r["us"] for r in sel if r[key]]
            if sp:
                summary["%s_%s" % (key[:-3], N)] = {
                    "geomean_speedup": round(math.exp(sum(math.log(x) for x in sp) / len(sp)), 3),
                    "faster_pct": round(100.0 * sum(1 for x in sp if x > 1.0) / len(sp), 1), "points": len(sp)}
    return summary


def run_sweep(args, cols=(32, 64, 128), narrow=False, ffn=False, square512=False):
    """Configuration 4: 48 magnitude-pruned matrices x bCols 32/64/128 against
    hipSPARSE CSR SpMM and rocBLAS SGEMM; geometric means of the speedups and the
    share of points where this library is faster (the shape of the paper's Table 1).
    narrow: the same on the 30 matrices with M, K >= 1024 for bCols 4/8/16, the
    widths below the kernel's narrowest tile (the paper's Figure 9 measures bCols 4).
    ffn: the same on the eight feed-forward matrices of configuration 2 (two shapes x four
    sparsities, lognormal row lengths).
    square512: the same on one 512 x 512 magnitude-pruned matrix per sparsity from 50 to
    99 % for bCols 64 and 4 (the sweep of the paper's Figure 9)."""
    import numpy as np
    import torch
    import paper_2506_15174_amd as spmm
    from workloads import generators as gen
    torch.cuda.set_device(0)
    t_start = time.perf_counter()
    if ffn:
        entries = [dict(index=4 * si + pi, sparsity=gen.FFN_SPARSITIES[pi], ffn=(si, pi))
                   for si in range(len(gen.FFN_SHAPES)) for pi in range(len(gen.FFN_SPARSITIES))]
        make = lambda e: gen.ffn(*e["ffn"])
    elif square512:
        entries = [dict(index=i, sparsity=sp, seed=9000 + i) for i, sp in enumerate(SPARSITY_SWEEP)]
        make = lambda e: gen.magnitude_pruned(512, 512, e["sparsity"], e["seed"])
    else:
        entries = _ladder_matrices(gen) if narrow else gen.sweep_entries()
        make = gen.sweep_matrix
    rows_out = _measure_points(torch, np, spmm, gen, entries, cols, make)
    summary = _summarise(rows_out, cols)
    total_flops = sum(2.0 * r["nnz"] * r["N"] for r in rows_out)
    total_s = sum(r["us"] for r in rows_out) * 1e-6
    out = {"metric": "fp32 CSR SpMM GFLOP/s (2*nnz*bCols)", "value": round(total_flops / total_s / 1e9, 2),
           "unit": "GFLOP/s", "n_gpus": 1, "steps": 1, "warmup": 10, "ms_per_step": round(total_s * 1e3, 4),
           "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
           "config": {"workload": ("ffn: 8 feed-forward matrices (lognormal rows) x bCols 32/64/128 (configs[2])" if ffn else
                                   "sparsity sweep: 512 x 512 magnitude-pruned, 50 to 99 % pruned, bCols 64 and 4" if square512 else
                                   "narrow B: 30 magnitude-pruned matrices (M, K >= 1024) x bCols 4/8/16" if narrow else
                                   "sweep: 48 magnitude-pruned matrices x bCols 32/64/128 (configs[4])"),
                      "wall_s": round(time.perf_counter() - t_start, 1)},
           "summary": summary, "points": rows_out}
    print(json.dumps(out))


def time_execute(torch, plan, B, C, N, samples=SAMPLES, inner=INNER):
    """(mean, median) duration in ms of one spmm_execute launch on the default stream,
    timed by the C loop of the shim with HIP events around `inner` back-to-back calls.
    Without the shim (it needs hipSPARSE and rocBLAS to link) the same loop runs in
    Python, where the interpreter paces kernels shorter than about 4 us."""
    import ctypes
    import paper_2506_15174_amd as spmm
    assert (torch.cuda.current_stream().cuda_stream or 0) == 0, "the timing loops launch on the default stream"
    pb, pc = B.data_ptr() or None, C.data_ptr() or None
    torch.cuda.synchronize()
    try:
        lib = _baseline_lib()
    except Exception as exc:
        print("timing shim unavailable (%r): timing from Python" % (exc,), file=sys.stderr)
        lib = None
    if lib is not None:
        fn = ctypes.cast(spmm.load().spmm_execute, ctypes.c_void_p)
        ms = (ctypes.c_float * 2)(-1, -1)
        rc = lib.baseline_time_spmm_execute(fn, plan.handle, pb, N, pc, samples, inner, ms)
        if rc != 0 or ms[0] <= 0:
            raise RuntimeError("timing loop failed (status %d)" % rc)
        return ms[1], ms[0]
    for _ in range(3):
        plan.execute_raw(pb, N, pc, None)
    torch.cuda.synchronize()
    ts = []
    for _ in range(samples):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(inner):
            plan.execute_raw(pb, N, pc, None)
        e1.record()
        e1.synchronize()
        ts.append(e0.elapsed_time(e1) / inner)
    ts.sort()
    return sum(ts) / len(ts), ts[len(ts) // 2]


GATHER_CEILING_GWLS = 32.0      # G wave-wide 16-byte-per-lane loads per second, measured (baselines/microbench_paths.hip)
COLD_WORKING_SET = 1 << 30      # bytes the rotating copies must exceed (four times the 256 MiB Infinity Cache)
COLD_MAX_COPIES = 256


def time_execute_cold(torch, csr, plan, B, N, samples=SAMPLES, inner=INNER):
    """Cold-cache duration of one spmm_execute: independent copies of (plan, B, C), at
    least 1 GiB together or 256 of them, taken in turn by the shim's C loop, so that no
    call finds its plan, B or C in L2 or in the Infinity Cache.  Returns a dict, or None
    without the shim."""
    import ctypes
    import paper_2506_15174_amd as spmm
    try:
        lib = _baseline_lib()
    except Exception:
        return None
    info = plan.describe()
    one = info["device_bytes"] + 4 * N * (csr.K + csr.M)
    copies = max(2, min(COLD_MAX_COPIES, -(-COLD_WORKING_SET // max(one, 1))))
    plans = [plan] + [spmm.plan_create(csr.M, csr.K, csr.row_ptr, csr.col_idx, csr.vals, n_hint=N)
                      for _ in range(copies - 1)]
    Bs = [B] + [B.clone() for _ in range(copies - 1)]
    Cs = [torch.empty((csr.M, N), dtype=torch.float32, device="cuda") for _ in range(copies)]
    vp = ctypes.c_void_p * copies
    fn = ctypes.cast(spmm.load().spmm_execute, ctypes.c_void_p)
    ms = (ctypes.c_float * 2)(-1, -1)
    torch.cuda.synchronize()
    # every sample walks all copies at least once
    inner = max(inner, copies)
    rc = lib.baseline_time_spmm_execute_rotating(fn, vp(*[p.handle for p in plans]), vp(*[b.data_ptr() for b in Bs]),
                                                 vp(*[c.data_ptr() for c in Cs]), copies, N, samples, inner, ms)
    torch.cuda.synchronize()
    for p in plans[1:]:
        p.destroy()
    if rc != 0 or ms[0] <= 0:
        raise RuntimeError("cold timing loop failed (status %d)" % rc)
    return {"copies": copies, "working_set_bytes": one * copies, "us": round(ms[0] * 1e3, 3),
            "mean_us": round(ms[1] * 1e3, 3)}


def _time_plan(torch, plan, B, C, N, reps=SAMPLES, batch=INNER):
    return time_execute(torch, plan, B, C, N, reps, batch)[1] * 1e3   # median, us


def _geomean(xs):
    import math
    return math.exp(sum(math.log(x) for x in xs) / len(xs))


def _ladder_matrices(gen):
    """The sweep's matrices with at least 1024 rows and columns (30 of the 48)."""
    return [e for e in gen.sweep_entries() if e["M"] >= 1024 and e["K"] >= 1024]


def run_ablation(args):
    """The ingredients of the method switched on one by one on 30 sweep matrices (paper
    Section 4.3, Figure 7: baseline -> + enumeration -> + coarsening), as geometric-mean
    GFLOP/s per column count:
      rows        one wave per row, rows never cut, no B row requested before the
                  previous chunk is multiplied (the paper's Figure 1a mapping with this
                  kernel's chunked B loads)
      +balance    nnz-balanced row groups: heavy rows cut into pieces that meet in LDS
      +enumerate  panels of 2, 4 or 8 rows enumerated by nonzero pattern, height by the
                  schedule rule; still one chunk at a time (pipeline depth 1)
      +coarsen    the chunks of B rows of the next D - 1 steps in flight while one is
                  multiplied (the paper's unroll(k, UFk), Section 3.3.2)
      full        the plan the inspector makes by itself: as +coarsen, and cut into column
                  ranges bound to the XCDs' L2 caches where a tile of B fills or exceeds one
                  (of these matrices only 8192 x 8192 at 50 to 80 % for 128 columns)"""
    import torch
    import paper_2506_15174_amd as spmm
    from workloads import generators as gen
    torch.cuda.set_device(0)
    cols = (32, 64, 128)
    rungs = ("rows", "+balance", "+enumerate", "+coarsen", "full")
    pts = []
    t_start = time.perf_counter()
    for entry in _ladder_matrices(gen):
        csr = gen.sweep_matrix(entry)
        nnz = int(csr.row_ptr[-1])
        a = (csr.M, csr.K, csr.row_ptr, csr.col_idx, csr.vals)
        for N in cols:
            B = torch.from_numpy(gen.activations_for(csr, N)).cuda()
            C = torch.empty((csr.M, N), dtype=torch.float32, device="cuda")
            plans = {"rows": spmm.plan_create(*a, ufi=1, group_nnz=1 << 30, group_panels=1, depth=1, kslices=1),
                     "+balance": spmm.plan_create(*a, ufi=1, n_hint=N, depth=1, kslices=1),
                     "+enumerate": spmm.plan_create(*a, n_hint=N, depth=1, kslices=1),
                     "+coarsen": spmm.plan_create(*a, n_hint=N, kslices=1),
                     "full": spmm.plan_create(*a, n_hint=N)}
            row = {"M": csr.M, "K": csr.K, "sparsity": entry["sparsity"], "N": N,
                   "ufi": plans["full"].describe()["ufi"], "k_slices": plans["full"].describe()["k_slices"]}
            for r in rungs:
                us = _time_plan(torch, plans[r], B, C, N)
                row[r + "_us"] = round(us, 3)
                row[r + "_gflops"] = round(2.0 * nnz * N / us / 1e3, 1)
                plans[r].destroy()
            pts.append(row)
            print(json.dumps(row), file=sys.stderr, flush=True)
    summary = {}
    for N in cols:
        sel = [p for p in pts if p["N"] == N]
        summary[str(N)] = {r: round(_geomean([p[r + "_gflops"] for p in sel]), 1) for r in rungs}
        summary[str(N)]["speedup_full_over_rows"] = round(
            _geomean([p["rows_us"] / p["full_us"] for p in sel]), 3)
        summary[str(N)]["speedup_coarsen_over_enumerate"] = round(
            _geomean([p["+enumerate_us"] / p["+coarsen_us"] for p in sel]), 3)
    full = [p["full_gflops"] for p in pts]
    print(json.dumps({"metric": "fp32 CSR SpMM GFLOP/s (2*nnz*bCols), geomean per rung", "value": round(_geomean(full), 2),
                      "unit": "GFLOP/s", "n_gpus": 1, "higher_is_better": True, "dtype": "f32", "data": "synthetic",
                      "config": {"workload": "ablation ladder on 30 sweep matrices (M, K >= 1024) x bCols 32/64/128",
                                 "wall_s": round(time.perf_counter() - t_start, 1)},
                      "summary": summary, "points": pts}))


# Shapes between those of the sweep that the schedule rule was fitted on as well (they were the
# held-out set of an earlier tuning run, which showed the rule's row-count thresholds to be too
# cautious between 1024 and 4096 rows), and the shapes it was never fitted on: the tuning run
# reports the rule's loss on the latter separately.
FIT_EXTRA = [dict(M=2048, K=8192, sparsity=0.7, seed=7001), dict(M=2048, K=8192, sparsity=0.95, seed=7002),
             dict(M=3072, K=768, sparsity=0.5, seed=7003), dict(M=3072, K=768, sparsity=0.9, seed=7004),
             dict(M=6144, K=1536, sparsity=0.8, seed=7005), dict(M=2048, K=2048, sparsity=0.6, seed=7006),
             dict(M=768, K=3072, sparsity=0.8, seed=7007), dict(M=12288, K=3072, sparsity=0.9, seed=7008)]
HELD_OUT = [dict(M=1536, K=6144, sparsity=0.8, seed=7101), dict(M=2560, K=2560, sparsity=0.7, seed=7102),
            dict(M=3584, K=1024, sparsity=0.6, seed=7103), dict(M=5120, K=5120, sparsity=0.9, seed=7104),
            dict(M=640, K=2560, sparsity=0.7, seed=7105), dict(M=10240, K=2560, sparsity=0.8, seed=7106),
            dict(M=2048, K=4096, sparsity=0.9, seed=7107), dict(M=3072, K=3072, sparsity=0.5, seed=7108)]


def run_tune(args):
    """Offline tuning run (paper Section 3.5): every panel height and three group budgets
    forced on each of the 30 larger sweep matrices per column count; reports what the
    inspector's closed rule loses against the best candidate, and the size of the plan
    against CSR (8 nnz + 4 (M+1) bytes) and dense (4 M K bytes), the comparison of the
    paper's Section 4.4."""
    import torch
    import paper_2506_15174_amd as spmm
    from workloads import generators as gen
    torch.cuda.set_device(0)
    cols = tuple(int(x) for x in args.cols.split(",")) if args.cols else (32, 64, 128)
    pts = []
    t_start = time.perf_counter()
    entries = ([dict(e, heldout=False) for e in _ladder_matrices(gen)] + [dict(e, heldout=False, extra=True) for e in FIT_EXTRA]
               + [dict(e, heldout=True) for e in HELD_OUT])
    for entry in entries:
        csr = gen.magnitude_pruned(entry["M"], entry["K"], entry["sparsity"], entry["seed"])
        nnz = int(csr.row_ptr[-1])
        a = (csr.M, csr.K, csr.row_ptr, csr.col_idx, csr.vals)
        for N in cols:
            B = torch.from_numpy(gen.activations_for(csr, N)).cuda()
            C = torch.empty((csr.M, N), dtype=torch.float32, device="cuda")
            auto = spmm.plan_create(*a, n_hint=N)
            ai = auto.describe()
            _time_plan(torch, auto, B, C, N, reps=3)          # clocks up before the first figure
            row = {"M": csr.M, "K": csr.K, "sparsity": entry["sparsity"], "N": N, "heldout": entry["heldout"],
                   "rule_ufi": ai["ufi"],
                   "rule_group_nnz": ai["group_nnz"], "rule_us": round(_time_plan(torch, auto, B, C, N), 3),
                   "plan_bytes_over_csr": round(ai["device_bytes"] / (8.0 * nnz + 4 * (csr.M + 1)), 3),
                   "plan_bytes_over_dense": round(ai["device_bytes"] / (4.0 * csr.M * csr.K), 3)}
            auto.destroy()
            best = None
            by_ufi = {}
            for ufi in (1, 2, 4, 8):
                g0 = spmm.plan_create(*a, ufi=ufi, n_hint=N, host_only=True).describe()["group_nnz"]
                for g in sorted({max(32, g0 // 2), g0, min(1024, g0 * 2)}):
                    plan = spmm.plan_create(*a, ufi=ufi, group_nnz=g, n_hint=N)
                    us = _time_plan(torch, plan, B, C, N, reps=5)
                    plan.destroy()
                    if best is None or us < best[0]:
                        best = (us, ufi, g)
                    if ufi not in by_ufi or us < by_ufi[ufi][0]:
                        by_ufi[ufi] = (round(us, 3), g)
            row.update(best_us=round(best[0], 3), best_ufi=best[1], best_group_nnz=best[2],
                       rule_over_best=round(row["rule_us"] / best[0], 3), by_ufi=by_ufi)
            pts.append(row)
            print(json.dumps(row), file=sys.stderr, flush=True)
    def loss(sel):
        return {str(N): {"geomean_rule_over_best": round(_geomean([p["rule_over_best"] for p in sel if p["N"] == N]), 3),
                         "worst": max(p["rule_over_best"] for p in sel if p["N"] == N)} for N in cols}
    summary = loss([p for p in pts if not p["heldout"]])
    summary_heldout = loss([p for p in pts if p["heldout"]])
    size = {}
    for sp in sorted({p["sparsity"] for p in pts if not p["heldout"]}):
        sel = [p for p in pts if p["sparsity"] == sp and p["N"] == max(cols) and not p["heldout"]]
        size[str(sp)] = {"plan_over_csr": round(_geomean([p["plan_bytes_over_csr"] for p in sel]), 3),
                         "plan_over_dense": round(_geomean([p["plan_bytes_over_dense"] for p in sel]), 3)}
    print(json.dumps({"metric": "time of the rule's plan / time of the best forced plan (geomean)",
                      "value": round(_geomean([p["rule_over_best"] for p in pts]), 3), "unit": "ratio", "n_gpus": 1,
                      "higher_is_better": False, "dtype": "f32", "data": "synthetic",
                      "config": {"workload": "tuning run on 30 sweep matrices (M, K >= 1024), 8 shapes between them and 8 held-out shapes x bCols " + "/".join(map(str, cols)),
                                 "wall_s": round(time.perf_counter() - t_start, 1)},
                      "summary": summary, "summary_heldout": summary_heldout,
                      "plan_size_by_sparsity_bcols128": size, "points": pts}))


def run_unhinted(args):
    """What the bCols hint is worth: every sweep matrix as ONE plan made without a hint (the
    inspector then assumes wide B), executed at 32, 64 and 128 columns, against the three
    hinted plans the other workloads create per matrix."""
    import torch
    import paper_2506_15174_amd as spmm
    from workloads import generators as gen
    torch.cuda.set_device(0)
    cols = (32, 64, 128)
    pts = []
    for entry in gen.sweep_entries():
        csr = gen.sweep_matrix(entry)
        a = (csr.M, csr.K, csr.row_ptr, csr.col_idx, csr.vals)
        plain = spmm.plan_create(*a)
        pi = plain.describe()
        for N in cols:
            B = torch.from_numpy(gen.activations_for(csr, N)).cuda()
            C = torch.empty((csr.M, N), dtype=torch.float32, device="cuda")
            hinted = spmm.plan_create(*a, n_hint=N)
            hi = hinted.describe()
            _time_plan(torch, hinted, B, C, N, reps=3)
            t_h = _time_plan(torch, hinted, B, C, N)
            t_p = _time_plan(torch, plain, B, C, N)
            hinted.destroy()
            pts.append({"M": csr.M, "K": csr.K, "sparsity": entry["sparsity"], "N": N, "hinted_us": round(t_h, 3),
                        "unhinted_us": round(t_p, 3), "hinted": [hi["ufi"], hi["ufk"], hi["group_nnz"], hi["k_slices"]],
                        "unhinted": [pi["ufi"], pi["ufk"], pi["group_nnz"], pi["k_slices"]],
                        "unhinted_over_hinted": round(t_p / t_h, 3)})
        plain.destroy()
    summary = {str(N): {"geomean_unhinted_over_hinted": round(_geomean([p["unhinted_over_hinted"] for p in pts if p["N"] == N]), 3),
                        "worst": max(p["unhinted_over_hinted"] for p in pts if p["N"] == N)} for N in cols}
    print(json.dumps({"metric": "time of the plan made without a bCols hint / time of the hinted plan (geomean)",
                      "value": round(_geomean([p["unhinted_over_hinted"] for p in pts]), 3), "unit": "ratio", "n_gpus": 1,
                      "higher_is_better": False, "dtype": "f32", "data": "synthetic",
                      "config": {"workload": "48 sweep matrices, one unhinted plan each, executed at bCols 32/64/128"},
                      "summary": summary, "points": pts}))


def kernel_report(torch, csr, plan, info, B, C, N, workload_key, samples=20, plan_kw=None):
    """Roofline block of one launch: algorithmic bytes over the launch's average duration
    (HIP events on the launch stream) against the HBM peak, the rate of wave-wide loads of
    B rows against the measured gather ceiling, the share of the fp32 vector peak."""
    nnz = int(csr.row_ptr[-1])
    avg_ms, med_ms = time_execute(torch, plan, B, C, N, samples=samples)
    bmin = bytes_min(csr.M, csr.K, nnz, N)
    achieved = bmin / (avg_ms * 1e-3) / 1e9
    kernel_tflops = 2.0 * nnz * N / (avg_ms * 1e-3) / 1e12
    traffic, prov = measured_traffic(workload_key, N)
    shape = kernel_shape(N, info["ufi"], csr.K, info["ufk"], info["k_slices"])
    roofline = {"bound": "hbm", "achieved": round(achieved, 2), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(achieved / HBM_PEAK_GBS, 5), "traffic": traffic, "traffic_source": prov,
                "kernel": "spmm_chunks_kernel<UFI=%d,%s> (bCols %d)" % (info["ufi"], shape, N),
                "cache_state": "hot",
                "avg_launch_us": round(avg_ms * 1e3, 3), "median_launch_us": round(med_ms * 1e3, 3),
                "launches_per_execute": 1 + (info["n_cross"] > 0) + (info["k_slices"] > 1), "algorithmic_bytes": bmin, "kernel_tflops": round(kernel_tflops, 3),
                "frac_of_fp32_valu_peak": round(kernel_tflops / FP32_VALU_PEAK_TFLOPS, 5),
                "traffic_gbs": round(traffic / (avg_ms * 1e-3) / 1e9, 2) if traffic else None,
                "counters_pct": measured_counters(workload_key, N)}
    # On-chip gather: each chunk of ufk enumerated columns costs ufk / S wave-wide loads of B
    # rows (S rows of B per load); the ceiling is the rate the gather microbenchmark
    # reaches on distinct rows of an L2-resident B.
    S = int(shape.split(",")[0][2:])
    tiles = 2 if (info["ufk"] == 8 and info["k_slices"] == 1 and tiles_of_64(N, csr.K)) else 1
    wave_loads = info["n_chunks"] * info["ufk"] // S * tiles
    roofline["gather"] = {"wave_loads_per_launch": wave_loads,
                          "g_wave_loads_per_s": round(wave_loads / (avg_ms * 1e-3) / 1e9, 2),
                          "measured_ceiling": GATHER_CEILING_GWLS,
                          "frac": round(wave_loads / (avg_ms * 1e-3) / 1e9 / GATHER_CEILING_GWLS, 4)}
    # The ceiling of the plan's own index stream: the same plan as a measuring plan, whose
    # launches request and await every B row as the product does and skip the multiply-adds.
    try:
        if plan_kw is False:
            raise RuntimeError("not measured: the plan forces a pipeline depth")
        import paper_2506_15174_amd as spmm
        kw = dict(plan_kw if plan_kw is not None else {"n_hint": N})
        probe = spmm.plan_create(csr.M, csr.K, csr.row_ptr, csr.col_idx, csr.vals, probe=True, **kw)
        scratch_c = torch.empty_like(C)
        p_avg, _ = time_execute(torch, probe, B, scratch_c, N, samples=samples)
        probe.destroy()
        roofline["gather"].update({"loads_only_us": round(p_avg * 1e3, 3),
                                   "loads_only_over_product": round(p_avg / avg_ms, 4)})
    except Exception as exc:   # a measuring plan is refused for 64-bit addressing and chunks wider than 16
        roofline["gather"]["loads_only_us"] = None
        roofline["gather"]["loads_only_note"] = repr(exc)
    return roofline


def cpu_baseline(csr, cols, gen, skip=False):
    """The oracle as it stands (row-parallel build of the same source), same products,
    host cores of this machine, on a bounded sample: whole passes until about 1.5 s of wall
    time have gone by (with 16 threads some 24 s of CPU work)."""
    from oracle import spmm_oracle
    nnz = int(csr.row_ptr[-1])
    host_B = {N: gen.activations_for(csr, N) for N in cols}
    cap_rows = csr.M
    sample = "full workload"
    if nnz * sum(cols) > 4e9:  # bound the CPU work to roughly 10-30 s
        cap_rows = max(4, int(csr.M * 4e9 / (nnz * sum(cols))) // 4 * 4)
        sample = "first %d of %d rows" % (cap_rows, csr.M)
    sub_ptr = csr.row_ptr[:cap_rows + 1]
    sub_nnz = int(sub_ptr[-1])
    passes, spent = 0, 0.0
    while not skip and (passes < 3 or spent < 1.5) and passes < 5000:
        t0 = time.perf_counter()
        for N in cols:
            spmm_oracle.spmm(sub_ptr, csr.col_idx[:sub_nnz], csr.vals[:sub_nnz], host_B[N],
                             K=csr.K, want_abs=False, parallel=True)
        spent += time.perf_counter() - t0
        passes += 1
    return {"value": round(2.0 * sub_nnz * sum(cols) * passes / spent / 1e9, 3) if passes else None, "unit": "GFLOP/s",
            "cores": spmm_oracle.threads(True), "kind": "oracle",
            "sample": "%s, %d passes in %.2f s, double accumulation, OpenMP over rows" % (sample, passes, spent)}


PLAN_KEYS = ("ufi", "ufk", "group_nnz", "group_panels", "n_groups", "n_blocks", "n_split", "n_enum", "n_chunks",
             "device_bytes", "sorted_rows", "n_cross", "scratch_bytes", "k_slices")


def run_headline(args):
    """The default workload: configuration 4 (48 magnitude-pruned matrices x bCols
    32/64/128, the sweep the metric and its comparison with hipSPARSE are stated on)
    together with configuration 3 (the 16384 x 16384 stress matrix at bCols 128, the
    largest single launch, on which the roofline figures are taken).  A step is one pass
    over all 145 products, every plan, B and C resident in HBM."""
    import numpy as np
    import torch
    import paper_2506_15174_amd as spmm
    from workloads import generators as gen

    assert torch.cuda.is_available(), "bench.py needs the MI355X"
    torch.cuda.set_device(0)
    t_start = time.perf_counter()
    cols = (32, 64, 128)
    resident = []
    points = _measure_points(torch, np, spmm, gen, gen.sweep_entries(), cols, gen.sweep_matrix, keep=resident,
                             with_baselines=not args.no_baselines)
    summary = _summarise(points, cols)
    sweep_flops = sum(2.0 * r["nnz"] * r["N"] for r in points)
    sweep_s = sum(r["us"] for r in points) * 1e-6

    # the stress product: roofline figures on the largest launch of the batch
    csr = gen.stress()
    nnz = int(csr.row_ptr[-1])
    Ns = 128
    t0 = time.perf_counter()
    plan = spmm.plan_create(csr.M, csr.K, csr.row_ptr, csr.col_idx, csr.vals, n_hint=Ns)
    plan_s = time.perf_counter() - t0
    info = plan.describe()
    B = torch.from_numpy(gen.activations_for(csr, Ns)).cuda()
    C = torch.empty((csr.M, Ns), dtype=torch.float32, device="cuda")
    resident.append((plan, B, C, Ns, nnz))
    hot = kernel_report(torch, csr, plan, info, B, C, Ns, "stress")
    roofline = dict(hot)
    cold = None if args.no_cold else time_execute_cold(torch, csr, plan, B, Ns)
    if cold is not None:
        # roofline claims are made on the cold figure: plan, B and C of every call come from HBM
        bmin = hot["algorithmic_bytes"]
        achieved = bmin / (cold["mean_us"] * 1e-6) / 1e9
        tflops = 2.0 * nnz * Ns / (cold["mean_us"] * 1e-6) / 1e12
        roofline.update({"achieved": round(achieved, 2), "frac": round(achieved / HBM_PEAK_GBS, 5),
                         "cache_state": "cold: %d copies of plan, B and C in turn, %d MiB together"
                                        % (cold["copies"], cold["working_set_bytes"] >> 20),
                         "avg_launch_us": cold["mean_us"], "median_launch_us": cold["us"],
                         "kernel_tflops": round(tflops, 3),
                         "frac_of_fp32_valu_peak": round(tflops / FP32_VALU_PEAK_TFLOPS, 5),
                         "hot": {k: hot[k] for k in ("achieved", "frac", "avg_launch_us", "median_launch_us",
                                                     "kernel_tflops")}})
        if roofline.get("traffic"):
            roofline["traffic_gbs"] = round(roofline["traffic"] / (cold["mean_us"] * 1e-6) / 1e9, 2)
        g = roofline["gather"]
        rate = g["wave_loads_per_launch"] / (cold["mean_us"] * 1e-6) / 1e9
        roofline["gather"] = dict(g, g_wave_loads_per_s=round(rate, 2), frac=round(rate / GATHER_CEILING_GWLS, 4))
    stress_base = {} if args.no_baselines else measure_baselines(torch, np, csr, (Ns,), {Ns: B}).get(str(Ns), {})

    # The timed steps: one pass over every product of the batch.  The products are independent
    # (each has its own plan, B and C), so they are issued round robin over args.streams HIP
    # streams of the default priority: a short product then starts while the previous one drains
    # (most of the batch takes 3 to 10 us per product, close to what a launch costs).  A product
    # always goes to the same stream, so the executes of one plan never overlap.  The per-product
    # figures above and the roofline block are single-stream launches of one product at a time.
    calls = [(p, b.data_ptr(), n, c.data_ptr()) for (p, b, c, n, _) in resident]

    def timed_steps(n_streams, steps, warmup):
        pool = [torch.cuda.Stream() for _ in range(n_streams)] if n_streams > 1 else [torch.cuda.current_stream()]
        handles = [q.cuda_stream or None for q in pool]
        torch.cuda.synchronize()

        def step():
            for i, (p, pb, n, pc) in enumerate(calls):
                p.execute_raw(pb, n, pc, handles[i % len(handles)])

        for _ in range(warmup):
            step()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            step()
        torch.cuda.synchronize()
        return 1e3 * (time.perf_counter() - t0) / steps

    single_ms = timed_steps(1, max(3, args.steps // 4), args.warmup) if args.streams > 1 else None
    ms_per_step = timed_steps(args.streams, args.steps, args.warmup)
    flops_step = sum(2.0 * z * n for (_, _, _, n, z) in resident)
    value = flops_step / (ms_per_step * 1e-3) / 1e9

    cpu = cpu_baseline(csr, (Ns,), gen, skip=args.no_cpu)
    out = {"metric": "fp32 CSR SpMM GFLOP/s (2*nnz*bCols)", "value": round(value, 2), "unit": "GFLOP/s",
           "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 5),
           "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
           "config": {"workload": "sweep: 48 magnitude-pruned matrices x bCols 32/64/128 (configs[4]) + stress "
                                  "16384x16384 @95% Zipf(1.5) rows, 5% empty, bCols 128 (configs[3]); one step = "
                                  "all 145 products, issued over " + str(args.streams) + " stream(s)",
                      "products_per_step": len(resident), "flops_per_step": flops_step,
                      "streams": args.streams,
                      "single_stream_ms_per_step": round(single_ms, 5) if single_ms else None,
                      "sweep_only": {"gflops_from_per_launch_medians": round(sweep_flops / sweep_s / 1e9, 2),
                                     "sum_of_launch_medians_ms": round(sweep_s * 1e3, 4)},
                      "stress": {"M": csr.M, "K": csr.K, "nnz": nnz, "bCols": Ns,
                                 "plan": {k: info[k] for k in PLAN_KEYS}, "plan_create_s": round(plan_s, 4),
                                 "row_stats": gen.row_stats(csr), "cold": cold,
                                 "hipsparse_best_us": stress_base.get("hipsparse_best_us"),
                                 "rocblas_sgemm_us": stress_base.get("rocblas_sgemm_us")},
                      "wall_s": round(time.perf_counter() - t_start, 1)},
           "roofline": roofline, "cpu_baseline": cpu, "summary": summary}
    if args.points_file:
        with open(args.points_file, "w") as f:
            json.dump(points, f)
    # the per-point figures went to stderr as they were measured; the line stays short
    print(json.dumps(out))


def run_single(args):
    import numpy as np
    import torch
    import paper_2506_15174_amd as spmm
    from workloads import generators as gen

    assert torch.cuda.is_available(), "bench.py needs the MI355X"
    torch.cuda.set_device(0)
    label, csr, cols = build_workload(args.workload, args)
    nnz = int(csr.row_ptr[-1])
    t0 = time.perf_counter()
    # one plan per column count: the schedule constants are chosen per bCols, as the
    # paper's tuner does (Section 3.5)
    plans = {N: spmm.plan_create(csr.M, csr.K, csr.row_ptr, csr.col_idx, csr.vals, n_hint=N, ufi=args.ufi,
                                 depth=args.depth, ufk=args.ufk, kslices=args.kslices) for N in cols}
    plan_s = (time.perf_counter() - t0) / len(cols)
    infos = {N: plans[N].describe() for N in cols}

    Bs = {N: torch.from_numpy(gen.activations_for(csr, N)).cuda() for N in cols}
    Cs = {N: torch.empty((csr.M, N), dtype=torch.float32, device="cuda") for N in cols}

    # spmm_execute through the binding's raw entry (device addresses marshalled once:
    # at these kernel lengths the tensor checks of Plan.execute would pace the launches)
    st = torch.cuda.current_stream().cuda_stream or None
    calls = {N: (plans[N], Bs[N].data_ptr(), N, Cs[N].data_ptr()) for N in cols}

    def step():
        for N in cols:
            plan, pb, n, pc = calls[N]
            plan.execute_raw(pb, n, pc, st)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = 1e3 * elapsed / args.steps
    flops_step = 2.0 * nnz * sum(cols)
    value = flops_step / (ms_per_step * 1e-3) / 1e9

    # dominant kernel: the widest column count; one launch per execute there (column tiles
    # of one width share a launch)
    Nd = max(cols)
    roofline = kernel_report(torch, csr, plans[Nd], infos[Nd], Bs[Nd], Cs[Nd], Nd, args.workload,
                             plan_kw=dict(n_hint=Nd, ufi=args.ufi, ufk=args.ufk, kslices=args.kslices) if args.depth == 0 else False)

    per_cols = {}
    for N in cols:
        a, m = time_execute(torch, plans[N], Bs[N], Cs[N], N, samples=20)
        per_cols[str(N)] = {"us": round(m * 1e3, 3), "gflops": round(2.0 * nnz * N / (m * 1e-3) / 1e9, 1),
                            "hbm_model_gbs": round(bytes_min(csr.M, csr.K, nnz, N) / (m * 1e-3) / 1e9, 1)}
    # cold timings after every hot one: creating their copies leaves the GPU idle for a while
    for N in () if args.no_cold else cols:
        cold = time_execute_cold(torch, csr, plans[N], Bs[N], N)
        if cold is not None:
            cold["hbm_model_gbs"] = round(bytes_min(csr.M, csr.K, nnz, N) / (cold["us"] * 1e-6) / 1e9, 1)
            cold["frac_of_hbm_peak"] = round(cold["hbm_model_gbs"] / HBM_PEAK_GBS, 5)
            per_cols[str(N)]["cold"] = cold

    baselines = {}
    if not args.no_baselines:
        baselines = measure_baselines(torch, np, csr, cols, Bs)

    if args.copy_calibration:
        src = torch.empty(64 << 20, dtype=torch.float32, device="cuda").normal_()
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()

    cpu = cpu_baseline(csr, cols, gen, skip=args.no_cpu)
    out = {"metric": "fp32 CSR SpMM GFLOP/s (2*nnz*bCols)", "value": round(value, 2), "unit": "GFLOP/s",
           "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 5),
           "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32",
           "data": "synthetic",
           "config": {"workload": label, "M": csr.M, "K": csr.K, "nnz": nnz, "bCols": list(cols),
                      "plans": {str(N): {k: infos[N][k] for k in PLAN_KEYS} for N in cols},
                      "plan_create_s": round(plan_s, 4), "row_stats": gen.row_stats(csr)},
           "roofline": roofline, "cpu_baseline": cpu, "per_bcols": per_cols, "baselines": baselines}
    print(json.dumps(out))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="headline",
                    help="headline (default: sweep + stress) | conv | stress | ffn | ffn-all | matrix | sweep | "
                         "narrow | sparsity | ablation | tune | unhinted")
    ap.add_argument("--shape", default="4096x4096", help="--workload matrix: rows x columns of A")
    ap.add_argument("--sparsity", type=float, default=0.5, help="--workload matrix: pruned share")
    ap.add_argument("--bcols", type=int, default=128, help="--workload matrix: columns of B")
    ap.add_argument("--seed", type=int, default=11, help="--workload matrix: generator seed")
    ap.add_argument("--ufi", type=int, default=0, help="single workloads: force the rows per panel (1, 2, 4, 8)")
    ap.add_argument("--kslices", type=int, default=0,
                    help="single workloads: cut the plan into so many column ranges (1 = never, 0 = the rule)")
    ap.add_argument("--ufk", type=int, default=0,
                    help="single workloads: force the enumerated columns per chunk (8, 16, 32, 64)")
    ap.add_argument("--depth", type=int, default=0,
                    help="single workloads: chunks of B rows in flight per wave (1, 2, 3, 4, 8; 0 = tuned)")
    ap.add_argument("--streams", type=int, default=2,
                    help="headline: HIP streams the independent products of a step are issued over (1 = one after the other)")
    ap.add_argument("--cols", default="", help="tune: comma-separated column counts instead of 32,64,128")
    ap.add_argument("--points-file", default="", help="headline: also write the per-point figures to this JSON file")
    ap.add_argument("--no-baselines", action="store_true")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle timing")
    ap.add_argument("--no-cold", action="store_true",
                    help="skip the cold-cache timing (copies of plan, B and C beyond the Infinity Cache, in turn)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run a plain 256 MiB device copy (reference for HBM byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        raise SystemExit("this build runs on one GPU only: the path would shard by rows of A (each GPU "
                         "plans and multiplies its own row range, B replicated), but no multi-GPU run "
                         "exists; use --gpus 1")
    if args.workload == "headline":
        return run_headline(args)
    if args.workload == "narrow":
        return run_sweep(args, cols=(4, 8, 16), narrow=True)
    if args.workload == "sparsity":
        return run_sweep(args, cols=(64, 4), square512=True)
    if args.workload == "ffn-all":
        return run_sweep(args, ffn=True)
    if args.workload in ("sweep", "ablation", "tune", "unhinted"):
        return {"sweep": run_sweep, "ablation": run_ablation, "tune": run_tune, "unhinted": run_unhinted}[args.workload](args)
    return run_single(args)


if __name__ == "__main__":
    main()
