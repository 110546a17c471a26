"""Parity of the HIP path with the CPU oracle, element by element, through the
C ABI (GPU machine only: run with -m gpu).

Bar (written out here): |C_gpu - C_ref| <= 1e-5 * S per element, where C_ref is
the oracle's double-precision value and S = sum |A_ik| |B_kj| over the same
terms; elements with S == 0 must be exactly zero.  With small-integer data every
summation order is exact in fp32, so those cases must match the oracle bit for
bit.
"""
import os

import numpy as np
import pytest

import paper_2506_15174_amd as spmm
from workloads import generators as gen

pytestmark = pytest.mark.gpu

TOL = 1e-5


@pytest.fixture(scope="module")
def torch_gpu():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    spmm.load()
    return torch


def gpu_product(torch, csr, B, guard_rows=0, stream=None, **plan_kw):
    """plan_create + execute through the C ABI; returns C as numpy (and the plan)."""
    plan = spmm.plan_create(csr.M, csr.K, csr.row_ptr, csr.col_idx, csr.vals, **plan_kw)
    dB = torch.from_numpy(np.ascontiguousarray(B)).cuda()
    N = B.shape[1]
    if guard_rows:
        full = torch.full((csr.M + 2 * guard_rows, N), float("nan"), dtype=torch.float32, device="cuda")
        dC = full[guard_rows:guard_rows + csr.M]
        plan.execute(dB, dC, stream=stream)
        torch.cuda.synchronize()
        host = full.cpu().numpy()
        assert np.isnan(host[:guard_rows]).all() and np.isnan(host[guard_rows + csr.M:]).all(), \
            "rows outside C were written"
        return host[guard_rows:guard_rows + csr.M].copy(), plan
    dC = torch.full((csr.M, N), float("nan"), dtype=torch.float32, device="cuda")
    plan.execute(dB, dC, stream=stream)
    torch.cuda.synchronize()
    return dC.cpu().numpy(), plan


from conftest import PARITY_WORST as WORST   # largest relative error seen, printed in the run's summary


def check(oracle, csr, B, C, parallel=False):
    """Whole product against the oracle.  parallel: the row-parallel build of the oracle's
    source (pinned bit-identical to the serial one by the CPU tests), for the large cases."""
    C_ref, S = oracle.spmm(csr.row_ptr, csr.col_idx, csr.vals, B, parallel=parallel)
    err, bad_zero = oracle.parity_error(C, C_ref, S)
    assert bad_zero == 0, "%d elements without terms are not exactly zero" % bad_zero
    assert err <= TOL, "max relative error %.3e" % err
    WORST["err"] = max(WORST["err"], err)
    return err


def heavy_tail(M, K, seed):
    rng = np.random.default_rng(seed)
    W = np.where(rng.random((M, K)) < 0.05, rng.standard_normal((M, K)), 0.0).astype(np.float32)
    W[3] = rng.standard_normal(K)
    W[M // 2] = rng.standard_normal(K)
    W[[0, 5, 6, 7, 8, M - 1]] = 0
    return gen.csr_from_dense(W)


# The configurations of the benchmark run as bench.py runs them: one plan per column
# count, created with that count as hint (hinted), and also with the hint left out.
@pytest.mark.parametrize("hinted", [True, False])
def test_tiny_config(torch_gpu, oracle, hinted):
    csr = gen.tiny()
    B = gen.activations_for(csr, 32)
    C, _ = gpu_product(torch_gpu, csr, B, guard_rows=8, n_hint=32 if hinted else 0)
    check(oracle, csr, B, C)


@pytest.mark.parametrize("hinted", [True, False])
@pytest.mark.parametrize("N", [32, 64, 128])
def test_conv_config(torch_gpu, oracle, N, hinted):
    csr = gen.conv_layer()
    B = gen.activations_for(csr, N)
    C, plan = gpu_product(torch_gpu, csr, B, guard_rows=4, n_hint=N if hinted else 0)
    check(oracle, csr, B, C)
    assert plan.describe()["n_split"] > 0  # 410 nonzeros per row: every panel is split
    assert plan.describe()["ufi"] < 4      # 512 rows: shorter panels give the chip enough workgroups


@pytest.mark.parametrize("N", [32, 64, 128])
@pytest.mark.parametrize("sparsity_index", [0, 1, 2, 3])
@pytest.mark.parametrize("shape_index", [0, 1])
def test_ffn_config(torch_gpu, oracle, shape_index, sparsity_index, N):
    # all eight feed-forward matrices (two shapes x four sparsities) at the three widths
    csr = gen.ffn(shape_index, sparsity_index)
    B = gen.activations_for(csr, N)
    for hint in (N, 0):
        C, _ = gpu_product(torch_gpu, csr, B, n_hint=hint)
        check(oracle, csr, B, C)


@pytest.mark.parametrize("N", [1, 2, 4, 8, 12, 16, 20, 31, 33, 63, 65, 96, 127, 130, 144, 200, 256, 257])
def test_any_column_count_with_ragged_rows_and_split_panels(torch_gpu, oracle, N):
    csr = heavy_tail(39, 1500, 40 + N)   # M % 8 != 0, dense rows, empty rows
    B = gen.dense_activations(csr.K, N, 50 + N)
    for ufi in (8, 4, 2, 1):
        C, plan = gpu_product(torch_gpu, csr, B, guard_rows=3, group_nnz=96, ufi=ufi)
        assert plan.describe()["n_split"] > 0 and plan.describe()["ufi"] == ufi
        check(oracle, csr, B, C)


@pytest.mark.parametrize("N", [4, 32, 64, 100, 128, 200])
@pytest.mark.parametrize("ufi", [1, 2, 4, 8])
def test_rows_sorted_by_length_write_c_in_the_callers_order(torch_gpu, oracle, N, ufi):
    # Zipf row lengths with empty rows, M % 8 != 0; the plan's rows are the matrix's
    # rows sorted by length, so every panel writes scattered rows of C
    csr = gen.zipf_rows(203, 1200, 0.85, 300 + ufi)
    B = gen.dense_activations(csr.K, N, 310 + N)
    C, plan = gpu_product(torch_gpu, csr, B, guard_rows=3, group_nnz=96, ufi=ufi, sort_rows=1)
    info = plan.describe()
    assert info["sorted_rows"] == 1 and info["ufi"] == ufi and info["n_split"] > 0
    check(oracle, csr, B, C)
    # the same product from the unsorted plan: same terms per element, maybe another order
    C2, plan2 = gpu_product(torch_gpu, csr, B, group_nnz=96, ufi=ufi, sort_rows=-1)
    assert plan2.describe()["sorted_rows"] == 0
    check(oracle, csr, B, C2)


def test_sorted_rows_with_small_integer_data_are_bit_exact(torch_gpu, oracle):
    rng = np.random.default_rng(77)
    M, K, N = 150, 640, 64
    dens = np.clip(0.6 / (1 + np.arange(M)) ** 0.7, 0.01, 1.0)[rng.permutation(M)]
    W = np.where(rng.random((M, K)) < dens[:, None], rng.integers(-8, 9, (M, K)), 0).astype(np.float32)
    csr = gen.csr_from_dense(W)
    B = rng.integers(-16, 17, (K, N)).astype(np.float32)
    C_ref, _ = oracle.spmm(csr.row_ptr, csr.col_idx, csr.vals, B)
    assert np.abs(C_ref).max() < 2 ** 24
    for ufi in (2, 4, 8):
        C, plan = gpu_product(torch_gpu, csr, B, group_nnz=64, ufi=ufi, sort_rows=1)
        assert plan.describe()["sorted_rows"] == 1
        assert np.array_equal(C.astype(np.float64), C_ref)


@pytest.mark.parametrize("group_nnz", [32, 64, 1000, 100000])
def test_group_budget_does_not_change_the_result_class(torch_gpu, oracle, group_nnz):
    csr = gen.lognormal_rows(300, 700, 0.8, 61)
    B = gen.dense_activations(csr.K, 128, 62)
    C, _ = gpu_product(torch_gpu, csr, B, group_nnz=group_nnz)
    check(oracle, csr, B, C)


@pytest.mark.parametrize("ufi", [0, 1, 2, 4, 8])
@pytest.mark.parametrize("N", [4, 8, 16, 32, 64, 128, 100])
def test_small_integer_data_is_bit_exact(torch_gpu, oracle, N, ufi):
    rng = np.random.default_rng(70 + N)
    M, K = 203, 900
    W = np.where(rng.random((M, K)) < 0.2, rng.integers(-8, 9, (M, K)), 0).astype(np.float32)
    W[17] = rng.integers(1, 9, K)          # a dense row: split panel, partial sums meet in LDS
    csr = gen.csr_from_dense(W)
    B = rng.integers(-16, 17, (K, N)).astype(np.float32)
    C, plan = gpu_product(torch_gpu, csr, B, group_nnz=128, ufi=ufi)
    assert plan.describe()["n_split"] > 0
    C_ref, _ = oracle.spmm(csr.row_ptr, csr.col_idx, csr.vals, B)
    assert np.abs(C_ref).max() < 2 ** 24
    assert np.array_equal(C.astype(np.float64), C_ref)


def test_identity_and_empty_matrices(torch_gpu, oracle):
    n = 130
    eye = gen.csr_from_dense(np.eye(n, dtype=np.float32))
    B = gen.dense_activations(n, 64, 80)
    C, _ = gpu_product(torch_gpu, eye, B)
    assert np.array_equal(C, B)
    empty = gen.csr_from_dense(np.zeros((11, n), dtype=np.float32))
    C0, _ = gpu_product(torch_gpu, empty, B)
    assert C0.shape == (11, 64) and not C0.any() and not np.signbit(C0).any()
    # no columns: every product is an empty sum; B holds no bytes and the kernels'
    # look-ahead loads go through a zero-length buffer range
    nocols = spmm.plan_create(5, 0, np.zeros(6, np.int32), np.zeros(0, np.int32), np.zeros(0, np.float32))
    for ncol in (8, 7):
        out0 = nocols.execute(torch_gpu.empty((0, ncol), dtype=torch_gpu.float32, device="cuda"),
                              torch_gpu.full((5, ncol), 3.0, dtype=torch_gpu.float32, device="cuda"))
        torch_gpu.cuda.synchronize()
        assert tuple(out0.shape) == (5, ncol) and not out0.cpu().numpy().any()
    # no rows at all: nothing to launch, nothing written
    none = spmm.plan_create(0, n, np.zeros(1, np.int32), np.zeros(0, np.int32), np.zeros(0, np.float32))
    dB = torch_gpu.from_numpy(B).cuda()
    out = none.execute(dB)
    assert tuple(out.shape) == (0, 64)


def test_column_order_inside_rows_does_not_matter(torch_gpu):
    rng = np.random.default_rng(81)
    csr = gen.uniform_positions(64, 300, 0.7, 82)
    col, val = csr.col_idx.copy(), csr.vals.copy()
    for i in range(csr.M):
        lo, hi = csr.row_ptr[i], csr.row_ptr[i + 1]
        perm = rng.permutation(hi - lo)
        col[lo:hi], val[lo:hi] = col[lo:hi][perm], val[lo:hi][perm]
    B = gen.dense_activations(csr.K, 128, 83)
    C0, _ = gpu_product(torch_gpu, csr, B)
    C1, _ = gpu_product(torch_gpu, gen.Csr(csr.M, csr.K, csr.row_ptr, col, val), B)
    assert np.array_equal(C0, C1)


def test_repeated_and_other_stream_executes_are_bit_identical(torch_gpu, oracle):
    csr = heavy_tail(64, 2000, 90)
    B = gen.dense_activations(csr.K, 128, 91)
    plan = spmm.plan_create(csr.M, csr.K, csr.row_ptr, csr.col_idx, csr.vals, group_nnz=64)
    assert plan.describe()["n_split"] > 0
    dB = torch_gpu.from_numpy(B).cuda()
    first = plan.execute(dB).cpu().numpy()
    check(oracle, csr, B, first)
    for _ in range(5):
        again = plan.execute(dB)
        torch_gpu.cuda.synchronize()
        assert np.array_equal(first, again.cpu().numpy())
    side = torch_gpu.cuda.Stream()
    side.wait_stream(torch_gpu.cuda.current_stream())
    with torch_gpu.cuda.stream(side):
        other = plan.execute(dB)
    side.synchronize()
    assert np.array_equal(first, other.cpu().numpy())


def test_wide_addressing_kernels(torch_gpu, oracle):
    csr = heavy_tail(50, 800, 95)
    for N in (32, 128, 77):
        B = gen.dense_activations(csr.K, N, 96 + N)
        C, _ = gpu_product(torch_gpu, csr, B, guard_rows=2, group_nnz=128, force_wide=True)
        check(oracle, csr, B, C)


# One case per compiled kernel instance <UFI, S, VW, D, WIDE>: the B rows of the software
# pipeline are loaded by hand-written asynchronous loads whose destination registers the
# compiler must leave alone until the matching wait; a toolchain that copies or spills one
# in between would hand stale data to the multiply-adds.  Small-integer data (any summation
# order exact) must match the oracle bit for bit, with groups of many more chunks than the
# deepest pipeline so that every stage of it runs in steady state.
INSTANCE_WIDTH = {2: 128, 4: 64, 8: 32}
INSTANCES = [(ufi, S, depth, wide)
             for ufi in (1, 2, 4, 8) for S in (2, 4, 8, 1) for wide in (False, True)
             for depth in ((0,) if wide else (0, 1, 2, 3, 4, 8))
             # the one-column-per-lane kernel (S == 1) is only reached through 64-bit addressing with N % 4 != 0
             if wide or S != 1]


@pytest.mark.parametrize("ufi,S,depth,wide", INSTANCES,
                         ids=["UFI%d-S%d-depth%d-%s" % (u, S, d, "wide" if w else "narrow") for u, S, d, w in INSTANCES])
def test_every_kernel_instance_is_bit_exact_on_integer_data(torch_gpu, oracle, ufi, S, depth, wide):
    rng = np.random.default_rng(1000 * ufi + 10 * S + depth)
    M, K = 67, 1800
    N = INSTANCE_WIDTH.get(S, 61)
    W = np.where(rng.random((M, K)) < 0.3, rng.integers(-8, 9, (M, K)), 0).astype(np.float32)
    W[5] = rng.integers(1, 9, K)          # a dense row: split panel
    W[[9, 10, 11, 12, 13, 14, 15, 16]] = 0   # a panel without entries
    csr = gen.csr_from_dense(W)
    B = rng.integers(-16, 17, (K, N)).astype(np.float32)
    C, plan = gpu_product(torch_gpu, csr, B, guard_rows=2, group_nnz=1024, ufi=ufi, depth=depth, force_wide=wide)
    info = plan.describe()
    assert info["ufi"] == ufi and info["n_split"] > 0
    assert info["n_chunks"] > 16 * info["n_groups"] > 0, "groups must be much longer than the pipeline"
    C_ref, _ = oracle.spmm(csr.row_ptr, csr.col_idx, csr.vals, B)
    assert np.abs(C_ref).max() < 2 ** 24
    assert np.array_equal(C.astype(np.float64), C_ref)


NARROW_INSTANCES = [(ufi, ufk, N) for ufi in (1, 2, 4, 8) for ufk, N in ((16, 32), (32, 16), (64, 8), (64, 4))]


@pytest.mark.parametrize("ufi,ufk,N", NARROW_INSTANCES,
                         ids=["UFI%d-UFK%d-S%d" % (u, k, 256 // n) for u, k, n in NARROW_INSTANCES])
def test_every_narrow_b_kernel_instance_is_bit_exact_on_integer_data(torch_gpu, oracle, ufi, ufk, N):
    """The instances for plans made for narrow B: chunks of 16 / 32 / 64 enumerated columns
    on waves cut into 8 / 16 / 32 or 64 slices (tiles of 32 / 16 / 8 / 4 columns).  Same
    demands as above: integer data, bit-exact, groups much longer than the pipeline."""
    rng = np.random.default_rng(7000 + 100 * ufi + ufk + N)
    M, K = 67, 4000
    W = np.where(rng.random((M, K)) < 0.3, rng.integers(-8, 9, (M, K)), 0).astype(np.float32)
    W[5] = rng.integers(1, 9, K)
    W[[9, 10, 11, 12, 13, 14, 15, 16]] = 0
    csr = gen.csr_from_dense(W)
    B = rng.integers(-16, 17, (K, N)).astype(np.float32)
    C, plan = gpu_product(torch_gpu, csr, B, guard_rows=2, group_nnz=1024, ufi=ufi, ufk=ufk)
    info = plan.describe()
    assert (info["ufi"], info["ufk"]) == (ufi, ufk) and info["n_split"] > 0
    assert info["n_chunks"] > 6 * info["n_groups"] > 0
    C_ref, _ = oracle.spmm(csr.row_ptr, csr.col_idx, csr.vals, B)
    assert np.abs(C_ref).max() < 2 ** 24
    assert np.array_equal(C.astype(np.float64), C_ref)


@pytest.mark.parametrize("N", [1, 2, 3, 4, 5, 8, 12, 16, 17, 31, 32, 33, 70, 130])
@pytest.mark.parametrize("hint", [4, 8, 16, 32])
def test_plans_made_for_narrow_b_compute_every_width(torch_gpu, oracle, hint, N):
    """A plan created with a narrow hint (chunks of 64 / 64 / 32 / 16 columns for hints of
    4 / 8 / 16 / 32 columns) stays valid for every N: wider B runs as several of the plan's
    narrow column tiles, the last one masked.  Ragged rows, dense rows (split panels, and
    with cross = 1 panels cut across workgroups), empty rows, M % 8 != 0."""
    csr = heavy_tail(39, 1500, 140 + hint)
    B = gen.dense_activations(csr.K, N, 150 + N)
    for ufi, cross in ((0, 0), (4, 1), (8, 0)):
        C, plan = gpu_product(torch_gpu, csr, B, guard_rows=3, group_nnz=96, ufi=ufi, n_hint=hint, cross=cross)
        assert plan.describe()["ufk"] == {4: 64, 8: 64, 16: 32, 32: 16}[hint]
        check(oracle, csr, B, C)


@pytest.mark.parametrize("depth", [1, 2, 3, 4, 8])
def test_pipeline_depth_setting_does_not_change_the_result(torch_gpu, oracle, depth):
    """The depth of the software pipeline (spmm_options_t.depth) only changes when a B
    row is requested, never what is added to what: results are bit-identical to the
    default depth's for every width."""
    csr = gen.lognormal_rows(300, 2000, 0.8, 161)
    for N in (32, 64, 128, 100):
        B = gen.dense_activations(csr.K, N, 162 + N)
        C0, _ = gpu_product(torch_gpu, csr, B, n_hint=N)
        C1, _ = gpu_product(torch_gpu, csr, B, n_hint=N, depth=depth)
        assert np.array_equal(C0, C1)
    check(oracle, csr, B, C1)


@pytest.mark.parametrize("N", [32, 64, 128, 100, 260, 700])
@pytest.mark.parametrize("ufi", [1, 2, 4, 8])
def test_panels_cut_across_workgroups(torch_gpu, oracle, ufi, N):
    """Dense rows far heavier than the group budget: their panels are cut across several
    workgroups whose sums meet in the plan's scratch memory, and a second launch adds them
    in workgroup order.  Small integers: bit-exact against the oracle; repeated executes are
    bit-identical (every launch overwrites what its second step reads, nothing is cleared
    in between); N = 700 needs more column tiles than one launch's scratch holds; the same
    matrix with cross < 0 (every panel inside one workgroup) gives the same C."""
    rng = np.random.default_rng(600 + ufi)
    M, K = 61, 2600
    W = np.where(rng.random((M, K)) < 0.04, rng.integers(-8, 9, (M, K)), 0).astype(np.float32)
    W[1] = rng.integers(1, 9, K)
    W[2, ::3] = rng.integers(1, 9, len(W[2, ::3]))
    W[40] = rng.integers(1, 9, K)
    W[[7, 8, 9]] = 0
    csr = gen.csr_from_dense(W)
    B = rng.integers(-16, 17, (K, N)).astype(np.float32)
    C_ref, _ = oracle.spmm(csr.row_ptr, csr.col_idx, csr.vals, B)
    assert np.abs(C_ref).max() < 2 ** 24
    C, plan = gpu_product(torch_gpu, csr, B, guard_rows=2, group_nnz=64, ufi=ufi, cross=1)
    info = plan.describe()
    assert info["n_cross"] >= 1 and info["scratch_bytes"] > 0
    assert np.array_equal(C.astype(np.float64), C_ref)
    dB = torch_gpu.from_numpy(B).cuda()
    for _ in range(3):
        again = plan.execute(dB)
        torch_gpu.cuda.synchronize()
        assert np.array_equal(C, again.cpu().numpy())
    C1, plan1 = gpu_product(torch_gpu, csr, B, group_nnz=64, ufi=ufi, cross=-1)
    assert plan1.describe()["n_cross"] == 0 and plan1.describe()["scratch_bytes"] == 0
    assert np.array_equal(C1.astype(np.float64), C_ref)


def test_panels_cut_across_workgroups_in_a_replayed_graph(torch_gpu, oracle):
    """Both launches of a plan with panels cut across workgroups are plain kernel nodes (no
    clearing call in between), so a captured execute replays correctly."""
    torch = torch_gpu
    csr = heavy_tail(64, 3000, 195)
    N = 128
    plan = spmm.plan_create(csr.M, csr.K, csr.row_ptr, csr.col_idx, csr.vals, group_nnz=64, ufi=4, cross=1)
    assert plan.describe()["n_cross"] > 0
    B = torch.from_numpy(gen.dense_activations(csr.K, N, 196)).cuda()
    C = torch.full((csr.M, N), float("nan"), dtype=torch.float32, device="cuda")
    eager = plan.execute(B).clone()
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        plan.execute(B, C)
    torch.cuda.current_stream().wait_stream(side)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        plan.execute(B, C)
    for replay in range(4):
        C.fill_(float("nan"))
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(C, eager), "replay %d differs from the eager result" % replay
        plan.execute(B)
        torch.cuda.synchronize()
    check(oracle, csr, B.cpu().numpy(), C.cpu().numpy())


@pytest.mark.parametrize("N", [1, 5, 32, 64, 100, 128, 129, 200, 257])
@pytest.mark.parametrize("ns,ufi,sort_rows,cross", [(2, 0, 0, 0), (4, 8, 1, 1), (8, 4, 1, -1), (4, 2, -1, 0), (8, 1, 0, 1),
                                                    (2, 8, -1, 1)])
def test_plans_cut_along_k(torch_gpu, oracle, ns, ufi, sort_rows, cross, N):
    """A plan cut into column ranges: every workgroup multiplies one range, the ranges' sums
    meet in the plan's scratch memory and a last launch adds them in range order, 128 columns
    of B at a time (N = 200 and 257 take two and three rounds).  Small integers: bit-exact
    against the oracle whatever the order of the additions; repeated executes are
    bit-identical; rows outside C stay untouched; M is not a multiple of the panel height."""
    rng = np.random.default_rng(700 + ns + ufi)
    M, K = 61, 2600
    W = np.where(rng.random((M, K)) < 0.04, rng.integers(-8, 9, (M, K)), 0).astype(np.float32)
    W[1] = rng.integers(1, 9, K)
    W[2, ::3] = rng.integers(1, 9, len(W[2, ::3]))
    W[40] = rng.integers(1, 9, K)
    W[[7, 8, 9]] = 0
    csr = gen.csr_from_dense(W)
    B = rng.integers(-16, 17, (K, N)).astype(np.float32)
    C_ref, _ = oracle.spmm(csr.row_ptr, csr.col_idx, csr.vals, B)
    assert np.abs(C_ref).max() < 2 ** 24
    C, plan = gpu_product(torch_gpu, csr, B, guard_rows=2, group_nnz=64, ufi=ufi, sort_rows=sort_rows, cross=cross,
                          kslices=ns)
    info = plan.describe()
    assert info["k_slices"] == ns and info["slice_rows"] == 64 and info["scratch_bytes"] >= ns * 64 * 128 * 4
    # heavy panels of a range are cut across workgroups as in any plan (a single row's share
    # of a range, 325 entries, stays below the bound of eight budgets)
    assert (info["n_cross"] > 0) == (cross > 0 and ufi == 8)
    assert np.array_equal(C.astype(np.float64), C_ref)
    dB = torch_gpu.from_numpy(B).cuda()
    for _ in range(2):
        again = plan.execute(dB)
        torch_gpu.cuda.synchronize()
        assert np.array_equal(C, again.cpu().numpy())
    # the entry point without allocations has no room for the ranges' sums
    with pytest.raises(spmm.SpmmError) as e:
        plan.execute_static_raw(dB.data_ptr(), N, again.data_ptr())
    assert e.value.status == spmm.SPMM_ERR_UNSUPPORTED


@pytest.mark.parametrize("N", [128, 64, 40])
def test_plans_cut_along_k_with_real_data_and_unsorted_columns(torch_gpu, oracle, N):
    """Column ranges of a matrix whose rows are stored with their columns in random order and
    with duplicates (the inspector orders every row before it cuts it), lognormal row
    lengths, real values: within the tolerance of the oracle."""
    csr = gen.lognormal_rows(700, 5000, 0.9, 31)
    rng = np.random.default_rng(32)
    rows = np.repeat(np.arange(csr.M), np.diff(csr.row_ptr))
    extra_rows = rng.integers(0, csr.M, 500)
    rows_all = np.concatenate([rows, extra_rows])
    cols_all = np.concatenate([csr.col_idx, rng.integers(0, csr.K, 500).astype(np.int32)])
    vals_all = np.concatenate([csr.vals, rng.standard_normal(500).astype(np.float32)])
    o = np.lexsort((rng.random(len(rows_all)), rows_all))       # rows together, columns shuffled
    row_ptr = np.concatenate(([0], np.cumsum(np.bincount(rows_all, minlength=csr.M)))).astype(np.int32)
    shuffled = gen.Csr(csr.M, csr.K, row_ptr, cols_all[o].astype(np.int32), vals_all[o].astype(np.float32))
    B = gen.dense_activations(csr.K, N, 33)
    for ns in (2, 8):
        C, plan = gpu_product(torch_gpu, shuffled, B, guard_rows=1, kslices=ns, n_hint=N)
        assert plan.describe()["k_slices"] == ns
        check(oracle, shuffled, B, C)


@pytest.mark.parametrize("N", [64, 37, 130])
def test_plans_cut_along_k_on_the_64_bit_addressing_kernels(torch_gpu, oracle, N):
    """force_wide: the kernels that address B with 64 bits (N = 37 and 130: one column per
    lane, tiles of 64 columns, so the column ranges' sums are added 64 columns at a time)."""
    csr = heavy_tail(70, 1200, 301)
    B = gen.dense_activations(csr.K, N, 302)
    for ufi in (1, 4):
        C, plan = gpu_product(torch_gpu, csr, B, guard_rows=1, force_wide=True, kslices=4, ufi=ufi, group_nnz=96)
        assert plan.describe()["k_slices"] == 4
        check(oracle, csr, B, C)


def test_plan_cut_along_k_in_a_replayed_graph(torch_gpu, oracle):
    """The three launches of a plan cut along K whose heavy panels are also cut across
    workgroups (product, sums of the cut panels, sums of the ranges) replay from a graph."""
    torch = torch_gpu
    csr = heavy_tail(64, 3000, 197)
    N = 128
    plan = spmm.plan_create(csr.M, csr.K, csr.row_ptr, csr.col_idx, csr.vals, group_nnz=64, ufi=4, cross=1, kslices=4)
    assert plan.describe()["n_cross"] > 0 and plan.describe()["k_slices"] == 4
    B = torch.from_numpy(gen.dense_activations(csr.K, N, 198)).cuda()
    C = torch.full((csr.M, N), float("nan"), dtype=torch.float32, device="cuda")
    eager = plan.execute(B).clone()
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        plan.execute(B, C)
    torch.cuda.current_stream().wait_stream(side)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        plan.execute(B, C)
    for replay in range(4):
        C.fill_(float("nan"))
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(C, eager), "replay %d differs from the eager result" % replay
        plan.execute(B)
        torch.cuda.synchronize()
    check(oracle, csr, B.cpu().numpy(), C.cpu().numpy())


def test_measuring_plans_load_everything_and_multiply_nothing(torch_gpu):
    """probe = 1: the launches request every row of B as the product does and skip the
    multiply-adds, so C is all zeros (never NaN: every element is still written); the
    setting is refused together with forced 64-bit addressing, a depth or chunks wider than 16."""
    csr = heavy_tail(70, 1800, 171)
    for N, kw in ((128, dict(ufi=8)), (64, dict(ufi=4, cross=1, group_nnz=64)), (32, dict(n_hint=32, ufi=2)), (100, dict())):
        B = gen.dense_activations(csr.K, N, 172)
        C, plan = gpu_product(torch_gpu, csr, B, guard_rows=2, probe=True, **kw)
        assert not C.any() and not np.isnan(C).any()
    for bad in (dict(force_wide=True), dict(depth=2), dict(ufk=32)):
        with pytest.raises(spmm.SpmmError) as err:
            spmm.plan_create(csr.M, csr.K, csr.row_ptr, csr.col_idx, csr.vals, probe=True, **bad)
        assert err.value.status == spmm.SPMM_ERR_INVALID_ARG


def test_plain_c_client_runs_on_the_device(tmp_path):
    """create -> execute -> destroy from plain C99 (no Python, no torch between the caller
    and the library): the client uploads B, runs the product and compares known elements."""
    import shutil
    import subprocess
    here = os.path.dirname(os.path.abspath(__file__))
    root = os.path.dirname(here)
    lib_dir = os.path.dirname(spmm.LIB_PATH)
    rocm_lib = os.path.join(os.environ.get("ROCM_PATH", "/opt/rocm"), "lib")
    assert shutil.which("gcc"), "needs gcc"
    exe = str(tmp_path / "device_client")
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-Werror", "-pedantic", "-I", os.path.join(root, "include"),
                    os.path.join(here, "c_abi_device_client.c"), "-L", lib_dir, "-lspmm_cdna4", "-L", rocm_lib,
                    "-lamdhip64", "-Wl,-rpath," + lib_dir, "-Wl,-rpath," + rocm_lib, "-o", exe], check=True)
    res = subprocess.run([exe], capture_output=True, text=True, timeout=120)
    assert res.returncode == 0, res.stdout + res.stderr
    assert "device client ok" in res.stdout


@pytest.mark.parametrize("N", [64, 66, 3, 127])
def test_pointers_with_only_four_byte_alignment(torch_gpu, oracle, N):
    """B and C that start 4 bytes past a 16-byte boundary, with rows that are (N = 64)
    or are not a multiple of 16 bytes long: the 16-byte loads and stores of the
    four-columns-per-lane kernels run at 4-byte alignment, the last lane of a tile
    with N % 4 columns stores only those, and nothing outside C is written."""
    csr = heavy_tail(45, 600, 97)
    B = gen.dense_activations(csr.K, N, 98 + N)
    plan = spmm.plan_create(csr.M, csr.K, csr.row_ptr, csr.col_idx, csr.vals, group_nnz=64)
    flatB = torch_gpu.zeros(csr.K * N + 1, dtype=torch_gpu.float32, device="cuda")
    flatC = torch_gpu.full((csr.M * N + 9,), float("nan"), dtype=torch_gpu.float32, device="cuda")
    flatB[1:] = torch_gpu.from_numpy(B).cuda().reshape(-1)
    plan.execute_raw(flatB.data_ptr() + 4, N, flatC.data_ptr() + 4, None)
    torch_gpu.cuda.synchronize()
    host = flatC.cpu().numpy()
    assert np.isnan(host[0]) and np.isnan(host[csr.M * N + 1:]).all(), "words outside C were written"
    check(oracle, csr, B, host[1:csr.M * N + 1].reshape(csr.M, N))


def test_b_ending_at_the_end_of_its_allocation_is_not_overrun(torch_gpu, oracle):
    """N = 5: the last active lane of the tile asks for columns 4 .. 7 of every row of B;
    for the last row that is past the end of B, which the buffer descriptor's range
    check answers with zeros.  B is the tail of an allocation, C is guarded."""
    csr = heavy_tail(40, 512, 131)
    N = 5
    B = gen.dense_activations(csr.K, N, 132)
    pool = torch_gpu.zeros(1 << 20, dtype=torch_gpu.float32, device="cuda")
    dB = pool[pool.numel() - csr.K * N:]
    dB.copy_(torch_gpu.from_numpy(B).cuda().reshape(-1))
    plan = spmm.plan_create(csr.M, csr.K, csr.row_ptr, csr.col_idx, csr.vals, ufi=4)
    flatC = torch_gpu.full((csr.M * N + 8,), float("nan"), dtype=torch_gpu.float32, device="cuda")
    plan.execute_raw(dB.data_ptr(), N, flatC.data_ptr(), None)
    torch_gpu.cuda.synchronize()
    host = flatC.cpu().numpy()
    assert np.isnan(host[csr.M * N:]).all()
    check(oracle, csr, B, host[:csr.M * N].reshape(csr.M, N))


def test_execute_rejects_bad_arguments(torch_gpu):
    csr = gen.tiny()
    plan = spmm.plan_create(csr.M, csr.K, csr.row_ptr, csr.col_idx, csr.vals)
    dB = torch_gpu.zeros((csr.K, 32), dtype=torch_gpu.float32, device="cuda")
    dC = torch_gpu.zeros((csr.M, 32), dtype=torch_gpu.float32, device="cuda")
    lib = spmm.load()
    assert lib.spmm_execute(plan.handle, dB.data_ptr(), 0, dC.data_ptr(), None) == spmm.SPMM_ERR_INVALID_ARG
    assert lib.spmm_execute(plan.handle, None, 32, dC.data_ptr(), None) == spmm.SPMM_ERR_INVALID_ARG
    assert lib.spmm_execute(plan.handle, dB.data_ptr(), 32, None, None) == spmm.SPMM_ERR_INVALID_ARG
    assert lib.spmm_execute(plan.handle, dB.data_ptr() + 2, 32, dC.data_ptr(), None) == spmm.SPMM_ERR_INVALID_ARG
    info = plan.describe()
    assert info["device_bytes"] > 0 and info["stream_words"] * 4 <= info["device_bytes"]
    # a plan on the device keeps its row groups but not the host mirror of its arrays
    assert len(plan.get_groups()) == info["n_groups"]
    with pytest.raises(spmm.SpmmError) as err:
        plan.get_array(spmm.ARRAY_STREAM)
    assert err.value.status == spmm.SPMM_ERR_INVALID_ARG


def test_stress_config_whole_product_at_full_size(torch_gpu, oracle):
    """Full 16384 x 16384 Zipf matrix at N = 128 in the launch configuration the
    benchmark times; every element against the oracle."""
    csr = gen.stress()
    B = gen.activations_for(csr, 128)
    C, plan = gpu_product(torch_gpu, csr, B, n_hint=128)
    # Zipf rows: the inspector sorts them by length and takes eight-row panels; 128 columns of
    # B (8 MiB) exceed one L2: the plan is cut into four column ranges, whose panels (at most
    # 8 x 4096 entries) all stay inside one workgroup
    info = plan.describe()
    assert (info["sorted_rows"], info["ufi"], info["k_slices"], info["n_cross"]) == (1, 8, 4, 0)
    assert info["scratch_bytes"] == 4 * 16384 * 128 * 4
    check(oracle, csr, B, C, parallel=True)
    lens = np.diff(csr.row_ptr)
    # every empty row of the full matrix is exactly zero
    assert not C[lens == 0].any()
    # the same matrix left whole (two tiles of 64 columns in one launch, the panels of the dense
    # rows cut across workgroups)
    C1, plan1 = gpu_product(torch_gpu, csr, B, n_hint=128, kslices=1)
    assert plan1.describe()["k_slices"] == 1 and plan1.describe()["n_cross"] > 50
    check(oracle, csr, B, C1, parallel=True)


@pytest.mark.parametrize("N,want_ufi", [(128, 8), (64, 8), (32, 8)])
def test_largest_sweep_entry_whole_product_at_full_size(torch_gpu, oracle, N, want_ufi):
    """The largest matrix of the sweep (8192 x 8192, half of the entries kept) in the
    launch configuration the benchmark times (eight-row panels at every width, chunks of 16
    columns for 32 columns of B); every element against the oracle, with guard rows around C."""
    entry = [e for e in gen.sweep_entries() if e["M"] == 8192 and e["sparsity"] == 0.5][0]
    csr = gen.sweep_matrix(entry)
    B = gen.activations_for(csr, N)
    C, plan = gpu_product(torch_gpu, csr, B, guard_rows=8, n_hint=N)
    assert plan.describe()["ufi"] == want_ufi
    check(oracle, csr, B, C, parallel=True)


@pytest.mark.parametrize("N", [128, 96])
def test_wide_b_beyond_one_l2_runs_as_tiles_of_64_columns(torch_gpu, oracle, N):
    """4096 x 12288 with rows of 3686 entries: 128 columns of B (6 MiB) exceed one L2, 64
    fit, so the product runs as 64-column tiles (with the 24 KiB of idle LDS that caps
    the workgroups per CU) over eight-row panels; every element against the oracle."""
    csr = gen.magnitude_pruned(4096, 12288, 0.7, 91)
    B = gen.activations_for(csr, N)
    C, plan = gpu_product(torch_gpu, csr, B, n_hint=N, kslices=1)
    assert plan.describe()["ufi"] == 8 and plan.describe()["sorted_rows"] == 0
    check(oracle, csr, B, C, parallel=True)
    # by default the plan is cut into four ranges of 3072 columns (1.5 MiB of B each) instead
    C, plan = gpu_product(torch_gpu, csr, B, n_hint=N)
    assert (plan.describe()["ufi"], plan.describe()["k_slices"], plan.describe()["slice_cols"]) == (8, 4, 3072)
    check(oracle, csr, B, C, parallel=True)


def test_sorted_zipf_matrix_with_eight_row_panels_at_full_size(torch_gpu, oracle):
    """16384 x 4096 with Zipf row lengths: rows sorted by length, eight-row panels
    (the longest row, 4096, is within twice a compute unit's share); every element
    against the oracle."""
    csr = gen.zipf_rows(16384, 4096, 0.9, 13)
    B = gen.activations_for(csr, 128)
    C, plan = gpu_product(torch_gpu, csr, B, n_hint=128)
    assert (plan.describe()["sorted_rows"], plan.describe()["ufi"]) == (1, 8)
    check(oracle, csr, B, C, parallel=True)
    lens = np.diff(csr.row_ptr)
    assert not C[lens == 0].any()


@pytest.mark.parametrize("seed", range(48))
def test_random_shapes_settings_and_widths(torch_gpu, oracle, seed):
    """Random shape, row-length law (uniform, a few dense rows, very short rows, duplicates
    and unsorted columns), panel height, budget, row order and width, with B and C at a
    random 4-byte offset inside guarded buffers."""
    rng = np.random.default_rng(4000 + seed)
    M, K = int(rng.integers(1, 300)), int(rng.integers(1, 1500))
    mode = seed % 4
    if mode == 0:
        lens = rng.integers(0, K + 1, M)
    elif mode == 1:
        lens = np.where(rng.random(M) < 0.1, K, rng.integers(0, 6, M))
    elif mode == 2:
        lens = rng.integers(0, 4, M)
    else:
        lens = np.where(rng.random(M) < 0.2, 0, rng.integers(0, 2 * K, M))       # duplicates
    row_ptr = np.concatenate(([0], np.cumsum(lens))).astype(np.int32)
    nnz = int(row_ptr[-1])
    col_idx = rng.integers(0, K, nnz).astype(np.int32)
    vals = rng.standard_normal(nnz).astype(np.float32)
    csr = gen.Csr(M, K, row_ptr, col_idx, vals)
    N = int(rng.choice([1, 3, 4, 7, 17, 32, 33, 64, 70, 100, 128, 129, 190, 260]))
    B = rng.standard_normal((K, N)).astype(np.float32)
    plan = spmm.plan_create(M, K, row_ptr, col_idx, vals, ufi=int(rng.choice([0, 1, 2, 4, 8])),
                            group_nnz=int(rng.choice([0, 16, 100, 1000])), sort_rows=int(rng.choice([-1, 0, 1])),
                            n_hint=int(rng.choice([0, 32, 64, 128])))
    check_random_plan(torch_gpu, oracle, rng, csr, plan, B, N)


@pytest.mark.parametrize("seed", range(32))
def test_random_shapes_settings_and_widths_with_cut_plans(torch_gpu, oracle, seed):
    """The same with plans cut along K into 2, 4 or 8 column ranges, with and without panels
    cut across workgroups, for hints of more than 32 columns or none."""
    rng = np.random.default_rng(4400 + seed)
    M, K = int(rng.integers(1, 300)), int(rng.integers(8, 1500))
    mode = seed % 4
    if mode == 0:
        lens = rng.integers(0, K + 1, M)
    elif mode == 1:
        lens = np.where(rng.random(M) < 0.1, K, rng.integers(0, 6, M))
    elif mode == 2:
        lens = rng.integers(0, 4, M)
    else:
        lens = np.where(rng.random(M) < 0.2, 0, rng.integers(0, 2 * K, M))       # duplicates
    row_ptr = np.concatenate(([0], np.cumsum(lens))).astype(np.int32)
    nnz = int(row_ptr[-1])
    csr = gen.Csr(M, K, row_ptr, rng.integers(0, K, nnz).astype(np.int32), rng.standard_normal(nnz).astype(np.float32))
    N = int(rng.choice([1, 3, 4, 7, 17, 32, 33, 64, 70, 100, 128, 129, 190, 260]))
    B = rng.standard_normal((K, N)).astype(np.float32)
    ns = int(rng.choice([2, 4, 8]))
    plan = spmm.plan_create(M, K, csr.row_ptr, csr.col_idx, csr.vals, ufi=int(rng.choice([0, 1, 2, 4, 8])),
                            group_nnz=int(rng.choice([0, 16, 100, 1000])), sort_rows=int(rng.choice([-1, 0, 1])),
                            n_hint=int(rng.choice([0, 64, 128])), cross=int(rng.choice([-1, 0, 1])), kslices=ns)
    assert plan.describe()["k_slices"] == ns
    check_random_plan(torch_gpu, oracle, rng, csr, plan, B, N)


def check_random_plan(torch_gpu, oracle, rng, csr, plan, B, N):
    M, K = csr.M, csr.K
    shift = int(rng.integers(0, 4))
    flatB = torch_gpu.zeros(K * N + 8, dtype=torch_gpu.float32, device="cuda")
    flatB[shift:shift + K * N] = torch_gpu.from_numpy(B).cuda().reshape(-1)
    flatC = torch_gpu.full((M * N + 16,), float("nan"), dtype=torch_gpu.float32, device="cuda")
    plan.execute_raw(flatB.data_ptr() + 4 * shift, N, flatC.data_ptr() + 4 * (4 + shift), None)
    torch_gpu.cuda.synchronize()
    host = flatC.cpu().numpy()
    lo = 4 + shift
    assert np.isnan(host[:lo]).all() and np.isnan(host[lo + M * N:]).all(), "words outside C were written"
    check(oracle, csr, B, host[lo:lo + M * N].reshape(M, N))


@pytest.mark.parametrize("index", range(48))
def test_every_sweep_matrix_at_the_three_widths(torch_gpu, oracle, index):
    """Configuration 4 as the benchmark runs it (one hinted plan per width): every
    element of every product against the oracle."""
    entry = gen.sweep_entries()[index]
    csr = gen.sweep_matrix(entry)
    for N in (32, 64, 128):
        B = gen.activations_for(csr, N)
        C, _ = gpu_product(torch_gpu, csr, B, n_hint=N)
        check(oracle, csr, B, C, parallel=csr.M > 1024)


def test_execute_can_be_captured_in_a_graph_and_replayed(torch_gpu, oracle):
    """spmm_execute allocates nothing, clears nothing and never synchronises, so it can
    sit in a captured graph: every replay (with eager work in between) reproduces the
    eager result bit for bit, also for split panels and for a second set of B values."""
    torch = torch_gpu
    csr = heavy_tail(64, 2000, 95)
    N = 128
    plan = spmm.plan_create(csr.M, csr.K, csr.row_ptr, csr.col_idx, csr.vals, group_nnz=64)
    assert plan.describe()["n_split"] > 0
    B = torch.from_numpy(gen.dense_activations(csr.K, N, 96)).cuda()
    C = torch.full((csr.M, N), float("nan"), dtype=torch.float32, device="cuda")
    eager = plan.execute(B).clone()
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        plan.execute(B, C)            # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        plan.execute(B, C)
    for replay in range(4):
        C.fill_(float("nan"))
        if replay == 2:               # new inputs in the captured buffers
            B.copy_(torch.from_numpy(gen.dense_activations(csr.K, N, 97)).cuda())
            eager = plan.execute(B).clone()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(C, eager), "replay %d differs from the eager result" % replay
        plan.execute(B)               # eager work between replays
        torch.cuda.synchronize()
    check(oracle, csr, B.cpu().numpy(), C.cpu().numpy())


def test_b_beyond_four_gib_is_addressed_with_64_bits(torch_gpu, oracle):
    """K * N * 4 just above 2^32: the executor must take the 64-bit addressing kernels by
    itself.  A has 16 rows whose columns include the last row of B and rows on both sides of
    the 4 GiB boundary; the oracle works on the rows of B that A touches."""
    torch = torch_gpu
    N = 128
    K = (1 << 23) + 4096                      # K * 512 bytes = 4 GiB + 2 MiB
    M = 16
    rng = np.random.default_rng(2024)
    rows = []
    for i in range(M):
        c = set(rng.integers(0, K, size=60).tolist())
        c.update((K - 1 - i, (1 << 23) - 1 - i, (1 << 23) + i))
        rows.append(np.array(sorted(c), dtype=np.int32))
    row_ptr = np.concatenate(([0], np.cumsum([len(r) for r in rows]))).astype(np.int32)
    col_idx = np.concatenate(rows)
    vals = rng.standard_normal(len(col_idx)).astype(np.float32)
    dB = torch.empty((K, N), dtype=torch.float32, device="cuda")
    dB.normal_()
    plan = spmm.plan_create(M, K, row_ptr, col_idx, vals)
    dC = plan.execute(dB)
    torch.cuda.synchronize()
    uniq, inverse = np.unique(col_idx, return_inverse=True)
    B_small = dB[torch.from_numpy(uniq.astype(np.int64)).cuda()].cpu().numpy()
    small = gen.Csr(M, len(uniq), row_ptr, inverse.astype(np.int32), vals)
    check(oracle, small, B_small, dC.cpu().numpy())
    del dB


def test_many_short_rows_share_waves(torch_gpu, oracle):
    """200 000 rows of 0-8 entries: the inspector packs 16 single-row panels per wave
    (one group closes by the panel cap, not by the budget); whole product against the oracle."""
    rng = np.random.default_rng(77)
    M, K, N = 200_000, 512, 32
    lens = rng.integers(0, 9, size=M)
    row_ptr = np.concatenate(([0], np.cumsum(lens))).astype(np.int32)
    col_idx = np.concatenate([np.sort(rng.choice(K, size=n, replace=False)) for n in lens]).astype(np.int32)
    vals = rng.standard_normal(int(row_ptr[-1])).astype(np.float32)
    csr = gen.Csr(M, K, row_ptr, col_idx, vals)
    B = gen.dense_activations(K, N, 78)
    C, plan = gpu_product(torch_gpu, csr, B, guard_rows=2, n_hint=N)
    info = plan.describe()
    assert info["ufi"] == 1 and info["group_panels"] == 16 and info["n_groups"] < M // 8
    check(oracle, csr, B, C)
