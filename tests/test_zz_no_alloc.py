"""The allocation-free entry point spmm_execute_static against spmm_execute, through the
C ABI (GPU machine only).

Plans whose heavy panels are cut across workgroups park partial sums in scratch memory:
spmm_execute uses memory the plan allocated, spmm_execute_static a device array that is
part of the library's code object.  Same kernels, same order of additions: the results
must be equal bit for bit.  Two calls in a row share the array, the second on a smaller
input; a plan whose single column tile does not fit the array is refused.
"""
import numpy as np
import pytest

import paper_2506_15174_amd as spmm
from workloads import generators as gen

pytestmark = pytest.mark.gpu


def _dense_rows_matrix(M, K, dense_rows, seed):
    rng = np.random.default_rng(seed)
    W = np.where(rng.random((M, K)) < 0.03, rng.standard_normal((M, K)), 0.0).astype(np.float32)
    for r in dense_rows:
        W[r] = rng.standard_normal(K)
    return gen.csr_from_dense(W)


def _both(torch, plan, B):
    """C from spmm_execute and from spmm_execute_static, each into NaN-filled memory."""
    info = plan.describe()
    N = B.shape[1]
    dB = torch.from_numpy(B).cuda()
    C0 = torch.full((info["M"], N), float("nan"), dtype=torch.float32, device="cuda")
    C1 = torch.full((info["M"], N), float("nan"), dtype=torch.float32, device="cuda")
    plan.execute_raw(dB.data_ptr(), N, C0.data_ptr(), None)
    torch.cuda.synchronize()
    plan.execute_static_raw(dB.data_ptr(), N, C1.data_ptr(), None)
    torch.cuda.synchronize()
    return C0.cpu().numpy(), C1.cpu().numpy()


def test_static_scratch_entry_point_matches_execute_on_two_calls_in_a_row(oracle):
    import torch
    assert torch.cuda.is_available(), "this test needs the MI355X"
    spmm.load()
    big = _dense_rows_matrix(150, 6000, (3, 4, 77, 140), 1)
    small = _dense_rows_matrix(40, 2100, (9,), 2)
    plans = {}
    for name, csr, ufi in (("big", big, 8), ("small", small, 4)):
        plans[name] = spmm.plan_create(csr.M, csr.K, csr.row_ptr, csr.col_idx, csr.vals, group_nnz=64, ufi=ufi, cross=1)
        info = plans[name].describe()
        assert info["n_cross"] >= 1 and info["scratch_bytes"] > 0
    # first call: the larger input, 200 columns (two column tiles in one launch); second call
    # right after it: a smaller input with fewer slots, which finds the first call's sums
    # still in the array
    for name, csr, N in (("big", big, 200), ("small", small, 96), ("big", big, 32)):
        B = gen.dense_activations(csr.K, N, 7 + N)
        C0, C1 = _both(torch, plans[name], B)
        assert np.isfinite(C1).all()
        assert np.array_equal(C0, C1), "%s, N = %d: the two entry points differ" % (name, N)
        C_ref, S = oracle.spmm(csr.row_ptr, csr.col_idx, csr.vals, B)
        err, bad_zero = oracle.parity_error(C1, C_ref, S)
        assert bad_zero == 0 and err <= 1e-5, "max relative error %.3e" % err


def test_static_scratch_entry_point_runs_plans_without_cut_panels_and_refuses_oversize(oracle):
    import torch
    spmm.load()
    # no panel cut across workgroups: nothing to park, same path as spmm_execute
    csr = gen.tiny()
    plan = spmm.plan_create(csr.M, csr.K, csr.row_ptr, csr.col_idx, csr.vals)
    assert plan.describe()["n_cross"] == 0
    C0, C1 = _both(torch, plan, gen.activations_for(csr, 32))
    assert np.array_equal(C0, C1)
    # about 1900 workgroups of cut eight-row panels: 512 * 8 bytes each per column tile, more
    # than the 6 MiB of the array: refused with a status, nothing enqueued, C untouched
    M, K = 7600, 520
    row_ptr = (np.arange(M + 1, dtype=np.int64) * K).astype(np.int32)
    col_idx = np.tile(np.arange(K, dtype=np.int32), M)
    vals = np.ones(M * K, dtype=np.float32)
    heavy = spmm.plan_create(M, K, row_ptr, col_idx, vals, group_nnz=256, ufi=8, cross=1, sort_rows=-1)
    info = heavy.describe()
    # the plan's scratch holds four column tiles
    assert info["n_cross"] == 950 and info["scratch_bytes"] // 4 > 6 << 20, "one tile must need more than the array holds"
    dB = torch.ones((K, 8), dtype=torch.float32, device="cuda")
    dC = torch.full((M, 8), float("nan"), dtype=torch.float32, device="cuda")
    lib = spmm.load()
    assert lib.spmm_execute_static(heavy.handle, dB.data_ptr(), 8, dC.data_ptr(), None) == spmm.SPMM_ERR_UNSUPPORTED
    torch.cuda.synchronize()
    assert torch.isnan(dC).all()
    # the plan's own scratch is large enough: spmm_execute runs it
    assert lib.spmm_execute(heavy.handle, dB.data_ptr(), 8, dC.data_ptr(), None) == spmm.SPMM_OK
    torch.cuda.synchronize()
    assert torch.equal(dC, torch.full_like(dC, float(K)))
