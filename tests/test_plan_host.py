"""Host logic of the library, checked without a GPU (host-only plans).

Covers: the exported C ABI, the row-group enumeration against an independent
re-derivation from row_ptr (bit-exact), the format round trip back to the
canonical CSR (bit-exact), the closed forms the paper gives for pattern
enumeration, the meaning of the chunk arrays (evaluated by a test-side
interpreter against the oracle) and the error codes of the boundary.
"""
import ctypes
import os
import re

import numpy as np
import pytest

import paper_2506_15174_amd as spmm
from workloads import generators as gen

from plan_reference import (UFK, canonical_csr, choose_group_budget, choose_kslices, choose_schedule, choose_ufi,
                            check_blocks, choose_ufi_skewed, cross_allowed, decode_plan, derive_groups, interpret_plan, skewed_rows,
                            derive_sliced_groups, plan_schedule, sliced_row_ptr, sorted_row_order, undeal_blocks,
                            walk_chunks)

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def host_plan(csr, **kw):
    return spmm.plan_create(csr.M, csr.K, csr.row_ptr, csr.col_idx, csr.vals, host_only=True, **kw)


def arrays(plan):
    return (plan.get_array(spmm.ARRAY_ITEMS), plan.get_array(spmm.ARRAY_HDR),
            plan.get_array(spmm.ARRAY_STREAM), plan.get_array(spmm.ARRAY_WINS))


def plan_rows(csr, plan):
    """(row map, row pointer of the plan's row order); the map is None when the
    plan's rows are the matrix's.  Checks the exported map against the sort the
    header describes (decreasing length, equal lengths in ascending row order)."""
    rowmap = plan.get_array(spmm.ARRAY_ROWMAP)
    if not plan.describe()["sorted_rows"]:
        assert len(rowmap) == 0
        return None, np.asarray(csr.row_ptr, dtype=np.int64)
    order, ptr = sorted_row_order(csr.row_ptr)
    assert len(rowmap) == csr.M and np.array_equal(rowmap, order)
    return rowmap, ptr


def heavy_tail_matrix(M, K, seed, heavy_rows=(3, 10), empty_rows=(0, 5, 6, 7, 8)):
    """Random sparse matrix with a few dense rows and a few empty ones."""
    rng = np.random.default_rng(seed)
    W = np.where(rng.random((M, K)) < 0.08, rng.standard_normal((M, K)), 0.0).astype(np.float32)
    for r in heavy_rows:
        if r < M:
            W[r] = rng.standard_normal(K).astype(np.float32)
    for r in empty_rows:
        if r < M:
            W[r] = 0
    return gen.csr_from_dense(W)


CASES = {
    "tiny": lambda: gen.tiny(),
    "uniform_half": lambda: gen.uniform_positions(64, 96, 0.5, 3),
    "ragged_rows": lambda: gen.uniform_positions(37, 50, 0.8, 4),       # M % 4 != 0
    "heavy_tail": lambda: heavy_tail_matrix(30, 700, 5),                # split panels + empty rows
    "all_empty": lambda: gen.csr_from_dense(np.zeros((9, 12), np.float32)),
    "single_row": lambda: gen.uniform_positions(1, 300, 0.3, 6),
    "lognormal": lambda: gen.lognormal_rows(128, 256, 0.9, 7),
}


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "spmm.h")).read()
    declared = set(re.findall(r"\b(spmm_[a-z_]+)\s*\(", header))
    assert declared == set(spmm.EXPORTS)
    lib = ctypes.CDLL(spmm.LIB_PATH)
    for name in declared:
        assert getattr(lib, name) is not None
    assert spmm.status_string(0) == "ok"
    assert "CSR" in spmm.status_string(spmm.SPMM_ERR_INVALID_CSR)


@pytest.mark.parametrize("name", sorted(CASES))
@pytest.mark.parametrize("group_nnz", [0, 32, 200])
@pytest.mark.parametrize("force_ufi", [0, 1, 2, 4, 8])
@pytest.mark.parametrize("sort_rows", [0, 1, -1])
def test_row_groups_match_python_rederivation(name, group_nnz, force_ufi, sort_rows):
    csr = CASES[name]()
    plan = host_plan(csr, group_nnz=group_nnz, ufi=force_ufi, sort_rows=sort_rows)
    info = plan.describe()
    assert (info["M"], info["K"], info["nnz"]) == (csr.M, csr.K, int(csr.row_ptr[-1]))
    assert info["ufk"] == UFK and info["ufi"] in (1, 2, 4, 8)
    nnz = int(csr.row_ptr[-1])
    UFI, is_sorted = choose_schedule(csr.row_ptr, csr.M, csr.K, 0, force_ufi, sort_rows)
    assert info["ufi"] == UFI and info["sorted_rows"] == int(is_sorted)
    auto_g, auto_gp = choose_group_budget(csr.M, nnz, UFI)
    assert info["group_nnz"] == (group_nnz or auto_g) and info["group_panels"] == auto_gp
    got = plan.get_groups()
    _, plan_ptr = plan_rows(csr, plan)
    want, blocks = derive_groups(plan_ptr, csr.M, info["group_nnz"], info["group_panels"], UFI,
                                 cross=cross_allowed(csr.row_ptr))
    assert blocks == info["n_blocks"]
    assert got.shape == want.shape and np.array_equal(got, want)
    assert info["n_groups"] == len(want) and info["n_split"] == int((want[:, 4] & 1).sum())
    assert info["n_blocks"] * 8 * 16 == len(plan.get_array(spmm.ARRAY_ITEMS))
    # invariants: whole rows and the whole nonzero range are covered exactly once
    by_row = got[np.lexsort((got[:, 2], got[:, 0]))]
    nnz_cover = 0
    next_row = 0
    for rb, re_, nb, ne, fl in by_row:
        assert ne >= nb
        if fl & 1:
            assert re_ - rb <= UFI and rb % UFI == 0 and ne > nb
            assert rb in (next_row, next_row - (re_ - rb))  # pieces share their panel's rows
            pn = int(plan_ptr[re_] - plan_ptr[rb])
            assert pn > info["group_nnz"]
            assert ne - nb <= max(info["group_nnz"], -(-pn // 8))
        else:
            assert rb == next_row and rb % UFI == 0
            assert (nb, ne) == (plan_ptr[rb], plan_ptr[re_])
            assert ne - nb <= info["group_nnz"]
        assert nb == nnz_cover
        nnz_cover = ne
        next_row = re_
    assert next_row == csr.M and nnz_cover == csr.row_ptr[-1]
    whole = got[(got[:, 4] & 1) == 0]
    assert np.all(np.diff(whole[:, 3] - whole[:, 2]) <= 0), "whole-panel groups: heaviest first"
    n_split = int((got[:, 4] & 1).sum())
    assert np.all((got[:n_split, 4] & 1) == 1), "pieces of split panels come first"


def _row_ptr_only_plan(M, K, per_row, **kw):
    """A host plan of M rows with `per_row` entries each (columns 0 .. per_row-1)."""
    row_ptr = (np.arange(M + 1, dtype=np.int64) * per_row).astype(np.int32)
    col_idx = np.tile(np.arange(per_row, dtype=np.int32), M)
    return spmm.plan_create(M, K, row_ptr, col_idx, np.ones(M * per_row, np.float32), host_only=True, **kw)


# (M, K, entries per row, hint) -> (ufi, group_nnz, group_panels), worked by hand
# from the rule the header of spmm_plan.cpp states
SCHEDULE_CASES = [
    # 512 x 2048 at 20 %: wide B -> 2 rows; 256 panels of 820 -> 8 pieces -> ceil(5*820/32) = 129 -> 160
    ((512, 2048, 410, 0), (2, 160, 1)),
    # the same for 32 columns of B: rows of 410 >= 256 on 512 rows -> 2 rows as well
    ((512, 2048, 410, 32), (2, 160, 1)),
    # ... but rows of 200 stay single: 512 panels of 200 -> 8 pieces -> ceil(5*200/32) = 32
    ((512, 2048, 200, 32), (1, 32, 1)),
    # 1024 single rows of 100 for narrow B are cut in two at most: ceil(5*100/8) = 63 -> 64; for wide B 8 pieces -> 16 -> 32
    ((1024, 1024, 100, 32), (1, 64, 1)),
    ((1024, 1024, 30, 128), (1, 32, 1)),
    # ... rows of 400 in 4096 columns for 64 columns of B: two such rows share 400 * 400 / 4096 = 39 < 128
    # columns: single rows, not cut below 128 entries either; rows of 1200 share 351: two rows, 512 panels
    # of 2400 -> 8 pieces -> ceil(5*2400/32) = 375 -> 384
    ((1024, 4096, 400, 64), (1, 128, 1)),
    ((1024, 4096, 1200, 64), (2, 384, 1)),
    # 2048 rows: eight rows for wide B from rows of 128 sharing 16 columns on (256 panels of 6560 -> 8
    # pieces -> 1025 -> 1024), four rows for 64 columns (row >= 256, shared >= 32: 512 panels of 3280 ->
    # 8 pieces -> 513 -> 544) and for 32 (row >= 384, rows an eighth full)
    ((2048, 2048, 820, 128), (8, 1024, 1)),
    ((2048, 2048, 820, 64), (4, 544, 1)),
    ((2048, 2048, 820, 32), (4, 544, 1)),
    # ... rows of 400 in 8192 columns share 19 columns: eight rows for wide B (256 panels of 3200 -> 500 ->
    # 512), single rows for 64 columns (shared < 32; 2048 rows of 400 -> 4 pieces -> 125 -> 128) and for 32
    # (rows less than an eighth full)
    ((2048, 8192, 400, 128), (8, 512, 1)),
    ((2048, 8192, 400, 64), (1, 128, 1)),
    ((2048, 8192, 400, 32), (1, 128, 1)),
    # 4096 x 4096 with rows of 204 (95 % pruned): two rows share 10 columns < 16: single rows for wide B
    ((4096, 4096, 204, 128), (1, 256, 1)),
    # B of at most 16 columns (chunks of 32 or 64): eight rows only where two rows share 160 / 320 / 640
    # columns (hints 16 / 8 / 4).  Rows of 819 in 4096 columns share 163: eight rows for 16 columns (512
    # panels of 6552 -> 8 pieces -> 1024), single rows for 8 and 4 (4096 whole rows of 819 -> 1024)
    ((4096, 4096, 819, 16), (8, 1024, 1)),
    ((4096, 4096, 819, 8), (1, 1024, 1)),
    ((4096, 4096, 2048, 4), (8, 1024, 1)),
    # ... about 4096 waves instead of 8192: 1024 single rows of 400 are cut in 4 (not 8): ceil(5*400/16) = 125 -> 128
    ((1024, 4096, 400, 8), (1, 128, 1)),
    # ... 9 .. 16 columns keep the four- and two-row panels of the rule for 17 .. 32 columns; fewer columns do not
    # (512 four-row panels of 3280 -> 8 pieces -> 513 -> 544; 2048 whole single rows of 820 -> 1025 -> 1024)
    ((2048, 2048, 820, 16), (4, 544, 1)),
    ((2048, 2048, 820, 8), (1, 1024, 1)),
    # 4096 x 1024 at 50 %, wide B: 8 rows; 512 panels of 4096 -> 8 pieces -> 640
    ((4096, 1024, 512, 128), (8, 640, 1)),
    # narrow B, 384 <= rows of 512 < 768, half full: four rows; 1024 panels of 2048 -> 8 pieces -> 5*2048/32 = 320
    ((4096, 1024, 512, 32), (4, 320, 1)),
    # ... rows of 400 in 4096 columns are less than an eighth full: single rows
    ((4096, 4096, 400, 32), (1, 512, 1)),
    # rows of 52 < 192: single rows; 4096 whole rows of 52 -> 65 -> 96
    ((4096, 1024, 52, 0), (1, 96, 1)),
    # 256 rows: too few panels for tall ones; 256 rows of 128 -> 8 pieces -> 20 -> 32
    ((256, 256, 128, 128), (1, 32, 1)),
    # 32768 single rows: 4 panels share a wave, budget 5*8*4/4 = 40 -> 64
    ((32768, 1024, 8, 0), (1, 64, 4)),
    # 8192 x 8192 at 50 %, narrow B: rows of 4096 >= 768 -> 8 rows; 1024 panels -> 8 pieces, capped
    ((8192, 8192, 4096, 32), (8, 1024, 1)),
    # ... medium and wide B: 8 rows as well
    ((8192, 8192, 4096, 64), (8, 1024, 1)),
    # (128 columns of B: 8192 rows of 512 bytes are exactly one L2 and the rows hold 1024 entries or
    # more: two column ranges; 2 x 8192 plan rows = 2048 panels of 16384 -> 4 pieces -> 5120 -> 1024)
    ((8192, 8192, 4096, 128), (8, 1024, 1, 2)),
    ((8192, 8192, 4096, 128, 1), (8, 1024, 1, 1)),
    ((8192, 8192, 1000, 128), (8, 1024, 1, 1)),
    # 64 columns of B: 8 rows from 4096 rows on when rows hold 256 or more
    ((4096, 1024, 512, 64), (8, 640, 1)),
    # ... 512 panels of 3280 -> 8 pieces -> ceil(5*3280/32) = 513 -> 544
    ((4096, 4096, 410, 64), (8, 544, 1)),
    # ... 1024 rows: 2 rows; 512 panels of 4096 -> 8 pieces -> 640
    ((1024, 4096, 2048, 64), (2, 640, 1)),
    # wide B, 1024 rows of 102 (64 <= 102 < 128): 2 rows; 512 panels of 204 -> ceil(1020/32) = 32
    ((1024, 1024, 102, 128), (2, 32, 1)),
    # 16384 rows of B of 512 bytes do not fit one L2.  Left whole (kslices = 1): single rows; 2 panels
    # per wave, capped budget
    ((16384, 16384, 800, 128, 1), (1, 1024, 2)),
    # ... but rows of 1100 take eight rows there (the product runs as 64-column tiles that fit):
    # 2048 panels of 8800 -> 4 pieces -> ceil(5*8800/16) = 2750 -> capped at 1024
    ((16384, 16384, 1100, 128, 1), (8, 1024, 1)),
    # K = 32768: no tile fits, single rows whatever the rows
    ((4096, 32768, 2000, 128, 1), (1, 1024, 1)),
    # By default such matrices are cut along K (13 M entries >= 2^20): 16384 columns in 4 ranges of
    # 4096 (2 MiB of B each).  The height is that of a 4096-column matrix (rows of 800 >= 192: eight
    # rows); 4 x 16384 plan rows = 8192 panels of 1600 -> whole panels, ceil(5*1600/4) = 2000 -> 1024
    ((16384, 16384, 800, 128), (8, 1024, 1, 4)),
    # ... 32768 columns in 8 ranges of 4096; 8 x 4096 plan rows = 4096 panels of 2000 -> 2500 -> 1024
    ((4096, 32768, 2000, 128), (8, 1024, 1, 8)),
    # ... 64 columns of B: 16384 rows of 256 bytes fit (not cut); 32768 do not: 4 ranges of 8192 (2 MiB)
    ((16384, 16384, 800, 64), (8, 1024, 1, 1)),
    ((8192, 32768, 800, 64), (8, 1024, 1, 4)),
    # ... rows too short for 4 ranges (rows of 100 < 4 x 32) or too few entries (2^20 > 16384 x 60): whole,
    # single rows, 2 per wave: ceil(5*100*2/4) = 250 -> 256, ceil(5*60*2/4) = 150 -> 160
    ((16384, 16384, 100, 128), (1, 256, 2, 1)),
    ((16384, 16384, 60, 128), (1, 160, 2, 1)),
    # ... a plan with chunks of 16 (hint of 32 columns or fewer) is never cut
    ((4096, 65536, 2000, 32), (1, 1024, 1, 1)),
]


@pytest.mark.parametrize("case,want", SCHEDULE_CASES)
def test_schedule_constants_rule(case, want):
    M, K, per_row, hint = case[:4]
    setting = case[4] if len(case) > 4 else 0
    info = _row_ptr_only_plan(M, K, per_row, n_hint=hint, kslices=setting).describe()
    assert (info["ufi"], info["group_nnz"], info["group_panels"]) == want[:3]
    nnz = M * per_row
    ns = choose_kslices(M, K, nnz, hint, setting, info["ufk"])
    assert info["k_slices"] == ns == (want[3] if len(want) > 3 else 1)
    assert info["slice_rows"] == (-(-M // 8) * 8 if ns > 1 else M) and info["slice_cols"] == -(-K // ns)
    ufi = choose_ufi(M, -(-K // ns), nnz, hint)
    assert (ufi,) + choose_group_budget(ns * info["slice_rows"], nnz, ufi, hint) == want[:3]


def _plan_from_row_lengths(lens, K, **kw):
    """A host plan whose row i holds columns 0 .. lens[i]-1."""
    lens = np.asarray(lens, dtype=np.int64)
    row_ptr = np.concatenate(([0], np.cumsum(lens))).astype(np.int32)
    col_idx = np.concatenate([np.arange(n, dtype=np.int32) for n in lens]) if len(lens) else np.zeros(0, np.int32)
    return row_ptr, spmm.plan_create(len(lens), K, row_ptr, col_idx, np.ones(len(col_idx), np.float32),
                                     host_only=True, **kw)


# (rows as (count, length) runs, K, hint) -> (ufi, sorted), worked by hand from the
# rule for skewed matrices in the header of spmm_plan.cpp
SKEWED_CASES = [
    # 256 rows of 2048 among 16128 of 60: nnz 1 491 968 (2^20 or more: heavy panels may be cut
    # across workgroups), mean 91, the long rows hold 35 %: skewed -> eight rows for wide B,
    # four for medium B, sorted
    (((256, 2048), (16128, 60)), 2048, 128, (8, 1)),
    (((256, 2048), (16128, 60)), 2048, 64, (4, 1)),
    # narrow B takes two rows where wide B takes four or eight
    (((256, 2048), (16128, 60)), 2048, 32, (2, 1)),
    # 256 rows of 2048 among 16128 of 20: nnz 846 848 (below 2^20: every panel stays inside one
    # workgroup), fair share 3308: 2 x 2048 <= 6616 < 4 x 2048 -> two rows; narrow B: single rows, not sorted
    (((256, 2048), (16128, 20)), 2048, 128, (2, 1)),
    (((256, 2048), (16128, 20)), 2048, 32, (1, 0)),
    # 64 rows of 4096 among 4032 of 100: skewed (39 %), fair share 2599: 2 x 4096 > 5198: single rows
    (((64, 4096), (4032, 100)), 4096, 128, (1, 0)),
    # 512 rows of 1024 among 15872 of 200: nnz 3 698 688, mean 226, 1024 > 4 x 226 holds 14 %:
    # not skewed, the ordinary rule (16384 rows, rows of 225 >= 192) gives eight rows
    (((512, 1024), (15872, 200)), 1024, 128, (8, 0)),
    # 1024 rows of 2000 among 15360 of 100: nnz 3 584 000, the long rows hold 57 %; fair share
    # 14000: 8 x 2000 <= 28000 -> eight rows; narrow B: two rows
    (((1024, 2000), (15360, 100)), 2048, 0, (8, 1)),
    (((1024, 2000), (15360, 100)), 2048, 32, (2, 1)),
    # K = 16384: 128 columns of B exceed one L2; the plan is cut into 4 column ranges (3.6 M entries
    # >= 32 x 4 x 16384) and takes the height of a 4096-column matrix; K = 32768 would need 8 ranges,
    # for which the rows are too short (3.6 M < 32 x 8 x 16384): left whole, single rows, unsorted
    (((1024, 2000), (15360, 100)), 16384, 128, (8, 1)),
    (((1024, 2000), (15360, 100)), 32768, 128, (1, 0)),
]


@pytest.mark.parametrize("runs,K,hint,want", SKEWED_CASES)
def test_schedule_of_skewed_matrices(runs, K, hint, want):
    lens = np.concatenate([np.full(c, n) for c, n in runs])
    lens = lens[np.random.default_rng(5).permutation(len(lens))]
    row_ptr, plan = _plan_from_row_lengths(lens, K, n_hint=hint)
    info = plan.describe()
    assert (info["ufi"], info["sorted_rows"]) == want
    col_idx = np.concatenate([np.arange(n, dtype=np.int32) for n in lens])
    assert plan_schedule(row_ptr, col_idx, len(lens), K, hint)[:3] == (info["k_slices"], want[0], bool(want[1]))
    if want[1]:
        rowmap = plan.get_array(spmm.ARRAY_ROWMAP)
        if info["k_slices"] > 1:
            # cut along K: one map per column range, the same order in each, shifted by the range's rows
            M, MS = len(lens), info["slice_rows"]
            maps = rowmap.reshape(info["k_slices"], MS)
            for sidx, m in enumerate(maps):
                assert np.array_equal(m[:M], maps[0][:M] + sidx * MS) and np.array_equal(m[M:], np.arange(M, MS) + sidx * MS)
            rowmap = maps[0][:M]
        assert sorted(rowmap.tolist()) == list(range(len(lens)))
        sl = lens[rowmap]
        assert np.all(np.diff(sl) <= 0), "longest rows first"
        same = np.flatnonzero(np.diff(sl) == 0)
        assert np.all(rowmap[same] < rowmap[same + 1]), "equal lengths keep the row order"


def test_skewed_schedule_without_cuts_across_workgroups():
    """cross < 0: a panel stays inside one workgroup, so the height follows the longest row
    against a compute unit's share (fair share 5828: 4 x 2048 <= 11656 < 8 x 2048 -> four
    rows) and the group budget is the ordinary one; by default the same matrix takes eight
    rows and half the budget, its heavy panels cut across workgroups."""
    lens = np.concatenate([np.full(256, 2048), np.full(16128, 60)])
    lens = lens[np.random.default_rng(5).permutation(len(lens))]
    row_ptr, plan = _plan_from_row_lengths(lens, 2048, n_hint=128, cross=-1)
    info = plan.describe()
    assert (info["ufi"], info["sorted_rows"], info["n_cross"]) == (4, 1, 0)
    assert choose_schedule(row_ptr, len(lens), 2048, 128, cross=-1) == (4, True)
    assert info["group_nnz"] == choose_group_budget(len(lens), int(row_ptr[-1]), 4)[0]
    _, plan = _plan_from_row_lengths(lens, 2048, n_hint=128)
    info = plan.describe()
    assert (info["ufi"], info["sorted_rows"]) == (8, 1) and info["n_cross"] == 32   # 256 rows of 2048 in 32 panels
    g8 = choose_group_budget(len(lens), int(row_ptr[-1]), 8)[0]
    assert info["group_nnz"] == max(32, g8 // 2 // 32 * 32)


def test_sorting_can_be_forced_and_forbidden():
    lens = [5, 300, 0, 17, 300, 2, 64, 0, 9]
    row_ptr, plan = _plan_from_row_lengths(lens, 400, sort_rows=1, ufi=2)
    assert plan.describe()["sorted_rows"] == 1
    assert plan.get_array(spmm.ARRAY_ROWMAP).tolist() == [1, 4, 6, 3, 8, 0, 5, 2, 7]
    # groups are stated in the sorted order: the first panel is rows (1, 4) = 600 entries
    g = plan.get_groups()
    assert g[np.lexsort((g[:, 2], g[:, 0]))][0, :2].tolist() == [0, 2]
    assert not skewed_rows(row_ptr)      # 300 x 9 rows < 4 x 697 entries: left alone, the order would stay
    _, plan = _plan_from_row_lengths(lens, 400, sort_rows=-1, ufi=2)
    assert plan.describe()["sorted_rows"] == 0 and len(plan.get_array(spmm.ARRAY_ROWMAP)) == 0
    with pytest.raises(spmm.SpmmError):
        plan.get_array(6)


def test_empty_matrix_schedule():
    info = spmm.plan_create(0, 5, np.array([0], np.int32), np.zeros(0, np.int32), np.zeros(0, np.float32),
                            host_only=True).describe()
    assert (info["ufi"], info["group_nnz"], info["group_panels"]) == (1, 32, 1)


def test_split_panels_have_power_of_two_piece_counts():
    # rows of 300, 500 and 900 entries with a budget of 128: 3 -> 4, 4 and 8 -> 8 pieces
    lens = [300, 500, 900]
    row_ptr = np.concatenate(([0], np.cumsum(lens))).astype(np.int32)
    col_idx = np.concatenate([np.arange(n, dtype=np.int32) for n in lens])
    plan = spmm.plan_create(3, 1000, row_ptr, col_idx, np.ones(len(col_idx), np.float32), host_only=True,
                            ufi=1, group_nnz=128)
    g = plan.get_groups()
    pieces = {int(r): int(np.sum(g[:, 0] == r)) for r in range(3)}
    assert pieces == {0: 4, 1: 4, 2: 8}
    # 4 + 4 share one workgroup, 8 fill another
    assert plan.describe()["n_blocks"] == 2


@pytest.mark.parametrize("name", sorted(CASES))
@pytest.mark.parametrize("group_nnz", [0, 32, 200])
@pytest.mark.parametrize("force_ufi", [0, 1, 2, 4, 8])
@pytest.mark.parametrize("sort_rows", [0, 1])
def test_format_round_trip_is_bit_exact(name, group_nnz, force_ufi, sort_rows):
    csr = CASES[name]()
    plan = host_plan(csr, group_nnz=group_nnz, ufi=force_ufi, sort_rows=sort_rows)
    items, hdr, stream, wins = arrays(plan)
    rows, cc, bits = decode_plan(items, hdr, stream, wins, plan.describe()["ufi"], plan_rows(csr, plan)[0])
    assert len(rows) == csr.row_ptr[-1] == plan.describe()["nnz"]
    order = np.lexsort((cc, rows))
    want_rows, want_cols, want_bits = canonical_csr(csr.row_ptr, csr.col_idx, csr.vals)
    assert np.array_equal(rows[order], want_rows)
    assert np.array_equal(cc[order], want_cols)
    assert np.array_equal(bits[order], want_bits)
    info = plan.describe()
    counts = (hdr[:info["n_chunks"]] >> 8) & 127
    assert int(counts.sum()) == info["n_enum"]
    assert len(hdr) >= info["n_chunks"] + 10 and not hdr[info["n_chunks"]:].any()
    pc = np.array([bin(int(h) & 255).count("1") for h in hdr[:info["n_chunks"]]])
    assert len(stream) == info["stream_words"] >= (UFK + 1) * len(pc) + UFK * int(pc.sum())


def slot_patterns(h, cols):
    """(own pattern, column index) of the real slots of a chunk: a slot's pattern is
    the top byte of its column word, or the chunk's when that byte is 0."""
    return [((int(c) >> 24) or (int(h) & 255), int(c) & 0xFFFFFF) for c in cols[:(int(h) >> 8) & 127]]


def test_leftovers_of_different_patterns_share_chunks():
    # 4-row panel, K = 64: columns 0..9 have pattern 0b0001, 10..12 pattern 0b0110,
    # 13..14 pattern 0b1000: one full chunk of pattern 1, then 2 + 3 + 2 leftovers
    # in one chunk whose header holds the union 0b1111
    W = np.zeros((4, 64), dtype=np.float32)
    W[0, 0:10] = np.arange(1, 11)
    W[1, 10:13] = 20 + np.arange(3)
    W[2, 10:13] = 30 + np.arange(3)
    W[3, 13:15] = 40 + np.arange(2)
    plan = host_plan(gen.csr_from_dense(W), ufi=4)
    items, hdr, stream, wins = arrays(plan)
    info = plan.describe()
    assert info["n_chunks"] == 2 and info["n_enum"] == 15
    chunks = [c for it in items.reshape(-1, 16) if not int(it[5]) & 2 for c in walk_chunks(it, hdr, stream, wins)]
    (h0, c0, v0), (h1, c1, v1) = chunks
    assert h0 & 255 == 0b0001 and (h0 >> 8) & 127 == 8 and not (h0 >> 15) & 1
    assert [x for _, x in slot_patterns(h0, c0)] == list(range(8)) and all(int(c) >> 24 == 0 for c in c0)
    assert h1 & 255 == 0b1111 and (h1 >> 8) & 127 == 7 and (h1 >> 15) & 1
    assert slot_patterns(h1, c1) == [(1, 8), (1, 9), (6, 10), (6, 11), (6, 12), (8, 13), (8, 14)]
    # four value blocks (rows 0..3); a slot holds zeros in the rows it lacks
    f = [b.view(np.float32) for b in v1]
    assert f[0].tolist() == [9, 10, 0, 0, 0, 0, 0, 0]
    assert f[1].tolist() == [0, 0, 20, 21, 22, 0, 0, 0]
    assert f[2].tolist() == [0, 0, 30, 31, 32, 0, 0, 0]
    assert f[3].tolist() == [0, 0, 0, 0, 0, 40, 41, 0]


def test_unsorted_and_duplicate_columns_are_canonicalised():
    row_ptr = np.array([0, 5, 5, 8, 9], dtype=np.int32)
    col_idx = np.array([7, 2, 7, 0, 2, 2, 7, 1, 7], dtype=np.int32)
    vals = np.array([1, 2, 3, 4, 5, 6, 7, 8, 9], dtype=np.float32)
    csr = gen.Csr(4, 8, row_ptr, col_idx, vals)
    plan = host_plan(csr, ufi=4)
    items, hdr, stream, wins = arrays(plan)
    rows, cc, bits = decode_plan(items, hdr, stream, wins, plan.describe()["ufi"])
    got = sorted(zip(rows.tolist(), cc.tolist(), bits.view(np.float32).tolist()))
    want = sorted(zip([0, 0, 0, 0, 0, 2, 2, 2, 3], col_idx.tolist(), vals.tolist()))
    assert got == want
    # column 7 is stored twice in row 0: its second occurrence cannot share an
    # enumerated column with the first, so 7 appears in two different column slots
    assert cc.tolist().count(7) == 4 and len(rows) == 9
    slots = []
    for it in items.reshape(-1, 16):
        if not int(it[5]) & 2:
            for h, cols, _ in walk_chunks(it, hdr, stream, wins):
                slots += [int(c) & 0xFFFFFF for c in cols[:(h >> 8) & 127]]
    assert slots.count(7) == 2 and slots.count(2) == 2
    # within a row, duplicates keep their stored order (3 after 1 for column 7 of row 0)
    B = np.eye(8, dtype=np.float32)
    C = interpret_plan(items, hdr, stream, wins, B, 4, 4)
    assert C[0, 7] == 4.0 and C[0, 2] == 7.0 and C[2, 2] == 6.0 and C[3, 7] == 9.0
    assert not C[1].any()


def test_every_pattern_of_a_four_row_panel_is_enumerated():
    # Paper Section 2: a tile of 4 rows has 15 possible nonzero patterns.
    W = np.zeros((4, 15), dtype=np.float32)
    for p in range(1, 16):
        for r in range(4):
            if (p >> r) & 1:
                W[r, p - 1] = 10 * p + r
    plan = host_plan(gen.csr_from_dense(W), ufi=4)
    items, hdr, stream, wins = arrays(plan)
    seen = {}
    for it in items.reshape(-1, 16):
        if not int(it[5]) & 2:
            for h, cols, _ in walk_chunks(it, hdr, stream, wins):
                for own, col in slot_patterns(h, cols):
                    seen[own] = col
    assert sorted(seen) == list(range(1, 16)) and len(seen) == 2 ** 4 - 1
    assert all(col == p - 1 for p, col in seen.items())
    # one column per pattern: all fifteen are leftovers and share two chunks
    assert plan.describe()["n_chunks"] == 2
    # three rows give 2^3 - 1 = 7 patterns (caption of the paper's Figure 4)
    plan3 = host_plan(gen.csr_from_dense(W[:3]), ufi=4)
    items3, hdr3, stream3, wins3 = arrays(plan3)
    pats3 = set()
    for it in items3.reshape(-1, 16):
        if not int(it[5]) & 2:
            for h, cols, _ in walk_chunks(it, hdr3, stream3, wins3):
                pats3 |= {own for own, _ in slot_patterns(h, cols)}
    assert pats3 == set(range(1, 8))


def test_pattern_histogram_of_uniform_sparsity_matches_closed_form():
    # With independent positions of density d a panel column shows pattern p with
    # probability d^r (1-d)^(4-r), r = popcount(p) (the paper's "nearly uniform
    # frequency" at d = 1/2, Section 3.2.2); the reuse factor nnz / n_enum is
    # 4 d / (1 - (1-d)^4).
    for d, seed in ((0.5, 21), (0.2, 22), (0.1, 23)):
        M, K = 256, 2048
        rng = np.random.default_rng(seed)
        W = np.where(rng.random((M, K)) < d, 1.0, 0.0).astype(np.float32)
        csr = gen.csr_from_dense(W)
        plan = host_plan(csr, group_nnz=1 << 20, group_panels=1 << 20, ufi=4)
        info = plan.describe()
        items, hdr, stream, wins = arrays(plan)
        hist = np.zeros(16)
        for it in items.reshape(-1, 16):
            if not int(it[5]) & 2:
                for h, cols, _ in walk_chunks(it, hdr, stream, wins):
                    for own, _ in slot_patterns(h, cols):
                        hist[own] += 1
        UFI = 4
        total_columns = (M // UFI) * K
        for p in range(1, 16):
            r = bin(p).count("1")
            prob = d ** r * (1 - d) ** (UFI - r)
            sigma = np.sqrt(total_columns * prob * (1 - prob))
            assert abs(hist[p] - total_columns * prob) < 6 * sigma + 1
        reuse = info["nnz"] / info["n_enum"]
        assert abs(reuse - UFI * d / (1 - (1 - d) ** UFI)) < 0.02


@pytest.mark.parametrize("name", ["tiny", "ragged_rows", "heavy_tail", "all_empty", "single_row"])
@pytest.mark.parametrize("group_nnz", [0, 32])
@pytest.mark.parametrize("force_ufi", [0, 1, 2, 4, 8])
@pytest.mark.parametrize("sort_rows", [0, 1])
def test_chunk_arrays_evaluate_to_the_product(oracle, name, group_nnz, force_ufi, sort_rows):
    csr = CASES[name]()
    B = gen.dense_activations(csr.K, 5, 99)
    plan = host_plan(csr, group_nnz=group_nnz, ufi=force_ufi, sort_rows=sort_rows)
    C = interpret_plan(*arrays(plan), B, csr.M, plan.describe()["ufi"], plan_rows(csr, plan)[0])
    C_ref, S = oracle.spmm(csr.row_ptr, csr.col_idx, csr.vals, B)
    err, bad_zero = oracle.parity_error(C, C_ref, S)
    assert err <= 1e-5 and bad_zero == 0


def test_many_empty_panels_in_one_group_keep_windows_short():
    # 400 empty rows packed into one group: 400 chunks without values; a window may
    # hold only as many as leave the kernels' look-ahead column reads inside it
    M = 400
    plan = spmm.plan_create(M, 16, np.zeros(M + 1, np.int32), np.zeros(0, np.int32), np.zeros(0, np.float32),
                            host_only=True, ufi=1, group_panels=1000)
    info = plan.describe()
    assert info["n_groups"] == 1 and info["n_chunks"] == M
    items, hdr, stream, wins = arrays(plan)
    rows, _, _ = decode_plan(items, hdr, stream, wins, 1)      # walks and checks every window
    assert len(rows) == 0
    counts = [int(w) & 0xFFFF for w in wins[:-1]]
    assert sum(counts) == M and len(counts) >= 4
    # without the bound a window of 1024 words would take 113 such chunks (9 words each)
    assert all(-(-wc // 8) * 8 + (wc + 8) * 8 <= 1024 for wc in counts) and max(counts) == 106


def _random_csr(rng, M, K, mode):
    """Random CSR with unsorted columns and duplicates; mode picks the row-length law."""
    lens = {0: lambda: rng.integers(0, K + 1, M),
            1: lambda: np.where(rng.random(M) < 0.15, K, rng.integers(0, 4, M)),       # a few dense rows
            2: lambda: rng.integers(0, 3, M),
            3: lambda: np.where(rng.random(M) < 0.2, 0, rng.integers(0, 2 * K, M))}[mode]()
    row_ptr = np.concatenate(([0], np.cumsum(lens))).astype(np.int32)
    col_idx = rng.integers(0, K, int(row_ptr[-1])).astype(np.int32)
    vals = rng.integers(-8, 9, int(row_ptr[-1])).astype(np.float32)
    return gen.Csr(M, K, row_ptr, col_idx, vals)


@pytest.mark.parametrize("seed", range(60))
def test_random_matrices_and_settings_round_trip(seed):
    """Random shapes, row-length laws, heights, budgets and row orders: the plan decodes
    to the canonical CSR bit for bit, its groups are those the reference derives, and
    the chunk arrays evaluate to the exact product (small integers: any order is exact)."""
    rng = np.random.default_rng(1000 + seed)
    M, K = int(rng.integers(0, 60)), int(rng.integers(1, 200))
    csr = _random_csr(rng, M, K, seed % 4)
    ufi = int(rng.choice([0, 1, 2, 4, 8]))
    group_nnz = int(rng.choice([0, 8, 40, 300]))
    sort_rows = int(rng.choice([-1, 0, 1]))
    hint = int(rng.choice([0, 4, 8, 16, 32, 64, 128]))
    ufk = int(rng.choice([0, 0, 8, 16, 32, 64]))
    plan = host_plan(csr, group_nnz=group_nnz, ufi=ufi, sort_rows=sort_rows, n_hint=hint, ufk=ufk)
    info = plan.describe()
    assert info["ufk"] == (ufk or (8 if hint == 0 or hint > 32 else 16 if hint > 16 else 32 if hint > 8 else 64))
    want_ufi, want_sorted = choose_schedule(csr.row_ptr, M, K, hint, ufi, sort_rows)
    assert (info["ufi"], info["sorted_rows"]) == (want_ufi, int(want_sorted))
    rowmap, plan_ptr = plan_rows(csr, plan)
    want, blocks = derive_groups(plan_ptr, M, info["group_nnz"], info["group_panels"], info["ufi"],
                                 cross=cross_allowed(csr.row_ptr))
    assert np.array_equal(plan.get_groups(), want) and blocks == info["n_blocks"]
    items, hdr, stream, wins = arrays(plan)
    rows, cc, bits = decode_plan(items, hdr, stream, wins, info["ufi"], rowmap, ufk=info["ufk"])
    # the same multiset of (row, column, value): values of a column stored twice in a row keep their order
    want_rows, want_cols, want_bits = canonical_csr(csr.row_ptr, csr.col_idx, csr.vals)
    got = sorted(zip(rows.tolist(), cc.tolist(), bits.tolist()))
    assert got == sorted(zip(want_rows.tolist(), want_cols.tolist(), want_bits.tolist()))
    B = rng.integers(-4, 5, (K, 3)).astype(np.float32)
    C = interpret_plan(items, hdr, stream, wins, B, M, info["ufi"], rowmap, ufk=info["ufk"])
    dense = np.zeros((M, K), dtype=np.float64)
    np.add.at(dense, (np.repeat(np.arange(M), np.diff(csr.row_ptr)), csr.col_idx), csr.vals.astype(np.float64))
    assert np.array_equal(C.astype(np.float64), dense @ B.astype(np.float64))


@pytest.mark.parametrize("ufi", [1, 2, 4, 8])
def test_heavy_panels_are_cut_across_blocks(ufi):
    """A panel heavier than eight group budgets and than 1/1024 of all entries is cut
    into more pieces than a block has waves: its pieces fill blocks of their own, eight
    each (the last may be short), every block gets a scratch slot, and the chunk arrays
    still evaluate to the exact product.  With the setting cross < 0 the same matrix
    keeps every panel in one block and needs no scratch."""
    rng = np.random.default_rng(50 + ufi)
    M, K = 37, 3000
    W = np.where(rng.random((M, K)) < 0.03, rng.integers(-8, 9, (M, K)), 0).astype(np.float32)
    W[2] = rng.integers(1, 9, K)
    W[3, ::2] = rng.integers(1, 9, K // 2)
    W[20] = rng.integers(1, 9, K)
    csr = gen.csr_from_dense(W)
    B = rng.integers(-4, 5, (K, 5)).astype(np.float32)
    dense = W.astype(np.float64) @ B.astype(np.float64)
    assert not cross_allowed(csr.row_ptr) and cross_allowed(csr.row_ptr, 1)    # a small matrix: only on request
    for cross in (1, 0, -1):
        plan = host_plan(csr, ufi=ufi, group_nnz=64, cross=cross)
        info = plan.describe()
        groups = plan.get_groups()
        rowmap, plan_ptr = plan_rows(csr, plan)     # tall panels of this matrix sort the rows by length
        want, blocks = derive_groups(plan_ptr, M, info["group_nnz"], info["group_panels"], ufi, cross=cross > 0)
        assert np.array_equal(groups, want) and blocks == info["n_blocks"]
        items, hdr, stream, wins = arrays(plan)
        slots = check_blocks(items, ufi, rowmap)
        if cross <= 0:
            assert info["n_cross"] == 0 and slots == 0 and not (groups[:, 4] & 8).any()
            assert max(np.bincount(groups[groups[:, 4] != 0, 0])) <= 8
        else:
            assert info["n_cross"] >= 1 and slots >= 2 * info["n_cross"]
            heavy = groups[(groups[:, 4] & 8) != 0]
            assert len(heavy) > 8 * info["n_cross"] and np.all(heavy[:, 4] == 9)
            # pieces of one budget or less: 8 budgets = 512 entries per block at most
            assert np.all(heavy[:, 3] - heavy[:, 2] <= 64)
        assert info["scratch_bytes"] == 0      # host-only plans own no device memory
        # the table the adding launch reads: one entry per cut panel, in the order of its workgroups
        table = plan.get_array(spmm.ARRAY_CROSS).reshape(-1, 12)
        assert len(table) == info["n_cross"]
        firsts = [blk for blk in items.reshape(-1, 8, 16) if int(blk[0, 5]) & 8 and int(blk[0, 15]) == 0]
        assert len(firsts) == len(table)
        for entry, blk in zip(table, firsts):
            live = blk[(blk[:, 5] & 2) == 0]
            rows_of_panel = int(live[0, 1])
            assert (int(entry[0]), int(entry[1]), int(entry[2]), int(entry[3])) == \
                (int(blk[0, 14]), int(blk[0, 13]), rows_of_panel, 0)
            want_rows = [int(rowmap[int(live[0, 0]) + r]) if rowmap is not None else int(live[0, 0]) + r
                         for r in range(rows_of_panel)]
            assert entry[4:4 + rows_of_panel].tolist() == want_rows and not entry[4 + rows_of_panel:].any()
        C = interpret_plan(items, hdr, stream, wins, B, M, ufi, rowmap)
        assert np.array_equal(C.astype(np.float64), dense)


def sliced_plan_rows(csr, plan):
    """(row map or None, row pointer of the plan's rows, row order or None) of a plan cut along K,
    with the exported map checked against the order the header describes."""
    info = plan.describe()
    ns, MS = info["k_slices"], info["slice_rows"]
    rowmap = plan.get_array(spmm.ARRAY_ROWMAP)
    order = None
    if info["sorted_rows"]:
        order, _ = sorted_row_order(csr.row_ptr)
        want = np.arange(ns * MS).reshape(ns, MS)
        want[:, :csr.M] = order[None, :] + (np.arange(ns) * MS)[:, None]
        assert np.array_equal(rowmap, want.reshape(-1))
    else:
        assert len(rowmap) == 0
        rowmap = None
    return rowmap, sliced_row_ptr(csr.row_ptr, csr.col_idx, csr.K, ns, order), order


@pytest.mark.parametrize("name", sorted(CASES))
@pytest.mark.parametrize("ns", [2, 4, 8])
@pytest.mark.parametrize("force_ufi", [0, 1, 4, 8])
@pytest.mark.parametrize("sort_rows,cross,group_nnz", [(0, 0, 0), (1, 1, 32), (-1, -1, 200)])
def test_plans_cut_along_k(oracle, name, ns, force_ufi, sort_rows, cross, group_nnz):
    """A plan cut into column ranges is the plan of the matrix's rows taken once per range
    (range s of row i as plan row s * slice_rows + i): same groups as the re-derivation
    from that row pointer, every block in one range, block b of the launch in range
    b mod k_slices, the entries of the matrix each exactly once and in their range, and the
    ranges' partial products adding up to the product."""
    csr = CASES[name]()
    plan = host_plan(csr, kslices=ns, ufi=force_ufi, sort_rows=sort_rows, cross=cross, group_nnz=group_nnz)
    info = plan.describe()
    nnz = int(csr.row_ptr[-1])
    want_ns = choose_kslices(csr.M, csr.K, nnz, 0, ns)
    assert info["k_slices"] == want_ns == (ns if csr.K >= 8 else 1)
    MS, KS = info["slice_rows"], info["slice_cols"]
    assert (info["M"], info["K"]) == (csr.M, csr.K) and MS == -(-csr.M // 8) * 8 and KS == -(-csr.K // ns)
    _, UFI, is_sorted, may_cross = plan_schedule(csr.row_ptr, csr.col_idx, csr.M, csr.K, 0, force_ufi, sort_rows, cross, ns)
    assert info["ufi"] == UFI and info["sorted_rows"] == int(is_sorted)
    rowmap, plan_ptr, order = sliced_plan_rows(csr, plan)
    assert plan_ptr[-1] == nnz
    auto_g, auto_gp = choose_group_budget(ns * MS, nnz, UFI)
    if may_cross:
        auto_g = max(32, auto_g // 2 // 32 * 32)
    elif skewed_rows(csr.row_ptr):
        auto_g = max(32, auto_g // 4 // 32 * 32)       # skewed rows, every panel inside one workgroup: a quarter
    assert info["group_nnz"] == (group_nnz or auto_g) and info["group_panels"] == auto_gp
    want, blocks = derive_sliced_groups(plan_ptr, MS, ns, info["group_nnz"], info["group_panels"], UFI, cross=may_cross)
    assert np.array_equal(plan.get_groups(), want) and info["n_blocks"] == blocks and blocks % ns == 0
    items, hdr, stream, wins = arrays(plan)
    # block b of the launch holds rows of range b mod ns only
    for b, blk in enumerate(items.reshape(-1, 8, 16)):
        live = blk[(blk[:, 5] & 2) == 0]
        assert np.all(live[:, 0] // MS == b % ns) and np.all((live[:, 0] + live[:, 1] - 1) // MS == b % ns)
    formed = undeal_blocks(items, ns)
    rows, cc, bits = decode_plan(formed, hdr, stream, wins, UFI, rowmap)
    assert len(rows) == nnz
    assert np.array_equal(rows // MS, cc // KS), "every entry sits in the range of its column"
    o = np.lexsort((cc, rows % MS))
    want_rows, want_cols, want_bits = canonical_csr(csr.row_ptr, csr.col_idx, csr.vals)
    assert np.array_equal((rows % MS)[o], want_rows) and np.array_equal(cc[o], want_cols)
    assert np.array_equal(bits[o], want_bits)
    # the ranges' products, added in range order as the last launch does
    B = gen.dense_activations(csr.K, 5, 99)
    parts = interpret_plan(formed, hdr, stream, wins, B, ns * MS, UFI, rowmap).reshape(ns, MS, 5)
    assert not np.isnan(parts).any(), "every row of every range is written"
    assert not parts[:, csr.M:].any(), "the rows that pad a range are empty"
    C = parts[0, :csr.M].copy()
    for sl in range(1, ns):
        C += parts[sl, :csr.M]
    C_ref, S = oracle.spmm(csr.row_ptr, csr.col_idx, csr.vals, B)
    err, bad_zero = oracle.parity_error(C, C_ref, S)
    assert err <= 1e-5 and bad_zero == 0


def test_options_of_plans_cut_along_k():
    csr = CASES["uniform_half"]()
    for bad in (3, 5, 16, -1):
        with pytest.raises(spmm.SpmmError) as e:
            host_plan(csr, kslices=bad)
        assert e.value.status == spmm.SPMM_ERR_INVALID_ARG
    with pytest.raises(spmm.SpmmError) as e:     # only plans with chunks of 8 columns are cut
        host_plan(csr, kslices=4, ufk=16)
    assert e.value.status == spmm.SPMM_ERR_INVALID_ARG
    assert host_plan(csr, kslices=4, n_hint=16).describe()["k_slices"] == 1      # the hint's wider chunks win
    assert host_plan(csr, kslices=1).describe()["k_slices"] == 1
    assert host_plan(csr).describe()["k_slices"] == 1                            # a small matrix is never cut by itself
    info = host_plan(gen.csr_from_dense(np.ones((3, 5), np.float32)), kslices=8).describe()
    assert (info["k_slices"], info["slice_rows"], info["slice_cols"]) == (1, 3, 5)   # fewer than 8 columns


@pytest.mark.parametrize("K", [(1 << 24) - 1, 1 << 24, (1 << 24) + 1, (1 << 24) + 77])
@pytest.mark.parametrize("ufi", [1, 4])
def test_column_words_at_and_beyond_the_24_bit_boundary(K, ufi):
    """A column word keeps a slot pattern in its top byte only while every column index
    fits 24 bits (K <= 2^24); beyond that the word is all index and leftovers of different
    patterns never share a chunk.  Few entries, columns next to K - 1 and around 2^24,
    rows that share and do not share columns; the plan decodes to the canonical CSR bit
    for bit and its chunk arrays evaluate to the exact product."""
    rng = np.random.default_rng(K % 1000 + ufi)
    M = 11
    near = [K - 1, K - 2, K - 3, (1 << 24) - 1, (1 << 24) - 2, 0, 1, 5, (1 << 23) + 3]
    if K > (1 << 24):
        near += [1 << 24]
    near = sorted(set(c for c in near if 0 <= c < K))
    rows = []
    for i in range(M):
        take = [c for c in near if rng.random() < 0.6]
        extra = rng.integers(0, K, size=int(rng.integers(0, 12))).tolist()
        rows.append(np.array(sorted(set(take + extra)), dtype=np.int32))
    rows[4] = np.zeros(0, dtype=np.int32)
    row_ptr = np.concatenate(([0], np.cumsum([len(r) for r in rows]))).astype(np.int32)
    col_idx = np.concatenate(rows)
    vals = rng.integers(-8, 9, len(col_idx)).astype(np.float32)
    csr = gen.Csr(M, K, row_ptr, col_idx, vals)
    plan = host_plan(csr, ufi=ufi, group_nnz=16)
    info = plan.describe()
    assert info["ufi"] == ufi and info["nnz"] == len(col_idx)
    items, hdr, stream, wins = arrays(plan)
    rows_d, cc, bits = decode_plan(items, hdr, stream, wins, ufi, K=K)
    want_rows, want_cols, want_bits = canonical_csr(csr.row_ptr, csr.col_idx, csr.vals)
    assert sorted(zip(rows_d.tolist(), cc.tolist(), bits.tolist())) == \
        sorted(zip(want_rows.tolist(), want_cols.tolist(), want_bits.tolist()))
    assert int(cc.max()) == K - 1
    # which column words carry a slot pattern
    col_words = []
    for it in items.reshape(-1, 16):
        if not int(it[5]) & 2:
            for h, cw, _ in walk_chunks(it, hdr, stream, wins):
                col_words += [int(w) for w in cw[:(h >> 8) & 127]]
    tagged = [w for w in col_words if w >> 24]
    if K > (1 << 24):
        # all index: any top byte is part of a column number of 2^24 or more
        assert all(w < K for w in col_words) and all(w >= (1 << 24) for w in tagged)
        shared = [h for h in hdr[:info["n_chunks"]] if bin(int(h) & 255).count("1") > 1]
        if ufi == 1:
            assert not shared
    elif ufi > 1:
        assert tagged, "leftovers of different patterns share chunks and tag their slots"
        assert all((w & 0xFFFFFF) < K for w in col_words)
    B = np.zeros((K, 1), dtype=np.float32)
    touched = np.unique(col_idx)
    B[touched, 0] = rng.integers(-4, 5, len(touched)).astype(np.float32)
    C = interpret_plan(items, hdr, stream, wins, B, M, ufi, K=K)
    want = np.zeros((M, 1))
    for i in range(M):
        want[i, 0] = float(np.dot(vals[row_ptr[i]:row_ptr[i + 1]].astype(np.float64),
                                  B[col_idx[row_ptr[i]:row_ptr[i + 1]], 0].astype(np.float64)))
    assert np.array_equal(C.astype(np.float64), want)


@pytest.mark.parametrize("name", ["heavy_tail", "lognormal", "uniform_half", "all_empty"])
def test_plan_does_not_depend_on_the_number_of_inspector_threads(name):
    """The inspector enumerates contiguous ranges of groups on several threads for large
    inputs; the `threads` setting forces that on small ones.  Every array must come out the same."""
    csr = CASES[name]()
    plans = {}
    for threads in (1, 2, 5, 64):
        for ufi in (1, 4):
            plan = host_plan(csr, ufi=ufi, group_nnz=40, sort_rows=1, threads=threads)
            got = [plan.get_array(w) for w in range(5)] + [plan.get_groups()]
            want = plans.setdefault(ufi, got)
            assert all(np.array_equal(x, y) for x, y in zip(got, want)), (threads, ufi)


def test_plan_bytes_against_csr_bytes_trend():
    # Paper Section 4.4: the transformed format is smaller than CSR at moderate
    # sparsity (one index per merged column instead of one per nonzero) and larger
    # at extreme sparsity (metadata).  Here: 4 bytes per value slot and per column
    # slot and per chunk header of the staged stream.
    def ratio(sparsity):
        csr = gen.uniform_positions(512, 512, sparsity, 31)
        info = host_plan(csr, ufi=4, group_nnz=4096).describe()  # whole panels, as in the paper's format
        plan_bytes = 4 * info["stream_words"]
        csr_bytes = 8 * info["nnz"] + 4 * (csr.M + 1)
        return plan_bytes / csr_bytes
    assert ratio(0.5) < ratio(0.9) < ratio(0.99)
    assert ratio(0.5) < 1.0 < ratio(0.99)


def test_error_codes_of_the_boundary():
    ok_rp = np.array([0, 1, 2], dtype=np.int32)
    ci = np.array([0, 1], dtype=np.int32)
    v = np.ones(2, dtype=np.float32)

    def status(*args, **kw):
        try:
            spmm.plan_create(*args, host_only=True, **kw)
        except spmm.SpmmError as e:
            return e.status
        return 0

    assert status(2, 2, ok_rp, ci, v) == 0
    assert status(-1, 2, ok_rp, ci, v) == spmm.SPMM_ERR_INVALID_ARG
    assert status(2, -1, ok_rp, ci, v) == spmm.SPMM_ERR_INVALID_ARG
    assert status(2, 2 ** 31, ok_rp, ci, v) == spmm.SPMM_ERR_INVALID_ARG
    assert status(2, 2, np.array([1, 1, 2], np.int32), ci, v) == spmm.SPMM_ERR_INVALID_CSR
    assert status(2, 2, np.array([0, 2, 1], np.int32), ci, v) == spmm.SPMM_ERR_INVALID_CSR
    assert status(2, 2, ok_rp, np.array([0, 2], np.int32), v) == spmm.SPMM_ERR_INVALID_CSR
    assert status(2, 2, ok_rp, np.array([0, -1], np.int32), v) == spmm.SPMM_ERR_INVALID_CSR
    assert status(2, 2, ok_rp, ci, v, group_nnz=-5) == spmm.SPMM_ERR_INVALID_ARG
    assert status(2, 2, ok_rp, ci, v, ufi=3) == spmm.SPMM_ERR_INVALID_ARG
    lib = spmm.load()
    h = ctypes.c_void_p(123)
    assert lib.spmm_plan_create(ctypes.byref(h), 2, 2, None, None, None) == spmm.SPMM_ERR_INVALID_ARG
    assert h.value is None
    assert lib.spmm_plan_create(None, 2, 2, ok_rp.ctypes.data, ci.ctypes.data, v.ctypes.data) \
        == spmm.SPMM_ERR_INVALID_ARG
    assert lib.spmm_plan_destroy(None) == spmm.SPMM_OK
    assert lib.spmm_plan_describe(None, None) == spmm.SPMM_ERR_INVALID_ARG
    assert lib.spmm_execute(None, None, 32, None, None) == spmm.SPMM_ERR_INVALID_ARG
    # a host-only plan refuses to execute (there is no CPU path)
    plan = spmm.plan_create(2, 2, ok_rp, ci, v, host_only=True)
    assert lib.spmm_execute(plan.handle, None, 32, None, None) == spmm.SPMM_ERR_INVALID_ARG
    small = np.zeros(1, dtype=np.uint32)
    assert lib.spmm_plan_get_array(plan.handle, spmm.ARRAY_STREAM, small.ctypes.data, 1, None) \
        == spmm.SPMM_ERR_INVALID_ARG
    assert lib.spmm_plan_get_array(plan.handle, 9, None, 0, None) == spmm.SPMM_ERR_INVALID_ARG
    out = np.zeros(5, dtype=np.int32)
    assert lib.spmm_plan_get_groups(plan.handle, out.ctypes.data, 0) == spmm.SPMM_ERR_INVALID_ARG


def test_plan_is_deterministic():
    csr = CASES["heavy_tail"]()
    a = arrays(host_plan(csr, group_nnz=64))
    b = arrays(host_plan(csr, group_nnz=64))
    assert all(np.array_equal(x, y) for x, y in zip(a, b))
