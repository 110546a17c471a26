"""Pins of the CPU oracle to things other than itself (CPU only).

Each test names the fact it pins: the definition (paper, Section 3.1,
Listing 1) written as a dense triple loop, a hand-worked example, library
routines for the special cases, and algebraic invariants.  Shapes are
non-square and data asymmetric so that a transposed operand, a dropped term
or a wrong index fails at least one of them.
"""
import os

import numpy as np
import pytest
import scipy.sparse as sp

from workloads import generators as gen

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "worked_example.txt")


def _random_csr(rng, M, K, density, sort=True):
    dense = np.where(rng.random((M, K)) < density,
                     rng.standard_normal((M, K)), 0.0).astype(np.float32)
    csr = gen.csr_from_dense(dense)
    return dense, csr


def _dense_triple_loop(A, B):
    """Listing 1 verbatim in Python floats (double), i-k-j order."""
    M, K = A.shape
    N = B.shape[1]
    C = [[0.0] * N for _ in range(M)]
    for i in range(M):
        for k in range(K):
            if A[i][k] != 0:
                a = float(A[i][k])
                for j in range(N):
                    C[i][j] += a * float(B[k][j])
    return np.array(C, dtype=np.float64).reshape(M, N)


def _read_golden():
    mats = {}
    with open(GOLDEN) as f:
        lines = [ln.strip() for ln in f if ln.strip() and not ln.startswith("#")]
    i = 0
    while i < len(lines):
        name, r, c = lines[i].split()
        r, c = int(r), int(c)
        rows = [[float(x) for x in lines[i + 1 + t].split()] for t in range(r)]
        mats[name] = np.array(rows, dtype=np.float64).reshape(r, c)
        i += 1 + r
    return mats


def test_hand_worked_example(oracle):
    m = _read_golden()
    csr = gen.csr_from_dense(m["A"].astype(np.float32))
    C, S = oracle.spmm(csr.row_ptr, csr.col_idx, csr.vals,
                       m["B"].astype(np.float32))
    assert np.array_equal(C, m["C"])
    assert np.array_equal(S, m["S"])


@pytest.mark.parametrize("M,K,N,density,seed", [
    (7, 13, 5, 0.3, 1), (16, 9, 33, 0.5, 2), (1, 64, 3, 0.2, 3),
    (40, 24, 1, 0.4, 4), (12, 12, 12, 1.0, 5), (9, 17, 4, 0.0, 6)])
def test_bit_equal_to_dense_triple_loop(oracle, M, K, N, density, seed):
    rng = np.random.default_rng(seed)
    A, csr = _random_csr(rng, M, K, density)
    B = rng.standard_normal((K, N)).astype(np.float32)
    C, _ = oracle.spmm(csr.row_ptr, csr.col_idx, csr.vals, B)
    assert np.array_equal(C, _dense_triple_loop(A, B))


def test_matches_numpy_and_scipy_float64(oracle):
    rng = np.random.default_rng(11)
    A, csr = _random_csr(rng, 96, 160, 0.15)
    B = rng.standard_normal((160, 48)).astype(np.float32)
    C, S = oracle.spmm(csr.row_ptr, csr.col_idx, csr.vals, B)
    ref_np = A.astype(np.float64) @ B.astype(np.float64)
    ref_sp = sp.csr_matrix((csr.vals.astype(np.float64), csr.col_idx,
                            csr.row_ptr), shape=(96, 160)) @ B.astype(np.float64)
    tol = 1e-12 * S + 1e-300
    assert np.all(np.abs(C - ref_np) <= tol)
    assert np.all(np.abs(C - ref_sp) <= tol)
    ref_S = np.abs(A).astype(np.float64) @ np.abs(B).astype(np.float64)
    assert np.all(np.abs(S - ref_S) <= 1e-12 * ref_S + 1e-300)


def test_single_column_is_textbook_spmv(oracle):
    rng = np.random.default_rng(12)
    A, csr = _random_csr(rng, 50, 70, 0.2)
    x = rng.standard_normal((70, 1)).astype(np.float32)
    C, _ = oracle.spmm(csr.row_ptr, csr.col_idx, csr.vals, x)
    y = np.zeros(50)
    for i in range(50):
        for p in range(csr.row_ptr[i], csr.row_ptr[i + 1]):
            y[i] += float(csr.vals[p]) * float(x[csr.col_idx[p], 0])
    assert np.array_equal(C[:, 0], y)


def test_fully_dense_reduces_to_gemm(oracle):
    rng = np.random.default_rng(13)
    A = rng.integers(-4, 5, size=(10, 14)).astype(np.float32)
    A[A == 0] = 1.0
    B = rng.integers(-4, 5, size=(14, 6)).astype(np.float32)
    csr = gen.csr_from_dense(A)
    C, _ = oracle.spmm(csr.row_ptr, csr.col_idx, csr.vals, B)
    assert np.array_equal(C, (A.astype(np.int64) @ B.astype(np.int64)))


def test_identity_returns_B_bit_exact(oracle):
    rng = np.random.default_rng(14)
    n = 37
    csr = gen.csr_from_dense(np.eye(n, dtype=np.float32))
    B = rng.standard_normal((n, 9)).astype(np.float32)
    C, S = oracle.spmm(csr.row_ptr, csr.col_idx, csr.vals, B)
    assert np.array_equal(C, B.astype(np.float64))
    assert np.array_equal(S, np.abs(B).astype(np.float64))


def test_empty_rows_and_empty_matrix_give_exact_zeros(oracle):
    rng = np.random.default_rng(15)
    A, _ = _random_csr(rng, 20, 11, 0.4)
    A[[0, 7, 19]] = 0
    csr = gen.csr_from_dense(A)
    B = rng.standard_normal((11, 5)).astype(np.float32)
    C, S = oracle.spmm(csr.row_ptr, csr.col_idx, csr.vals, B)
    for r in (0, 7, 19):
        assert not C[r].any() and not S[r].any()
        assert not np.signbit(C[r]).any()
    csr0 = gen.csr_from_dense(np.zeros((6, 11), dtype=np.float32))
    C0, S0 = oracle.spmm(csr0.row_ptr, csr0.col_idx, csr0.vals, B)
    assert C0.shape == (6, 5) and not C0.any() and not S0.any()
    Cm, _ = oracle.spmm(np.zeros(1, np.int32), np.zeros(0, np.int32),
                        np.zeros(0, np.float32), B)
    assert Cm.shape == (0, 5)


def test_linearity_in_B_with_exact_integer_data(oracle):
    rng = np.random.default_rng(16)
    A = np.where(rng.random((18, 25)) < 0.3,
                 rng.integers(-8, 9, (18, 25)), 0).astype(np.float32)
    csr = gen.csr_from_dense(A)
    B1 = rng.integers(-16, 17, (25, 7)).astype(np.float32)
    B2 = rng.integers(-16, 17, (25, 7)).astype(np.float32)
    f = lambda B: oracle.spmm(csr.row_ptr, csr.col_idx, csr.vals, B)[0]
    assert np.array_equal(f(B1 + B2), f(B1) + f(B2))
    assert np.array_equal(f(4.0 * B1), 4.0 * f(B1))
    assert np.array_equal(f(B1 - 0.5 * B2), f(B1) - 0.5 * f(B2))


def test_power_of_two_scaling_of_A_is_exact(oracle):
    rng = np.random.default_rng(17)
    A, csr = _random_csr(rng, 15, 21, 0.35)
    B = rng.standard_normal((21, 6)).astype(np.float32)
    C, S = oracle.spmm(csr.row_ptr, csr.col_idx, csr.vals, B)
    C8, S8 = oracle.spmm(csr.row_ptr, csr.col_idx, csr.vals * np.float32(0.125), B)
    assert np.array_equal(C8, C * 0.125) and np.array_equal(S8, S * 0.125)


def test_within_row_column_permutation(oracle):
    rng = np.random.default_rng(18)
    A, csr = _random_csr(rng, 14, 40, 0.5)
    B = rng.standard_normal((40, 8)).astype(np.float32)
    col = csr.col_idx.copy()
    val = csr.vals.copy()
    for i in range(14):
        lo, hi = csr.row_ptr[i], csr.row_ptr[i + 1]
        perm = rng.permutation(hi - lo)
        col[lo:hi] = col[lo:hi][perm]
        val[lo:hi] = val[lo:hi][perm]
    C0, S = oracle.spmm(csr.row_ptr, csr.col_idx, csr.vals, B)
    C1, S1 = oracle.spmm(csr.row_ptr, col, val, B)
    assert np.all(np.abs(C0 - C1) <= 1e-12 * S)
    # with small-integer data every summation order is exact
    Ai = np.rint(4 * A)
    Ai[(A != 0) & (Ai == 0)] = 1.0
    Ai = Ai.astype(np.float32)
    Bi = np.rint(4 * B).astype(np.float32)
    csri = gen.csr_from_dense(Ai)
    assert np.array_equal(csri.row_ptr, csr.row_ptr)
    vali = csri.vals.copy()
    coli = csri.col_idx.copy()
    for i in range(14):
        lo, hi = csr.row_ptr[i], csr.row_ptr[i + 1]
        perm = rng.permutation(hi - lo)
        coli[lo:hi] = coli[lo:hi][perm]
        vali[lo:hi] = vali[lo:hi][perm]
    Ci0, _ = oracle.spmm(csri.row_ptr, csri.col_idx, csri.vals, Bi)
    Ci1, _ = oracle.spmm(csri.row_ptr, coli, vali, Bi)
    assert np.array_equal(Ci0, Ci1)


def test_duplicate_columns_are_summed_and_explicit_zeros_are_terms(oracle):
    row_ptr = np.array([0, 4, 5], dtype=np.int32)
    col_idx = np.array([2, 0, 2, 1, 1], dtype=np.int32)
    vals = np.array([1.5, -2.0, 0.25, 0.0, 3.0], dtype=np.float32)
    B = np.array([[1, 2], [3, 4], [5, 6]], dtype=np.float32)
    C, S = oracle.spmm(row_ptr, col_idx, vals, B)
    dense = np.array([[-2.0, 0.0, 1.75], [0.0, 3.0, 0.0]])
    assert np.array_equal(C, dense @ B.astype(np.float64))
    assert np.array_equal(S, np.abs(dense) @ np.abs(B).astype(np.float64))


def test_normaliser_is_the_product_of_absolute_values(oracle):
    rng = np.random.default_rng(19)
    A, csr = _random_csr(rng, 23, 31, 0.25)
    B = rng.standard_normal((31, 10)).astype(np.float32)
    _, S = oracle.spmm(csr.row_ptr, csr.col_idx, csr.vals, B)
    Cabs, _ = oracle.spmm(csr.row_ptr, csr.col_idx, np.abs(csr.vals), np.abs(B))
    assert np.array_equal(S, Cabs)


def test_openmp_build_is_bit_identical(oracle):
    csr = gen.tiny()
    B = gen.activations_for(csr, 32)
    C0, S0 = oracle.spmm(csr.row_ptr, csr.col_idx, csr.vals, B)
    C1, S1 = oracle.spmm(csr.row_ptr, csr.col_idx, csr.vals, B, parallel=True)
    assert np.array_equal(C0, C1) and np.array_equal(S0, S1)
    assert oracle.threads(False) == 1 and oracle.threads(True) >= 1


def test_malformed_csr_is_rejected(oracle):
    B = np.ones((3, 2), dtype=np.float32)
    with pytest.raises(ValueError):
        oracle.spmm(np.array([1, 2], np.int32), np.array([0], np.int32),
                    np.ones(1, np.float32), B)
    with pytest.raises(ValueError):
        oracle.spmm(np.array([0, 2, 1], np.int32), np.array([0, 1], np.int32),
                    np.ones(2, np.float32), B)
    with pytest.raises(ValueError):
        oracle.spmm(np.array([0, 1], np.int32), np.array([3], np.int32),
                    np.ones(1, np.float32), B)


def test_parity_metric(oracle):
    C_ref = np.array([[1.0, 0.0], [10.0, -4.0]])
    S = np.array([[2.0, 0.0], [10.0, 8.0]])
    ok = C_ref.copy()
    assert oracle.parity_error(ok, C_ref, S) == (0.0, 0)
    off = C_ref.copy()
    off[1, 1] += 8e-5
    err, bad = oracle.parity_error(off, C_ref, S)
    assert abs(err - 1e-5) < 1e-12 and bad == 0
    off[0, 1] = 1e-30
    assert oracle.parity_error(off, C_ref, S)[1] == 1
    off[0, 0] = np.nan
    assert oracle.parity_error(off, C_ref, S)[0] == float("inf")


def test_generators_are_seeded_and_sized():
    a, b = gen.tiny(), gen.tiny()
    assert a.row_ptr[-1] == 6554
    assert np.array_equal(a.col_idx, b.col_idx) and np.array_equal(a.vals, b.vals)
    c = gen.conv_layer()
    assert (c.M, c.K, int(c.row_ptr[-1])) == (512, 2048, 209715)
    f = gen.ffn(0, 3)
    assert (f.M, f.K) == (4096, 1024)
    lens = np.diff(f.row_ptr)
    assert 0.9 * 83886 < lens.sum() < 1.1 * 83886 and lens.max() > 2 * lens.mean()
    for csr in (a, c, f):
        for i in range(0, csr.M, 37):
            seg = csr.col_idx[csr.row_ptr[i]:csr.row_ptr[i + 1]]
            assert np.all(np.diff(seg) > 0) and (seg.size == 0 or seg.max() < csr.K)
    assert len(gen.sweep_entries()) == 48
