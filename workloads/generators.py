"""Seeded synthetic inputs shared by the tests, the oracle-side checks and the
HIP-side checks.  This module holds no arithmetic of the method: it only draws
sparse weight matrices (as CSR) and dense activations.

The matrices stand in for the pruned ResNet-50 / Transformer weights of the
paper's evaluation (Section 4.1 "Dataset"): unstructured element-wise sparsity
of 50 % and more, 1x1-convolution and feed-forward shapes, fp32 values, dense
right-hand sides with 32, 64 or 128 columns (Table 1).  Every generator is a
pure function of its arguments and its seed (numpy ``PCG64``).

CSR convention: ``row_ptr`` int32 of length M+1, ``col_idx`` int32 sorted
ascending inside each row, ``vals`` float32.
"""
from collections import namedtuple

import numpy as np

Csr = namedtuple("Csr", "M K row_ptr col_idx vals")


def _rng(seed):
    return np.random.Generator(np.random.PCG64(int(seed)))


def csr_from_dense(W):
    """CSR of the nonzero entries of a dense matrix (row-major scan order)."""
    W = np.asarray(W, dtype=np.float32)
    M, K = W.shape
    mask = W != 0
    counts = mask.sum(axis=1)
    row_ptr = np.zeros(M + 1, dtype=np.int64)
    np.cumsum(counts, out=row_ptr[1:])
    rows, cols = np.nonzero(mask)
    del rows
    return Csr(M, K, row_ptr.astype(np.int32), cols.astype(np.int32),
               W[mask].astype(np.float32))


def csr_from_row_columns(M, K, row_cols, vals):
    """CSR from a per-row list of sorted column arrays and a flat value array."""
    counts = np.array([len(c) for c in row_cols], dtype=np.int64)
    row_ptr = np.zeros(M + 1, dtype=np.int64)
    np.cumsum(counts, out=row_ptr[1:])
    col_idx = (np.concatenate(row_cols).astype(np.int32) if row_ptr[-1] > 0
               else np.zeros(0, dtype=np.int32))
    return Csr(M, K, row_ptr.astype(np.int32), col_idx,
               np.asarray(vals, dtype=np.float32))


def dense_activations(K, N, seed):
    """B: K x N, N(0, 1), float32, row-major."""
    return _rng(seed).standard_normal((K, N), dtype=np.float32)


def uniform_positions(M, K, sparsity, seed):
    """Exactly round((1 - sparsity) M K) nonzeros at uniformly random positions
    (drawn without replacement), values N(0, 1)."""
    rng = _rng(seed)
    nnz = int(round((1.0 - sparsity) * M * K))
    flat = np.sort(rng.permutation(M * K)[:nnz])
    rows = flat // K
    cols = flat % K
    row_ptr = np.zeros(M + 1, dtype=np.int64)
    np.add.at(row_ptr, rows + 1, 1)
    np.cumsum(row_ptr, out=row_ptr)
    vals = rng.standard_normal(nnz, dtype=np.float32)
    return Csr(M, K, row_ptr.astype(np.int32), cols.astype(np.int32), vals)


def magnitude_pruned(M, K, sparsity, seed):
    """Global magnitude pruning of a dense N(0, 1) matrix: keep exactly the
    round((1 - sparsity) M K) entries of largest |w| (ties at the threshold
    are resolved towards the lower row-major position)."""
    rng = _rng(seed)
    W = rng.standard_normal((M, K), dtype=np.float32)
    keep = int(round((1.0 - sparsity) * M * K))
    if keep <= 0:
        W[:] = 0
    elif keep < M * K:
        absw = np.abs(W).ravel()
        thresh = np.partition(absw, M * K - keep)[M * K - keep]
        above = absw > thresh
        # float32 draws can tie at the threshold: keep the first ties in
        # row-major order until the count is exact.
        ties = np.flatnonzero(absw == thresh)
        need = keep - int(np.count_nonzero(above))
        above[ties[:need]] = True
        W.ravel()[~above] = 0
    return csr_from_dense(W)


def lognormal_rows(M, K, sparsity, seed, sigma=0.5, std=0.02):
    """Feed-forward-layer stand-in with skewed row lengths: the density of row
    i is d * exp(sigma z_i - sigma^2 / 2) clipped to [0, 1] (mean-preserving
    lognormal around the target density d), columns uniform without
    replacement inside the row, values N(0, std)."""
    rng = _rng(seed)
    d = 1.0 - sparsity
    z = rng.standard_normal(M)
    dens = np.clip(d * np.exp(sigma * z - 0.5 * sigma * sigma), 0.0, 1.0)
    counts = np.rint(dens * K).astype(np.int64)
    row_cols = [np.sort(rng.permutation(K)[:c]) for c in counts]
    vals = (rng.standard_normal(int(counts.sum())) * std).astype(np.float32)
    return csr_from_row_columns(M, K, row_cols, vals)


def zipf_rows(M, K, mean_sparsity, seed, exponent=1.5, empty_fraction=0.05):
    """Load-balance stress: round(empty_fraction M) empty rows; the other rows
    have lengths proportional to Zipf(exponent) draws capped at K, rescaled (at
    most 8 passes) so the total is within 1 % of (1 - mean_sparsity) M K; rows
    in random order; columns uniform without replacement; values N(0, 1)."""
    rng = _rng(seed)
    n_empty = int(round(empty_fraction * M))
    order = rng.permutation(M)
    live = order[n_empty:]
    z = np.minimum(rng.zipf(exponent, size=live.shape[0]), K).astype(np.float64)
    target = (1.0 - mean_sparsity) * M * K
    s = target / z.sum()
    for _ in range(8):
        counts_live = np.clip(np.rint(s * z), 1, K)
        total = counts_live.sum()
        if abs(total - target) <= 0.01 * target:
            break
        s *= target / total
    counts = np.zeros(M, dtype=np.int64)
    counts[live] = counts_live.astype(np.int64)
    row_cols = [np.sort(rng.permutation(K)[:c]) if c < K else np.arange(K)
                for c in counts]
    vals = rng.standard_normal(int(counts.sum()), dtype=np.float32)
    return csr_from_row_columns(M, K, row_cols, vals)


# ---------------------------------------------------------------------------
# The five named configurations
# ---------------------------------------------------------------------------

SWEEP_SHAPES = ((256, 256), (1024, 1024), (4096, 4096), (8192, 8192),
                (1024, 256), (256, 1024), (4096, 1024), (1024, 4096))
SWEEP_SPARSITIES = (0.50, 0.70, 0.80, 0.90, 0.95, 0.98)
BCOLS = (32, 64, 128)


def config_seed(config_index, running_index):
    return 1000 * int(config_index) + int(running_index)


def tiny():
    """Configuration 0: 256 x 256 at 90 %, uniform positions; N = 32."""
    return uniform_positions(256, 256, 0.90, config_seed(0, 0))


def conv_layer():
    """Configuration 1: 512 x 2048 1x1-convolution weight at 80 %."""
    return magnitude_pruned(512, 2048, 0.80, config_seed(1, 0))


FFN_SHAPES = ((4096, 1024), (1024, 4096))
FFN_SPARSITIES = (0.70, 0.90, 0.95, 0.98)


def ffn(shape_index, sparsity_index):
    """Configuration 2: feed-forward weights with lognormal row densities."""
    M, K = FFN_SHAPES[shape_index]
    sp = FFN_SPARSITIES[sparsity_index]
    return lognormal_rows(M, K, sp,
                          config_seed(2, 4 * shape_index + sparsity_index))


def stress():
    """Configuration 3: 16384 x 16384, Zipf rows, 95 % mean sparsity."""
    return zipf_rows(16384, 16384, 0.95, config_seed(3, 0))


def sweep_entries():
    """Configuration 4: the 48 (shape, sparsity) pairs with their seeds."""
    out = []
    for si, (M, K) in enumerate(SWEEP_SHAPES):
        for pi, sp in enumerate(SWEEP_SPARSITIES):
            out.append(dict(index=len(out), M=M, K=K, sparsity=sp,
                            seed=config_seed(4, len(out))))
    return out


def sweep_matrix(entry):
    return magnitude_pruned(entry["M"], entry["K"], entry["sparsity"],
                            entry["seed"])


def activations_for(csr, N, seed_offset=0):
    """The dense right-hand side paired with a matrix (seed derived from its
    shape so that every consumer sees the same bytes)."""
    return dense_activations(csr.K, N, 7919 * csr.K + 31 * N + 17 + seed_offset)


def row_stats(csr):
    """Achieved nnz, mean / max row length and the Gini coefficient of the row
    lengths (reported with every measurement)."""
    lens = np.diff(csr.row_ptr.astype(np.int64))
    nnz = int(lens.sum())
    if csr.M == 0 or nnz == 0:
        return dict(nnz=nnz, mean_row=0.0, max_row=0, gini=0.0)
    srt = np.sort(lens)
    n = srt.shape[0]
    gini = float((2.0 * np.sum((np.arange(1, n + 1)) * srt) / (n * srt.sum()))
                 - (n + 1.0) / n)
    return dict(nnz=nnz, mean_row=float(lens.mean()), max_row=int(lens.max()),
                gini=gini)
