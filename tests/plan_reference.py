"""Test-side, independent re-derivations of what the inspector produces.

Nothing here is used by the product path.  `derive_groups` re-derives the row
groups from row_ptr and the constants the plan reports; `decode_plan` turns the
plan's chunk arrays back into (row, column, value-bits) triples; `interpret_plan`
evaluates the product from the chunk arrays the way the kernel consumes them.
"""
import numpy as np

UFI = 4
UFK = 8
ITEM_WORDS = 16


def derive_groups(row_ptr, M, group_nnz, group_panels):
    """Row groups in launch order as an (n, 5) int32 array, from row_ptr only."""
    rp = [int(x) for x in row_ptr]
    groups = []
    cur = None
    cur_panels = 0
    P = (M + UFI - 1) // UFI
    for p in range(P):
        r0, r1 = p * UFI, min(M, p * UFI + UFI)
        a, b = rp[r0], rp[r1]
        pn = b - a
        if pn > group_nnz:
            if cur is not None:
                groups.append(cur)
                cur = None
            nseg = -(-pn // group_nnz)
            for s in range(nseg):
                groups.append([r0, r1, a + s * group_nnz, min(b, a + (s + 1) * group_nnz), 1])
            continue
        if cur is not None and (cur[3] - cur[2] + pn > group_nnz or cur_panels == group_panels):
            groups.append(cur)
            cur = None
        if cur is None:
            cur = [r0, r1, a, b, 0]
            cur_panels = 0
        cur[1], cur[3] = r1, b
        cur_panels += 1
    if cur is not None:
        groups.append(cur)
    # heaviest first, ties in creation order
    order = sorted(range(len(groups)), key=lambda i: (-(groups[i][3] - groups[i][2]), i))
    return np.array([groups[i] for i in order], dtype=np.int32).reshape(-1, 5)


def canonical_csr(row_ptr, col_idx, vals):
    """Rows stably sorted by column; returns (rows, cols, value bits) arrays."""
    rows = np.repeat(np.arange(len(row_ptr) - 1), np.diff(row_ptr))
    order = np.lexsort((np.arange(len(col_idx)), col_idx, rows))
    return rows[order], np.asarray(col_idx)[order], np.asarray(vals, dtype=np.float32).view(np.uint32)[order]


def decode_plan(items, hdr, cols, vals):
    """Chunk arrays -> list of (row, col, value bits, group index, position) in the
    order the kernel consumes them.  Also checks the structural invariants of the
    format and raises AssertionError on any violation."""
    items = items.reshape(-1, ITEM_WORDS)
    out_rows, out_cols, out_bits = [], [], []
    for gi, it in enumerate(items):
        row0, nrows, chunk0, nchunks, vals0, flags = (int(x) for x in it[:6])
        assert nchunks >= 1
        v = vals0
        row = row0
        rows_left = nrows
        for c in range(chunk0, chunk0 + nchunks):
            h = int(hdr[c])
            pattern, count, end = h & 15, (h >> 4) & 15, (h >> 8) & 1
            assert h >> 9 == 0 and count <= UFK
            assert (count == 0) == (pattern == 0)
            if count == 0:
                assert end, "an empty chunk is the only chunk of an empty panel"
            assert rows_left > 0, "chunks after the last panel of the group"
            rows_here = min(UFI, rows_left)
            assert pattern < (1 << rows_here), "pattern names a row beyond the panel"
            cc = cols[c * UFK:(c + 1) * UFK]
            if count:
                assert np.all(cc[count:] == cc[count - 1]), "unused slots repeat the last real column"
            for r in range(UFI):
                if not (pattern >> r) & 1:
                    continue
                block = vals[v:v + UFK]
                assert not block[count:].any(), "unused value slots must be zero"
                for u in range(count):
                    out_rows.append(row + r)
                    out_cols.append(int(cc[u]))
                    out_bits.append(int(block[u]))
                v += UFK
            if end:
                row += rows_here
                rows_left -= rows_here
        assert rows_left == 0 or (flags & 1), "whole-panel groups end with their last panel"
        if flags & 1:
            assert nrows <= UFI and rows_left == 0
    return (np.array(out_rows, dtype=np.int64), np.array(out_cols, dtype=np.int64),
            np.array(out_bits, dtype=np.uint32))


def interpret_plan(items, hdr, cols, vals, B, M):
    """Evaluates C from the chunk arrays in float32, chunk by chunk, FMA by FMA in
    the kernel's order (row blocks in ascending row, slots in ascending order;
    pieces of a split panel summed in piece order)."""
    items = items.reshape(-1, ITEM_WORDS)
    N = B.shape[1]
    C = np.full((M, N), np.nan, dtype=np.float32)
    partial = {}
    fvals = vals.view(np.float32)
    B64 = B.astype(np.float64)
    for it in items:
        row0, nrows, chunk0, nchunks, vals0, flags, ticket, nseg, slot0, seg = (int(x) for x in it[:10])
        acc = np.zeros((UFI, N), dtype=np.float32)
        v = vals0
        row, rows_left = row0, nrows
        for c in range(chunk0, chunk0 + nchunks):
            h = int(hdr[c])
            pattern, end = h & 15, (h >> 8) & 1
            cc = cols[c * UFK:(c + 1) * UFK]
            for r in range(UFI):
                if not (pattern >> r) & 1:
                    continue
                for u in range(UFK):
                    a = np.float64(fvals[v + u])
                    # fused multiply-add in float32: exact product and sum in double, one rounding
                    acc[r] = (a * B64[cc[u]] + acc[r].astype(np.float64)).astype(np.float32)
                v += UFK
            if end:
                rows_here = min(UFI, rows_left)
                if flags & 1:
                    partial.setdefault(ticket, {})[seg] = (acc.copy(), row, rows_here, nseg)
                else:
                    C[row:row + rows_here] = acc[:rows_here]
                row += rows_here
                rows_left -= rows_here
                acc[:] = 0
    for ticket, pieces in partial.items():
        nseg = next(iter(pieces.values()))[3]
        assert sorted(pieces) == list(range(nseg))
        total = np.zeros((UFI, N), dtype=np.float32)
        for s in range(nseg):
            total = total + pieces[s][0]
        _, row, rows_here, _ = pieces[0]
        C[row:row + rows_here] = total[:rows_here]
    return C
