"""Test-side, independent re-derivations of what the inspector produces.

Nothing here is used by the product path.  `derive_groups` re-derives the row
groups from row_ptr and the constants the plan reports; `decode_plan` turns the
plan's chunk arrays back into (row, column, value-bits) triples; `interpret_plan`
evaluates the product from the chunk arrays the way the kernel consumes them.
"""
import numpy as np

MAX_UFI = 8
UFK = 8
ITEM_WORDS = 16
WIN_WORDS = 1024
LOOKAHEAD = 8
COL_PATTERN_SHIFT = 24
COL_INDEX_MASK = (1 << COL_PATTERN_SHIFT) - 1


WAVES_PER_WG = 8
FLAG_SPLIT, FLAG_IDLE, FLAG_SYNC, FLAG_CROSS = 1, 2, 4, 8
CROSS_SHARE = 1024
MAX_CROSS_PARTS = 64


def _groups_for(rp, M, ufi, group_nnz, group_panels, cross=True):
    whole, split = [], []          # split: list of panels, each a list of pieces
    cur = None
    cur_panels = 0
    P = (M + ufi - 1) // ufi
    # a panel heavier than this (and than the budget of eight groups) is cut across workgroups
    part_bound = max(WAVES_PER_WG * group_nnz, rp[M] // CROSS_SHARE)
    for p in range(P):
        r0, r1 = p * ufi, min(M, p * ufi + ufi)
        a, b = rp[r0], rp[r1]
        pn = b - a
        if pn > group_nnz:
            if cur is not None:
                whole.append(cur)
                cur = None
            want = min(WAVES_PER_WG, -(-pn // group_nnz))
            while want & (want - 1):
                want += 1
            want = max(want, ufi)      # a block holds 8 / ufi split panels
            across = cross and pn > part_bound
            if across:
                want = WAVES_PER_WG * min(MAX_CROSS_PARTS, -(-pn // part_bound))
            size = -(-pn // want)
            nseg = -(-pn // size)
            flag = FLAG_SPLIT | FLAG_CROSS if across else FLAG_SPLIT
            split.append([[r0, r1, a + s * size, min(b, a + (s + 1) * size), flag] for s in range(nseg)])
            continue
        if cur is not None and (cur[3] - cur[2] + pn > group_nnz or cur_panels == group_panels):
            whole.append(cur)
            cur = None
        if cur is None:
            cur = [r0, r1, a, b, 0]
            cur_panels = 0
        cur[1], cur[3] = r1, b
        cur_panels += 1
    if cur is not None:
        whole.append(cur)
    # split panels first, heaviest panel first; then whole-panel groups, heaviest
    # first; ties keep row order
    split.sort(key=lambda pieces: -(pieces[-1][3] - pieces[0][2]))
    whole.sort(key=lambda g: -(g[3] - g[2]))
    return split, whole


def _blocks_for(split, whole, ufi):
    blocks = -(-len(whole) // WAVES_PER_WG)
    used, panels = WAVES_PER_WG, WAVES_PER_WG // ufi
    for pieces in split:
        if pieces[0][4] & FLAG_CROSS:
            blocks += -(-len(pieces) // WAVES_PER_WG)       # blocks of their own, eight pieces each
            used, panels = WAVES_PER_WG, WAVES_PER_WG // ufi
            continue
        if used + len(pieces) > WAVES_PER_WG or panels == WAVES_PER_WG // ufi:
            blocks += 1
            used, panels = 0, 0
        used += len(pieces)
        panels += 1
    return blocks


def choose_ufi(M, K, nnz, n_hint=0):
    """The inspector's panel height as a function of the shape, the number of
    entries and the number of B columns the plan is meant for (0 = unknown)."""
    row = nnz // M if M else 0
    narrow, medium = 0 < n_hint <= 32, 32 < n_hint <= 64
    if K * (128 if narrow else 256 if medium else 512) > 4 << 20:
        # wide B run as 64-column tiles that still fit one L2
        wide_tiles = not narrow and not medium and K * 256 <= 4 << 20
        return 8 if (wide_tiles and M >= 4096 and row >= 1024) else 1
    shared = row * row // K if K else 0      # columns two rows of the mean length have in common
    if 0 < n_hint <= 16:                      # chunks of 32 or 64 columns
        need = 640 if n_hint <= 4 else 320 if n_hint <= 8 else 160
        if M >= 4096 and shared >= need:
            return 8
        if n_hint > 8:
            if M >= 2048:
                return 4 if (row >= 384 and 8 * row >= K) else 1
            if M >= 1024:
                return 2 if (row >= 256 and 3 * row >= K) else 1
        return 1
    if narrow:
        if M >= 4096:
            return 8 if row >= 768 else 4 if (row >= 384 and 8 * row >= K) else 1
        if M >= 2048:
            return 4 if (row >= 384 and 8 * row >= K) else 1
        if M >= 1024:
            return 2 if (row >= 256 and 3 * row >= K) else 1
        return 2 if (M >= 512 and row >= 256) else 1
    if medium:
        if M >= 4096:
            return 8 if (row >= 128 and shared >= 16) else 1
        if M >= 2048:
            return 4 if (row >= 256 and shared >= 32) else 1
        if M >= 1024:
            return 2 if shared >= 128 else 1
        return 2 if (M >= 512 and row >= 64) else 1
    if M >= 2048:
        return 8 if (row >= 128 and shared >= 16) else 1
    if M >= 1024:
        return 4 if row >= 128 else 2 if row >= 64 else 1
    return 2 if (M >= 512 and row >= 128) else 1


def skewed_rows(row_ptr):
    """True when the rows longer than four times the mean hold at least a quarter of
    the entries: the inspector then considers sorting the rows by length."""
    lens = np.diff(np.asarray(row_ptr, dtype=np.int64))
    M, nnz = len(lens), int(lens.sum())
    if M < 2 or nnz == 0:
        return False
    heavy = int(lens[lens * M > 4 * nnz].sum())
    return 4 * heavy >= nnz


def cross_allowed(row_ptr, setting=0, n_hint=0):
    """Whether panels may be cut across workgroups: the caller's setting, or skewed row
    lengths, at least 2^20 entries and no hint of 32 columns or fewer."""
    if setting != 0:
        return setting > 0
    return bool(skewed_rows(row_ptr)) and not 0 < n_hint <= 32 and int(row_ptr[-1]) >= 1 << 20


def choose_ufi_skewed(K, nnz, max_row, n_hint=0, cross=False):
    """Panel height for rows sorted by length: the largest power of two h <= 8 with
    h * (longest row) <= 2 * (nnz // 256); narrow B takes 2 where that gives 4 or 8,
    else 1; single rows when the tile of B exceeds one L2 (wide tiles narrow to 64
    columns first).  When panels may be cut across workgroups: 8 for wide, 4 for medium B."""
    narrow, medium = 0 < n_hint <= 32, 32 < n_hint <= 64
    l2 = 4 << 20
    tile_row_bytes = 128 if narrow else 256 if medium else 256 if K * 512 > l2 else 512
    if K * tile_row_bytes > l2:
        return 1
    if cross and not narrow:
        return 4 if medium else 8
    fair = max(1, nnz // 256)
    h = 1
    while h < MAX_UFI and 2 * h * max_row <= 2 * fair:
        h *= 2
    if narrow:
        return 2 if h >= 4 else 1
    return h


def choose_kslices(M, K, nnz, n_hint=0, setting=0, ufk=UFK):
    """Column ranges a plan is cut into (1 = not cut): the caller's setting (2, 4, 8; any
    other nonzero value = 1), else the smallest power of two whose share of a column tile
    of B (512 bytes per row, 256 for hints of 33 to 64 columns) takes at most half of a
    4 MiB L2, when the whole tile exceeds one L2, the matrix holds 2^20 entries or more and
    its rows at least 32 entries per range on average (a tile of exactly one L2: rows of
    1024 entries on average); plans with chunks wider than 8 are never cut."""
    if ufk != UFK or M <= 0 or K < 8 or (M + MAX_UFI) * 8 > 2**31 - 1:
        return 1
    if setting in (2, 4, 8):
        return setting
    if setting != 0:
        return 1
    tile_row_bytes = 256 if 32 < n_hint <= 64 else 512
    l2 = 4 << 20
    if K * tile_row_bytes < l2 or nnz < 1 << 20:
        return 1
    ns = 2
    while ns < 8 and -(-K // ns) * tile_row_bytes > l2 // 2:
        ns *= 2
    min_row = 32 * ns if K * tile_row_bytes > l2 else 1024       # a tile of exactly one L2: long rows only
    return ns if nnz >= min_row * M else 1


def sliced_row_ptr(row_ptr, col_idx, K, ns, order=None):
    """Row pointer of the rows of a plan cut into `ns` column ranges: range s of row i
    (of row order[i] when given) is plan row s * MS + i, MS = M rounded up to 8."""
    row_ptr = np.asarray(row_ptr, dtype=np.int64)
    M = len(row_ptr) - 1
    MS = -(-M // MAX_UFI) * MAX_UFI
    KS = -(-K // ns)
    lens = np.diff(row_ptr)
    rows = np.repeat(np.arange(M), lens)
    if order is not None:
        pos = np.empty(M, dtype=np.int64)
        pos[np.asarray(order)] = np.arange(M)
        rows = pos[rows]
    cnt = np.bincount((np.asarray(col_idx, dtype=np.int64) // KS) * MS + rows, minlength=ns * MS)
    return np.concatenate(([0], np.cumsum(cnt)))


def plan_schedule(row_ptr, col_idx, M, K, n_hint=0, ufi=0, sort_rows=0, cross=0, kslices=0, ufk=UFK):
    """(column ranges, panel height, rows sorted?, panels cut across workgroups allowed?) as
    the inspector decides them; `ufi`, `sort_rows`, `cross` and `kslices` are the caller's
    settings (0 = choose).  A plan cut along K chooses its height as for the columns of one
    range and the longest row of a range, and cuts panels across workgroups only where the
    tallest panels would otherwise be too heavy for one workgroup."""
    lens = np.diff(np.asarray(row_ptr, dtype=np.int64))
    nnz = int(lens.sum())
    ns = choose_kslices(M, K, nnz, n_hint, kslices, ufk)
    may_cross = cross_allowed(row_ptr, cross, n_hint)
    max_row = int(lens.max()) if M else 0
    KS = -(-K // ns)
    if ns > 1:
        rows = np.repeat(np.arange(M), lens)
        per = np.bincount(rows * ns + np.asarray(col_idx, dtype=np.int64) // KS, minlength=M * ns)
        max_row = int(per.max()) if len(per) else 0
        if cross == 0 and may_cross:
            if choose_ufi_skewed(KS, nnz, max_row, n_hint, False) >= (4 if 32 < n_hint <= 64 else 8):
                may_cross = False
    skewed = skewed_rows(row_ptr)
    if ufi not in (1, 2, 4, 8):
        as_sorted = sort_rows > 0 or (sort_rows == 0 and skewed)
        ufi = choose_ufi_skewed(KS, nnz, max_row, n_hint, may_cross) if as_sorted else choose_ufi(M, KS, nnz, n_hint)
    return ns, ufi, bool(sort_rows > 0 or (sort_rows == 0 and skewed and ufi > 1)), may_cross


def choose_schedule(row_ptr, M, K, n_hint=0, ufi=0, sort_rows=0, cross=0):
    """(panel height, rows sorted?) of a plan that is not cut along K."""
    lens = np.diff(np.asarray(row_ptr, dtype=np.int64))
    nnz = int(lens.sum())
    skewed = skewed_rows(row_ptr)
    if ufi not in (1, 2, 4, 8):
        as_sorted = sort_rows > 0 or (sort_rows == 0 and skewed)
        ufi = (choose_ufi_skewed(K, nnz, int(lens.max()) if M else 0, n_hint, cross_allowed(row_ptr, cross, n_hint))
               if as_sorted else choose_ufi(M, K, nnz, n_hint))
    return ufi, bool(sort_rows > 0 or (sort_rows == 0 and skewed and ufi > 1))


def sorted_row_order(row_ptr):
    """Rows by decreasing length, equal lengths in ascending row order; also the row
    pointer of that order."""
    lens = np.diff(np.asarray(row_ptr, dtype=np.int64))
    order = np.argsort(-lens, kind="stable")
    return order, np.concatenate(([0], np.cumsum(lens[order])))


def choose_group_budget(M, nnz, ufi, n_hint=0):
    """(nonzero budget, panel cap) of a row group for panels of `ufi` rows."""
    P = max(1, -(-M // ufi))
    mean = -(-nnz // P)
    waves = 4096 if 0 < n_hint <= 16 else 8192      # B of at most 16 columns: half as many waves
    ppt = min(8, -(-waves // P)) if P < waves // 2 else 1
    GP = min(16, max(1, -(-P // 8192)))
    g = -(-(5 * mean * GP) // (4 * ppt))
    if ufi == 1 and 1024 <= M < 2048 and 0 < n_hint <= 64:   # single rows of small matrices for narrow B: not cut below 128 entries
        g = max(g, min(-(-(5 * mean) // 8), 128))
    g = -(-g // 32) * 32
    return min(1024, max(32, g)), GP


def derive_groups(row_ptr, M, group_nnz, group_panels, ufi, cross=True):
    """(row groups in launch order as an (n, 5) int32 array, workgroups), from
    row_ptr only, for a given panel height, budget and panel cap."""
    rp = [int(x) for x in row_ptr]
    split, whole = _groups_for(rp, M, ufi, group_nnz, group_panels, cross)
    blocks = _blocks_for(split, whole, ufi)
    out = [piece for pieces in split for piece in pieces] + whole
    return np.array(out, dtype=np.int32).reshape(-1, 5), blocks


def derive_sliced_groups(plan_ptr, slice_rows, ns, group_nnz, group_panels, ufi, cross=True):
    """derive_groups for a plan cut into `ns` column ranges (plan_ptr from sliced_row_ptr):
    groups and blocks are formed range by range, and every range gets as many blocks as
    the one with the most (they are dealt to the ranges in turn)."""
    rp = [int(x) for x in plan_ptr]
    split, whole = _groups_for(rp, ns * slice_rows, ufi, group_nnz, group_panels, cross)
    out_split, out_whole, most = [], [], 0
    for sl in range(ns):
        sp = [pieces for pieces in split if pieces[0][0] // slice_rows == sl]
        wh = [g for g in whole if g[0] // slice_rows == sl]
        most = max(most, _blocks_for(sp, wh, ufi))
        out_split += [piece for pieces in sp for piece in pieces]
        out_whole += wh
    return np.array(out_split + out_whole, dtype=np.int32).reshape(-1, 5), most * ns


def undeal_blocks(items, ns):
    """The wave-slot table of a plan cut into `ns` ranges with its blocks back in the order
    they were formed: range by range (block b of the launch belongs to range b mod ns)."""
    blocks = np.asarray(items).reshape(-1, WAVES_PER_WG, ITEM_WORDS)
    assert len(blocks) % ns == 0
    return np.concatenate([blocks[sl::ns] for sl in range(ns)]).reshape(-1)


def canonical_csr(row_ptr, col_idx, vals):
    """Rows stably sorted by column; returns (rows, cols, value bits) arrays."""
    rows = np.repeat(np.arange(len(row_ptr) - 1), np.diff(row_ptr))
    order = np.lexsort((np.arange(len(col_idx)), col_idx, rows))
    return rows[order], np.asarray(col_idx)[order], np.asarray(vals, dtype=np.float32).view(np.uint32)[order]


def check_blocks(items, ufi, rowmap=None):
    """Structural invariants of the wave-slot table.  rowmap: the matrix row of every
    plan row when the plan's rows are sorted by length."""
    items = items.reshape(-1, WAVES_PER_WG, ITEM_WORDS)
    to_c = (lambda r: int(rowmap[r])) if rowmap is not None and len(rowmap) else (lambda r: r)
    expect = None      # (parts, first slot, next part, panel rows) of a panel cut across blocks
    slots_used = 0
    for blk in items:
        flags = blk[:, 5]
        crossing = (flags & FLAG_CROSS) != 0
        assert crossing.all() or not crossing.any(), "a panel cut across blocks fills its blocks alone"
        if crossing.any():
            nparts, slot0, part = (int(x) for x in blk[0, 13:16])
            assert np.all(blk[:, 13] == nparts) and np.all(blk[:, 14] == slot0) and np.all(blk[:, 15] == part)
            live = blk[(flags & FLAG_IDLE) == 0]
            assert len(live) >= 1 and len(set(live[:, 0])) == 1 and len(set(live[:, 1])) == 1
            rows = (int(live[0, 0]), int(live[0, 1]))
            if expect is None:
                assert part == 0 and nparts >= 2 and slot0 == slots_used
                expect = [nparts, slot0, 0, rows]
            assert [nparts, slot0, part, rows] == expect
            assert len(live) == WAVES_PER_WG or part == nparts - 1, "only the last block may be short"
            expect[2] += 1
            if expect[2] == nparts:
                slots_used += nparts
                expect = None
        else:
            assert expect is None, "the blocks of a panel cut across blocks are adjacent"
            assert not blk[:, 13:16].any()
        sync = (flags & FLAG_SYNC) != 0
        assert sync.all() or not sync.any(), "the barrier flag is a property of the block"
        idle = (flags & FLAG_IDLE) != 0
        assert np.all(blk[idle, 3] == 0) and np.all(blk[~idle, 3] >= 1)
        is_split = (flags & FLAG_SPLIT) != 0
        if not sync.any():
            assert not is_split.any() and not blk[:, 6].any()
            continue
        assert not (is_split & idle).any() and (not crossing.any() or sync.all())
        assert np.all(is_split | idle), "blocks with split panels hold nothing else"
        # every split panel of the block has one adding wave per row, covering
        # exactly the slots of its pieces
        slots = np.flatnonzero(is_split)
        covered = np.zeros(WAVES_PER_WG, dtype=int)
        rows_written = set()
        for w in range(WAVES_PER_WG):
            nseg, slot0, r, crow = (int(x) for x in blk[w, 6:10])
            if nseg == 0:
                continue
            pieces = blk[slot0:slot0 + nseg]
            assert np.all((pieces[:, 5] & FLAG_SPLIT) != 0)
            assert len(set(pieces[:, 0])) == 1 and len(set(pieces[:, 1])) == 1
            assert crow == to_c(int(pieces[0, 0]) + r) and r < int(pieces[0, 1])
            assert crow not in rows_written
            rows_written.add(crow)
            if r == 0:
                covered[slot0:slot0 + nseg] += 1
        assert np.all(covered[slots] == 1) and covered.sum() == len(slots)
        for w in slots:
            for r in range(int(blk[w, 1])):
                assert to_c(int(blk[w, 0]) + r) in rows_written
    assert expect is None
    return slots_used


def win_words(ufk):
    return 2048 if ufk >= 32 else WIN_WORDS


def lookahead(ufk):
    return 4 if ufk > 8 else LOOKAHEAD


def walk_chunks(it, hdr, stream, wins, ufk=UFK):
    """Yields (header word, column slots, [value block per set row]) for every chunk
    of one wave slot, following the windows and checking the window table and the
    host-side header copy.  ufk: columns per chunk of the plan."""
    UFK = ufk
    WIN_WORDS, LOOKAHEAD = win_words(ufk), lookahead(ufk)
    row0, nrows, chunk0, nchunks, stream0, flags = (int(x) for x in it[:6])
    win0, nwins = int(it[10]), int(it[11])
    assert int(it[12]) == (int(wins[win0]) if nwins else 0), "descriptor's copy of the first window entry"
    at = stream0
    c = chunk0
    for w in range(win0, win0 + nwins):
        wc, ww = int(wins[w]) & 0xFFFF, int(wins[w]) >> 16
        assert 1 <= wc and ww <= WIN_WORDS and ww % 8 == 0
        assert -(-wc // 8) * 8 + (wc + LOOKAHEAD) * UFK <= WIN_WORDS, "look-ahead column reads leave the window"
        hdr_words = -(-wc // 8) * 8
        assert not stream[at + wc:at + hdr_words].any()
        cols_at = at + hdr_words
        vals_at = cols_at + wc * UFK
        for k in range(wc):
            h = int(stream[at + k])
            assert h == int(hdr[c]), "window header differs from the header list"
            pc = bin(h & 255).count("1")
            cc = stream[cols_at + k * UFK:cols_at + (k + 1) * UFK]
            blocks = [stream[vals_at + UFK * t:vals_at + UFK * (t + 1)] for t in range(pc)]
            yield h, cc, blocks
            vals_at += UFK * pc
            c += 1
        assert vals_at - at == ww, "window table disagrees with the window's content"
        at += ww
    assert c == chunk0 + nchunks


def decode_plan(items, hdr, stream, wins, ufi, rowmap=None, K=0, ufk=UFK):
    """Chunk arrays -> (row, col, value bits) arrays in the order the kernel
    consumes them.  Also checks the structural invariants of the format and
    raises AssertionError on any violation.  K: columns of the matrix; beyond 2^24
    columns a column word is all index (no slot pattern in its top byte)."""
    check_blocks(items, ufi, rowmap)
    wide_cols = K > (1 << COL_PATTERN_SHIFT)
    index_mask = 0xFFFFFFFF if wide_cols else COL_INDEX_MASK
    UFK = ufk
    to_c = (lambda r: int(rowmap[r])) if rowmap is not None and len(rowmap) else (lambda r: r)
    items = items.reshape(-1, ITEM_WORDS)
    out_rows, out_cols, out_bits = [], [], []
    for it in items:
        row0, nrows, chunk0, nchunks, stream0, flags = (int(x) for x in it[:6])
        if flags & FLAG_IDLE:
            assert int(it[11]) == 0
            continue
        row = row0
        rows_left = nrows
        for h, cc, blocks in walk_chunks(it, hdr, stream, wins, ufk):
            pattern, count, end = h & 255, (h >> 8) & 127, (h >> 15) & 1
            assert h >> 16 == 0 and count <= UFK
            assert (count == 0) == (pattern == 0)
            if count == 0:
                assert end, "an empty chunk is the only chunk of an empty panel"
            assert rows_left > 0, "chunks after the last panel of the group"
            rows_here = min(ufi, rows_left)
            assert pattern < (1 << rows_here), "pattern names a row beyond the panel"
            # a slot's own pattern: the top byte of its column word, or the chunk's
            own = [pattern if wide_cols else (int(cc[u]) >> COL_PATTERN_SHIFT) or pattern for u in range(count)]
            union = 0
            for u in range(count):
                assert own[u] & ~pattern == 0 and own[u] != 0, "a slot's pattern lies inside the chunk's"
                assert wide_cols or (int(cc[u]) >> COL_PATTERN_SHIFT) != pattern, "a full slot pattern is stored as 0"
                union |= own[u]
            assert union == pattern, "the chunk's pattern is the union of its slots'"
            if count:
                assert np.all((cc[count:] & index_mask) == (cc[count - 1] & index_mask)), \
                    "unused slots repeat the last real column"
            t = 0
            for r in range(ufi):
                if not (pattern >> r) & 1:
                    continue
                block = blocks[t]
                t += 1
                assert not block[count:].any(), "unused value slots must be zero"
                for u in range(count):
                    if (own[u] >> r) & 1:
                        out_rows.append(to_c(row + r))
                        out_cols.append(int(cc[u]) & index_mask)
                        out_bits.append(int(block[u]))
                    else:
                        assert block[u] == 0, "a slot without the row holds a zero there"
            if end:
                row += rows_here
                rows_left -= rows_here
        assert rows_left == 0
        if flags & FLAG_SPLIT:
            assert nrows <= ufi
    return (np.array(out_rows, dtype=np.int64), np.array(out_cols, dtype=np.int64),
            np.array(out_bits, dtype=np.uint32))


def interpret_plan(items, hdr, stream, wins, B, M, ufi, rowmap=None, K=0, ufk=UFK):
    """Evaluates C from the chunk arrays in float32, block by block, chunk by
    chunk, FMA by FMA (row blocks in ascending row, slots in ascending order;
    pieces of a split panel added in slot order by the wave slot the table names).
    The kernel's slices add the same terms in a different order."""
    blocks = items.reshape(-1, WAVES_PER_WG, ITEM_WORDS)
    to_c = (lambda r: int(rowmap[r])) if rowmap is not None and len(rowmap) else (lambda r: r)
    N = B.shape[1]
    C = np.full((M, N), np.nan, dtype=np.float32)
    B64 = B.astype(np.float64)
    index_mask = 0xFFFFFFFF if K > (1 << COL_PATTERN_SHIFT) else COL_INDEX_MASK
    parked = {}     # scratch slot -> sums of one block of a panel cut across blocks, per tile row
    for blk in blocks:
        tiles = np.zeros((WAVES_PER_WG, ufi, N), dtype=np.float32)
        for w, it in enumerate(blk):
            row0, nrows, chunk0, nchunks, stream0, flags = (int(x) for x in it[:6])
            if flags & FLAG_IDLE:
                continue
            acc = np.zeros((ufi, N), dtype=np.float32)
            row, rows_left = row0, nrows
            for h, cc, vblocks in walk_chunks(it, hdr, stream, wins, ufk):
                pattern, end = h & 255, (h >> 15) & 1
                t = 0
                for r in range(ufi):
                    if not (pattern >> r) & 1:
                        continue
                    fv = vblocks[t].view(np.float32)
                    t += 1
                    for u in range(ufk):
                        a = np.float64(fv[u])
                        # fused multiply-add: exact product and sum in double, one rounding
                        acc[r] = (a * B64[int(cc[u]) & index_mask] + acc[r].astype(np.float64)).astype(np.float32)
                if end:
                    rows_here = min(ufi, rows_left)
                    if flags & FLAG_SPLIT:
                        tiles[w] = acc
                    else:
                        for r in range(rows_here):
                            C[to_c(row + r)] = acc[r]
                    row += rows_here
                    rows_left -= rows_here
                    acc[:] = 0
        for it in blk:
            nseg, slot0, r, crow = (int(x) for x in it[6:10])
            if int(it[5]) & FLAG_SYNC and nseg:
                total = np.zeros(N, dtype=np.float32)
                for p in range(nseg):
                    total = total + tiles[slot0 + p, r]
                if not int(it[5]) & FLAG_CROSS:
                    C[crow] = total
                    continue
                # the block parks its sums; the second launch adds the blocks' sums in block order
                nparts, xslot0, part = (int(x) for x in it[13:16])
                parked[(xslot0 + part, r)] = total
                if part == nparts - 1:
                    final = np.zeros(N, dtype=np.float32)
                    for q in range(nparts):
                        final = final + parked[(xslot0 + q, r)]
                    C[crow] = final
    return C
