"""Pins for the reference row partition (integer definition of the analysis
pass; the per-row form of the vector-length estimate of Section 4.2)."""
import math
import os

import numpy as np
import pytest

import gen
import oracle


def test_constants():
    assert oracle._load().oracle_partition_num_bins(64) == oracle.NUM_BINS == 10
    assert oracle._load().oracle_partition_num_bins(32) == 9


def test_hand_worked_bins(golden_dir):
    pairs = [tuple(map(int, l.split())) for l in open(os.path.join(golden_dir, "partition_bins.txt"))
             if l.strip() and not l.startswith("#")]
    lengths = np.array([p[0] for p in pairs], dtype=np.int64)
    rowptr = np.zeros(lengths.size + 1, dtype=np.int32)
    np.cumsum(lengths, out=rowptr[1:])
    part = oracle.partition(rowptr)
    bin_of_row = np.empty(lengths.size, dtype=np.int64)
    for b in range(10):
        bin_of_row[part["row_perm"][part["bin_offset"][b]:part["bin_offset"][b + 1]]] = b
    assert bin_of_row.tolist() == [p[1] for p in pairs]


def _independent_partition(rowptr, wave, long_threshold, tile_nnz, stream_rows, stream_min_nnz):
    """The same definition through different primitives: reduceat, log2, stable argsort, searchsorted."""
    L = np.diff(rowptr).astype(np.int64)
    n = L.size
    starts = np.arange(0, n, stream_rows)
    ends = np.minimum(starts + stream_rows, n)
    chunk_max = np.maximum.reduceat(L, starts) if n else np.zeros(0, dtype=np.int64)
    chunk_nnz = rowptr[ends].astype(np.int64) - rowptr[starts]
    ratio = np.maximum(chunk_max, 1) / stream_rows
    cls = np.clip(np.ceil(np.log2(np.maximum(ratio, 1e-9))).astype(np.int64), 1, None)   # 2^k * rows >= max
    fit = np.clip(np.ceil(np.log2(np.maximum(chunk_nnz, 1) / (16.0 * stream_rows))).astype(np.int64), 1, None)
    cls = np.where((cls <= 4) & (fit <= 4), np.maximum(cls, fit), cls)                    # entries <= 2^k * 16 * rows
    cls[(cls > 4) | (chunk_nnz < stream_min_nnz)] = 0
    is_stream = cls > 0
    order = np.argsort(np.where(is_stream, cls, 99), kind="stable")
    stream_chunks = order[:is_stream.sum()].astype(np.int32)
    stream_offset = np.concatenate([[0], np.cumsum(np.bincount(cls, minlength=5)[1:5])]).astype(np.int32)
    binned = np.flatnonzero(~np.repeat(is_stream, ends - starts))
    top = int(math.log2(wave)) + 1
    Lb = L[binned]
    b = np.zeros(Lb.size, dtype=np.int64)
    pos = Lb > 0
    b[pos] = 1 + np.ceil(np.log2(Lb[pos])).astype(np.int64)
    b[Lb > wave] = top + 1
    b[Lb > long_threshold] = top + 2
    nb = top + 3
    perm = binned[np.argsort(b, kind="stable")].astype(np.int32)
    off = np.concatenate([[0], np.cumsum(np.bincount(b, minlength=nb))]).astype(np.int32)
    long_rows = perm[off[nb - 1]:]
    lp = np.concatenate([[0], np.cumsum(L[long_rows])]).astype(np.int64)
    T = -(-int(lp[-1]) // tile_nnz)
    tstarts = np.arange(T, dtype=np.int64) * tile_nnz
    tr = np.searchsorted(lp, tstarts, side="right") - 1
    tn = tstarts - lp[tr]
    return stream_chunks, stream_offset, off, perm, lp, np.append(tr, long_rows.size), np.append(tn, 0)


@pytest.mark.parametrize("wave,lt,tile,srows,smin", [(64, 4096, 4096, 32, 256), (64, 100, 64, 32, 256),
                                                      (32, 40, 16, 8, 20), (64, 64, 7, 16, 1), (64, 4096, 4096, 32, 0)])
@pytest.mark.parametrize("seed", [1, 2])
def test_partition_matches_independent_construction(wave, lt, tile, srows, smin, seed):
    n = 3001
    u = gen.uniform(seed, 0, n, 0.0, 1.0)
    L = np.floor(np.exp(u * u * 9.5)).astype(np.int64) - 1      # 0 .. ~13000, mostly short
    L[1000:2000] = np.minimum(L[1000:2000], wave)                 # a stretch without long rows
    L[1200:1300] = 0                                               # ... part of it empty
    L[::97] = 0
    L[5::211] = wave
    L[7::223] = lt
    L[9::227] = lt + 1
    rowptr = np.zeros(n + 1, dtype=np.int32)
    np.cumsum(L, out=rowptr[1:])
    part = oracle.partition(rowptr, wave, lt, tile, srows, smin)
    sc, so, off, perm, lp, tr, tn = _independent_partition(rowptr, wave, lt, tile, srows, smin)
    assert sc.size > 0 and perm.size > 0
    assert np.array_equal(part["stream_chunks"], sc)
    assert np.array_equal(part["stream_offset"], so)
    assert np.array_equal(part["bin_offset"], off)
    assert np.array_equal(part["row_perm"], perm)
    assert np.array_equal(part["long_off"], lp)
    assert np.array_equal(part["tile_row"], tr)
    assert np.array_equal(part["tile_nz"], tn)


def test_stream_chunks_hand_worked():
    """Chunks of 32 rows; class k = smallest k with max row length <= 2^k * 32 and entries <=
    2^k * 512 (k <= 4; the length alone if no k fits the entries), class 0 (binned) when the chunk
    holds fewer than 256 entries or a row exceeds 512 entries."""
    L = np.array([8] * 32            # chunk 0: 256 entries, max 8                -> class 1
                 + [8] * 31 + [65]   # chunk 1: max 65                            -> class 2
                 + [7] * 32          # chunk 2: 224 entries, below the minimum    -> binned
                 + [64] * 32         # chunk 3: rows at 64, 2048 entries > 2*512  -> class 2
                 + [0] * 31 + [64]   # chunk 4: 64 entries                        -> binned
                 + [128] * 2 + [1] * 30   # chunk 5: max 128                      -> class 2
                 + [129] + [5] * 31  # chunk 6: max 129 (284 entries)             -> class 3
                 + [512] + [0] * 31  # chunk 7: max 512                           -> class 4
                 + [513] + [9] * 31  # chunk 8: a row above 512                   -> binned
                 + [40] * 7,         # chunk 9 (ragged, 7 rows): 280 entries      -> class 1
                 dtype=np.int64)
    rowptr = np.zeros(L.size + 1, dtype=np.int32)
    np.cumsum(L, out=rowptr[1:])
    part = oracle.partition(rowptr)
    assert part["stream_chunks"].tolist() == [0, 9, 1, 3, 5, 6, 7]
    assert part["stream_offset"].tolist() == [0, 2, 5, 6, 7]
    # 32 rows of 300 entries: by length class 4 (300 <= 512); 9600 entries fit no 2^k * 512 -> stays 4
    rp = np.arange(33, dtype=np.int32) * 300
    assert oracle.partition(rp)["stream_offset"].tolist() == [0, 0, 0, 0, 1]
    # 32 rows of 81 entries (2592 entries): by length class 2, by entries class 3
    rp = np.arange(33, dtype=np.int32) * 81
    assert oracle.partition(rp)["stream_offset"].tolist() == [0, 0, 0, 1, 1]
    binned = list(range(64, 96)) + list(range(128, 160)) + list(range(256, 288))
    assert sorted(part["row_perm"].tolist()) == binned
    # bins: 31 empty rows; 32 rows of 7 (bin 4); 31 rows of 9 (bin 5); one row of 64 (bin 7); one of 513 (bin 8)
    assert np.diff(part["bin_offset"]).tolist() == [31, 0, 0, 0, 32, 31, 0, 1, 1, 0]
    # with 6 rows in the ragged chunk: 240 entries -> binned
    part = oracle.partition(rowptr[:-1].copy())
    assert part["stream_chunks"].tolist() == [0, 1, 3, 5, 6, 7]


def test_partition_invariants_on_power_law_workload():
    w = gen.workload(4, {"n": 1 << 17, "cap": 50000})
    part = oracle.partition(w.rowptr)
    n = w.nrows
    off, perm = part["bin_offset"], part["row_perm"]
    L = np.diff(w.rowptr)
    assert off[0] == 0 and np.all(np.diff(off) >= 0)
    in_stream = np.zeros(n, dtype=bool)
    for c in part["stream_chunks"]:
        in_stream[32 * c:32 * c + 32] = True
    assert off[-1] == n - in_stream.sum()
    assert np.array_equal(np.sort(perm), np.flatnonzero(~in_stream))   # bins partition the other rows
    lo = [0, 1, 2, 3, 5, 9, 17, 33, 65, 4097]
    hi = [0, 1, 2, 4, 8, 16, 32, 64, 4096, 2 ** 31]
    for b in range(10):
        rows = perm[off[b]:off[b + 1]]
        assert np.all(np.diff(rows) > 0)                         # ascending inside a bin
        assert np.all((L[rows] >= lo[b]) & (L[rows] <= hi[b]))
    long_rows = perm[off[9]:]
    lp, tr, tn = part["long_off"], part["tile_row"], part["tile_nz"]
    assert long_rows.size > 0
    assert np.array_equal(np.diff(lp), L[long_rows])
    T = tr.size - 1
    assert T == -(-int(lp[-1]) // 4096)
    assert tr[T] == long_rows.size and tn[T] == 0
    pos = lp[tr[:T]] + tn[:T]
    assert np.array_equal(pos, 4096 * np.arange(T))              # tiles start every 4096 long entries
    assert np.all(tn[:T] >= 0) and np.all(tn[:T] < L[long_rows][tr[:T]])
    assert np.all(np.diff(tr) >= 0)


def test_partition_degenerate_inputs():
    part = oracle.partition(np.zeros(1, dtype=np.int32))          # zero rows
    assert np.all(part["bin_offset"] == 0) and part["row_perm"].size == 0
    assert part["tile_row"].tolist() == [0] and part["long_off"].tolist() == [0]
    part = oracle.partition(np.zeros(6, dtype=np.int32))          # only empty rows
    assert part["bin_offset"].tolist() == [0] + [5] * 10
    assert part["row_perm"].tolist() == [0, 1, 2, 3, 4]
    rp = np.array([0, 10000], dtype=np.int32)                      # one long row: 3 tiles
    part = oracle.partition(rp)
    assert part["tile_row"].tolist() == [0, 0, 0, 1]
    assert part["tile_nz"].tolist() == [0, 4096, 8192, 0]
    rp = np.array([0, 4097, 4097, 8194 + 4095], dtype=np.int32)    # two long rows around an empty one
    part = oracle.partition(rp)
    assert part["row_perm"].tolist() == [1, 0, 2]
    assert part["long_off"].tolist() == [0, 4097, 4097 + 8192]
    # 12289 long entries -> 4 tiles starting at 0, 4096, 8192, 12288
    assert part["tile_row"].tolist() == [0, 0, 1, 1, 2]
    assert part["tile_nz"].tolist() == [0, 4096, 4095, 8191, 0]


def test_split_geometry():
    assert oracle.split_geometry(1 << 23, 4) == (16, 1 << 19)       # 32 MiB of floats: 16 blocks of 2 MiB
    assert oracle.split_geometry(1 << 22, 8) == (16, 1 << 18)
    assert oracle.split_geometry(1 << 18, 8) == (0, 0)              # 2 MiB: not worth it
    assert oracle.split_geometry((1 << 18) + 1, 8) == (2, (1 << 17) + 1)
    assert oracle.split_geometry(1 << 30, 8) == (32, 1 << 25)       # capped at 32 blocks
    assert oracle.split_geometry(1000003, 4) == (2, 500002)


def test_split_cuts_hand_worked():
    """Two rows above 64 entries in a 30-column-block world: blocks of width 10 (nb = 3)."""
    cols0 = list(range(0, 70))                   # row 0: columns 0..69 -> cuts at 10, 20, then the end
    cols1 = [5] * 3 + [12] * 60 + [29] * 7        # row 2: duplicates allowed (non-decreasing)
    rowptr = np.array([0, 70, 72, 142], dtype=np.int32)
    colidx = np.array(cols0 + [1, 2] + cols1, dtype=np.int32)
    part = oracle.partition(rowptr)
    assert part["row_perm"].tolist() == [1, 0, 2]                   # bin 2 (row 1), bin 8 (rows 0, 2)
    assert part["stream_chunks"].size == 0                           # 142 entries: below the minimum
    sp = oracle.split_partition(rowptr, colidx, 30, 8, part, block_bytes=80, max_blocks=32)
    assert (sp["num_blocks"], sp["block_width"], sp["num_split_rows"]) == (3, 10, 2)
    # cut[b*S + r]: b = 0..3, r = 0 (row 0), 1 (row 2)
    assert sp["cut"].tolist() == [0, 72, 10, 75, 20, 135, 70, 142]
    # virtual rows (b, r): lengths 10, 3, 10, 60, 50, 7 -> bins 5, 3, 5, 7, 7, 4
    assert np.diff(sp["bin_offset"]).tolist() == [0, 0, 0, 1, 1, 2, 0, 2, 0, 0]
    assert sp["row_perm"].tolist() == [1, 5, 0, 2, 3, 4]
    # an unsorted split row switches the split off
    colidx[3], colidx[4] = colidx[4], colidx[3]
    assert oracle.split_partition(rowptr, colidx, 30, 8, part, block_bytes=80)["num_blocks"] == 0


def test_split_matches_searchsorted():
    n, ncols = 400, 1 << 20
    L = np.full(n, 3, dtype=np.int64)
    L[::7] = 100 + 37 * np.arange(L[::7].size)        # rows above 64 entries, some above 4096
    L[5] = 9000
    rowptr, colidx, _ = gen.random_csr(n, ncols, L, 99)
    part = oracle.partition(rowptr)
    sp = oracle.split_partition(rowptr, colidx, ncols, 8, part)
    nb, W, S = sp["num_blocks"], sp["block_width"], sp["num_split_rows"]
    rows = part["row_perm"][part["bin_offset"][8]:]          # rows above 64 entries outside stream chunks
    assert sp["num_huge_rows"] == 0 and np.array_equal(sp["split_rows"], rows)
    assert (nb, W) == (4, 1 << 18) and S == rows.size and 0 < S <= (L > 64).sum()
    for r, row in enumerate(rows):
        cols = colidx[rowptr[row]:rowptr[row + 1]]
        expect = rowptr[row] + np.searchsorted(cols, np.arange(nb + 1) * W, side="left")
        expect[-1] = rowptr[row + 1]
        assert np.array_equal(sp["cut"][r::S], expect)
    vlen = sp["cut"][S:] - sp["cut"][:-S]
    assert vlen.sum() == L[rows].sum() and np.all(vlen >= 0)
    assert np.array_equal(np.sort(sp["row_perm"]), np.arange(nb * S))


def test_split_huge_rows_hand_worked():
    """Threshold 70 entries and 32-byte LDS blocks (4 doubles) in a 30-column world: the row of 72
    entries is 'huge' and cut at columns 0, 4, 8, ..., the row of 66 stays a split row."""
    cols0 = np.sort(np.concatenate([np.arange(30), np.arange(30), np.arange(12)])).tolist()   # 72 entries
    cols2 = np.sort(np.concatenate([np.arange(30), np.arange(30), np.arange(6)])).tolist()    # 66 entries
    rowptr = np.array([0, 72, 74, 140], dtype=np.int32)
    colidx = np.array(cols0 + [1, 2] + cols2, dtype=np.int32)
    part = oracle.partition(rowptr)
    sp = oracle.split_partition(rowptr, colidx, 30, 8, part, block_bytes=80, huge_row=70, lds_block_bytes=32)
    assert (sp["num_blocks"], sp["num_split_rows"], sp["num_huge_rows"]) == (3, 1, 1)
    assert sp["split_rows"].tolist() == [2] and sp["huge_rows"].tolist() == [0]
    assert (sp["num_fblocks"], sp["fblock_width"]) == (8, 4)
    # row 0 holds columns 0..11 three times and 12..29 twice: 12 entries per block of 4 up to
    # column 11, then 8 per block; the last block (28, 29) holds 4
    assert np.diff(sp["fcut"]).tolist() == [12, 12, 12, 8, 8, 8, 8, 4]
    assert sp["fcut"][0] == 0 and sp["fcut"][-1] == 72
    # the split row alone: cuts at columns 10 and 20 of row 2 (entries 74..139)
    assert sp["cut"].tolist() == [74, 74 + 26, 74 + 46, 140]
    # an unsorted huge row switches everything off, as an unsorted split row does
    colidx[2], colidx[3] = colidx[3], colidx[2]
    assert colidx[2] > colidx[3]
    assert oracle.split_partition(rowptr, colidx, 30, 8, part, block_bytes=80, huge_row=70,
                                  lds_block_bytes=32)["num_blocks"] == 0


def test_split_huge_rows_match_searchsorted_on_power_law_rows():
    w = gen.workload(4, {"n": 1 << 20, "cap": 100000})
    part = oracle.partition(w.rowptr)
    sp = oracle.split_partition(w.rowptr, w.colidx, w.ncols, 4, part)
    L = np.diff(w.rowptr)
    rows = part["row_perm"][part["bin_offset"][8]:]
    assert sp["num_blocks"] > 0 and sp["num_huge_rows"] > 0
    assert np.array_equal(sp["huge_rows"], rows[L[rows] > oracle.HUGE_ROW])
    assert np.array_equal(sp["split_rows"], rows[L[rows] <= oracle.HUGE_ROW])
    assert np.all(np.diff(sp["huge_rows"]) > 0)                       # all in the last bin: ascending ids
    H, nbf, fW = sp["num_huge_rows"], sp["num_fblocks"], sp["fblock_width"]
    assert fW == 16384 and nbf == -(-w.ncols // fW)
    for h in (0, H // 2, H - 1):
        row = sp["huge_rows"][h]
        cols = w.colidx[w.rowptr[row]:w.rowptr[row + 1]]
        expect = w.rowptr[row] + np.searchsorted(cols, np.arange(nbf + 1) * fW, side="left")
        expect[-1] = w.rowptr[row + 1]
        assert np.array_equal(sp["fcut"][h::H], expect)
    # every entry of every row above 64 entries is owned exactly once
    flen = sp["fcut"][H:] - sp["fcut"][:-H]
    S = sp["num_split_rows"]
    vlen = sp["cut"][S:] - sp["cut"][:-S]
    assert flen.sum() == L[sp["huge_rows"]].sum() and vlen.sum() == L[sp["split_rows"]].sum()
    assert np.all(flen >= 0) and np.all(vlen >= 0)
    assert part["bin_offset"][8] == part["bin_offset"][10] - S - H


# ---- level 1b: 16-bit column offsets of narrow stream chunks ----------------
def _index16_brute(rowptr, colidx, part):
    """Straight from the definition, chunk by chunk, with numpy min / max / unique."""
    n = rowptr.size - 1
    nchunks = (n + oracle.STREAM_ROWS - 1) // oracle.STREAM_ROWS
    base = np.full(nchunks, -1, dtype=np.int32)
    table = np.zeros(32 * nchunks, dtype=np.int32)
    col16 = np.zeros(colidx.size, dtype=np.uint16)
    narrow = framed = 0
    for c in part["stream_chunks"]:
        b, e = rowptr[c * oracle.STREAM_ROWS], rowptr[min((c + 1) * oracle.STREAM_ROWS, n)]
        cols = colidx[b:e]
        if int(cols.max()) - int(cols.min()) <= 65535:
            base[c] = cols.min()
            col16[b:e] = cols - cols.min()
            narrow += e - b
            continue
        frames = np.unique(cols >> 11)
        if frames.size <= 32:
            base[c] = -2
            table[32 * c:32 * c + 32] = frames[-1]
            table[32 * c:32 * c + frames.size] = frames
            col16[b:e] = (np.searchsorted(frames, cols >> 11) << 11) | (cols & 2047)
            framed += e - b
    return base, table, col16, narrow, framed


def _decode_index16(rowptr, got):
    """Columns back from the codes: base + offset, or frame_table[code >> 11] * 2048 + (code & 2047)."""
    n = rowptr.size - 1
    chunk_of_entry = np.repeat(np.arange(n) // oracle.STREAM_ROWS, np.diff(rowptr))
    b = got["chunk_base"][chunk_of_entry].astype(np.int64)
    code = got["col16"].astype(np.int64)
    frame = got["frame_table"][32 * chunk_of_entry + (code >> 11)].astype(np.int64)
    cols = np.where(b >= 0, b + code, frame * 2048 + (code & 2047))
    return cols, b


@pytest.mark.parametrize("cfg,scale", [(1, None), (2, {"nx": 24, "ny": 24, "nz": 24}),
                                       (2, {"nx": 200, "ny": 200, "nz": 6}),
                                       (3, {"n": 1 << 18}), (4, {"n": 1 << 15, "cap": 5000}),
                                       (8, {"grid": 12})])
def test_index16_matches_definition_and_reconstructs_columns(cfg, scale):
    w = gen.workload(cfg, scale)
    part = oracle.partition(w.rowptr)
    got = oracle.index16(w.rowptr, w.colidx)
    base, table, col16, narrow, framed = _index16_brute(w.rowptr, w.colidx, part)
    assert got["chunk_base"].dtype == np.int32 and got["col16"].dtype == np.uint16
    assert np.array_equal(got["chunk_base"], base) and np.array_equal(got["col16"], col16)
    assert np.array_equal(got["frame_table"], table)
    assert (got["narrow_entries"], got["framed_entries"]) == (narrow, framed)
    assert got["enabled"] == (narrow + framed > 0 and 2 * (narrow + framed) >= w.nnz)
    # the point of the structure: every column of a narrow or framed chunk comes back from its code
    cols, b = _decode_index16(w.rowptr, got)
    ok = b != -1
    assert np.array_equal(cols[ok], w.colidx[ok])
    assert np.all(got["col16"][~ok] == 0)
    if cfg == 2 and scale["nx"] == 200:
        assert framed > narrow                     # 200 x 200 planes: interior chunks span 2*(200^2+201) columns


def test_index16_frames_hand_worked():
    """One chunk of 32 rows x 8 entries: columns 0..3 and 100000..100003 in every row: two frames
    (0 and 48); a second chunk touching 33 frames is left alone."""
    n, per = 64, 8
    rowptr = (np.arange(n + 1) * per).astype(np.int32)
    row_a = np.array([0, 1, 2, 3, 100000, 100001, 100002, 100003], dtype=np.int32)
    chunk_b = (np.arange(32 * per) % 33 * 2048 + 5).astype(np.int32)          # 33 distinct frames
    colidx = np.concatenate([np.tile(row_a, 32), np.sort(chunk_b.reshape(32, per), axis=1).ravel()]).astype(np.int32)
    got = oracle.index16(rowptr, colidx)
    assert got["chunk_base"].tolist() == [-2, -1]
    assert got["frame_table"][:32].tolist() == [0] + [48] * 31 and np.all(got["frame_table"][32:] == 0)
    assert got["col16"][:8].tolist() == [0, 1, 2, 3, 2048 + 100000 % 2048, 2048 + 100001 % 2048,
                                          2048 + 100002 % 2048, 2048 + 100003 % 2048]
    assert np.all(got["col16"][256:] == 0)
    assert (got["narrow_entries"], got["framed_entries"], got["enabled"]) == (0, 256, True)
    # 32 frames is still fine
    chunk_c = (np.arange(32 * per) % 32 * 4096 + 7).astype(np.int32)
    colidx[256:] = np.sort(chunk_c.reshape(32, per), axis=1).ravel()
    got = oracle.index16(rowptr, colidx)
    assert got["chunk_base"].tolist() == [-2, -2]
    assert got["frame_table"][32:].tolist() == list(range(0, 64, 2))


def test_index16_threshold_is_65535():
    """Two chunks of 32 rows x 8 entries; the second spans exactly 65535 / 65536 columns."""
    n, per = 64, 8
    rowptr = (np.arange(n + 1) * per).astype(np.int32)
    for span, narrow in ((65535, True), (65536, False)):
        colidx = np.tile(np.arange(per, dtype=np.int32), n)
        colidx[32 * per:] += 1000
        colidx[-1] = 1000 + span                  # largest column of chunk 1; its smallest is 1000
        got = oracle.index16(rowptr, colidx)
        assert got["chunk_base"][0] == 0
        assert got["chunk_base"][1] == (1000 if narrow else -2)       # not narrow: two frames, 0 and 32
        assert got["col16"][-1] == (span if narrow else (1 << 11) | ((1000 + span) & 2047))
        assert got["enabled"]                     # chunk 0 alone holds half of the entries


def test_index16_off_without_stream_chunks_and_below_half():
    rowptr = (np.arange(33) * 4).astype(np.int32)            # 128 entries: below the stream minimum
    colidx = np.tile(np.arange(4, dtype=np.int32), 32)
    got = oracle.index16(rowptr, colidx)
    assert not got["enabled"] and np.all(got["chunk_base"] == -1) and got["narrow_entries"] == 0
    # one narrow chunk of 256 entries and one chunk of 320 entries over 40 frames: 256 * 2 < 576
    lens = np.concatenate([np.full(32, 8), np.full(32, 10)])
    rowptr = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    wide = np.sort(((np.arange(32)[:, None] * 10 + np.arange(10)[None, :]) % 40) * 10000, axis=1)
    colidx = np.concatenate([np.tile(np.arange(8), 32), wide.ravel()]).astype(np.int32)
    got = oracle.index16(rowptr, colidx)
    assert got["chunk_base"].tolist() == [0, -1] and got["narrow_entries"] == 256 and not got["enabled"]
    assert got["framed_entries"] == 0


# ---- demotion of stream chunks whose gathers would have no locality ----------
def test_demoted_chunks_rule():
    """Four chunks of 32 rows over 2^20 double columns (x = 8 MiB: the split's condition holds):
    0: rows of 16 scattered columns (wide, but no row above 64)   -> streams
    1: one row of 100 scattered columns, 31 rows of 8              -> demoted
    2: one row of 100 consecutive columns (narrow), 31 rows of 8   -> streams
    3: one row of 100 columns in 4 far-apart clusters (framed)     -> streams"""
    ncols = 1 << 20
    rng = np.random.default_rng(3)
    rows = []
    for c in range(4):
        for r in range(32):
            if c == 0:
                rows.append(np.sort(rng.choice(ncols, 16, replace=False)))
            elif r == 0 and c == 1:
                rows.append(np.sort(rng.choice(ncols, 100, replace=False)))
            elif r == 0 and c == 2:
                rows.append(5000 + np.arange(100))
            elif r == 0 and c == 3:
                rows.append(np.sort(np.concatenate([k * 200000 + np.arange(25) for k in range(4)])))
            else:
                rows.append(5000 + c + np.arange(8))
    rowptr = np.concatenate([[0], np.cumsum([len(r) for r in rows])]).astype(np.int32)
    colidx = np.concatenate(rows).astype(np.int32)
    plain = oracle.partition(rowptr)
    assert plain["stream_chunks"].size == 4
    base = oracle.index16(rowptr, colidx)["chunk_base"]
    assert base[0] == -1 and base[1] == -1 and base[2] >= 0 and base[3] == -2
    dem = oracle.demoted_chunks(rowptr, colidx, ncols, 8)
    assert dem.tolist() == [0, 1, 0, 0]
    part = oracle.partition(rowptr, colidx=colidx, ncols=ncols, itemsize=8)
    assert sorted(part["stream_chunks"].tolist()) == [0, 2, 3]
    assert np.array_equal(np.sort(part["row_perm"]), np.arange(32, 64))       # the demoted chunk's rows are binned
    assert part["bin_offset"][8] == 31 and part["bin_offset"][9] == 32        # 31 rows of 8 (bin 4), one of 100 (bin 8)
    # x of 2 MiB or less: nothing is demoted
    assert oracle.demoted_chunks(rowptr, np.minimum(colidx, (1 << 18) - 1), 1 << 18, 8).sum() == 0
    # the codes are those of the undemoted view: a demoted chunk had none anyway
    again = oracle.index16(rowptr, colidx)
    assert np.array_equal(again["chunk_base"], base)


def test_demotion_on_power_law_rows():
    w = gen.workload(4, {"n": 1 << 20, "cap": 100000})
    plain = oracle.partition(w.rowptr)
    part = oracle.partition(w.rowptr, colidx=w.colidx, ncols=w.ncols, itemsize=4)
    dem = oracle.demoted_chunks(w.rowptr, w.colidx, w.ncols, 4)
    assert dem.sum() > 0
    assert np.array_equal(np.setdiff1d(plain["stream_chunks"], part["stream_chunks"]), np.flatnonzero(dem))
    L = np.diff(w.rowptr)
    for c in np.flatnonzero(dem)[:50]:
        assert L[c * 32:(c + 1) * 32].max() > 64
    for c in part["stream_chunks"][:2000]:
        cols = w.colidx[w.rowptr[c * 32]:w.rowptr[min((c + 1) * 32, w.nrows)]]
        coded = int(cols.max()) - int(cols.min()) <= 65535 or np.unique(cols >> 11).size <= 32
        assert coded or L[c * 32:(c + 1) * 32].max() <= 64
    assert part["bin_offset"][-1] == plain["bin_offset"][-1] + sum(
        min(32, w.nrows - c * 32) for c in np.flatnonzero(dem))
