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
    holds fewer than 64 entries or a row exceeds 512 entries."""
    L = np.array([2] * 32            # chunk 0: 64 entries, max 2                 -> class 1
                 + [8] * 31 + [65]   # chunk 1: max 65                            -> class 2
                 + [1] * 31 + [32]   # chunk 2: 63 entries, below the minimum     -> binned
                 + [64] * 32         # chunk 3: rows at 64, 2048 entries > 2*512  -> class 2
                 + [0] * 31 + [63]   # chunk 4: 63 entries                        -> binned
                 + [128] * 2 + [1] * 30   # chunk 5: max 128                      -> class 2
                 + [129] + [5] * 31  # chunk 6: max 129 (284 entries)             -> class 3
                 + [512] + [0] * 31  # chunk 7: max 512                           -> class 4
                 + [513] + [9] * 31  # chunk 8: a row above 512                   -> binned
                 + [10] * 7,         # chunk 9 (ragged, 7 rows): 70 entries       -> class 1
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
    # bins: 31 empty rows; 31 rows of 1 (bin 1); 31 rows of 9 (bin 5); rows of 32 and 63 (bins 6, 7); one of 513 (bin 8)
    assert np.diff(part["bin_offset"]).tolist() == [31, 31, 0, 0, 0, 31, 1, 1, 1, 0]
    # with 6 rows in the ragged chunk: 60 entries -> binned
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
    part = oracle.partition(rowptr, stream_min_nnz=1000)            # no stream chunk: the rows are binned
    assert part["row_perm"].tolist() == [1, 0, 2]                   # bin 2 (row 1), bin 8 (rows 0, 2)
    assert part["stream_chunks"].size == 0
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
    part = oracle.partition(rowptr, stream_min_nnz=1000)            # no stream chunk: the rows are binned
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
    rowptr = np.concatenate([np.arange(32), [63]]).astype(np.int32)   # 63 entries: below the stream minimum
    colidx = np.arange(63, dtype=np.int32) % 32
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


# ---- level 1c: row patterns ---------------------------------------------------
def _csr_from_rows(rows):
    rowptr = np.zeros(len(rows) + 1, dtype=np.int32)
    np.cumsum([len(r) for r in rows], out=rowptr[1:])
    colidx = np.array([c for r in rows for c in r], dtype=np.int32)
    return rowptr, colidx


def _banded(n, half):
    return [[j for j in range(i - half, i + half + 1) if 0 <= j < n] for i in range(n)]


def _columns_from_patterns(rowptr, got):
    """Columns back from the patterns (-1 where the chunk has none): row + shift + pool[pat_off + start + k]."""
    n = rowptr.size - 1
    L = np.diff(rowptr)
    row_of_entry = np.repeat(np.arange(n, dtype=np.int64), L)
    k = np.arange(rowptr[-1], dtype=np.int64) - np.repeat(rowptr[:-1].astype(np.int64), L)
    chunk = row_of_entry // oracle.STREAM_ROWS
    has = (got["pat_off"][1:] > got["pat_off"][:-1])[chunk]
    start, shift = oracle.pattern_start_shift(got["row_pat"])
    at = got["pat_off"][chunk].astype(np.int64) + start[row_of_entry] + k
    cols = np.full(rowptr[-1], -1, dtype=np.int64)
    cols[has] = row_of_entry[has] + shift[row_of_entry][has] + got["pool"][at[has]]
    return cols, has


def test_row_patterns_hand_worked_band():
    # 9 diagonals, 64 rows: chunk 0 needs the four cut-off patterns of rows 0-3 (5, 6, 7, 8 entries)
    # and the full one; chunk 1 the full one and the four cut-off ones of rows 60-63
    rowptr, colidx = _csr_from_rows(_banded(64, 4))
    got = oracle.row_patterns(rowptr, colidx)
    assert got["pat_off"].tolist() == [0, 35, 70]
    assert got["row_pat"][:6].tolist() == [0, 5, 11, 18, 26, 26] and np.all(got["row_pat"][4:32] == 26)
    assert got["pool"][:35].tolist() == (list(range(0, 5)) + list(range(-1, 5)) + list(range(-2, 5))
                                        + list(range(-3, 5)) + list(range(-4, 5)))
    assert np.all(got["row_pat"][32:60] == 0) and got["row_pat"][60:].tolist() == [9, 17, 24, 30]
    assert got["pool"][35:].tolist() == (list(range(-4, 5)) + list(range(-4, 4)) + list(range(-4, 3))
                                        + list(range(-4, 2)) + list(range(-4, 1)))
    assert got["entries"] == colidx.size and got["enabled"]
    assert got["row_pat"].dtype == np.uint16 and got["pool"].dtype == np.int32


def test_row_patterns_first_appearance_order_and_prefixes():
    # A B A C(prefix of A) in the first rows; the stored order of a row matters (unsorted, duplicates)
    n = 32
    A = [0, 3, 1, 1, 7, 9, 12, 15, 2]
    B = [5, 4, 3, 2, 1, 0, 6, 7, 8]
    C = A[:8]
    pats = [A, B, A, C] + [A] * (n - 4)
    rows = [[i + d for d in p] for i, p in enumerate(pats)]
    rowptr, colidx = _csr_from_rows(rows)
    got = oracle.row_patterns(rowptr, colidx)
    assert got["pat_off"].tolist() == [0, 26]
    assert got["row_pat"][:5].tolist() == [0, 9, 0, 18, 0]
    assert got["pool"].tolist() == A + B + C


def test_row_patterns_with_shifts_hand_worked():
    """Three unknowns per grid point, 1-D grid with neighbours -1, 0, +1: row 3p + a holds the columns
    3(p-1) .. 3(p+1)+2 whatever a is, so the three rows of a point have the list of its first row moved
    by 0, -1, -2: one stored list of 9 for the interior, the two cut-off lists of the end points, and the
    shift in bits 9..15 of row_pat."""
    npts = 16                                                  # 48 rows: one full chunk and half a chunk
    rows = []
    for p in range(npts):
        cols = [3 * q + c for q in (p - 1, p, p + 1) if 0 <= q < npts for c in range(3)]
        rows += [cols] * 3
    rowptr, colidx = _csr_from_rows(rows)
    got = oracle.row_patterns(rowptr, colidx)
    start, shift = oracle.pattern_start_shift(got["row_pat"])
    # chunk 0 (rows 0..31): point 0 has 6 columns 0..5: list (0..5) stored at 0; rows 1, 2 are it moved by -1, -2;
    # point 1 (rows 3, 4, 5) has columns 0..8: list (-3..5) stored at 6; every later row has that shape
    assert got["pat_off"].tolist() == [0, 15, 30]
    assert got["pool"][:15].tolist() == [0, 1, 2, 3, 4, 5] + [-3, -2, -1, 0, 1, 2, 3, 4, 5]
    assert start[:32].tolist() == [0, 0, 0] + [6] * 29
    assert shift[:32].tolist() == [0, -1, -2] + [0, -1, -2] * 9 + [0, -1]
    assert got["row_pat"][1] == (127 << 9) and got["row_pat"][5] == 6 | (126 << 9)
    # chunk 1 (rows 32..47) starts with the third row of point 10: ITS list (-5..3) is stored, and the rows
    # of the next points are that list moved by +2, +1, 0; the last point (rows 45, 46, 47) has 6 columns
    assert got["pool"][15:30].tolist() == [-5, -4, -3, -2, -1, 0, 1, 2, 3] + [-3, -2, -1, 0, 1, 2]
    assert start[32:].tolist() == [0] * 13 + [9] * 3
    assert shift[32:].tolist() == [0] + [2, 1, 0] * 4 + [0, -1, -2]
    cols, has = _columns_from_patterns(rowptr, got)
    assert has.all() and np.array_equal(cols, colidx)


def test_row_patterns_shift_limits_and_order_of_the_search():
    """A row whose shift to a stored list of its shape is outside [-64, 63] does not take that list: it
    stores its own, and later rows take whichever stored list of the shape comes first within reach."""
    shape = [0, 1, 2, 3, 4, 5, 6, 7]
    firsts = [0, 63, 64, -64, -65, 100, 128 + 63, 1]            # first diagonal of rows 0..7 (row i: columns i + first + shape)
    rows = [[i + f + d for d in shape] for i, f in enumerate(firsts)]
    rows += [[i + 10 + d for d in shape] for i in range(8, 32)]
    rows = [[c + 200 for c in r] for r in rows]                 # keep every column non-negative
    rowptr, colidx = _csr_from_rows(rows)
    got = oracle.row_patterns(rowptr, colidx)
    start, shift = oracle.pattern_start_shift(got["row_pat"])
    # row 0 stores list A (first 200).  row 1: +63 -> A.  row 2: +64 is too far -> stores B (first 264).
    # row 3: -64 -> A.  row 4: -65 from A, -129 from B -> stores C (first 135).  row 5: first 300: +100 from A,
    # +36 from B -> B.  row 6: first 391: from A 191, from B 127, from C 256 -> stores D.  row 7: +1 -> A.
    assert got["pat_off"].tolist() == [0, 32]
    assert start[:8].tolist() == [0, 0, 8, 0, 16, 8, 24, 0]
    assert shift[:8].tolist() == [0, 63, 0, -64, 0, 36, 0, 1]
    assert np.all(start[8:] == 0) and np.all(shift[8:] == 10)
    assert got["pool"].tolist() == [200 + d for d in shape] + [264 + d for d in shape] + [135 + d for d in shape] + [391 + d for d in shape]
    cols, has = _columns_from_patterns(rowptr, got)
    assert has.all() and np.array_equal(cols, colidx)


# ---- level 1d: which chunks share rows of X in the product with a block of vectors ------------
def _share(rows):
    rowptr, colidx = _csr_from_rows(rows)
    part = oracle.partition(rowptr)
    pats = oracle.row_patterns(rowptr, colidx)
    return oracle.share_classes(rowptr, part, pats)


def _block_rows(npts, dof, nbrs):
    """dof unknowns per point of a 1-D grid: row dof*p + a holds the columns dof*q + b, q = p + a neighbour."""
    rows = []
    for p in range(npts):
        cols = [dof * (p + d) + b for d in nbrs if 0 <= p + d < npts for b in range(dof)]
        rows += [cols] * dof
    return rows


def test_share_classes_hand_worked():
    P, N, B3, B2 = oracle.SHARE_PLAIN, oracle.SHARE_NONE, oracle.SHARE_BLOCK3, oracle.SHARE_BLOCK2
    # a band of 9 diagonals over 96 rows: rows 0-3 and 92-95 are cut off (4 odd rows in the end chunks)
    assert _share(_banded(96, 4)).tolist() == [P, P, P]
    # 11 diagonals: 5 cut-off rows at each end are one too many
    assert _share(_banded(96, 5)).tolist() == [N, P, N]
    # the three-unknowns example of the row patterns above: rows 0-2 are odd (the first point), the others
    # stand at v = 3, 3, 3, 6, 6, 6, ...: every aligned four rows see two points, three apart
    assert _share(_block_rows(16, 3, (-1, 0, 1))).tolist() == [B3, B3]
    # two unknowns per point: the four rows of a group are two points, two apart
    assert _share(_block_rows(40, 2, (-1, 0, 1))).tolist() == [B2, B2, B2]
    # four unknowns: every aligned group is ONE point, all its rows need the same rows of X: no class for that
    assert _share(_block_rows(24, 4, (-1, 0, 1))).tolist() == [N, N, N]
    # five unknowns: groups see steps of 5
    assert _share(_block_rows(16, 5, (-1, 0, 1))).tolist() == [N, N, N]
    # the reference list must ascend: every row with the same two runs, the second first
    assert _share([[i + 50, i + 51, i + 52, i + 10, i + 11] for i in range(64)]).tolist() == [N, N]
    assert _share([[i + 10, i + 11, i + 50, i + 51, i + 52] for i in range(64)]).tolist() == [P, P]


def test_share_classes_limits():
    P, N, B3 = oracle.SHARE_PLAIN, oracle.SHARE_NONE, oracle.SHARE_BLOCK3
    # plain rows: at most 64 diagonals, and the chunk's values within one window of 1024 with 64 to spare
    wide = lambda w, n=64: [[i + d for d in range(w)] for i in range(n)]
    assert _share(wide(30)).tolist() == [P, P]                   # 960 + 64 = 1024
    assert _share(wide(31)).tolist() == [N, N]                   # 992 + 64 > 1024
    # ... counted from the chunk's first entry rounded down to a multiple of 8: 28 entries before the second chunk
    rows = [[0]] * 28 + [[]] * 4 + wide(30, 32)
    assert _share(rows).tolist() == [0, N]                       # chunk 0 has too few entries to stream; 28 % 8 = 4 more
    rows = [[0]] * 24 + [[]] * 8 + wide(30, 32)
    assert _share(rows).tolist() == [0, P]
    # block rows: up to 128 diagonals (the longest row a pattern may have), values unlimited
    got = _share(_block_rows(200, 3, range(-21, 21))).tolist()   # 42 points * 3 = 126 diagonals; points 21 .. 178 are whole
    assert got[2:16] == [B3] * 14
    assert _share(_block_rows(200, 3, range(-21, 22))) is None   # 129 diagonals: rows too long for a pattern
    # odd rows: empty rows count, rows past the end of the matrix do not
    rows = _block_rows(32, 3, (-1, 0, 1))[:80]                   # 2.5 chunks; the last point is cut like an inner one
    for i in (35, 40, 41, 50):
        rows[i] = []
    assert _share(rows).tolist() == [B3, B3, B3]
    rows[51] = rows[51][:-1]
    assert _share(rows).tolist() == [B3, N, B3]
    # a shorter reference list among longer odd rows is not looked for: the first longest row decides
    rows = _banded(64, 4)
    rows[40] = list(range(30, 45))
    assert _share(rows).tolist() == [P, N]


def test_share_classes_off_without_patterns():
    rowptr, colidx, _ = gen.random_csr(256, 256, np.full(256, 12, dtype=np.int64), 5, np.float64)
    part = oracle.partition(rowptr)
    pats = oracle.row_patterns(rowptr, colidx)
    assert not pats["enabled"] and oracle.share_classes(rowptr, part, pats) is None


def test_row_patterns_limits():
    base = list(range(9))

    def chunk_with(patterns):
        rows = [[i + d for d in patterns[i % len(patterns)]] for i in range(32)]
        return _csr_from_rows(rows)

    eight = [base[:-1] + [20 + p] for p in range(8)]
    nine = eight + [base[:-1] + [40]]
    assert oracle.row_patterns(*chunk_with(eight))["pat_off"].tolist() == [0, 72]
    got = oracle.row_patterns(*chunk_with(nine))                       # a ninth pattern: none at all
    assert got["pat_off"].tolist() == [0, 0] and not got["row_pat"].any() and got["entries"] == 0 and not got["enabled"]
    # table of exactly 512 diagonals fits (8 patterns of 64), 513 do not
    wide = [[q * 100 + t for t in range(64)] for q in range(8)]
    assert oracle.row_patterns(*chunk_with(wide))["pat_off"].tolist() == [0, 512]
    wider = [w[:] for w in wide]
    wider[7] = wider[7] + [999]
    assert oracle.row_patterns(*chunk_with(wider))["pat_off"].tolist() == [0, 0]
    # a row of 128 entries is allowed, 129 is not (one pattern, 4 rows of it)
    for length, expect in ((128, [0, 128]), (129, [0, 0])):
        rows = [list(range(i, i + length)) if i < 4 else [] for i in range(32)]
        assert oracle.row_patterns(*_csr_from_rows(rows))["pat_off"].tolist() == expect
    # the table must pay for itself: 8 rows, all different, 40 entries each: 2 * 320 > 320
    rows = [[i + 3 * t + (t == 39) * i for t in range(40)] for i in range(8)]
    assert oracle.row_patterns(*_csr_from_rows(rows))["pat_off"].tolist() == [0, 0]
    # exactly twice the table: two patterns, each used twice
    rows = [[i + t * (1 + i % 2) for t in range(64)] for i in range(4)]
    assert oracle.row_patterns(*_csr_from_rows(rows))["pat_off"].tolist() == [0, 128]
    # chunks below the stream minimum (63 entries) have no patterns
    rows = [list(range(i, i + 2)) for i in range(31)] + [[31]]
    assert oracle.row_patterns(*_csr_from_rows(rows))["pat_off"].tolist() == [0, 0]


def test_row_patterns_of_the_27_point_stencil_are_its_neighbour_offsets():
    nx, ny, nz = 32, 6, 5                                               # one grid line per chunk
    w = gen.workload(2, {"nx": nx, "ny": ny, "nz": nz})
    got = oracle.row_patterns(w.rowptr, w.colidx)
    assert got["enabled"] and got["entries"] == w.nnz
    lens = np.diff(got["pat_off"])
    for z in range(nz):
        for y in range(ny):
            c = z * ny + y
            dz = [d for d in (-1, 0, 1) if 0 <= z + d < nz]
            dy = [d for d in (-1, 0, 1) if 0 <= y + d < ny]
            left = [a * nx * ny + b * nx + e for a in dz for b in dy for e in (0, 1)]
            mid = [a * nx * ny + b * nx + e for a in dz for b in dy for e in (-1, 0, 1)]
            right = [a * nx * ny + b * nx + e for a in dz for b in dy for e in (-1, 0)]
            # the row on the right face holds the list of the row on the left face moved by -1: the same
            # stored list, shift -1 (bits 9..15 of row_pat = 127)
            assert [r - right[0] for r in right] == [l - left[0] for l in left] and right[0] - left[0] == -1
            assert lens[c] == len(left) + len(mid)
            assert got["pool"][got["pat_off"][c]:got["pat_off"][c + 1]].tolist() == left + mid
            rp = got["row_pat"][32 * c:32 * c + 32]
            assert rp[0] == 0 and np.all(rp[1:31] == len(left)) and rp[31] == (127 << 9)


@pytest.mark.parametrize("cfg,scale", [(1, None), (2, {"nx": 24, "ny": 24, "nz": 24}),
                                       (2, {"nx": 50, "ny": 7, "nz": 9}),
                                       (3, {"n": 1 << 14}), (4, {"n": 1 << 15, "cap": 5000}),
                                       (7, {"scale": 0.01}), (8, {"grid": 12})])
def test_row_patterns_reconstruct_columns_and_are_minimal(cfg, scale):
    w = gen.workload(cfg, scale)
    got = oracle.row_patterns(w.rowptr, w.colidx, w.ncols, w.vals.dtype.itemsize)
    cols, has = _columns_from_patterns(w.rowptr, got)
    assert np.array_equal(cols[has], w.colidx[has])
    assert got["entries"] == int(has.sum())
    part = oracle.partition(w.rowptr, colidx=w.colidx, ncols=w.ncols, itemsize=w.vals.dtype.itemsize)
    streams = set(part["stream_chunks"].tolist())
    L = np.diff(w.rowptr)
    start, shift = oracle.pattern_start_shift(got["row_pat"])
    for c in range(got["pat_off"].size - 1):
        rows = range(32 * c, min(32 * c + 32, w.nrows))
        # the table built again, directly from the rule: a row takes the first stored list with its length,
        # its shape (the list minus its first element) and a shift within [-64, 63], else stores its own
        stored, where, expect = [], 0, {}
        for i in rows:
            if not L[i]:
                continue
            lst = (w.colidx[w.rowptr[i]:w.rowptr[i + 1]].astype(np.int64) - i).tolist()
            for at, other in stored:
                if len(other) == len(lst) and -64 <= lst[0] - other[0] <= 63 and \
                        [a - lst[0] for a in lst] == [a - other[0] for a in other]:
                    expect[i] = (at, lst[0] - other[0])
                    break
            else:
                stored.append((where, lst))
                expect[i] = (where, 0)
                where += len(lst)
        size = where
        entries = int(w.rowptr[rows[-1] + 1] - w.rowptr[rows[0]])
        fits = (c in streams and len(stored) <= 8 and size <= 512 and 2 * size <= entries
                and max(L[i] for i in rows) <= 128)
        assert got["pat_off"][c + 1] - got["pat_off"][c] == (size if fits else 0), c
        if fits:
            assert got["pool"][got["pat_off"][c]:got["pat_off"][c + 1]].tolist() == sum((l for _, l in stored), [])
            for i in rows:
                assert (int(start[i]), int(shift[i])) == expect.get(i, (0, 0)), i
        else:
            assert not got["row_pat"][rows[0]:rows[-1] + 1].any()
    if cfg in (3, 4):         # random columns repeat nothing
        assert not got["enabled"]
    if cfg == 1:              # every chunk of the 5-point grid is patterned
        assert got["enabled"] and got["entries"] == w.nnz
    if cfg == 2:              # everything but a last chunk below the stream minimum
        assert got["enabled"] and got["entries"] >= w.nnz - 255
