"""Host-side replay of the index arithmetic of the SpMV stream kernel (csrc/spmv_kernels.hpp,
spmv_stream_kernel / stream_share / stream_batch / stream_fill): every LDS slot a lane reads a
column code from, live or discarded, must hold an entry of the wavefront's OWN rows, because a
16-bit code is decoded with the base or the frame table of the wavefront's chunk and a foreign
code can decode to a column past the end of x.  Parity tests cannot see such a read (its product
is discarded), so the rules are modelled here on the oracle's partition and 16-bit codes:

  * window w of a wavefront covers entries [w0, w1), w0 = (first entry of its rows) & ~7 + 1024 w;
  * lane (row r, sub s) owns the entries ub + s, ub + s + G, ... of its row inside the window;
    lanes with fewer entries than the batch repeat their own last entry;
  * lanes without an entry in the window re-read the first entry of the window that belongs to
    the wavefront's rows;
  * 16-byte loads of values / columns stop at nnz & ~3, those of the 16-bit codes within the
    array's padding of 8 beyond nnz rounded up to 8.
"""
import numpy as np
import pytest

import gen
import oracle

WINDOW = 1024


def wave_reads(rowptr, nrows, nnz, chunk, wave_in_chunk, G):
    """Yields (w0, w1, base, end, slots) per window: the LDS slots (relative to w0) every lane
    of the wavefront reads codes from, and the memory ranges the fill touches."""
    rows_per_wave = 64 // G
    lanes = np.arange(64)
    row = chunk * 32 + wave_in_chunk * rows_per_wave + lanes // G
    sub = lanes % G
    row_ok = row < nrows
    row_c = np.where(row_ok, row, nrows - 1)
    p0, p1 = rowptr[row_c].astype(np.int64), rowptr[row_c + 1].astype(np.int64)
    rb = np.where(row_ok, p0, p1)
    re = p1
    base, end = int(rb[0]), int(re[63])
    w0 = base & ~7
    while w0 < end:
        w1 = end if end - w0 < WINDOW else w0 + WINDOW
        ub = np.maximum(rb, w0) - w0
        ue = np.minimum(re, w1) - w0
        my_n = (ue - ub - sub + G - 1) // G
        own0 = max(base, w0) - w0
        slots = []
        if (my_n > 0).any():                      # otherwise no batch runs and nothing is gathered
            for lane in range(64):
                if my_n[lane] > 0:
                    first = int(ub[lane] + sub[lane])
                    slots.append(first + G * np.arange(int(my_n[lane])))
                else:
                    slots.append(np.array([own0]))
        yield w0, w1, base, end, (np.concatenate(slots) if slots else np.zeros(0, dtype=np.int64))
        w0 += WINDOW


def check_matrix(rowptr, colidx, ncols, itemsize):
    nrows = rowptr.size - 1
    nnz = int(rowptr[-1])
    part = oracle.partition(rowptr, colidx=colidx, ncols=ncols, itemsize=itemsize)
    idx = oracle.index16(rowptr, colidx)
    nnz4 = nnz & ~3
    col16_len = (nnz + 7) // 8 * 8 + 8
    seen_foreign_window_start = 0
    for cls in range(1, 5):
        G = 1 << cls
        for chunk in part["stream_chunks"][part["stream_offset"][cls - 1]:part["stream_offset"][cls]]:
            cb = int(idx["chunk_base"][chunk]) if idx["enabled"] else -1
            tab = idx["frame_table"][32 * chunk:32 * chunk + 32]
            for wv in range(G // 2):
                for w0, w1, base, end, slots in wave_reads(rowptr, nrows, nnz, int(chunk), wv, G):
                    if w0 < base:
                        seen_foreign_window_start += 1
                    # fill side: vector loads
                    vec_end = ((w1 + 3) & ~3) if w1 < nnz4 else nnz4
                    n_vec = max(vec_end - w0, 0)
                    assert w0 % 8 == 0 and w0 + n_vec <= nnz4 and n_vec <= WINDOW
                    assert w0 + ((n_vec + 7) & ~7) <= col16_len
                    if slots.size == 0:
                        continue
                    j = w0 + slots
                    assert j.min() >= base and j.max() < end, (
                        f"chunk {chunk} wave {wv} window {w0}: a lane reads entry {j.min()}..{j.max()} "
                        f"outside its wavefront's entries [{base}, {end})")
                    # decode as the kernel does, with THIS chunk's base / table
                    if cb >= 0:
                        cols = cb + idx["col16"][j].astype(np.int64)
                    elif cb == -2:
                        code = idx["col16"][j].astype(np.int64)
                        cols = (tab[code >> 11].astype(np.int64) << 11) | (code & 2047)
                    else:
                        cols = colidx[j].astype(np.int64)
                    assert np.array_equal(cols, colidx[j]) and cols.max() < ncols and cols.min() >= 0
    return seen_foreign_window_start


def banded(n, half_band, lo_len, hi_len, seed):
    u = gen.uniform(seed, 0, n, 0.0, 1.0)
    L = (lo_len + np.floor(u * (hi_len - lo_len + 1))).astype(np.int64)
    rowptr, colidx, vals = gen.random_csr(n, n, L, seed + 1, np.float64)
    v = gen.uniform(seed + 2, 5, int(rowptr[-1]), 0.0, 1.0)
    rows = np.repeat(np.arange(n, dtype=np.int64), L)
    cols = np.clip(rows - half_band + (v * (2 * half_band + 1)).astype(np.int64), 0, n - 1)
    order = np.lexsort((cols, rows))
    colidx[:] = cols[order].astype(np.int32)
    return rowptr, colidx


@pytest.mark.parametrize("n,half_band,lo_len,hi_len", [
    (4096, 1000, 0, 29),        # chunks that do not start at a multiple of 8, empty and 1-entry rows
    (4096 + 19, 1000, 0, 29),   # nrows % 32 != 0
    (3000, 700, 9, 70),         # two lane-group sizes
    (2048 + 5, 900, 100, 300),  # several windows per wavefront
    (1500, 40000, 8, 20),       # framed / 32-bit chunks (band wider than 2^16 columns would need n larger)
])
def test_every_code_a_lane_reads_belongs_to_its_wavefront(n, half_band, lo_len, hi_len):
    half_band = min(half_band, (n - 2) // 2)
    rowptr, colidx = banded(n, half_band, lo_len, hi_len, 4100 + n)
    unaligned_starts = check_matrix(rowptr, colidx, n, 8)
    if lo_len == 0:
        assert unaligned_starts > 0, "the case is meant to have windows that begin in a foreign chunk"


def test_wide_matrix_with_framed_chunks():
    """Columns in a few distant clusters: chunks that are framed, not narrow."""
    n, ncols = 2048 + 7, 3_000_000
    u = gen.uniform(31, 0, n, 0.0, 1.0)
    L = (5 + np.floor(u * 20)).astype(np.int64)
    L[::17] = 0
    rowptr, colidx, _ = gen.random_csr(n, ncols, L, 32, np.float64)
    rows = np.repeat(np.arange(n, dtype=np.int64), L)
    v = gen.uniform(33, 5, int(rowptr[-1]), 0.0, 1.0)
    cluster = (v * 4).astype(np.int64)                     # 4 clusters 700 000 columns apart
    cols = cluster * 700_000 + rows + (v * 4000).astype(np.int64) % 1500
    order = np.lexsort((cols, rows))
    colidx[:] = cols[order].astype(np.int32)
    idx = oracle.index16(rowptr, colidx)
    assert idx["enabled"] and idx["framed_entries"] > 0
    check_matrix(rowptr, colidx, ncols, 8)


def test_idle_lane_rule_matters():
    """The rule the kernel had before (idle lanes re-read slot 0 of the window) does leave the
    wavefront's own entries on the first case above: this model would have caught it."""
    n = 4096
    rowptr, colidx = banded(n, 1000, 0, 29, 4100 + n)
    part = oracle.partition(rowptr, colidx=colidx, ncols=n, itemsize=8)
    idx = oracle.index16(rowptr, colidx)
    assert idx["enabled"]
    worst = -1
    for cls in range(1, 5):
        G = 1 << cls
        for chunk in part["stream_chunks"][part["stream_offset"][cls - 1]:part["stream_offset"][cls]]:
            cb = int(idx["chunk_base"][chunk])
            for wv in range(G // 2):
                for w0, w1, base, end, slots in wave_reads(rowptr, n, int(rowptr[-1]), int(chunk), wv, G):
                    if slots.size and w0 < base and cb >= 0:
                        worst = max(worst, cb + int(idx["col16"][w0]))     # slot 0 decoded with this chunk's base
    assert worst >= n, "expected the old rule to decode a foreign code to a column past the end of x"
