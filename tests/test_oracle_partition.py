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


def _independent_partition(rowptr, wave, long_threshold, tile_nnz):
    """The same definition through different primitives: log2, stable argsort, searchsorted."""
    L = np.diff(rowptr).astype(np.int64)
    top = int(math.log2(wave)) + 1
    b = np.zeros(L.size, dtype=np.int64)
    pos = L > 0
    b[pos] = 1 + np.ceil(np.log2(L[pos])).astype(np.int64)
    b[L > wave] = top + 1
    b[L > long_threshold] = top + 2
    nb = top + 3
    perm = np.argsort(b, kind="stable").astype(np.int32)
    off = np.concatenate([[0], np.cumsum(np.bincount(b, minlength=nb))]).astype(np.int32)
    long_rows = perm[off[nb - 1]:]
    lp = np.concatenate([[0], np.cumsum(L[long_rows])]).astype(np.int64)
    T = -(-int(lp[-1]) // tile_nnz)
    starts = np.arange(T, dtype=np.int64) * tile_nnz
    tr = np.searchsorted(lp, starts, side="right") - 1
    tn = starts - lp[tr]
    return off, perm, lp, np.append(tr, long_rows.size), np.append(tn, 0)


@pytest.mark.parametrize("wave,lt,tile", [(64, 4096, 4096), (64, 100, 64), (32, 40, 16), (64, 64, 7)])
@pytest.mark.parametrize("seed", [1, 2])
def test_partition_matches_independent_construction(wave, lt, tile, seed):
    n = 3000
    u = gen.uniform(seed, 0, n, 0.0, 1.0)
    L = np.floor(np.exp(u * u * 9.5)).astype(np.int64) - 1      # 0 .. ~13000, mostly short
    L[::97] = 0
    L[5::211] = wave
    L[7::223] = lt
    L[9::227] = lt + 1
    rowptr = np.zeros(n + 1, dtype=np.int32)
    np.cumsum(L, out=rowptr[1:])
    part = oracle.partition(rowptr, wave, lt, tile)
    off, perm, lp, tr, tn = _independent_partition(rowptr, wave, lt, tile)
    assert np.array_equal(part["bin_offset"], off)
    assert np.array_equal(part["row_perm"], perm)
    assert np.array_equal(part["long_off"], lp)
    assert np.array_equal(part["tile_row"], tr)
    assert np.array_equal(part["tile_nz"], tn)


def test_partition_invariants_on_power_law_workload():
    w = gen.workload(4, {"n": 1 << 17, "cap": 50000})
    part = oracle.partition(w.rowptr)
    n = w.nrows
    off, perm = part["bin_offset"], part["row_perm"]
    L = np.diff(w.rowptr)
    assert off[0] == 0 and off[-1] == n and np.all(np.diff(off) >= 0)
    assert np.array_equal(np.sort(perm), np.arange(n))          # bins partition the rows
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
