"""GPU parity of lapis_spmv_transpose (y = alpha*A^T*x + beta*y, the column-wise traversal of
Section 4.2) against the oracle.  The additions into one element come in no fixed order, so the
comparison uses the rounding bound with the entry count of the COLUMN; integer-valued data,
where every order gives the same bits, is compared exactly."""
import numpy as np
import pytest

import gen
import oracle
from helpers import DeviceCsr, assert_close, general_bound, literal_bound
from test_gpu_parity import mixed_lengths, say

pytestmark = pytest.mark.gpu


def check_transpose(dev, rowptr, colidx, vals, ncols, x, alpha=1.0, beta=0.0, y0=None, what=""):
    ref, absATx = oracle.spmv_transpose(rowptr, colidx, vals, ncols, x, alpha, beta, y0)
    got = dev.spmv_transpose(x, alpha, beta, y0)
    assert got.dtype == vals.dtype and got.shape == (ncols,)
    counts = np.bincount(colidx, minlength=ncols) if colidx.size else np.zeros(ncols, dtype=np.int64)
    assert_close(got, ref, general_bound(counts, absATx, vals.dtype, alpha, beta, y0), what)
    return got


@pytest.mark.parametrize("dtype", [np.float64, np.float32])
@pytest.mark.parametrize("n,ncols,longest,srt,dup", [
    (1, 1, 1, True, False),
    (5, 3, 3, True, False),
    (257, 100, 100, True, False),
    (4099, 5000, 700, False, False),          # two entry tiles and a ragged tail; unsorted
    (20000, 777, 777, True, True),            # duplicates, many tiles, heavy column reuse
    (3001, 40000, 30000, True, False),        # rows longer than an entry tile
])
def test_transpose_general_matrices(dtype, n, ncols, longest, srt, dup):
    say(f"transpose general n={n} ncols={ncols} longest={longest} {np.dtype(dtype).name}")
    L = np.minimum(mixed_lengths(n, 31, longest), ncols)
    if n < 10:
        L = np.minimum(np.arange(n) % (longest + 1), ncols)
    rowptr, colidx, vals = gen.random_csr(n, ncols, L, 4321, dtype, sorted_cols=srt, allow_duplicates=dup)
    x = gen.uniform(21, gen.STREAM_X, n).astype(dtype)
    y0 = gen.uniform(21, gen.STREAM_Y0, ncols).astype(dtype)
    dev = DeviceCsr(n, ncols, rowptr, colidx, vals)
    try:
        check_transpose(dev, rowptr, colidx, vals, ncols, x, what="alpha=1 beta=0")
        check_transpose(dev, rowptr, colidx, vals, ncols, x, -1.5, 0.25, y0, what="alpha=-1.5 beta=0.25")
        check_transpose(dev, rowptr, colidx, vals, ncols, x, 0.0, 2.0, y0, what="alpha=0 beta=2")
    finally:
        dev.close()


@pytest.mark.parametrize("dtype", [np.float64, np.float32])
def test_transpose_exact_on_small_integers(dtype):
    say(f"transpose exact ints {np.dtype(dtype).name}")
    n, ncols = 6000, 900
    L = np.minimum(mixed_lengths(n, 32, 500), ncols)
    rowptr, colidx, vals = gen.random_csr(n, ncols, L, 99, dtype, small_ints=True)
    x = np.floor(gen.uniform(22, gen.STREAM_X, n, -8.0, 9.0)).astype(dtype)
    y0 = np.floor(gen.uniform(22, gen.STREAM_Y0, ncols, -8.0, 9.0)).astype(dtype)
    dev = DeviceCsr(n, ncols, rowptr, colidx, vals)
    try:
        ref, _ = oracle.spmv_transpose(rowptr, colidx, vals, ncols, x, 2.0, -3.0, y0)
        assert np.array_equal(dev.spmv_transpose(x, 2.0, -3.0, y0), ref)
    finally:
        dev.close()


def test_transpose_degenerate_shapes():
    say("transpose degenerate shapes")
    # long runs of empty rows between entries: the tile's row range does not fit the LDS window
    n, ncols = 50000, 64
    L = np.zeros(n, dtype=np.int64)
    L[::5000] = 40
    L[-1] = 64
    rowptr, colidx, vals = gen.random_csr(n, ncols, L, 5, np.float64)
    x = gen.uniform(23, gen.STREAM_X, n)
    dev = DeviceCsr(n, ncols, rowptr, colidx, vals)
    try:
        check_transpose(dev, rowptr, colidx, vals, ncols, x, what="sparse rows")
    finally:
        dev.close()
    # no entries at all: y = beta*y, NaN in y ignored when beta == 0
    rowptr = np.zeros(8, dtype=np.int32)
    dev = DeviceCsr(7, 11, rowptr, np.zeros(0, dtype=np.int32), np.zeros(0))
    try:
        assert np.array_equal(dev.spmv_transpose(np.ones(7)), np.zeros(11))
        y0 = np.arange(11.0)
        assert np.array_equal(dev.spmv_transpose(np.ones(7), 1.0, -2.0, y0), -2.0 * y0)
    finally:
        dev.close()
    # beta == 0 ignores what y held (NaN), empty columns give exactly 0
    rowptr = np.array([0, 2, 2, 3], dtype=np.int32)
    colidx = np.array([0, 3, 3], dtype=np.int32)
    vals = np.array([1.0, 2.0, 4.0])
    dev = DeviceCsr(3, 5, rowptr, colidx, vals)
    try:
        got = dev.spmv_transpose(np.array([1.0, 100.0, -1.0]), 2.0, 0.0)
        assert np.array_equal(got, [2.0, 0.0, 0.0, -4.0, 0.0])
    finally:
        dev.close()


def test_transpose_symmetric_matrix_matches_forward_product():
    """For the symmetric 5-point Laplacian, A^T x is A x: the two entry points, which share no
    kernel, agree within the bound."""
    say("transpose symmetric")
    w = gen.workload(1)
    dev = DeviceCsr(w.nrows, w.ncols, w.rowptr, w.colidx, w.vals)
    try:
        fwd = dev.spmv(w.x)
        _, absAx = oracle.spmv(w.rowptr, w.colidx, w.vals, w.x)
        tr = dev.spmv_transpose(w.x)
        assert_close(tr, fwd, 2 * general_bound(np.diff(w.rowptr), absAx, np.float64, 1.0, 0.0, None))
    finally:
        dev.close()


@pytest.mark.parametrize("cfg", [2, 4])
def test_transpose_full_workloads(cfg):
    say(f"transpose workload {cfg} full size")
    w = gen.workload(cfg)
    x = gen.uniform(24, gen.STREAM_X, w.nrows).astype(w.vals.dtype)
    dev = DeviceCsr(w.nrows, w.ncols, w.rowptr, w.colidx, w.vals)
    try:
        check_transpose(dev, w.rowptr, w.colidx, w.vals, w.ncols, x, what=w.name)
    finally:
        dev.close()


# ---- explicit transposition on the device -----------------------------------
def check_transposed_handle(rowptr, colidx, vals, nrows, ncols, x=None, what=""):
    """Arrays of the transposed handle are bit-identical to the oracle's transposition, its
    partition to the oracle's partition of those arrays, and products on it match the oracle."""
    dev = DeviceCsr(nrows, ncols, rowptr, colidx, vals)
    t = dev.mat.transposed()
    try:
        ref = oracle.transpose(rowptr, colidx, vals, ncols)
        got = t.arrays()
        for name, g, r in zip(("rowptr", "colidx", "vals"), got, ref):
            assert g.dtype == r.dtype and np.array_equal(g, r), f"{what}: transposed {name} differs"
        part, pref = t.partition(), oracle.partition(ref[0], colidx=ref[1], ncols=nrows, itemsize=vals.itemsize)
        for key in ("stream_chunks", "stream_offset", "bin_offset", "row_perm", "long_off", "tile_row", "tile_nz"):
            assert np.array_equal(part[key], pref[key]), f"{what}: partition field {key} of the transposed handle differs"
        if x is not None:
            import torch
            dx = torch.from_numpy(x).cuda()
            dy = torch.full((ncols,), float("nan"), dtype=dx.dtype, device="cuda:0")
            t.spmv(dx, dy)
            torch.cuda.synchronize()
            yref, absATx = oracle.spmv_transpose(rowptr, colidx, vals, ncols, x)
            counts = np.bincount(colidx, minlength=ncols) if colidx.size else np.zeros(ncols, dtype=np.int64)
            assert_close(dy.cpu().numpy(), yref, literal_bound(counts, absATx, vals.dtype), what)
    finally:
        t.close()
        dev.close()


@pytest.mark.parametrize("dtype", [np.float64, np.float32])
@pytest.mark.parametrize("n,ncols,longest,srt,dup", [
    (1, 1, 1, True, False),
    (5, 3, 3, True, False),
    (257, 100, 100, True, False),
    (4099, 5000, 700, False, False),
    (20000, 777, 777, True, True),            # columns of about 2000 entries: the in-memory sort
    (3001, 40000, 30000, True, False),
    (30000, 1500, 1024, False, True),         # columns around the LDS / memory sort threshold
])
def test_transposed_handle_general_matrices(dtype, n, ncols, longest, srt, dup):
    say(f"transposed handle n={n} ncols={ncols} longest={longest} {np.dtype(dtype).name}")
    L = np.minimum(mixed_lengths(n, 33, longest), ncols)
    if n < 10:
        L = np.minimum(np.arange(n) % (longest + 1), ncols)
    rowptr, colidx, vals = gen.random_csr(n, ncols, L, 4322, dtype, sorted_cols=srt, allow_duplicates=dup)
    x = gen.uniform(25, gen.STREAM_X, n).astype(dtype)
    check_transposed_handle(rowptr, colidx, vals, n, ncols, x, what="general")


def test_transposed_handle_degenerate_shapes():
    say("transposed handle degenerate shapes")
    z = np.zeros(0, dtype=np.int32)
    check_transposed_handle(np.zeros(8, dtype=np.int32), z, np.zeros(0), 7, 11, np.ones(7), "no entries")
    check_transposed_handle(np.zeros(1, dtype=np.int32), z, np.zeros(0), 0, 5, None, "no rows")
    check_transposed_handle(np.zeros(4, dtype=np.int32), z, np.zeros(0), 3, 0, None, "no columns")
    # one dense column of 5000 entries and one dense row: a single long column, sorted in memory
    n, ncols = 5000, 3000
    L = np.ones(n, dtype=np.int64)
    L[17] = ncols
    rowptr, colidx, vals = gen.random_csr(n, ncols, L, 6, np.float64)
    single = np.flatnonzero(np.diff(rowptr) == 1)
    colidx[rowptr[single]] = 7                       # every one-entry row sits in column 7
    check_transposed_handle(rowptr, colidx, vals, n, ncols, gen.uniform(26, gen.STREAM_X, n), "dense column")
    # empty columns between occupied ones, entries only in the last rows
    n, ncols = 4000, 100000
    L = np.zeros(n, dtype=np.int64)
    L[-3:] = 900
    rowptr, colidx, vals = gen.random_csr(n, ncols, L, 8, np.float32)
    check_transposed_handle(rowptr, colidx, vals, n, ncols, gen.uniform(27, gen.STREAM_X, n).astype(np.float32), "sparse columns")


@pytest.mark.parametrize("cfg", [1, 2, 4])
def test_transposed_handle_full_workloads(cfg):
    say(f"transposed handle workload {cfg} full size")
    w = gen.workload(cfg)
    x = gen.uniform(28, gen.STREAM_X, w.nrows).astype(w.vals.dtype)
    check_transposed_handle(w.rowptr, w.colidx, w.vals, w.nrows, w.ncols, x, w.name)


def test_transposing_twice_restores_sorted_matrices():
    say("transposed handle twice")
    w = gen.workload(4, {"n": 1 << 16, "cap": 20000})       # long rows become long columns on the way back
    dev = DeviceCsr(w.nrows, w.ncols, w.rowptr, w.colidx, w.vals)
    t = dev.mat.transposed()
    tt = t.transposed()
    try:
        for g, r in zip(tt.arrays(), (w.rowptr, w.colidx, w.vals)):
            assert np.array_equal(g, r)
    finally:
        tt.close(); t.close(); dev.close()
