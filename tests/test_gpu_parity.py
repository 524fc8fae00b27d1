"""GPU parity: the HIP library, called through its C ABI, against the CPU oracle
on the same seeded inputs.  Index structures must match bit for bit; floating
point per element within 8*nnz_row*eps*(|A||x|)_i (eps = 2^-53 double, 2^-24
float), extended by the alpha/beta terms for the generic unit cases."""
import sys

import numpy as np
import pytest

import gen
import oracle
from helpers import DeviceCsr, assert_close, general_bound, literal_bound

pytestmark = pytest.mark.gpu


def say(msg):
    print(f"[case] {msg}", file=sys.stderr, flush=True)


def check_half_bandwidth(dev, rowptr, colidx):
    rows = np.repeat(np.arange(rowptr.size - 1, dtype=np.int64), np.diff(rowptr))
    expect = int(np.abs(colidx.astype(np.int64) - rows).max()) if colidx.size else 0
    assert dev.L.lapis_csr_half_bandwidth(dev.mat.handle) == expect


def check_index16(dev):
    """The 16-bit column offsets of the handle against the oracle's, bit for bit."""
    ref = oracle.index16(dev.h_rowptr, dev.h_colidx)
    got = dev.index16()
    assert got["enabled"] == ref["enabled"] and got["narrow_entries"] == ref["narrow_entries"]
    assert got["framed_entries"] == ref["framed_entries"]
    if ref["enabled"]:
        assert got["chunk_base"].dtype == np.int32 and got["col16"].dtype == np.uint16
        assert np.array_equal(got["chunk_base"], ref["chunk_base"]), "chunk_base differs"
        assert np.array_equal(got["frame_table"], ref["frame_table"]), "frame_table differs"
        assert np.array_equal(got["col16"], ref["col16"]), "col16 differs"
    return ref["enabled"]


def check_patterns(dev):
    """The row patterns of the handle against the oracle's, bit for bit."""
    ref = oracle.row_patterns(dev.h_rowptr, dev.h_colidx, dev.ncols, np.dtype(dev.np_dtype).itemsize)
    got = dev.patterns()
    assert got["enabled"] == ref["enabled"] and got["entries"] == ref["entries"]
    assert got["pool_size"] == ref["pool"].size
    if ref["enabled"]:
        assert got["pat_off"].dtype == np.int32 and got["row_pat"].dtype == np.uint16
        assert np.array_equal(got["pat_off"], ref["pat_off"]), "pat_off differs"
        assert np.array_equal(got["row_pat"], ref["row_pat"]), "row_pat differs"
        assert np.array_equal(got["pool"], ref["pool"]), "pattern pool differs"
    return ref["enabled"]


def check_share_classes(dev, part):
    """How lapis_spmm treats every chunk against the oracle's reading of the same rule (all chunks, or
    4000 of them spread over the matrix)."""
    pats = oracle.row_patterns(dev.h_rowptr, dev.h_colidx, dev.ncols, np.dtype(dev.np_dtype).itemsize)
    nchunks = (dev.nrows + 31) // 32
    only = None if nchunks <= 6000 else sorted(set(np.linspace(0, nchunks - 1, 4000).astype(np.int64).tolist()))
    ref = oracle.share_classes(dev.h_rowptr, part, pats, only=only)
    got = dev.share_classes()
    assert (got is None) == (ref is None)
    if ref is not None:
        assert got.dtype == np.int32 and got.size == nchunks
        sel = ref >= 0
        assert np.array_equal(got[sel], ref[sel]), f"share classes differ at chunks {np.flatnonzero(sel & (got != ref))[:8]}"
    return got


def check_partition(dev, rowptr):
    assert rowptr is dev.h_rowptr or np.array_equal(rowptr, dev.h_rowptr)
    ref = oracle.partition(rowptr, colidx=dev.h_colidx, ncols=dev.ncols, itemsize=np.dtype(dev.np_dtype).itemsize)
    got = dev.partition()
    for key in ("stream_chunks", "stream_offset", "bin_offset", "row_perm", "long_off", "tile_row", "tile_nz"):
        assert got[key].dtype == np.int32
        assert np.array_equal(got[key], ref[key]), f"partition field {key} differs"
    check_index16(dev)
    check_patterns(dev)
    check_share_classes(dev, ref)


def check_split(dev, rowptr, colidx, ncols, itemsize, expect_on=None):
    ref = oracle.split_partition(rowptr, colidx, ncols, itemsize)
    got = dev.split()
    if expect_on is not None:
        assert (ref["num_blocks"] > 0) == expect_on
    for key in ("num_blocks", "block_width", "num_split_rows", "num_huge_rows"):
        assert got[key] == ref[key], f"split field {key} differs"
    if ref["num_blocks"]:
        for key in ("num_fblocks", "fblock_width"):
            assert got[key] == ref[key], f"split field {key} differs"
        for key in ("split_rows", "huge_rows", "cut", "fcut", "bin_offset", "row_perm", "long_off", "tile_row",
                    "tile_nz"):
            assert got[key].dtype == np.int32
            assert np.array_equal(got[key], ref[key]), f"split field {key} differs"
    return ref


def check_spmv(dev, rowptr, colidx, vals, x, alpha=1.0, beta=0.0, y0=None, literal=False, what="",
               paper_shape=False):
    ref, absAx = oracle.spmv(rowptr, colidx, vals, x, alpha, beta, y0)
    got = dev.spmv(x, alpha, beta, y0, paper_shape=paper_shape)
    nnz_row = np.diff(rowptr)
    tol = literal_bound(nnz_row, absAx, vals.dtype) if literal else general_bound(
        nnz_row, absAx, vals.dtype, alpha, beta, y0)
    assert got.dtype == vals.dtype
    assert_close(got, ref, tol, what)
    empty = nnz_row == 0
    if empty.any():  # rows without entries: exactly beta*y0, +0 when beta == 0
        assert np.array_equal(got[empty], ref[empty])
        if beta == 0.0:
            assert not np.any(np.signbit(got[empty]))
    return got


def check_spmm(dev, rowptr, colidx, vals, X, alpha=1.0, beta=0.0, Y0=None, literal=False, what="",
               ldx=None, ldy=None):
    ref, absAX = oracle.spmm(rowptr, colidx, vals, X, alpha, beta, Y0)
    got = dev.spmm(X, alpha, beta, Y0, ldx, ldy)
    nnz_row = np.diff(rowptr)[:, None]
    tol = literal_bound(nnz_row, absAX, vals.dtype) if literal else general_bound(
        nnz_row, absAX, vals.dtype, alpha, beta, Y0)
    assert_close(got, ref, tol, what)
    return got


# ---------------------------------------------------------------------------
# small general matrices: every bin, ragged tails, duplicates, unsorted columns
# ---------------------------------------------------------------------------
def mixed_lengths(n, seed, longest):
    u = gen.uniform(seed, 0, n, 0.0, 1.0)
    L = np.floor(np.exp(u ** 3 * np.log(longest + 1))).astype(np.int64) - 1
    L[::53] = 0
    for i, v in enumerate([1, 2, 3, 4, 5, 8, 9, 16, 17, 32, 33, 63, 64, 65, 127, 128, 129, 4095, 4096, 4097]):
        if v <= longest and 7 + 11 * i < n:
            L[7 + 11 * i] = v
    return L


@pytest.mark.parametrize("dtype", [np.float64, np.float32])
@pytest.mark.parametrize("n,ncols,longest,srt,dup", [
    (1, 1, 1, True, False),
    (5, 3, 3, True, False),
    (777, 5000, 70, True, False),
    (3001, 20000, 20000, True, False),       # includes rows beyond the long threshold
    (3001, 4000, 300, False, True),          # duplicates, unsorted
    (40, 30000, 30000, False, False),        # few rows, mostly long, unsorted
])
def test_spmv_general_matrices(dtype, n, ncols, longest, srt, dup):
    say(f"spmv general n={n} ncols={ncols} longest={longest} sorted={srt} dup={dup} {np.dtype(dtype).name}")
    L = np.minimum(mixed_lengths(n, 40 + n, longest), ncols)
    rowptr, colidx, vals = gen.random_csr(n, ncols, L, 900 + n, dtype, sorted_cols=srt, allow_duplicates=dup)
    x = gen.uniform(31, gen.STREAM_X, ncols).astype(dtype)
    y0 = gen.uniform(31, gen.STREAM_Y0, n).astype(dtype)
    dev = DeviceCsr(n, ncols, rowptr, colidx, vals)
    try:
        check_partition(dev, rowptr)
        check_spmv(dev, rowptr, colidx, vals, x, what="alpha=1 beta=0")
        check_spmv(dev, rowptr, colidx, vals, x, -2.5, 0.75, y0, what="alpha=-2.5 beta=0.75")
        check_spmv(dev, rowptr, colidx, vals, x, 0.0, 2.0, y0, what="alpha=0")
        check_spmv(dev, rowptr, colidx, vals, x, what="paper shape", paper_shape=True)
        check_spmv(dev, rowptr, colidx, vals, x, -2.5, 0.75, y0, what="paper shape, alpha beta", paper_shape=True)
        a = check_spmv(dev, rowptr, colidx, vals, x, 3.0, 0.0, what="run 1")
        b = dev.spmv(x, 3.0, 0.0)
        assert np.array_equal(a, b), "two runs differ: result depends on scheduling"
    finally:
        dev.close()


def test_spmv_exact_small_integers():
    """Integer data: any summation order is exact, so the GPU must match bit for bit."""
    n, ncols = 2000, 9000
    L = np.minimum(mixed_lengths(n, 5, 9000), ncols)
    for dtype in (np.float64, np.float32):
        rowptr, colidx, vals = gen.random_csr(n, ncols, L, 77, dtype, small_ints=True)
        x = np.floor(gen.uniform(3, gen.STREAM_X, ncols, -8.0, 9.0)).astype(dtype)
        y0 = np.floor(gen.uniform(3, gen.STREAM_Y0, n, -8.0, 9.0)).astype(dtype)
        dev = DeviceCsr(n, ncols, rowptr, colidx, vals)
        try:
            ref, _ = oracle.spmv(rowptr, colidx, vals, x, 2.0, -3.0, y0)
            assert np.array_equal(dev.spmv(x, 2.0, -3.0, y0), ref)
        finally:
            dev.close()


def test_beta_zero_ignores_old_y_and_degenerate_shapes():
    # beta == 0: NaN in the old y must not leak (DeviceCsr.spmv pre-fills y with NaN)
    w = gen.workload(1)
    dev = DeviceCsr(w.nrows, w.ncols, w.rowptr, w.colidx, w.vals)
    try:
        got = dev.spmv(w.x)
        assert np.all(np.isfinite(got))
    finally:
        dev.close()
    # rows but no entries at all
    rowptr = np.zeros(101, dtype=np.int32)
    dev = DeviceCsr(100, 7, rowptr, np.empty(0, np.int32), np.empty(0, np.float64))
    try:
        check_partition(dev, rowptr)
        y0 = gen.uniform(1, gen.STREAM_Y0, 100)
        assert np.array_equal(dev.spmv(np.ones(7), 1.0, 0.0), np.zeros(100))
        assert np.array_equal(dev.spmv(np.ones(7), 1.0, -0.5, y0), -0.5 * y0)
        X = gen.uniform(1, gen.STREAM_X, 7 * 3).reshape(7, 3)
        assert np.array_equal(dev.spmm(X), np.zeros((100, 3)))
    finally:
        dev.close()
    # no rows
    dev = DeviceCsr(0, 5, np.zeros(1, dtype=np.int32), np.empty(0, np.int32), np.empty(0, np.float32))
    try:
        part = dev.partition()
        assert np.all(part["bin_offset"] == 0)
        assert dev.spmv(np.ones(5, dtype=np.float32)).size == 0
    finally:
        dev.close()


def test_create_rejects_bad_structure_on_device():
    import torch
    import paper_2509_25605_amd as L
    rowptr = torch.tensor([0, 2, 1, 3], dtype=torch.int32, device="cuda:0")      # decreasing
    colidx = torch.tensor([0, 1, 2], dtype=torch.int32, device="cuda:0")
    vals = torch.ones(3, dtype=torch.float64, device="cuda:0")
    with pytest.raises(L.LapisError) as e:
        L.CsrMatrix(3, 3, rowptr, colidx, vals)
    assert e.value.code == L.LAPIS_ERR_INVALID_ARG
    rowptr = torch.tensor([0, 1, 2, 3], dtype=torch.int32, device="cuda:0")
    for bad in (3, -1):                                                           # column out of range
        colidx = torch.tensor([0, bad, 2], dtype=torch.int32, device="cuda:0")
        with pytest.raises(L.LapisError) as e:
            L.CsrMatrix(3, 3, rowptr, colidx, vals)
        assert e.value.code == L.LAPIS_ERR_INVALID_ARG
    rowptr = torch.tensor([1, 1, 2, 3], dtype=torch.int32, device="cuda:0")      # rowptr[0] != 0
    with pytest.raises(L.LapisError):
        L.CsrMatrix(3, 3, rowptr, torch.tensor([0, 1, 2], dtype=torch.int32, device="cuda:0"), vals)
    A = L.CsrMatrix(3, 3, torch.tensor([0, 1, 2, 3], dtype=torch.int32, device="cuda:0"),
                    torch.tensor([0, 1, 2], dtype=torch.int32, device="cuda:0"), vals)
    x = torch.ones(3, dtype=torch.float64, device="cuda:0")
    for k, ldx, ldy in ((0, 4, 4), (-1, 4, 4), (4, 3, 4), (4, 4, 3)):
        with pytest.raises(L.LapisError) as e:
            L.lapis_spmm(A.handle, k, 1.0, x, ldx, 0.0, x, ldy)
        assert e.value.code == L.LAPIS_ERR_INVALID_ARG
    A.close()



# ---------------------------------------------------------------------------
# stream chunks: windows, alignment offsets, the matrix's last nnz % 4 entries
# ---------------------------------------------------------------------------
STREAM_LAYOUTS = {
    # chunk-by-chunk row lengths (32 rows per chunk unless ragged)
    "tail1": [[9] * 31 + [10]],                                  # nnz % 4 == 1... see below
    "tail2": [[9] * 31 + [11]],
    "tail3": [[9] * 31 + [12]],
    "dense": [[64] * 32, [64] * 32],                             # 2048 entries per chunk: 2 windows
    "offset": [[3] * 31 + [70], [64] * 32, [33] * 32, [17] * 32, [8] * 32],   # odd prefix, mixed
    "ragged": [[27] * 32, [27] * 32, [27] * 11],                 # last chunk has 11 rows (297 entries)
    "mixed": [[8] * 32, [0] * 16 + [16] * 16, [1] * 32, [64] + [7] * 31, [5] * 32, [40] * 7],
    "classes": [[81] * 32, [128] + [3] * 31, [129] * 32, [256] * 32, [300, 0, 512] + [77] * 29, [513] + [9] * 31,
                [345] + [60] * 10],
}


@pytest.mark.parametrize("dtype", [np.float64, np.float32])
@pytest.mark.parametrize("mix", ["small_below", "small_between", "two_small", "too_many", "scattered16"])
def test_spmv_small_stream_classes_ride_with_the_next_class(mix, dtype):
    """Stream classes with few chunks are launched with the next class up that has chunks (its lane
    groups, its kernel variant) when they are at most an eighth of it; the results must not care."""
    say(f"stream classes {mix} {np.dtype(dtype).name}")
    # (row length, number of chunks) per population; rows of 20 / 60 / 100 / 200 entries make chunks of class 1 / 2 / 3 / 4
    chunks = {
        "small_below": [(20, 3), (60, 60)],               # class 1 rides with class 2
        "small_between": [(20, 80), (60, 4), (100, 70)],  # class 2 rides with class 3; class 1 is too large to
        "two_small": [(20, 2), (60, 3), (200, 64)],       # classes 1 and 2 ride with class 4
        "too_many": [(20, 30), (100, 60)],                # half as many: a launch of its own
        "scattered16": [(20, 4), (100, 70)],              # few columns: 16-bit offsets, grouped wavefronts above class 1
    }[mix]
    L = np.concatenate([np.full(32 * c, length, dtype=np.int64) for length, c in chunks])
    order = np.argsort(gen.uniform(17, 0, L.size // 32, 0.0, 1.0), kind="stable")     # shuffle whole chunks
    L = L.reshape(-1, 32)[order].ravel()
    n = L.size
    ncols = 200_000                                       # x within one column block: no chunk is demoted
    if mix == "scattered16":
        ncols = 3000
        rowptr, colidx, vals = gen.random_csr(n, ncols, L, 19, dtype)
    else:
        rowptr, colidx, vals = gen.random_csr(n, ncols, L, 19, dtype)
    x = gen.uniform(20, gen.STREAM_X, ncols).astype(dtype)
    y0 = gen.uniform(20, gen.STREAM_Y0, n).astype(dtype)
    dev = DeviceCsr(n, ncols, rowptr, colidx, vals)
    try:
        part = dev.partition()
        sizes = np.diff(part["stream_offset"])
        assert np.count_nonzero(sizes) >= 2, f"class sizes {sizes}: the case needs several stream classes"
        check_partition(dev, rowptr)
        check_spmv(dev, rowptr, colidx, vals, x, what="alpha=1 beta=0")
        check_spmv(dev, rowptr, colidx, vals, x, 0.75, -1.25, y0, what="alpha=0.75 beta=-1.25")
    finally:
        dev.close()


@pytest.mark.parametrize("dtype", [np.float64, np.float32])
@pytest.mark.parametrize("layout", sorted(STREAM_LAYOUTS))
def test_spmv_stream_chunks(layout, dtype):
    say(f"stream layout={layout} {np.dtype(dtype).name}")
    L = np.array(sum(STREAM_LAYOUTS[layout], []), dtype=np.int64)
    n, ncols = L.size, 5000
    rowptr, colidx, vals = gen.random_csr(n, ncols, L, 4242, dtype, sorted_cols=(layout != "mixed"))
    x = gen.uniform(77, gen.STREAM_X, ncols).astype(dtype)
    y0 = gen.uniform(77, gen.STREAM_Y0, n).astype(dtype)
    dev = DeviceCsr(n, ncols, rowptr, colidx, vals)
    try:
        part = dev.partition()
        assert part["stream_chunks"].size > 0
        check_partition(dev, rowptr)
        check_spmv(dev, rowptr, colidx, vals, x, what="alpha=1 beta=0")
        check_spmv(dev, rowptr, colidx, vals, x, 0.5, -1.5, y0, what="alpha=0.5 beta=-1.5")
        X = gen.uniform(78, gen.STREAM_X, ncols * 16).astype(dtype).reshape(ncols, 16)
        check_spmm(dev, rowptr, colidx, vals, X, what="spmm k=16")
    finally:
        dev.close()
    if layout.startswith("tail"):
        assert int(rowptr[-1]) % 4 == int(layout[-1])


def test_unaligned_arrays_fall_back_to_bins():
    """colidx / vals that are not 16-byte aligned: no stream chunks, same results."""
    import torch
    import paper_2509_25605_amd as L
    w = gen.workload(2, {"nx": 16, "ny": 16, "nz": 16})
    ref, absAx = oracle.spmv(w.rowptr, w.colidx, w.vals, w.x)
    pad_c = torch.zeros(w.nnz + 1, dtype=torch.int32, device="cuda:0")
    pad_v = torch.zeros(w.nnz + 1, dtype=torch.float64, device="cuda:0")
    pad_c[1:] = torch.from_numpy(w.colidx).cuda()
    pad_v[1:] = torch.from_numpy(w.vals).cuda()
    rowptr = torch.from_numpy(w.rowptr).cuda()
    x = torch.from_numpy(w.x).cuda()
    for colidx, vals, expect_stream in ((pad_c[1:], pad_v[1:], False), (pad_c[1:].clone(), pad_v[1:].clone(), True)):
        y = torch.full((w.nrows,), float("nan"), dtype=torch.float64, device="cuda:0")
        A = L.CsrMatrix(w.nrows, w.ncols, rowptr, colidx, vals)
        assert (A.partition()["stream_chunks"].size > 0) == expect_stream
        A.spmv(x, y)
        torch.cuda.synchronize()
        A.close()
        assert_close(y.cpu().numpy(), ref, literal_bound(np.diff(w.rowptr), absAx, np.float64))


# ---------------------------------------------------------------------------
# column split: wide matrices whose x exceeds the split block size
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("dtype", [np.float64, np.float32])
@pytest.mark.parametrize("srt", [True, False])
def test_spmv_column_split(dtype, srt):
    say(f"column split sorted={srt} {np.dtype(dtype).name}")
    n, ncols = 3000, 3 * (1 << 19) + 12345          # 12.6 MB (f64) / 6.3 MB (f32) of x
    L = mixed_lengths(n, 71, 40000)
    L[3::17] = 65 + (np.arange(L[3::17].size) * 61) % 4000   # plenty of rows in bin 8
    L = np.minimum(L, ncols)
    rowptr, colidx, vals = gen.random_csr(n, ncols, L, 555, dtype, sorted_cols=srt)
    x = gen.uniform(12, gen.STREAM_X, ncols).astype(dtype)
    y0 = gen.uniform(12, gen.STREAM_Y0, n).astype(dtype)
    dev = DeviceCsr(n, ncols, rowptr, colidx, vals)
    try:
        check_partition(dev, rowptr)
        check_split(dev, rowptr, colidx, ncols, np.dtype(dtype).itemsize, expect_on=srt)
        check_spmv(dev, rowptr, colidx, vals, x, what="alpha=1 beta=0")
        check_spmv(dev, rowptr, colidx, vals, x, -1.5, 0.25, y0, what="alpha=-1.5 beta=0.25")
        a = dev.spmv(x, 2.0, 0.0)
        assert np.array_equal(a, dev.spmv(x, 2.0, 0.0)), "two runs differ"
        X = gen.uniform(13, gen.STREAM_X, ncols * 4).astype(dtype).reshape(ncols, 4)
        check_spmm(dev, rowptr, colidx, vals, X, what="spmm k=4")
    finally:
        dev.close()


def test_column_split_looks_only_at_the_split_rows():
    """Unsorted columns in rows of at most 64 entries do not switch the split off; a single
    descent inside one split row does."""
    say("column split with unsorted short rows")
    n, ncols = 2000, (1 << 19) + 777
    L = mixed_lengths(n, 72, 30000)
    L[5::13] = 65 + (np.arange(L[5::13].size) * 37) % 3000
    L = np.minimum(L, ncols)
    rowptr, colidx, vals = gen.random_csr(n, ncols, L, 556, np.float64, sorted_cols=True)
    x = gen.uniform(14, gen.STREAM_X, ncols)
    short = np.flatnonzero((np.diff(rowptr) >= 2) & (np.diff(rowptr) <= 64))
    for r in short[::3]:                             # reverse the columns of some short rows
        a, b = rowptr[r], rowptr[r + 1]
        colidx[a:b] = colidx[a:b][::-1].copy()
        vals[a:b] = vals[a:b][::-1].copy()
    dev = DeviceCsr(n, ncols, rowptr, colidx, vals)
    try:
        check_split(dev, rowptr, colidx, ncols, 8, expect_on=True)
        check_spmv(dev, rowptr, colidx, vals, x, what="short rows unsorted")
    finally:
        dev.close()
    long_row = int(np.flatnonzero(np.diff(rowptr) > 4096)[0])
    a = rowptr[long_row] + 2000
    colidx[a], colidx[a + 1] = colidx[a + 1], colidx[a]      # the last pair of a check tile or not: any place
    dev = DeviceCsr(n, ncols, rowptr, colidx, vals)
    try:
        check_split(dev, rowptr, colidx, ncols, 8, expect_on=False)
        check_spmv(dev, rowptr, colidx, vals, x, what="one descent in a long row")
    finally:
        dev.close()


def _banded_and_random(n, ncols, per_row, narrow_rows, seed, dtype):
    """Rows [0, narrow_rows) get columns row, row+1, ... (a band); the rest keeps random columns."""
    rowptr, colidx, vals = gen.random_csr(n, ncols, np.full(n, per_row), seed, dtype)
    band = (np.arange(narrow_rows)[:, None] + np.arange(per_row)[None, :]) % ncols
    colidx[: narrow_rows * per_row] = np.sort(band, axis=1).ravel().astype(np.int32)
    return rowptr, colidx, vals


@pytest.mark.parametrize("dtype", [np.float64, np.float32])
@pytest.mark.parametrize("narrow_rows,expect_on", [(6400, True), (4480, True), (1600, False), (0, False)])
def test_index16_mixed_narrow_and_wide_chunks(dtype, narrow_rows, expect_on):
    """Chunks with 16-bit offsets and chunks with 32-bit columns in one launch (and the structure
    dropped when the narrow chunks hold less than half of the entries)."""
    say(f"index16 mixed narrow_rows={narrow_rows} {np.dtype(dtype).name}")
    n, ncols = 6400, 1 << 20
    rowptr, colidx, vals = _banded_and_random(n, ncols, 16, narrow_rows, 808, dtype)
    x = gen.uniform(15, gen.STREAM_X, ncols).astype(dtype)
    dev = DeviceCsr(n, ncols, rowptr, colidx, vals)
    try:
        check_partition(dev, rowptr)
        assert check_index16(dev) == expect_on
        if expect_on:
            base = dev.index16()["chunk_base"]
            assert np.all(base[: narrow_rows // 32] >= 0) and np.all(base[narrow_rows // 32:] == -1)
        check_spmv(dev, rowptr, colidx, vals, x, what="spmv")
        X = gen.uniform(16, gen.STREAM_X, ncols * 8).astype(dtype).reshape(ncols, 8)
        check_spmm(dev, rowptr, colidx, vals, X, what="spmm k=8")
    finally:
        dev.close()


def test_index16_framed_chunks():
    """Stencil planes of 200 x 200: chunks span 2*(200^2 + 201) columns, far beyond 2^16, but touch
    only 9 runs of columns: frame tables.  Also a matrix mixing narrow, framed and plain chunks."""
    say("index16 framed")
    w = gen.workload(2, {"nx": 200, "ny": 200, "nz": 12})
    dev = DeviceCsr(w.nrows, w.ncols, w.rowptr, w.colidx, w.vals)
    try:
        check_partition(dev, w.rowptr)
        assert check_index16(dev) and dev.index16()["framed_entries"] > 0
        check_spmv(dev, w.rowptr, w.colidx, w.vals, w.x, literal=True, what="stencil 200x200x12")
        X = gen.uniform(32, gen.STREAM_X, w.ncols * 16).reshape(w.ncols, 16)
        check_spmm(dev, w.rowptr, w.colidx, w.vals, X, what="spmm k=16")
    finally:
        dev.close()
    for dtype in (np.float64, np.float32):
        n, ncols, per = 9600, 1 << 22, 16
        rowptr, colidx, vals = _banded_and_random(n, ncols, per, 3200, 810, dtype)   # rows 0..3199 narrow
        # rows 3200..6399: four clusters of four columns far apart (4 frames per row, few per chunk)
        r = np.arange(3200, 6400)
        clusters = (np.arange(4)[None, :, None] * 700001 + (r[:, None, None] // 64) * 2048 + np.arange(4)[None, None, :])
        colidx[3200 * per:6400 * per] = np.sort(clusters.reshape(3200, per) % ncols, axis=1).ravel().astype(np.int32)
        x = gen.uniform(33, gen.STREAM_X, ncols).astype(dtype)
        dev = DeviceCsr(n, ncols, rowptr, colidx, vals)
        try:
            check_partition(dev, rowptr)
            assert check_index16(dev)
            base = dev.index16()["chunk_base"]
            assert np.all(base[:100] >= 0) and np.all(base[100:200] == -2) and np.all(base[200:] == -1)
            check_spmv(dev, rowptr, colidx, vals, x, what="mixed kinds")
            X = gen.uniform(34, gen.STREAM_X, ncols * 4).astype(dtype).reshape(ncols, 4)
            check_spmm(dev, rowptr, colidx, vals, X, what="mixed kinds spmm k=4")
        finally:
            dev.close()


def _rows_from_diagonals(n, lists, seed, dtype, empty=()):
    """CSR whose row i has the columns i + d for d in lists[i % len(lists)] (stored in that order);
    rows in `empty` have no entries."""
    rows = [[] if i in empty else [i + d for d in lists[i % len(lists)]] for i in range(n)]
    rowptr = np.zeros(n + 1, dtype=np.int32)
    np.cumsum([len(r) for r in rows], out=rowptr[1:])
    colidx = np.array([c for r in rows for c in r], dtype=np.int32)
    vals = gen.uniform(seed, gen.STREAM_VALUES, colidx.size).astype(dtype)
    return rowptr, colidx, vals


@pytest.mark.parametrize("dtype", [np.float64, np.float32])
@pytest.mark.parametrize("kind", ["band9", "band81", "band120", "three_lists", "unsorted_dups", "holes"])
def test_row_patterns_every_chunk_patterned(kind, dtype):
    """Matrices whose stream chunks all have row patterns: the kernels read no column per entry."""
    say(f"row patterns {kind} {np.dtype(dtype).name}")
    n = 3211                                            # ragged last chunk of 11 rows
    empty = ()
    if kind.startswith("band"):
        lists = [list(range(int(kind[4:])))]
    elif kind == "three_lists":
        lists = [list(range(0, 54, 2)), list(range(1, 37, 2)) + [900], list(range(27))]
    elif kind == "unsorted_dups":
        lists = [[5, 0, 5, 2, 700, 3, 3, 1, 64, 9, 8, 7], [0, 1, 2, 3, 4, 5, 6, 7, 8, 9, 10, 11]]
    else:
        lists = [list(range(40))]
        empty = set(range(0, 40)) | set(range(100, 131)) | {n - 1, n - 3}     # a chunk starting with empty rows
    ncols = n + 1000
    rowptr, colidx, vals = _rows_from_diagonals(n, lists, 911, dtype, empty)
    x = gen.uniform(912, gen.STREAM_X, ncols).astype(dtype)
    y0 = gen.uniform(912, gen.STREAM_Y0, n).astype(dtype)
    dev = DeviceCsr(n, ncols, rowptr, colidx, vals)
    try:
        check_partition(dev, rowptr)
        got = dev.patterns()
        assert got["enabled"]
        streams = dev.partition()["stream_chunks"]
        assert streams.size > 0 and np.all(np.diff(got["pat_off"])[streams] > 0)
        check_spmv(dev, rowptr, colidx, vals, x, what="alpha=1 beta=0")
        check_spmv(dev, rowptr, colidx, vals, x, -0.25, 2.0, y0, what="alpha=-0.25 beta=2")
        X = gen.uniform(913, gen.STREAM_X, ncols * 4).astype(dtype).reshape(ncols, 4)
        check_spmm(dev, rowptr, colidx, vals, X, what="spmm k=4")
    finally:
        dev.close()


@pytest.mark.parametrize("dtype", [np.float64, np.float32])
@pytest.mark.parametrize("dof,grid", [(3, (9, 7, 5)), (2, (17, 6, 4)), (4, (8, 5, 5)), (6, (6, 5, 3))])
def test_row_patterns_with_shifts_block_rows(dof, grid, dtype):
    """Several unknowns per grid point: the rows of a point hold the same columns, i.e. one list of
    diagonals moved by 0, -1, -2, ...: the chunk stores the list once and every row carries its shift.
    Structure bit for bit against the oracle, SpMV and SpMM element by element."""
    nx, ny, nz = grid
    say(f"block rows: {dof} unknowns per point, grid {nx}x{ny}x{nz} {np.dtype(dtype).name}")
    rowptr, colidx, vals = gen.block_stencil(nx, ny, nz, dof, 61)
    vals = vals.astype(dtype)
    n = nx * ny * nz * dof
    x = gen.uniform(62, gen.STREAM_X, n).astype(dtype)
    y0 = gen.uniform(62, gen.STREAM_Y0, n).astype(dtype)
    dev = DeviceCsr(n, n, rowptr, colidx, vals)
    try:
        check_partition(dev, rowptr)
        pats = dev.patterns()
        if dof * 27 <= 128:                                     # rows of at most 128 entries can be patterned
            assert pats["enabled"]
            start, shift = oracle.pattern_start_shift(pats["row_pat"])
            assert shift.min() < 0                              # rows that take a stored list moved to the left
        check_spmv(dev, rowptr, colidx, vals, x, what="alpha=1 beta=0")
        check_spmv(dev, rowptr, colidx, vals, x, -1.25, 0.75, y0, what="alpha=-1.25 beta=0.75")
        X = gen.uniform(63, gen.STREAM_X, n * 16).astype(dtype).reshape(n, 16)
        check_spmm(dev, rowptr, colidx, vals, X, what="spmm k=16")
        for j in (0, n // 2, n - 1):                             # a non-finite x[j] reaches exactly the rows with column j
            xi = x.copy()
            xi[j] = np.inf
            ref, _ = oracle.spmv(rowptr, colidx, vals, xi)
            got = dev.spmv(xi)
            assert np.array_equal(np.isfinite(got), np.isfinite(ref))
    finally:
        dev.close()


@pytest.mark.parametrize("dtype", [np.float64, np.float32])
@pytest.mark.parametrize("others", ["narrow", "framed", "plain", "few_patterned"])
def test_row_patterns_beside_other_chunks(others, dtype):
    """Patterned chunks in one launch with chunks that have 16-bit codes, and matrices where a
    class also holds chunks with neither (the patterns are then left unused for that class)."""
    say(f"row patterns beside {others} {np.dtype(dtype).name}")
    n, per = 6400, 16
    patterned_rows = 1600 if others == "few_patterned" else 4480
    ncols = 1 << 22
    rowptr, colidx, vals = gen.random_csr(n, ncols, np.full(n, per), 915, dtype)
    r = np.arange(n)
    # rows below patterned_rows: one list of 16 diagonals; above: random columns near the diagonal
    # (narrow), in four far clusters (framed), or anywhere (neither)
    colidx[: patterned_rows * per] = (r[:patterned_rows, None] + 3 * np.arange(per)[None, :]).ravel().astype(np.int32)
    rest = r[patterned_rows:]
    if others in ("narrow", "few_patterned"):
        jitter = (gen.uniform(916, 5, rest.size * per, 0.0, 1.0) * 3000).astype(np.int64).reshape(rest.size, per)
        colidx[patterned_rows * per:] = np.sort(rest[:, None] + jitter, axis=1).ravel().astype(np.int32)
    elif others == "framed":
        jitter = (gen.uniform(916, 5, rest.size * per, 0.0, 1.0) * 500).astype(np.int64).reshape(rest.size, 4, 4)
        clusters = np.arange(4)[None, :, None] * 900001 + (rest[:, None, None] // 64) * 2048 + jitter
        colidx[patterned_rows * per:] = np.sort(clusters.reshape(rest.size, per), axis=1).ravel().astype(np.int32)
    x = gen.uniform(917, gen.STREAM_X, ncols).astype(dtype)
    dev = DeviceCsr(n, ncols, rowptr, colidx, vals)
    try:
        check_partition(dev, rowptr)
        got = dev.patterns()
        assert got["enabled"] == (others != "few_patterned")
        assert got["entries"] == patterned_rows * per
        if got["enabled"]:
            lens = np.diff(got["pat_off"])
            assert np.all(lens[: patterned_rows // 32] == per) and not lens[patterned_rows // 32:].any()
        base = dev.index16()["chunk_base"]
        if others == "framed":
            assert np.all(base[patterned_rows // 32:] == -2)
        elif others == "plain":
            assert np.all(base[patterned_rows // 32:] == -1)
        check_spmv(dev, rowptr, colidx, vals, x, what="spmv")
        X = gen.uniform(918, gen.STREAM_X, ncols * 8).astype(dtype).reshape(ncols, 8)
        check_spmm(dev, rowptr, colidx, vals, X, what="spmm k=8")
    finally:
        dev.close()


@pytest.mark.parametrize("dtype", [np.float64, np.float32])
@pytest.mark.parametrize("per_row,half_band", [(12, 700), (40, 900), (81, 1000), (200, 600), (300, 1000), (12, 1100)])
def test_spmv_scattered_columns_in_a_narrow_band(per_row, half_band, dtype):
    """Random columns inside a band around the diagonal: every gather its own cache line, the
    columns of a chunk inside a window that fits LDS (or just not: the last case in doubles)."""
    say(f"band per_row={per_row} half_band={half_band} {np.dtype(dtype).name}")
    n = 4000 + 13
    ncols = n
    L = np.full(n, per_row, dtype=np.int64)
    L[5] = 0
    L[64:96] = 0                                        # an empty chunk
    L[n - 40:n - 20] = 0                                # empty rows in the last chunks
    rowptr, colidx, vals = gen.random_csr(n, ncols, L, 921, dtype)
    u = gen.uniform(922, 5, int(rowptr[-1]), 0.0, 1.0)
    rows = np.repeat(np.arange(n, dtype=np.int64), L)
    lo = np.clip(rows - half_band, 0, ncols - 2 * half_band - 1)
    cols = lo + (u * (2 * half_band)).astype(np.int64)
    order = np.lexsort((cols, rows))                    # ascending inside a row (duplicates stay)
    colidx[:] = cols[order].astype(np.int32)
    x = gen.uniform(923, gen.STREAM_X, ncols).astype(dtype)
    y0 = gen.uniform(923, gen.STREAM_Y0, n).astype(dtype)
    dev = DeviceCsr(n, ncols, rowptr, colidx, vals)
    try:
        check_partition(dev, rowptr)
        assert dev.partition()["stream_chunks"].size > 0
        check_spmv(dev, rowptr, colidx, vals, x, what="alpha=1 beta=0")
        check_spmv(dev, rowptr, colidx, vals, x, 1.5, -0.5, y0, what="alpha=1.5 beta=-0.5")
    finally:
        dev.close()


def test_index16_last_entries_of_the_matrix():
    """nnz % 4 = 1, 2, 3: the entries past the last vector load take the scalar path."""
    for extra in (1, 2, 3):
        say(f"index16 tail nnz%4={extra}")
        n = 640
        L = np.full(n, 12)
        L[-1] = 12 + extra
        rowptr, colidx, vals = gen.random_csr(n, 2000, L, 809, np.float64)
        assert int(rowptr[-1]) % 4 == extra
        dev = DeviceCsr(n, 2000, rowptr, colidx, vals)
        try:
            assert check_index16(dev)
            check_spmv(dev, rowptr, colidx, vals, gen.uniform(17, gen.STREAM_X, 2000), what="tail")
        finally:
            dev.close()


def test_spmm_row_lengths_and_wide_leading_dimension():
    """Stream chunks with 16-bit offsets: rows of 16 / 24 / 27 / 33 entries exercise the whole
    batches of 16, 8, 2 and 1 and the ragged remainder; a row of X longer than 64 KiB switches the
    32-bit row offsets off."""
    say("spmm batches and wide ldx")
    n, ncols = 1280, 900
    for lengths, tag in ((np.full(n, 16), "16"), (np.full(n, 24), "24"), (np.full(n, 27), "27"),
                         (np.full(n, 33), "33"), (16 + (np.arange(n) * 7) % 20, "ragged 16..35")):
        rowptr, colidx, vals = gen.random_csr(n, ncols, lengths, 4242, np.float64)
        dev = DeviceCsr(n, ncols, rowptr, colidx, vals)
        try:
            assert check_index16(dev)
            X = gen.uniform(18, gen.STREAM_X, ncols * 16).reshape(ncols, 16)
            Y0 = gen.uniform(18, gen.STREAM_Y0, n * 16).reshape(n, 16)
            check_spmm(dev, rowptr, colidx, vals, X, what=f"rows of {tag}")
            check_spmm(dev, rowptr, colidx, vals, X, -0.5, 2.0, Y0, what=f"rows of {tag}, beta")
            if tag == "27":
                check_spmm(dev, rowptr, colidx, vals, X, what="ldx 8200", ldx=8200, ldy=20)
                Xf = gen.uniform(19, gen.STREAM_X, ncols * 4).reshape(ncols, 4)
                check_spmm(dev, rowptr, colidx, vals, Xf, what="k = 4")
        finally:
            dev.close()


def test_spmv_huge_rows_lds_blocks():
    """Rows above 16384 entries with the split on: pieces per 64 KiB block of x (one that ends
    inside the last, partial block; empty pieces; a row that fills whole blocks)."""
    say("huge rows")
    for dtype, ncols in ((np.float32, (1 << 20) + 4321), (np.float64, (1 << 19) + 123)):
        n = 700
        L = mixed_lengths(n, 73, 3000)
        L[3] = 20000
        L[100] = 16385
        L[101] = 16384                       # not huge: stays a split row
        L[350] = min(ncols, 300000)
        L[699] = 65536
        rowptr, colidx, vals = gen.random_csr(n, ncols, L, 557, dtype)
        # one huge row whose columns are one contiguous run: most of its blocks are empty
        a = rowptr[100]
        colidx[a:a + 16385] = np.arange(777, 777 + 16385, dtype=np.int32)
        x = gen.uniform(29, gen.STREAM_X, ncols).astype(dtype)
        y0 = gen.uniform(29, gen.STREAM_Y0, n).astype(dtype)
        dev = DeviceCsr(n, ncols, rowptr, colidx, vals)
        try:
            check_partition(dev, rowptr)
            ref = check_split(dev, rowptr, colidx, ncols, np.dtype(dtype).itemsize, expect_on=True)
            assert ref["huge_rows"].tolist() == [3, 100, 350, 699]
            check_spmv(dev, rowptr, colidx, vals, x, what="alpha=1 beta=0")
            check_spmv(dev, rowptr, colidx, vals, x, -1.5, 0.25, y0, what="alpha=-1.5 beta=0.25")
            a1 = dev.spmv(x, 2.0, 0.0)
            assert np.array_equal(a1, dev.spmv(x, 2.0, 0.0)), "two runs differ"
            xn = x.copy()
            xn[5], xn[ncols // 2], xn[ncols - 1] = np.inf, np.nan, -np.inf
            with np.errstate(invalid="ignore", over="ignore"):
                refn, _ = oracle.spmv(rowptr, colidx, vals, xn)
                gotn = dev.spmv(xn)
            assert np.array_equal(np.isnan(gotn), np.isnan(refn)) and np.array_equal(np.isinf(gotn), np.isinf(refn))
        finally:
            dev.close()


def test_non_finite_values_propagate_like_the_reference():
    """Inf and NaN in x, X and vals reach exactly the rows the serial evaluation says (padding
    lanes repeat an entry and discard the product after the multiply, so they add nothing)."""
    say("non-finite values")
    n, ncols = 4000, 3000
    L = mixed_lengths(n, 74, 5000)
    L = np.minimum(L, ncols)
    rowptr, colidx, vals = gen.random_csr(n, ncols, L, 558, np.float64)
    x = gen.uniform(30, gen.STREAM_X, ncols)
    x[17] = np.inf
    x[1234] = -np.inf
    x[2999] = np.nan
    vals[rowptr[500]] = np.inf                      # first entry of a row
    vals[rowptr[2001] - 1] = np.nan                 # last entry of a row
    X = gen.uniform(31, gen.STREAM_X, ncols * 16).reshape(ncols, 16)
    X[17, 3] = np.inf
    X[2999, :] = np.nan
    dev = DeviceCsr(n, ncols, rowptr, colidx, vals)
    try:
        with np.errstate(invalid="ignore", over="ignore"):
            ref, _ = oracle.spmv(rowptr, colidx, vals, x)
            got = dev.spmv(x)
            assert np.array_equal(np.isnan(got), np.isnan(ref)), "NaN pattern differs (SpMV)"
            assert np.array_equal(np.isposinf(got), np.isposinf(ref)) and np.array_equal(np.isneginf(got), np.isneginf(ref))
            refm, _ = oracle.spmm(rowptr, colidx, vals, X)
            gotm = dev.spmm(X)
            assert np.array_equal(np.isnan(gotm), np.isnan(refm)), "NaN pattern differs (SpMM)"
            assert np.array_equal(np.isposinf(gotm), np.isposinf(refm)) and np.array_equal(np.isneginf(gotm), np.isneginf(refm))
        assert np.isnan(ref).sum() > 10 and np.isinf(ref).sum() > 10      # the case is not vacuous
    finally:
        dev.close()


def test_byte_offsets_beyond_4_gib():
    """288^3 27-point stencil: 640.5 M entries, so the value array is 5.1 GB and byte offsets
    into it pass 2^32 (and its chunks span more than 2^16 columns: framed 16-bit codes)."""
    w = gen.workload(2, {"nx": 288, "ny": 288, "nz": 288})
    say(f"large {w.name} nnz={w.nnz}")
    assert w.nnz * 8 > 2 ** 32
    dev = DeviceCsr(w.nrows, w.ncols, w.rowptr, w.colidx, w.vals)
    try:
        got = dev.mat.index16()
        assert got["enabled"] and got["framed_entries"] > 0.9 * w.nnz
        check_spmv(dev, w.rowptr, w.colidx, w.vals, w.x, literal=True, what=w.name)
        check_spmv(dev, w.rowptr, w.colidx, w.vals, w.x, literal=True, what=w.name + " (paper shape)", paper_shape=True)
    finally:
        dev.close()


def test_workload4_wide_reduced():
    """Power-law rows over 2^21 columns: x = 8 MB of floats, so the column split is on."""
    run_workload(4, {"n": 1 << 21, "cap": 200000})

# ---------------------------------------------------------------------------
# SpMM
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("dtype", [np.float64, np.float32])
@pytest.mark.parametrize("k,ldx,ldy", [(1, None, None), (1, 3, 2), (2, None, None), (3, 5, 4), (16, None, None),
                                       (16, 20, 24), (17, None, None), (40, 40, 44), (130, None, None)])
def test_spmm_general_matrices(dtype, k, ldx, ldy):
    say(f"spmm general k={k} ldx={ldx} ldy={ldy} {np.dtype(dtype).name}")
    n, ncols = 1500, 6000
    L = np.minimum(mixed_lengths(n, 60, 6000), ncols)
    rowptr, colidx, vals = gen.random_csr(n, ncols, L, 1234, dtype, sorted_cols=False)
    X = gen.uniform(8, gen.STREAM_X, ncols * k).astype(dtype).reshape(ncols, k)
    Y0 = gen.uniform(8, gen.STREAM_Y0, n * k).astype(dtype).reshape(n, k)
    dev = DeviceCsr(n, ncols, rowptr, colidx, vals)
    try:
        check_spmm(dev, rowptr, colidx, vals, X, what="alpha=1 beta=0", ldx=ldx, ldy=ldy)
        check_spmm(dev, rowptr, colidx, vals, X, 1.25, -0.5, Y0, what="alpha=1.25 beta=-0.5", ldx=ldx, ldy=ldy)
        if k == 1:  # the single-column product agrees with SpMV
            y = dev.spmv(X[:, 0])
            ref, absAx = oracle.spmv(rowptr, colidx, vals, np.ascontiguousarray(X[:, 0]))
            assert_close(dev.spmm(X)[:, 0], ref, general_bound(np.diff(rowptr), absAx, dtype, 1.0, 0.0, None))
            assert_close(y, ref, general_bound(np.diff(rowptr), absAx, dtype, 1.0, 0.0, None))
    finally:
        dev.close()


@pytest.mark.parametrize("dtype,k", [(np.float64, 16), (np.float64, 32), (np.float32, 32), (np.float64, 8), (np.float64, 11),
                                     (np.float32, 70)])
@pytest.mark.parametrize("per_row", [9, 70])
def test_spmm_few_stream_chunks_long_and_short_rows(per_row, dtype, k):
    """Few stream chunks without shared rows of X: with long rows (48 entries per row or more on average)
    every pass of a chunk - the 4, 8 or 16 rows that the slots of a wavefront take together - gets a
    wavefront of its own, with short rows a chunk keeps its one wavefront.  Rows of mixed lengths, a ragged
    last chunk, leading dimensions wider than k."""
    say(f"spmm few stream chunks, about {per_row} per row, k={k} {np.dtype(dtype).name}")
    n = 32 * 150 + 21
    L = (per_row - 4 + np.floor(gen.uniform(94, 0, n, 0.0, 1.0) * 9)).astype(np.int64)
    L[::53] = 0
    L[7::211] = 3 * per_row
    rowptr, colidx, vals = gen.random_csr(n, n, L, 95, dtype, sorted_cols=False)
    X = gen.uniform(96, gen.STREAM_X, n * k).astype(dtype).reshape(n, k)
    Y0 = gen.uniform(96, gen.STREAM_Y0, n * k).astype(dtype).reshape(n, k)
    dev = DeviceCsr(n, n, rowptr, colidx, vals)
    try:
        assert dev.partition()["stream_chunks"].size > 100
        assert (colidx.size >= 48 * n) == (per_row == 70)
        check_spmm(dev, rowptr, colidx, vals, X, what="alpha=1 beta=0")
        check_spmm(dev, rowptr, colidx, vals, X, 1.5, -0.25, Y0, what="alpha=1.5 beta=-0.25", ldx=k + 2, ldy=k + 1)
    finally:
        dev.close()


@pytest.mark.parametrize("ldx", [(1 << 21) - 8, 1 << 21])
def test_spmm_rows_of_x_sixteen_mebibytes_apart(ldx):
    """The kernels that share rows of X address them with 32-bit offsets from a row near the chunk's own and
    are used while a row of X is shorter than 16 MiB; at that length and beyond the ordinary path runs.
    A band matrix whose chunks all qualify, with leading dimensions just below and at the limit."""
    say(f"spmm with ldx={ldx} doubles")
    n, k = 32 * 6 + 5, 16
    rows = [[j for j in range(i - 4, i + 5) if 0 <= j < n] for i in range(n)]
    rowptr = np.zeros(n + 1, dtype=np.int32)
    rowptr[1:] = np.cumsum([len(r) for r in rows])
    colidx = np.array([c for r in rows for c in r], dtype=np.int32)
    vals = gen.uniform(71, gen.STREAM_VALUES, colidx.size)
    X = gen.uniform(71, gen.STREAM_X, n * k).reshape(n, k)
    dev = DeviceCsr(n, n, rowptr, colidx, vals)
    try:
        classes = dev.share_classes()
        assert classes is not None and np.all(classes[:-1] == oracle.SHARE_PLAIN)     # the last 5 rows are too few to stream
        check_spmm(dev, rowptr, colidx, vals, X, what="alpha=1 beta=0", ldx=ldx, ldy=k + 1)
    finally:
        dev.close()


@pytest.mark.parametrize("dtype,k", [(np.float64, 16), (np.float32, 8), (np.float64, 3)])
def test_spmm_many_stream_chunks_one_wavefront_per_chunk(dtype, k):
    """More than 8192 stream chunks without shared rows of X: the launch with one wavefront per chunk."""
    say(f"spmm over 9000 stream chunks k={k} {np.dtype(dtype).name}")
    n = 32 * 9000 + 13
    L = (6 + np.floor(gen.uniform(91, 0, n, 0.0, 1.0) * 7)).astype(np.int64)      # 6..12 entries per row
    L[::97] = 0
    rowptr, colidx, vals = gen.random_csr(n, n, L, 92, dtype)
    X = gen.uniform(93, gen.STREAM_X, n * k).astype(dtype).reshape(n, k)
    Y0 = gen.uniform(93, gen.STREAM_Y0, n * k).astype(dtype).reshape(n, k)
    dev = DeviceCsr(n, n, rowptr, colidx, vals)
    try:
        assert dev.partition()["stream_chunks"].size > 8192
        check_spmm(dev, rowptr, colidx, vals, X, what="alpha=1 beta=0")
        check_spmm(dev, rowptr, colidx, vals, X, -0.5, 2.0, Y0, what="alpha=-0.5 beta=2", ldx=k + 1, ldy=k + 3)
    finally:
        dev.close()


@pytest.mark.parametrize("dtype,k", [(np.float64, 16), (np.float64, 13), (np.float32, 32), (np.float32, 16),
                                     (np.float64, 32), (np.float64, 40), (np.float32, 64)])
@pytest.mark.parametrize("grid", [(128, 5, 4), (96, 3, 3), (64, 6, 5), (33, 9, 7)])
def test_spmm_rows_of_x_shared_between_neighbouring_rows(grid, dtype, k):
    """27-point stencils with grid lines of 4, 3, 2 and about 1 chunks: chunks whose rows all repeat
    one list of diagonals, chunks with a boundary row in their first or last slot (a shorter,
    masked list), and chunks that straddle grid lines.  With 8 lanes per row of X (f64 k = 16,
    f32 k = 32) a slot takes 4 consecutive rows and loads 6 rows of X per run of 3 diagonals, with 16
    lanes (f64 k = 32, f32 k = 64) 8 rows and 10 rows of X; k = 40 adds a second block of 8 columns."""
    nx, ny, nz = grid
    say(f"spmm shared rows of X, stencil {nx}x{ny}x{nz} k={k} {np.dtype(dtype).name}")
    rowptr, colidx, vals = gen.stencil27(nx, ny, nz, 41)
    vals = vals.astype(dtype)
    n = nx * ny * nz
    X = gen.uniform(43, gen.STREAM_X, n * k).astype(dtype).reshape(n, k)
    Y0 = gen.uniform(43, gen.STREAM_Y0, n * k).astype(dtype).reshape(n, k)
    dev = DeviceCsr(n, n, rowptr, colidx, vals)
    try:
        check_spmm(dev, rowptr, colidx, vals, X, what="alpha=1 beta=0")
        check_spmm(dev, rowptr, colidx, vals, X, -0.75, 0.5, Y0, what="alpha=-0.75 beta=0.5", ldx=k + 3, ldy=k + 1)
        # a row of X that is not finite reaches exactly the rows of Y whose matrix rows hold that column:
        # no product of an absent entry (a masked diagonal, a row of X loaded for a neighbour) may leak in
        for j in (0, n // 2 + 1, n - 1):
            Xi = X.copy()
            Xi[j, :] = np.inf
            ref, _ = oracle.spmm(rowptr, colidx, vals, Xi)
            got = dev.spmm(Xi)
            assert np.array_equal(np.isfinite(got), np.isfinite(ref)), f"non-finite row {j} of X spread differently"
            hit = ~np.isfinite(ref)
            assert np.array_equal(got[hit], ref[hit])
            assert hit.any(axis=1).sum() == np.count_nonzero(colidx == j)
    finally:
        dev.close()


@pytest.mark.parametrize("k", [16, 32])
def test_spmm_shared_rows_of_x_rectangular_and_a_few_other_rows(k):
    """Every row holds the same 27 diagonals (9 runs of 3, all to the right of the main diagonal, so
    the matrix is wider than tall), except that a few rows per chunk are emptied, shortened or given
    other columns: exactly 4 such rows in some chunks (still handled beside the shared rows), 5 in
    others (the ordinary path)."""
    say(f"spmm shared rows of X, rectangular band, k={k}")
    n, per = 32 * 40 + 7, 27
    diag = np.array([10 * r + e for r in range(9) for e in range(3)], dtype=np.int64)
    ncols = n + int(diag[-1]) + 1
    rows = [list(i + diag) for i in range(n)]
    for c in range(0, n // 32):
        base = 32 * c
        changed = [1, 9, 17, 30] if c % 3 == 0 else ([0, 5, 6, 21, 31] if c % 3 == 1 else [13])
        for j, r in enumerate(changed):
            i = base + r
            if j % 3 == 0:
                rows[i] = []                                      # empty
            elif j % 3 == 1:
                rows[i] = rows[i][2:20]                           # a subset of the list
            else:
                rows[i] = [(i * 7 + 3 * t) % ncols for t in range(27)][::-1]   # other columns, descending
    rowptr = np.zeros(n + 1, dtype=np.int32)
    rowptr[1:] = np.cumsum([len(r) for r in rows])
    colidx = np.array([c for r in rows for c in r], dtype=np.int32)
    vals = gen.uniform(47, gen.STREAM_VALUES, colidx.size)
    X = gen.uniform(47, gen.STREAM_X, ncols * k).reshape(ncols, k)
    Y0 = gen.uniform(47, gen.STREAM_Y0, n * k).reshape(n, k)
    dev = DeviceCsr(n, ncols, rowptr, colidx, vals)
    try:
        assert dev.patterns()["enabled"]
        check_spmm(dev, rowptr, colidx, vals, X, what="alpha=1 beta=0")
        check_spmm(dev, rowptr, colidx, vals, X, 2.0, -1.0, Y0, what="alpha=2 beta=-1")
    finally:
        dev.close()


SHARE_LISTS = {
    # reference lists of diagonals (ascending); runs of consecutive diagonals are cut into pieces of 3, 2 and 1
    "runs_of_3": [-40, -39, -38, -1, 0, 1, 50, 51, 52],                       # three pieces of 3
    "seven_point": [-400, -20, -1, 0, 1, 20, 400],                            # 1, 1, 3, 1, 1
    "pairs": [-31, -30, -11, -10, 0, 1, 10, 11, 30, 31, 60, 61],              # six pieces of 2
    "singles": [-90, -70, -50, -30, -10, 0, 10, 30, 50, 70, 90, 110, 130],    # thirteen pieces of 1
    "long_runs": list(range(-9, 2)) + list(range(20, 27)) + [40, 41, 50],     # 11 = 3+3+3+2, 7 = 3+3+1, 2, 1
    "dense_band": list(range(-30, 31)),                                       # one run of 61: 20 pieces of 3 and a 1
    "five_pieces_of_3": list(range(0, 15)),                                   # more pieces than are in flight
}


@pytest.mark.parametrize("dtype,k", [(np.float64, 16), (np.float32, 32), (np.float64, 32), (np.float64, 11),
                                     (np.float32, 7), (np.float64, 48)])
@pytest.mark.parametrize("kind", sorted(SHARE_LISTS))
def test_spmm_shared_rows_every_piece_length(kind, dtype, k):
    """Band matrices whose rows all hold one list of diagonals, so that every chunk away from the ends
    shares rows of X between neighbouring rows: pieces of 3, 2 and 1 diagonals, runs longer than 3,
    more pieces than are in flight at once; a few emptied or shortened rows per chunk (computed apart);
    8 and 16 lanes per row of X, element-wise loads (k = 11, 7), two column blocks (k = 48).  The first
    and last chunks would reach outside X with the rows they load for neighbours and clamp the row numbers."""
    say(f"spmm shared rows, list {kind} k={k} {np.dtype(dtype).name}")
    lst = SHARE_LISTS[kind]
    n = 32 * 37 + 11
    rows = []
    for i in range(n):
        cols = [i + d for d in lst if 0 <= i + d < n]
        c = i // 32
        if i % 32 == 5 and c % 2 == 0:
            cols = []                                            # an empty row
        elif i % 32 == 30 and c % 3 == 0:
            cols = cols[1:-1]                                    # a subset of the list
        elif i % 32 == 17 and c % 5 == 0:
            cols = cols[::-1]                                    # the same columns, descending
        rows.append(cols)
    rowptr = np.zeros(n + 1, dtype=np.int32)
    rowptr[1:] = np.cumsum([len(r) for r in rows])
    colidx = np.array([c for r in rows for c in r], dtype=np.int32)
    vals = gen.uniform(53, gen.STREAM_VALUES, colidx.size).astype(dtype)
    X = gen.uniform(53, gen.STREAM_X, n * k).astype(dtype).reshape(n, k)
    Y0 = gen.uniform(53, gen.STREAM_Y0, n * k).astype(dtype).reshape(n, k)
    dev = DeviceCsr(n, n, rowptr, colidx, vals)
    try:
        if len(lst) * 32 >= 256:
            assert dev.patterns()["enabled"]
        check_partition(dev, rowptr)
        check_spmm(dev, rowptr, colidx, vals, X, what="alpha=1 beta=0")
        check_spmm(dev, rowptr, colidx, vals, X, 0.5, -2.0, Y0, what="alpha=0.5 beta=-2", ldx=k + 1, ldy=k + 2)
        for j in (3, n // 2, n - 2):                             # a non-finite row of X reaches exactly its column's rows
            Xi = X.copy()
            Xi[j, :] = np.nan
            ref, _ = oracle.spmm(rowptr, colidx, vals, Xi)
            got = dev.spmm(Xi)
            assert np.array_equal(np.isnan(got), np.isnan(ref)), f"NaN row {j} of X spread differently"
    finally:
        dev.close()


BLOCK_GRIDS = {
    # (unknowns per point, neighbour offsets of a point on a line of points)
    "seven_point_3": (3, [-400, -20, -1, 0, 1, 20, 400]),                 # 21 diagonals: runs of 3, 3, 9, 3, 3
    "nine_point_2": (2, [-21, -20, -19, -1, 0, 1, 19, 20, 21]),           # 18 diagonals: three runs of 6
    "singles_3": (3, [-50, -30, -10, 0, 10, 30, 50, 70]),                 # 24 diagonals, eight runs of 3
    "plane27_3": (3, [z * 400 + y * 20 + x for z in (-1, 0, 1) for y in (-1, 0, 1) for x in (-1, 0, 1)]),   # 81: three passes
    "dense_3": (3, list(range(-20, 21))),                                 # one run of 123 diagonals: both halves of the list
    "dense_2": (2, list(range(-31, 33))),                                 # 128 diagonals, the most a pattern may have
    "pairs_2": (2, [-7, -3, 0, 5, 9]),                                    # 10 diagonals: pieces of 2 only
}


@pytest.mark.parametrize("dtype,k", [(np.float64, 16), (np.float32, 32), (np.float64, 32), (np.float64, 13),
                                     (np.float32, 7), (np.float64, 40)])
@pytest.mark.parametrize("kind", sorted(BLOCK_GRIDS))
def test_spmm_block_rows_share_rows_of_x(kind, dtype, k):
    """Two or three unknowns per grid point: the rows of a point hold the same columns, the chunk stores one
    list of diagonals and the rows differ in their shifts; the product loads a point's rows of X once for
    its rows.  Lists of up to 128 diagonals worked through in passes, a few emptied or shortened rows per
    chunk (computed apart), chunks at the ends of the matrix (cut-off lists; row numbers clamped),
    unaligned k (element-wise loads), two column blocks; the share classes bit for bit against the oracle."""
    dof, nbrs = BLOCK_GRIDS[kind]
    say(f"spmm block rows, {kind} k={k} {np.dtype(dtype).name}")
    npts = 1000 if len(nbrs) * dof <= 30 else 700
    n = npts * dof
    rows = []
    for p in range(npts):
        cols = [dof * (p + d) + b for d in nbrs if 0 <= p + d < npts for b in range(dof)]
        rows += [list(cols) for _ in range(dof)]
    for i in range(n):
        c = i // 32
        if i % 32 == 7 and c % 2 == 0:
            rows[i] = []                                         # an empty row
        elif i % 32 == 29 and c % 3 == 0:
            rows[i] = rows[i][1:-1]                              # a subset of the list
        elif i % 32 == 16 and c % 5 == 0:
            rows[i] = rows[i][::-1]                              # the same columns, descending
    rowptr = np.zeros(n + 1, dtype=np.int32)
    rowptr[1:] = np.cumsum([len(r) for r in rows])
    colidx = np.array([c for r in rows for c in r], dtype=np.int32)
    vals = gen.uniform(57, gen.STREAM_VALUES, colidx.size).astype(dtype)
    X = gen.uniform(57, gen.STREAM_X, n * k).astype(dtype).reshape(n, k)
    Y0 = gen.uniform(57, gen.STREAM_Y0, n * k).astype(dtype).reshape(n, k)
    dev = DeviceCsr(n, n, rowptr, colidx, vals)
    try:
        check_partition(dev, rowptr)
        classes = dev.share_classes()
        want = oracle.SHARE_BLOCK3 if dof == 3 else oracle.SHARE_BLOCK2
        assert classes is not None and np.count_nonzero(classes == want) * 2 > classes.size, \
            f"classes {np.bincount(classes, minlength=5)}: the block rows are not shared"
        check_spmm(dev, rowptr, colidx, vals, X, what="alpha=1 beta=0")
        check_spmm(dev, rowptr, colidx, vals, X, 0.5, -2.0, Y0, what="alpha=0.5 beta=-2", ldx=k + 1, ldy=k + 2)
        for j in (1, n // 2, n - 2):                             # a non-finite row of X reaches exactly its column's rows
            Xi = X.copy()
            Xi[j, :] = np.nan
            ref, _ = oracle.spmm(rowptr, colidx, vals, Xi)
            got = dev.spmm(Xi)
            assert np.array_equal(np.isnan(got), np.isnan(ref)), f"NaN row {j} of X spread differently"
    finally:
        dev.close()


# ---------------------------------------------------------------------------
# the five workloads: reduced sizes (several tiles + ragged tail) and full size
# ---------------------------------------------------------------------------
REDUCED = {
    6: {"scale": 0.03}, 7: {"scale": 0.04}, 8: {"scale": 0.02}, 9: {"scale": 0.03},
    1: None,
    2: {"nx": 37, "ny": 29, "nz": 31},
    3: {"n": 100003},
    4: {"n": 200003, "cap": 60000},
    5: {"nx": 23, "ny": 19, "nz": 17, "k": 16},
}


def run_workload(cfg, scale):
    w = gen.workload(cfg, scale)
    say(f"workload {cfg} {w.name} nrows={w.nrows} nnz={w.nnz}")
    dev = DeviceCsr(w.nrows, w.ncols, w.rowptr, w.colidx, w.vals)
    try:
        check_partition(dev, w.rowptr)
        check_half_bandwidth(dev, w.rowptr, w.colidx)
        check_split(dev, w.rowptr, w.colidx, w.ncols, w.vals.itemsize)
        if w.k == 0:
            check_spmv(dev, w.rowptr, w.colidx, w.vals, w.x, w.alpha, w.beta, w.y0, literal=True, what=w.name)
            check_spmv(dev, w.rowptr, w.colidx, w.vals, w.x, w.alpha, w.beta, w.y0, literal=True,
                       what=w.name + " (paper shape)", paper_shape=True)
        else:
            check_spmm(dev, w.rowptr, w.colidx, w.vals, w.x, w.alpha, w.beta, w.y0, literal=True, what=w.name)
    finally:
        dev.close()


@pytest.mark.parametrize("cfg", [1, 2, 3, 4, 5, 6, 7, 8, 9])
def test_workload_reduced(cfg):
    run_workload(cfg, REDUCED[cfg])


@pytest.mark.parametrize("cfg", [2, 3, 4, 5, 6, 7, 8, 9])
def test_workload_full_size(cfg):
    run_workload(cfg, None)


def test_workload4_exponent_two_full_size():
    """The labelled variant of workload 4 with Zipf exponent 2.0 (mean row length about 8)."""
    run_workload(4, {"s": 2.0})


# ---------------------------------------------------------------------------
# the largest matrix the interface takes: LAPIS_MAX_NNZ entries (entry ids up to 2^31 - 2^16 - 1)
# ---------------------------------------------------------------------------
MAX_NNZ = 2 ** 31 - 2 ** 16          # LAPIS_MAX_NNZ of the header


def test_one_handle_two_streams_products_are_ordered():
    """A handle with scratch (column split, tiles, LDS blocks) used from two streams at once: the
    library orders its products (event recorded by each, waited for by the next on another stream), so
    both results match the oracle however the streams interleave."""
    import torch
    say("one handle, two streams")
    w = gen.workload(4, {"n": 1_200_000, "cap": 50_000})
    ref, absAx = oracle.spmv(w.rowptr, w.colidx, w.vals, w.x, 1.0, 0.0, None)
    x2 = gen.uniform(99, gen.STREAM_X, w.ncols).astype(w.vals.dtype)
    ref2, absAx2 = oracle.spmv(w.rowptr, w.colidx, w.vals, x2, 1.0, 0.0, None)
    dev = DeviceCsr(w.nrows, w.ncols, w.rowptr, w.colidx, w.vals)
    try:
        assert dev.L.lapis_spmv_scratch_bytes(dev.mat.handle) > 0
        xa, xb = torch.from_numpy(w.x).cuda(), torch.from_numpy(x2).cuda()
        ya = torch.full((w.nrows,), float("nan"), dtype=xa.dtype, device="cuda:0")
        yb = torch.full_like(ya, float("nan"))
        sa, sb = torch.cuda.Stream(), torch.cuda.Stream()
        torch.cuda.synchronize()
        for _ in range(20):                                    # alternate the streams without waiting in between
            dev.mat.spmv(xa, ya, 1.0, 0.0, stream=sa)
            dev.mat.spmv(xb, yb, 1.0, 0.0, stream=sb)
        torch.cuda.synchronize()
        nnz_row = np.diff(w.rowptr)
        assert_close(ya.cpu().numpy(), ref, literal_bound(nnz_row, absAx, w.vals.dtype), "stream a")
        assert_close(yb.cpu().numpy(), ref2, literal_bound(nnz_row, absAx2, w.vals.dtype), "stream b")
    finally:
        dev.close()


@pytest.mark.parametrize("kind", ["diagonals", "scattered"])
def test_spmv_at_the_entry_limit(kind):
    """32 entries in every row, built on the device.  All values are small integers, so every sum is
    exact in float and the whole result can be compared with one computed by plain tensor operations
    (a property that holds at any size); rows sampled across the range, the ones holding the entries
    around 2^30 and the last ones among them, are also computed by the oracle from a copy of their entries."""
    import torch
    import paper_2509_25605_amd as lapis
    per = 32
    nnz = MAX_NNZ
    n = nnz // per
    assert n * per == nnz
    say(f"entry limit, {kind}: nrows={n} nnz={nnz} float32")
    dev = torch.device("cuda")
    step = 1 << 22

    def columns(r0, r1):
        i = torch.arange(r0, r1, dtype=torch.int64, device=dev).view(-1, 1)
        t = torch.arange(per, dtype=torch.int64, device=dev).view(1, -1)
        if kind == "diagonals":                       # the same 32 diagonals in every row
            c = i + (t - 16) * 1025
        else:                                         # anywhere within 2046 columns of the diagonal
            c = i + (t * 2654435761 + i * 40503) % 4093 - 2046
        return c.clamp_(0, n - 1), (1 + (i + t) % 3).to(torch.float32)

    rowptr = (torch.arange(n + 1, dtype=torch.int64, device=dev) * per).to(torch.int32)
    colidx = torch.empty(nnz, dtype=torch.int32, device=dev)
    vals = torch.empty(nnz, dtype=torch.float32, device=dev)
    for r0 in range(0, n, step):
        r1 = min(n, r0 + step)
        c, v = columns(r0, r1)
        colidx[r0 * per:r1 * per] = c.reshape(-1).to(torch.int32)
        vals[r0 * per:r1 * per] = v.reshape(-1)
    x = (torch.arange(n, dtype=torch.int64, device=dev) % 7).to(torch.float32)
    expected = torch.empty(n, dtype=torch.float32, device=dev)
    for r0 in range(0, n, step):
        r1 = min(n, r0 + step)
        c, v = columns(r0, r1)
        expected[r0:r1] = (v.double() * x[c].double()).sum(1).to(torch.float32)
    del c, v
    rows = np.unique(np.concatenate([
        [0, 1, 31, 32, n // 2, (2 ** 30) // per - 1, (2 ** 30) // per, n - 33, n - 32, n - 2, n - 1],
        (gen.uniform(77, 1, 40, 0.0, 1.0) * n).astype(np.int64)]))
    pick = torch.from_numpy(rows).to(dev)
    sub_col = colidx.view(n, per)[pick].cpu().numpy().reshape(-1)
    sub_val = vals.view(n, per)[pick].cpu().numpy().reshape(-1)
    sub_ptr = (np.arange(rows.size + 1) * per).astype(np.int32)
    ref, absAx = oracle.spmv(sub_ptr, sub_col, sub_val, x.cpu().numpy())
    assert np.array_equal(ref, expected[pick].cpu().numpy())       # the two references agree

    say("create")
    M = lapis.CsrMatrix(n, n, rowptr, colidx, vals)
    try:
        y = torch.full((n,), float("nan"), dtype=torch.float32, device=dev)
        say("tuned product")
        M.spmv(x, y)
        torch.cuda.synchronize()
        assert torch.equal(y, expected)
        assert np.array_equal(y[pick].cpu().numpy(), ref)
        say("paper-shape product")
        y.fill_(float("nan"))
        lapis.lapis_spmv_paper_shape(M.handle, 1.0, x, 0.0, y)
        torch.cuda.synchronize()
        assert torch.equal(y, expected)
        say("two columns")
        X = torch.stack([x, 2.0 * x], dim=1).contiguous()
        Y = torch.full((n, 2), float("nan"), dtype=torch.float32, device=dev)
        M.spmm(X, Y)
        torch.cuda.synchronize()
        assert torch.equal(Y[:, 0], expected) and torch.equal(Y[:, 1], 2.0 * expected)
        del X, Y
        # the transposed product, by atomics and through a handle for A^T (integer sums below 2^24:
        # exact in float in any order)
        expected_t = torch.zeros(n, dtype=torch.float64, device=dev)
        for r0 in range(0, n, step):
            r1 = min(n, r0 + step)
            c, v = columns(r0, r1)
            expected_t.index_add_(0, c.reshape(-1), (v.double() * x[r0:r1].double().view(-1, 1)).reshape(-1))
        del c, v
        assert float(expected_t.max()) < 2 ** 24
        expected_t = expected_t.to(torch.float32)
        say("transposed product by atomics")
        y.fill_(float("nan"))
        M.spmv_transpose(x, y)
        torch.cuda.synchronize()
        assert torch.equal(y, expected_t)
        say("transposed handle")
        T = M.transposed()
        try:
            y.fill_(float("nan"))
            T.spmv(x, y)
            torch.cuda.synchronize()
            assert torch.equal(y, expected_t)
        finally:
            T.close()
    finally:
        M.close()


# ---------------------------------------------------------------------------
# seeded sweep over structures: sections of a matrix built in different ways, so that patterned,
# narrow, framed and plain chunks, grouped and single wavefronts, bins and tiles meet in one handle
# ---------------------------------------------------------------------------
def _section(kind, r0, r1, ncols, seed):
    """Rows r0..r1-1 as lists of columns."""
    n = r1 - r0
    u = gen.uniform(seed, 9, n * 8 + 8, 0.0, 1.0)
    rows = []
    if kind == "stencil":                                # a few diagonals, every row the same list
        diags = sorted(set(int(d) for d in (np.floor(u[:9] * 400) - 200)))
        rows = [[min(max(i + d, 0), ncols - 1) for d in diags] for i in range(r0, r1)]
    elif kind == "band":                                 # a dense band of varying width
        w = 3 + int(u[0] * 90)
        rows = [[min(i + d, ncols - 1) for d in range(w)] for i in range(r0, r1)]
    elif kind == "short":                                # 0-6 random columns
        for k, i in enumerate(range(r0, r1)):
            m = int(u[k] * 7)
            rows.append(sorted(int(c) for c in np.floor(gen.uniform(seed + i, 10, m, 0.0, 1.0) * ncols)))
    elif kind == "jitter":                               # 20-150 columns scattered near the diagonal
        for k, i in enumerate(range(r0, r1)):
            m = 20 + int(u[k] * 130)
            c = i + np.floor(gen.uniform(seed + i, 11, m, 0.0, 1.0) * 3000).astype(np.int64) - 1500
            rows.append(sorted(int(v) for v in np.clip(c, 0, ncols - 1)))
    elif kind == "wide":                                 # 10-40 columns anywhere, unsorted
        for k, i in enumerate(range(r0, r1)):
            m = 10 + int(u[k] * 30)
            rows.append([int(c) for c in np.floor(gen.uniform(seed + i, 12, m, 0.0, 1.0) * ncols)])
    else:                                                # "long": one row of a few thousand entries among short ones
        for k, i in enumerate(range(r0, r1)):
            m = 5000 + int(u[0] * 3000) if k == n // 2 else 3
            rows.append(sorted(int(c) for c in np.floor(gen.uniform(seed + i, 13, m, 0.0, 1.0) * ncols)))
    return rows


@pytest.mark.parametrize("seed", range(12))
def test_seeded_structure_sweep(seed):
    kinds = ["stencil", "band", "short", "jitter", "wide", "long"]
    pick = gen.uniform(4000 + seed, 1, 16, 0.0, 1.0)
    dtype = np.float64 if seed % 2 == 0 else np.float32
    ncols = [3000, 70000, 1 << 20][seed % 3]
    sections, r = [], 0
    for t in range(3 + seed % 3):
        length = 32 * (2 + int(pick[t] * 20)) + (int(pick[t + 8] * 31) if t % 2 else 0)
        sections.append((kinds[int(pick[t + 4] * len(kinds)) % len(kinds)], r, r + length))
        r += length
    n = r
    say(f"sweep seed={seed} n={n} ncols={ncols} {np.dtype(dtype).name} " + " ".join(k for k, _, _ in sections))
    rows = []
    for k, a, b in sections:
        rows += _section(k, a, b, ncols, 5000 + 97 * seed + a)
    rowptr = np.zeros(n + 1, dtype=np.int32)
    np.cumsum([len(x) for x in rows], out=rowptr[1:])
    colidx = np.array([c for x in rows for c in x], dtype=np.int32)
    vals = gen.uniform(6000 + seed, gen.STREAM_VALUES, colidx.size).astype(dtype)
    x = gen.uniform(6000 + seed, gen.STREAM_X, ncols).astype(dtype)
    y0 = gen.uniform(6000 + seed, gen.STREAM_Y0, n).astype(dtype)
    dev = DeviceCsr(n, ncols, rowptr, colidx, vals)
    try:
        check_partition(dev, rowptr)
        check_half_bandwidth(dev, rowptr, colidx)
        check_spmv(dev, rowptr, colidx, vals, x, what="alpha=1 beta=0")
        check_spmv(dev, rowptr, colidx, vals, x, -2.0, 0.75, y0, what="alpha=-2 beta=0.75")
        k = 1 + seed % 5 * 4
        X = gen.uniform(6100 + seed, gen.STREAM_X, ncols * k).astype(dtype).reshape(ncols, k)
        check_spmm(dev, rowptr, colidx, vals, X, what=f"spmm k={k}")
    finally:
        dev.close()


def _grid_section(kind, r0, r1, ncols, seed):
    """Rows r0..r1-1 of a grid-like section: every row the same neighbours, with 1, 2 or 3 unknowns per point."""
    u = gen.uniform(seed, 14, 16, 0.0, 1.0)
    dof = {"scalar": 1, "block2": 2, "block3": 3}[kind]
    nbrs = sorted(set([0] + [int(d) for d in (np.floor(u[:6] * 60) - 30)] + [int(u[6] * 3) * 40 + e for e in (-1, 0, 1)]))
    rows = []
    for i in range(r0, r1):
        p, base = (i - r0) // dof, r0
        cols = [base + dof * (p + d) + b for d in nbrs for b in range(dof)]
        rows.append([c for c in cols if 0 <= c < ncols])       # cut off at the ends of the matrix only
    for t in range(int(u[7] * 4)):                              # a few rows emptied or shortened
        j = int(u[8 + t] * (r1 - r0))
        rows[j] = rows[j][::2] if t % 2 else []
    return rows


@pytest.mark.parametrize("seed", range(10))
def test_seeded_share_class_sweep(seed):
    """Sections of scalar grids and of grids with 2 and 3 unknowns per point, of lengths that are not multiples
    of 32, so that chunks straddle two kinds, start in the middle of a grid point and hold a few altered rows:
    every share class beside every other in one matrix; classes bit for bit, SpMM with 8 and 16 lanes per row of X."""
    kinds = ["scalar", "block2", "block3"]
    pick = gen.uniform(4100 + seed, 1, 24, 0.0, 1.0)
    dtype = np.float64 if seed % 2 == 0 else np.float32
    sections, r = [], 0
    for t in range(4 + seed % 3):
        length = 32 * (3 + int(pick[t] * 12)) + int(pick[t + 8] * 31)
        sections.append((kinds[int(pick[t + 16] * 3) % 3], r, r + length))
        r += length
    n = r
    say(f"share sweep seed={seed} n={n} {np.dtype(dtype).name} " + " ".join(k for k, _, _ in sections))
    rows = []
    for kd, a, b in sections:
        rows += _grid_section(kd, a, b, n, 5100 + 89 * seed + a)
    rowptr = np.zeros(n + 1, dtype=np.int32)
    np.cumsum([len(x) for x in rows], out=rowptr[1:])
    colidx = np.array([c for x in rows for c in x], dtype=np.int32)
    vals = gen.uniform(6200 + seed, gen.STREAM_VALUES, colidx.size).astype(dtype)
    dev = DeviceCsr(n, n, rowptr, colidx, vals)
    try:
        check_partition(dev, rowptr)
        classes = dev.share_classes()
        assert classes is not None and np.count_nonzero(classes != oracle.SHARE_NONE) > 0
        x = gen.uniform(6200 + seed, gen.STREAM_X, n).astype(dtype)
        check_spmv(dev, rowptr, colidx, vals, x, what="alpha=1 beta=0")
        for k in ((16, 32) if dtype == np.float64 else (32, 64)):
            X = gen.uniform(6300 + seed, gen.STREAM_X, n * k).astype(dtype).reshape(n, k)
            Y0 = gen.uniform(6300 + seed, gen.STREAM_Y0, n * k).astype(dtype).reshape(n, k)
            check_spmm(dev, rowptr, colidx, vals, X, what=f"spmm k={k}")
            check_spmm(dev, rowptr, colidx, vals, X, -1.5, 0.5, Y0, what=f"spmm k={k} alpha=-1.5 beta=0.5", ldx=k + 4, ldy=k + 2)
            Xi = X.copy()
            Xi[n // 3, :] = np.nan
            ref, _ = oracle.spmm(rowptr, colidx, vals, Xi)
            assert np.array_equal(np.isnan(dev.spmm(Xi)), np.isnan(ref)), "a NaN row of X spread differently"
    finally:
        dev.close()
