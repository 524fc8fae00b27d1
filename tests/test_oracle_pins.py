"""Pins for the CPU oracle (CSR SpMV / SpMM of Section 6.2, loop nest of
Section 4.2).  The paper prints no worked numeric example for this kernel, so
the oracle is tied to what the mathematics fixes: dense brute force, identity
and diagonal matrices, closed forms of the 5-point Laplacian, exact integer
cases, linearity, independent libraries, and rounding-order facts.  Each pin
is meant to break under one plausible mistake (dropped entry, wrong sign or
index, transposed operand, float instead of double accumulation, y0 read when
beta == 0).
"""
import numpy as np
import pytest

import gen
import oracle

EPS = {np.dtype(np.float64): 2.0 ** -53, np.dtype(np.float32): 2.0 ** -24}


def dense_reference(nrows, ncols, rowptr, colidx, vals, X, alpha, beta, Y0):
    """Densify (duplicates add) and do the textbook dense product in Python floats."""
    A = [[0.0] * ncols for _ in range(nrows)]
    for i in range(nrows):
        for j in range(int(rowptr[i]), int(rowptr[i + 1])):
            A[i][int(colidx[j])] += float(vals[j])
    k = X.shape[1]
    Y = np.zeros((nrows, k))
    for i in range(nrows):
        for c in range(k):
            s = 0.0
            for q in range(ncols):
                s += A[i][q] * float(X[q, c])
            Y[i, c] = alpha * s + (beta * float(Y0[i, c]) if beta != 0.0 else 0.0)
    return Y


def bound(nnz_row, absAx, dtype, alpha=1.0, beta=0.0, y0=None):
    extra = 0.0 if y0 is None else abs(beta) * np.abs(y0.astype(np.float64))
    return 8.0 * (nnz_row + 2) * EPS[np.dtype(dtype)] * (abs(alpha) * absAx + extra)


TINY_CASES = [
    # nrows, ncols, lengths, sorted, duplicates
    (1, 1, [1], True, False),
    (1, 1, [0], True, False),
    (7, 1, [1, 0, 1, 1, 0, 0, 1], True, False),            # n x 1
    (1, 9, [9], True, False),                               # one full row
    (12, 12, [0, 12, 3, 0, 0, 5, 1, 12, 7, 2, 0, 4], True, False),
    (33, 20, list(np.arange(33) % 8), False, False),        # unsorted columns
    (25, 6, [9, 0, 4, 6, 11] * 5, True, True),              # duplicates, sorted
    (25, 6, [9, 0, 4, 6, 11] * 5, False, True),             # duplicates, unsorted
    (64, 64, list((np.arange(64) * 7) % 65 % 64), True, False),
]


@pytest.mark.parametrize("dtype", [np.float64, np.float32])
@pytest.mark.parametrize("case", range(len(TINY_CASES)))
@pytest.mark.parametrize("alpha,beta", [(1.0, 0.0), (-2.5, 0.75), (0.0, 2.0), (3.0, 1.0)])
def test_dense_brute_force(case, dtype, alpha, beta):
    nrows, ncols, lengths, srt, dup = TINY_CASES[case]
    rowptr, colidx, vals = gen.random_csr(nrows, ncols, np.array(lengths), 100 + case, dtype,
                                          sorted_cols=srt, allow_duplicates=dup)
    x = gen.uniform(7 + case, gen.STREAM_X, ncols, dtype=np.float64).astype(dtype)
    y0 = gen.uniform(7 + case, gen.STREAM_Y0, nrows, dtype=np.float64).astype(dtype)
    y, absAx = oracle.spmv(rowptr, colidx, vals, x, alpha, beta, y0)
    ref = dense_reference(nrows, ncols, rowptr, colidx, vals, x[:, None], alpha, beta, y0[:, None])[:, 0]
    tol = bound(np.diff(rowptr), absAx, dtype, alpha, beta, y0)
    assert y.dtype == dtype
    assert np.all(np.abs(y.astype(np.float64) - ref) <= tol)
    # |A||x| itself: brute force with absolute values
    ref_abs = dense_reference(nrows, ncols, rowptr, colidx, np.abs(vals), np.abs(x)[:, None],
                              1.0, 0.0, None)[:, 0]
    if not dup:  # with duplicates |a+b| != |a|+|b|, the oracle's is the entrywise one
        assert np.allclose(absAx, ref_abs, rtol=1e-12, atol=0)
    else:
        assert np.all(absAx >= ref_abs * (1 - 1e-12))


@pytest.mark.parametrize("dtype", [np.float64, np.float32])
@pytest.mark.parametrize("case", range(len(TINY_CASES)))
def test_dense_brute_force_exact_small_integers(case, dtype):
    """Small integer data: every partial sum is exact, so any order gives the same bits."""
    nrows, ncols, lengths, srt, dup = TINY_CASES[case]
    rowptr, colidx, vals = gen.random_csr(nrows, ncols, np.array(lengths), 300 + case, dtype,
                                          sorted_cols=srt, allow_duplicates=dup, small_ints=True)
    x = np.floor(gen.uniform(9 + case, gen.STREAM_X, ncols, -8.0, 9.0)).astype(dtype)
    y0 = np.floor(gen.uniform(9 + case, gen.STREAM_Y0, nrows, -8.0, 9.0)).astype(dtype)
    y, _ = oracle.spmv(rowptr, colidx, vals, x, 2.0, -3.0, y0)
    ref = dense_reference(nrows, ncols, rowptr, colidx, vals, x[:, None], 2.0, -3.0, y0[:, None])[:, 0]
    assert np.array_equal(y.astype(np.float64), ref)


@pytest.mark.parametrize("dtype", [np.float64, np.float32])
def test_spmm_dense_brute_force(dtype):
    nrows, ncols, k = 19, 23, 5
    lengths = (np.arange(nrows) * 5) % 12
    rowptr, colidx, vals = gen.random_csr(nrows, ncols, lengths, 55, dtype, sorted_cols=False)
    X = gen.uniform(1, gen.STREAM_X, ncols * k).astype(dtype).reshape(ncols, k)
    Y0 = gen.uniform(1, gen.STREAM_Y0, nrows * k).astype(dtype).reshape(nrows, k)
    Y, absAX = oracle.spmm(rowptr, colidx, vals, X, 1.25, -0.5, Y0)
    ref = dense_reference(nrows, ncols, rowptr, colidx, vals, X, 1.25, -0.5, Y0)
    tol = bound(np.diff(rowptr)[:, None], absAX, dtype, 1.25, -0.5, Y0)
    assert np.all(np.abs(Y.astype(np.float64) - ref) <= tol)
    # a transposed X (column-major read) must not pass: the pin is sensitive to layout
    Yt, _ = oracle.spmm(rowptr, colidx, vals,
                        np.ascontiguousarray(X.T.reshape(ncols, k)), 1.25, -0.5, Y0)
    assert not np.all(np.abs(Yt.astype(np.float64) - ref) <= tol)


def test_spmm_leading_dimension():
    """X given as a strided view (ldx > k) gives the same bits as its compact copy."""
    nrows, ncols, k = 40, 31, 3
    rowptr, colidx, vals = gen.random_csr(nrows, ncols, (np.arange(nrows) % 9), 77)
    Xw = gen.uniform(2, gen.STREAM_X, ncols * 8).reshape(ncols, 8)
    Y1, _ = oracle.spmm(rowptr, colidx, vals, Xw[:, :k])
    Y2, _ = oracle.spmm(rowptr, colidx, vals, np.ascontiguousarray(Xw[:, :k]))
    assert np.array_equal(Y1, Y2)


@pytest.mark.parametrize("dtype", [np.float64, np.float32])
def test_identity_and_diagonal(dtype):
    n = 257
    rowptr = np.arange(n + 1, dtype=np.int32)
    colidx = np.arange(n, dtype=np.int32)
    x = gen.uniform(3, gen.STREAM_X, n).astype(dtype)
    y0 = gen.uniform(3, gen.STREAM_Y0, n).astype(dtype)
    y, absAx = oracle.spmv(rowptr, colidx, np.ones(n, dtype=dtype), x)
    assert np.array_equal(y, x)                       # I x == x, bit for bit
    assert np.array_equal(absAx, np.abs(x).astype(np.float64))
    y, _ = oracle.spmv(rowptr, colidx, np.ones(n, dtype=dtype), x, 2.0, 0.5, y0)
    assert np.array_equal(y, (2.0 * x.astype(np.float64) + 0.5 * y0.astype(np.float64)).astype(dtype))
    d = gen.uniform(3, gen.STREAM_VALUES, n).astype(dtype)
    y, _ = oracle.spmv(rowptr, colidx, d, x)
    assert np.array_equal(y, (d.astype(np.float64) * x.astype(np.float64)).astype(dtype))
    # a permutation matrix picks x[perm]: catches row/column index mix-ups
    perm = np.argsort(gen.uniform(4, 0, n, 0.0, 1.0)).astype(np.int32)
    y, _ = oracle.spmv(rowptr, perm, np.ones(n, dtype=dtype), x)
    assert np.array_equal(y, x[perm])


def test_laplacian_constant_and_linear_closed_forms():
    """5-point Laplacian (diag 4, off-diag -1, out-of-grid neighbours dropped):
    on a constant c row i gives c*(4 - deg_i); on f(i,j) = a*i + b*j + c interior
    rows vanish and a boundary row gives the sum of f over its missing (ghost)
    neighbours.  All integers, so the equalities are exact."""
    nx, ny = 64, 64
    rowptr, colidx, vals = gen.poisson2d(nx, ny)
    n = nx * ny
    deg = np.diff(rowptr) - 1
    for c in (1.0, -3.0, 7.0):
        y, _ = oracle.spmv(rowptr, colidx, vals, np.full(n, c))
        assert np.array_equal(y, c * (4 - deg))
    ii, jj = np.meshgrid(np.arange(nx), np.arange(ny), indexing="ij")
    interior = ((ii > 0) & (ii < nx - 1) & (jj > 0) & (jj < ny - 1)).ravel()
    y, _ = oracle.spmv(rowptr, colidx, vals, np.ones(n))
    assert np.all(y[interior] == 0.0) and np.all(y[~interior] > 0.0)
    for a, b, c in ((1.0, 0.0, 0.0), (0.0, 1.0, 0.0), (2.0, -3.0, 5.0)):
        f = lambda i, j: a * i + b * j + c
        y, _ = oracle.spmv(rowptr, colidx, vals, f(ii, jj).ravel().astype(np.float64))
        ghost = np.zeros((nx, ny))
        ghost[0, :] += f(-1, np.arange(ny))
        ghost[nx - 1, :] += f(nx, np.arange(ny))
        ghost[:, 0] += f(np.arange(nx), -1)
        ghost[:, ny - 1] += f(np.arange(nx), ny)
        assert np.array_equal(y, ghost.ravel())
        assert np.all(y[interior] == 0.0)


def test_laplacian_quadratic_closed_form():
    """On f = i^2 the interior value is -2 (second difference of i^2), exactly."""
    nx, ny = 16, 24
    rowptr, colidx, vals = gen.poisson2d(nx, ny)
    ii, jj = np.meshgrid(np.arange(nx), np.arange(ny), indexing="ij")
    interior = ((ii > 0) & (ii < nx - 1) & (jj > 0) & (jj < ny - 1)).ravel()
    y, _ = oracle.spmv(rowptr, colidx, vals, (ii * ii).ravel().astype(np.float64))
    assert np.all(y[interior] == -2.0)
    y, _ = oracle.spmv(rowptr, colidx, vals, (ii * jj).ravel().astype(np.float64))
    assert np.all(y[interior] == 0.0)


def test_float_matrix_accumulates_in_double_and_rounds_once():
    # 2^24 + 1 + 1: float accumulation would stall at 2^24, double gives 2^24 + 2 exactly
    rowptr = np.array([0, 3], dtype=np.int32)
    colidx = np.array([0, 1, 2], dtype=np.int32)
    vals = np.array([2.0 ** 24, 1.0, 1.0], dtype=np.float32)
    y, _ = oracle.spmv(rowptr, colidx, vals, np.ones(3, dtype=np.float32))
    assert y[0] == np.float32(2.0 ** 24 + 2)
    # left-to-right order in double: (1 + 2^53) - 2^53 == 0, whereas 1 + (2^53 - 2^53) == 1
    vals = np.array([1.0, 2.0 ** 53, -(2.0 ** 53)], dtype=np.float64)
    y, _ = oracle.spmv(rowptr, colidx, vals, np.ones(3))
    assert y[0] == 0.0
    vals = np.array([2.0 ** 53, -(2.0 ** 53), 1.0], dtype=np.float64)
    y, _ = oracle.spmv(rowptr, colidx, vals, np.ones(3))
    assert y[0] == 1.0


def test_no_fused_multiply_add():
    # a*b + c with a*b inexact: fma and mul+add differ in the last bit for this triple
    a = 1.0 + 2.0 ** -30
    b = 1.0 + 2.0 ** -30
    c = -(1.0 + 2.0 ** -29)
    rowptr = np.array([0, 2], dtype=np.int32)
    colidx = np.array([0, 1], dtype=np.int32)
    y, _ = oracle.spmv(rowptr, colidx, np.array([c, a]), np.array([1.0, b]))
    assert y[0] == (a * b) + c            # Python: separate rounding of the product
    assert y[0] == 0.0                    # the fused result would be 2^-60


def test_beta_zero_never_reads_y0_and_alpha_zero_scales():
    rowptr, colidx, vals = gen.random_csr(30, 30, np.arange(30) % 6, 11)
    x = gen.uniform(5, gen.STREAM_X, 30)
    y_a, _ = oracle.spmv(rowptr, colidx, vals, x, 1.0, 0.0, None)
    y_b, _ = oracle.spmv(rowptr, colidx, vals, x, 1.0, 0.0, np.full(30, np.nan))
    assert np.array_equal(y_a, y_b) and np.all(np.isfinite(y_b))
    y0 = gen.uniform(5, gen.STREAM_Y0, 30)
    y, _ = oracle.spmv(rowptr, colidx, vals, x, 0.0, 2.0, y0)
    assert np.array_equal(y, 2.0 * y0)
    empty = np.diff(rowptr) == 0
    y, _ = oracle.spmv(rowptr, colidx, vals, x, 3.0, -1.5, y0)
    assert empty.any() and np.array_equal(y[empty], -1.5 * y0[empty])
    y, _ = oracle.spmv(rowptr, colidx, vals, x)
    assert np.all(y[empty] == 0.0) and not np.any(np.signbit(y[empty]))


@pytest.mark.parametrize("dtype", [np.float64, np.float32])
def test_spmm_column_equals_spmv_bitwise(dtype):
    w = gen.workload(5, {"nx": 6, "ny": 5, "nz": 7, "k": 16})
    vals = w.vals.astype(dtype)
    X = w.x.astype(dtype)
    Y0 = gen.uniform(8, gen.STREAM_Y0, w.nrows * 16).astype(dtype).reshape(w.nrows, 16)
    Y, absAX = oracle.spmm(w.rowptr, w.colidx, vals, X, 0.5, 2.0, Y0)
    for c in range(16):
        y, absAx = oracle.spmv(w.rowptr, w.colidx, vals, np.ascontiguousarray(X[:, c]), 0.5, 2.0,
                               np.ascontiguousarray(Y0[:, c]))
        assert np.array_equal(Y[:, c], y) and np.array_equal(absAX[:, c], absAx)


def test_linearity_within_bound():
    w = gen.workload(3, {"n": 5000, "per_row": 16})
    x2 = gen.uniform(12, gen.STREAM_X, w.ncols)
    y1, a1 = oracle.spmv(w.rowptr, w.colidx, w.vals, w.x)
    y2, a2 = oracle.spmv(w.rowptr, w.colidx, w.vals, x2)
    y12, a12 = oracle.spmv(w.rowptr, w.colidx, w.vals, w.x + x2)
    tol = 8 * 18 * 2.0 ** -53 * (a1 + a2 + a12)
    assert np.all(np.abs(y12 - (y1 + y2)) <= tol)
    yab, _ = oracle.spmv(w.rowptr, w.colidx, w.vals, w.x, w.alpha, w.beta, w.y0)
    assert np.all(np.abs(yab - (w.alpha * y1 + w.beta * w.y0)) <= 8 * 18 * 2.0 ** -53 * (1.5 * a1 + 0.5))


SCALED = [
    (1, None),
    (2, {"nx": 20, "ny": 17, "nz": 23}),
    (3, {"n": 20000}),
    (4, {"n": 30000, "cap": 9000}),
    (5, {"nx": 12, "ny": 9, "nz": 10, "k": 16}),
]


@pytest.mark.parametrize("cfg,scale", SCALED)
def test_against_scipy_and_torch(cfg, scale):
    """The defining call of Section 6.2 is torch.mv(A, x) with A a sparse CSR tensor;
    SciPy's CSR product is a second independent implementation."""
    import scipy.sparse as sp
    import torch

    w = gen.workload(cfg, scale)
    A = sp.csr_matrix((w.vals, w.colidx, w.rowptr), shape=(w.nrows, w.ncols))
    At = torch.sparse_csr_tensor(torch.from_numpy(w.rowptr.astype(np.int64)),
                                 torch.from_numpy(w.colidx.astype(np.int64)),
                                 torch.from_numpy(w.vals), size=(w.nrows, w.ncols))
    nnz_row = np.diff(w.rowptr)
    if w.k == 0:
        y, absAx = oracle.spmv(w.rowptr, w.colidx, w.vals, w.x, w.alpha, w.beta, w.y0)
        base = A @ w.x
        tbase = torch.mv(At, torch.from_numpy(w.x)).numpy()
        y0 = w.y0 if w.y0 is not None else np.zeros(w.nrows, dtype=w.dtype)
    else:
        y, absAx = oracle.spmm(w.rowptr, w.colidx, w.vals, w.x, w.alpha, w.beta, w.y0)
        base = A @ w.x
        tbase = (At @ torch.from_numpy(w.x)).numpy()
        y0 = np.zeros_like(y)
        nnz_row = nnz_row[:, None]
    for lib in (base, tbase):
        ref = w.alpha * lib.astype(np.float64) + w.beta * y0.astype(np.float64)
        # the libraries accumulate in the matrix dtype: allow their error too
        tol = 2 * bound(nnz_row, absAx, w.dtype, w.alpha, w.beta, y0)
        assert np.all(np.abs(y.astype(np.float64) - ref) <= tol)


def test_absAx_is_result_for_nonnegative_data():
    rowptr, colidx, vals = gen.random_csr(200, 150, np.arange(200) % 37, 21)
    x = np.abs(gen.uniform(6, gen.STREAM_X, 150))
    y, absAx = oracle.spmv(rowptr, colidx, np.abs(vals), x)
    assert np.array_equal(y, absAx)
    _, absAx2 = oracle.spmv(rowptr, colidx, -np.abs(vals), x)
    assert np.array_equal(absAx, absAx2)
