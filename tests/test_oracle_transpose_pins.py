"""Pins for the oracle's transposed product y = alpha*A^T*x + beta*y0 (the column-wise traversal
of the loop pattern of Section 4.2): dense brute force on A^T, exact integer cases, the adjoint
identity <A u, v> = <u, A^T v>, symmetric matrices (A^T x = A x through the independent row-wise
function), a library cross-check, and the float rounding rule."""
import numpy as np
import pytest
import scipy.sparse as sp

import gen
import oracle
from test_oracle_pins import EPS, TINY_CASES, bound


def dense_transpose_reference(nrows, ncols, rowptr, colidx, vals, x, alpha, beta, y0):
    """Textbook: densify, then y[c] = alpha * sum_i A[i][c] * x[i] + beta * y0[c], Python floats."""
    A = [[0.0] * ncols for _ in range(nrows)]
    for i in range(nrows):
        for j in range(int(rowptr[i]), int(rowptr[i + 1])):
            A[i][int(colidx[j])] += float(vals[j])
    y = np.zeros(ncols)
    for c in range(ncols):
        s = 0.0
        for i in range(nrows):
            s += A[i][c] * float(x[i])
        y[c] = alpha * s + (beta * float(y0[c]) if beta != 0.0 else 0.0)
    return y


def col_counts(colidx, ncols):
    return np.bincount(colidx, minlength=ncols)


@pytest.mark.parametrize("dtype", [np.float64, np.float32])
@pytest.mark.parametrize("case", range(len(TINY_CASES)))
@pytest.mark.parametrize("alpha,beta", [(1.0, 0.0), (-2.5, 0.75), (0.0, 2.0)])
def test_dense_brute_force(case, dtype, alpha, beta):
    nrows, ncols, lengths, srt, dup = TINY_CASES[case]
    rowptr, colidx, vals = gen.random_csr(nrows, ncols, np.array(lengths), 100 + case, dtype,
                                          sorted_cols=srt, allow_duplicates=dup)
    x = gen.uniform(17 + case, gen.STREAM_X, nrows).astype(dtype)
    y0 = gen.uniform(17 + case, gen.STREAM_Y0, ncols).astype(dtype)
    y, absATx = oracle.spmv_transpose(rowptr, colidx, vals, ncols, x, alpha, beta, y0)
    ref = dense_transpose_reference(nrows, ncols, rowptr, colidx, vals, x, alpha, beta, y0)
    assert y.dtype == dtype and y.shape == (ncols,)
    tol = bound(col_counts(colidx, ncols), absATx, dtype, alpha, beta, y0)
    assert np.all(np.abs(y.astype(np.float64) - ref) <= tol)
    ref_abs = dense_transpose_reference(nrows, ncols, rowptr, colidx, np.abs(vals), np.abs(x), 1.0, 0.0, None)
    if not dup:
        assert np.allclose(absATx, ref_abs, rtol=1e-12, atol=0)
    else:
        assert np.all(absATx >= ref_abs * (1 - 1e-12))


@pytest.mark.parametrize("dtype", [np.float64, np.float32])
@pytest.mark.parametrize("case", range(len(TINY_CASES)))
def test_exact_small_integers(case, dtype):
    nrows, ncols, lengths, srt, dup = TINY_CASES[case]
    rowptr, colidx, vals = gen.random_csr(nrows, ncols, np.array(lengths), 300 + case, dtype,
                                          sorted_cols=srt, allow_duplicates=dup, small_ints=True)
    x = np.floor(gen.uniform(19 + case, gen.STREAM_X, nrows, -8.0, 9.0)).astype(dtype)
    y0 = np.floor(gen.uniform(19 + case, gen.STREAM_Y0, ncols, -8.0, 9.0)).astype(dtype)
    y, _ = oracle.spmv_transpose(rowptr, colidx, vals, ncols, x, 2.0, -3.0, y0)
    ref = dense_transpose_reference(nrows, ncols, rowptr, colidx, vals, x, 2.0, -3.0, y0)
    assert np.array_equal(y.astype(np.float64), ref)


def test_not_the_untransposed_product():
    """A rectangular matrix with one entry: A = e_0 e_2^T (1 x 3).  A^T x = x[0] * e_2."""
    rowptr = np.array([0, 1], dtype=np.int32)
    colidx = np.array([2], dtype=np.int32)
    vals = np.array([3.0])
    y, t = oracle.spmv_transpose(rowptr, colidx, vals, 3, np.array([-2.0]))
    assert np.array_equal(y, [0.0, 0.0, -6.0]) and np.array_equal(t, [0.0, 0.0, 6.0])


def test_adjoint_identity():
    """<A u, v> == <u, A^T v> up to rounding, with A u from the row-wise oracle function."""
    n, ncols = 700, 450
    L = (np.arange(n) * 13) % 40
    rowptr, colidx, vals = gen.random_csr(n, ncols, L, 77, np.float64, sorted_cols=False)
    u = gen.uniform(3, gen.STREAM_X, ncols)
    v = gen.uniform(3, gen.STREAM_Y0, n)
    Au, absAu = oracle.spmv(rowptr, colidx, vals, u)
    ATv, absATv = oracle.spmv_transpose(rowptr, colidx, vals, ncols, v)
    lhs, rhs = float(np.dot(Au, v)), float(np.dot(u, ATv))
    scale = float(np.dot(absAu, np.abs(v)))
    assert abs(lhs - rhs) <= 64 * (40 + n) * 2.0 ** -53 * scale
    assert abs(lhs) > 1e-3 * scale / n        # the identity is not satisfied by zeros


def test_symmetric_matrix_equals_rowwise_product():
    """The 5-point Laplacian is symmetric: A^T x and A x have the same terms per element (in a
    different order only where the column order differs from the row order: here they agree,
    both ascending, so the bits agree too)."""
    w = gen.workload(1)
    y1, a1 = oracle.spmv(w.rowptr, w.colidx, w.vals, w.x)
    y2, a2 = oracle.spmv_transpose(w.rowptr, w.colidx, w.vals, w.ncols, w.x)
    assert np.array_equal(y1, y2) and np.array_equal(a1, a2)


@pytest.mark.parametrize("dtype", [np.float64, np.float32])
def test_against_scipy(dtype):
    n, ncols = 3000, 2100
    L = (np.arange(n) * 7) % 60
    rowptr, colidx, vals = gen.random_csr(n, ncols, L, 91, dtype)
    x = gen.uniform(5, gen.STREAM_X, n).astype(dtype)
    y0 = gen.uniform(5, gen.STREAM_Y0, ncols).astype(dtype)
    y, absATx = oracle.spmv_transpose(rowptr, colidx, vals, ncols, x, 1.25, -0.5, y0)
    A = sp.csr_matrix((vals.astype(np.float64), colidx, rowptr), shape=(n, ncols))
    ref = 1.25 * (A.T @ x.astype(np.float64)) - 0.5 * y0.astype(np.float64)
    assert np.all(np.abs(y.astype(np.float64) - ref) <= bound(col_counts(colidx, ncols), absATx, dtype, 1.25, -0.5, y0))


def test_float_matrix_accumulates_in_double_and_rounds_once():
    """2^24 + 1 + 1 in a column: float accumulation would lose both ones, double keeps them and
    the single final rounding gives 2^24 + 2."""
    rowptr = np.array([0, 1, 2, 3], dtype=np.int32)
    colidx = np.zeros(3, dtype=np.int32)
    vals = np.array([2.0 ** 24, 1.0, 1.0], dtype=np.float32)
    y, _ = oracle.spmv_transpose(rowptr, colidx, vals, 1, np.ones(3, dtype=np.float32))
    assert y.dtype == np.float32 and y[0] == np.float32(2.0 ** 24 + 2)


def test_beta_zero_never_reads_y0_and_empty_columns():
    rowptr = np.array([0, 2, 2, 3], dtype=np.int32)
    colidx = np.array([0, 3, 3], dtype=np.int32)
    vals = np.array([1.0, 2.0, 4.0])
    x = np.array([1.0, 100.0, -1.0])
    y, t = oracle.spmv_transpose(rowptr, colidx, vals, 5, x, 2.0, 0.0, None)
    assert np.array_equal(y, [2.0, 0.0, 0.0, -4.0, 0.0]) and np.array_equal(t, [1.0, 0.0, 0.0, 6.0, 0.0])
    y, _ = oracle.spmv_transpose(rowptr, colidx, vals, 5, x, 0.0, 3.0, np.arange(5.0))
    assert np.array_equal(y, 3.0 * np.arange(5.0))


# ---- explicit transposition -------------------------------------------------
def dense(nrows, ncols, rowptr, colidx, vals):
    A = np.zeros((nrows, ncols))
    for i in range(nrows):
        for j in range(int(rowptr[i]), int(rowptr[i + 1])):
            A[i, int(colidx[j])] += float(vals[j])
    return A


@pytest.mark.parametrize("dtype", [np.float64, np.float32])
@pytest.mark.parametrize("case", range(len(TINY_CASES)))
def test_transpose_dense_brute_force_and_order(case, dtype):
    nrows, ncols, lengths, srt, dup = TINY_CASES[case]
    rowptr, colidx, vals = gen.random_csr(nrows, ncols, np.array(lengths), 100 + case, dtype,
                                          sorted_cols=srt, allow_duplicates=dup, small_ints=dup)
    tptr, tidx, tvals = oracle.transpose(rowptr, colidx, vals, ncols)
    assert tptr.dtype == np.int32 and tidx.dtype == np.int32 and tvals.dtype == dtype
    assert tptr[0] == 0 and tptr[-1] == colidx.size and np.all(np.diff(tptr) >= 0)
    assert np.array_equal(np.diff(tptr), col_counts(colidx, ncols))
    assert np.array_equal(dense(ncols, nrows, tptr, tidx, tvals), dense(nrows, ncols, rowptr, colidx, vals).T)
    # the unique order: brute force, column by column, scanning A in row order
    rows_of = np.repeat(np.arange(nrows), np.diff(rowptr))
    for c in range(ncols):
        js = [j for j in range(colidx.size) if colidx[j] == c]
        assert np.array_equal(tidx[tptr[c]:tptr[c + 1]], rows_of[js])
        assert np.array_equal(tvals[tptr[c]:tptr[c + 1]], vals[js])


def test_transpose_hand_example():
    """A = [[a . b], [. . .], [c d .]]  ->  A^T rows: [a c], [d], [b]."""
    rowptr = np.array([0, 2, 2, 4], dtype=np.int32)
    colidx = np.array([0, 2, 0, 1], dtype=np.int32)
    vals = np.array([1.0, 2.0, 3.0, 4.0])
    tptr, tidx, tvals = oracle.transpose(rowptr, colidx, vals, 3)
    assert tptr.tolist() == [0, 2, 3, 4] and tidx.tolist() == [0, 2, 2, 0] and tvals.tolist() == [1.0, 3.0, 4.0, 2.0]


def test_transpose_twice_is_identity_for_sorted_rows():
    n, ncols = 900, 1300
    L = (np.arange(n) * 11) % 70
    rowptr, colidx, vals = gen.random_csr(n, ncols, L, 13, np.float64)
    t = oracle.transpose(rowptr, colidx, vals, ncols)
    b = oracle.transpose(*t, n)
    assert np.array_equal(b[0], rowptr) and np.array_equal(b[1], colidx) and np.array_equal(b[2], vals)


@pytest.mark.parametrize("cfg,scale", [(1, None), (4, {"n": 1 << 12, "cap": 1000})])
def test_transpose_against_scipy(cfg, scale):
    w = gen.workload(cfg, scale)
    tptr, tidx, tvals = oracle.transpose(w.rowptr, w.colidx, w.vals, w.ncols)
    ref = sp.csr_matrix((w.vals, w.colidx, w.rowptr), shape=(w.nrows, w.ncols)).T.tocsr()
    ref.sort_indices()
    assert np.array_equal(tptr, ref.indptr) and np.array_equal(tidx, ref.indices) and np.array_equal(tvals, ref.data)


def test_product_with_transposed_arrays_is_the_transposed_product_bitwise():
    """Row c of A^T lists column c of A in row order, which is the order the transposed product
    adds in: the two oracle functions must agree to the bit."""
    n, ncols = 1200, 800
    L = (np.arange(n) * 5) % 90
    rowptr, colidx, vals = gen.random_csr(n, ncols, L, 14, np.float64, sorted_cols=False)
    x = gen.uniform(6, gen.STREAM_X, n)
    y0 = gen.uniform(6, gen.STREAM_Y0, ncols)
    t = oracle.transpose(rowptr, colidx, vals, ncols)
    y1, a1 = oracle.spmv(*t, x, 1.5, -2.0, y0)
    y2, a2 = oracle.spmv_transpose(rowptr, colidx, vals, ncols, x, 1.5, -2.0, y0)
    assert np.array_equal(y1, y2) and np.array_equal(a1, a2)
