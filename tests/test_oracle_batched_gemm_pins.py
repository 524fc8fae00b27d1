"""Pins for the batched GEMM of the oracle (Section 5: many small products C[b] = A[b] B[b], the
batch dimension being the one that is vectorised): things the definition fixes without the oracle."""
import itertools

import numpy as np
import pytest

import gen
import oracle


def _ints(seed, shape, lo=-4, hi=5):
    u = gen.uniform(seed, 7, int(np.prod(shape)), 0.0, 1.0)
    return (np.floor(u * (hi - lo)) + lo).reshape(shape)


@pytest.mark.parametrize("dtype", [np.float64, np.float32])
@pytest.mark.parametrize("m,n,k", [(1, 1, 1), (2, 3, 4), (5, 1, 7), (1, 6, 2), (8, 8, 8), (3, 16, 5), (16, 16, 16)])
def test_small_integers_are_exact_and_match_the_triple_loop(m, n, k, dtype):
    batch = 5
    A = _ints(11, (batch, m, k)).astype(dtype)
    B = _ints(12, (batch, k, n)).astype(dtype)
    C0 = _ints(13, (batch, m, n)).astype(dtype)
    C, absAB = oracle.batched_gemm(A, B, 2.0, -3.0, C0)
    for b, i, j in itertools.product(range(batch), range(m), range(n)):   # the definition, entry by entry
        s = sum(int(A[b, i, l]) * int(B[b, l, j]) for l in range(k))
        t = sum(abs(int(A[b, i, l])) * abs(int(B[b, l, j])) for l in range(k))
        assert C[b, i, j] == 2 * s - 3 * int(C0[b, i, j])
        assert absAB[b, i, j] == t
    assert C.dtype == dtype and C.shape == (batch, m, n)


def test_identity_diagonal_and_permutation_factors():
    batch, m = 4, 6
    A = gen.uniform(21, 1, batch * m * m).reshape(batch, m, m)
    eye = np.broadcast_to(np.eye(m), (batch, m, m)).copy()
    C, _ = oracle.batched_gemm(A, eye)
    assert np.array_equal(C, A)                                          # A I = A, bit for bit
    C, _ = oracle.batched_gemm(eye, A)
    assert np.array_equal(C, A)
    d = gen.uniform(22, 2, batch * m).reshape(batch, m)
    D = np.zeros((batch, m, m))
    D[:, np.arange(m), np.arange(m)] = d
    C, _ = oracle.batched_gemm(D, A)                                     # rows scaled: one rounding each
    assert np.array_equal(C, d[:, :, None] * A)
    C, _ = oracle.batched_gemm(A, D)                                     # columns scaled
    assert np.array_equal(C, A * d[:, None, :])
    perm = np.array([3, 0, 5, 1, 2, 4])
    P = np.zeros((batch, m, m))
    P[:, np.arange(m), perm] = 1.0                                       # (P A)[i] = A[perm[i]]
    C, _ = oracle.batched_gemm(P, A)
    assert np.array_equal(C, A[:, perm, :])


def test_not_transposed_not_mixed_between_batches():
    # A[b] = b+1 everywhere except one marked entry; a transposed operand or a wrong batch stride
    # moves the mark
    batch, m, n, k = 3, 2, 4, 3
    A = np.zeros((batch, m, k))
    B = np.zeros((batch, k, n))
    for b in range(batch):
        A[b, 1, 2] = b + 1.0                                             # picks row 2 of B[b] into row 1 of C[b]
        B[b, 2, :] = np.arange(n) + 10.0 * (b + 1)
    C, _ = oracle.batched_gemm(A, B)
    for b in range(batch):
        expect = np.zeros((m, n))
        expect[1, :] = (b + 1.0) * (np.arange(n) + 10.0 * (b + 1))
        assert np.array_equal(C[b], expect)


def test_outer_product_and_rank_one_update():
    u = np.array([[1.0, 2.0, 3.0]]).reshape(1, 3, 1)
    v = np.array([[4.0, 5.0]]).reshape(1, 1, 2)
    C, _ = oracle.batched_gemm(u, v)                                     # k = 1: the outer product
    assert np.array_equal(C[0], np.array([[4.0, 5.0], [8.0, 10.0], [12.0, 15.0]]))
    C0 = np.ones((1, 3, 2))
    C, _ = oracle.batched_gemm(u, v, alpha=-1.0, beta=0.5, C0=C0)
    assert np.array_equal(C[0], 0.5 - np.array([[4.0, 5.0], [8.0, 10.0], [12.0, 15.0]]))


def test_beta_zero_does_not_read_c0_and_alpha_zero_scales_it():
    A = gen.uniform(31, 1, 2 * 3 * 4).reshape(2, 3, 4)
    B = gen.uniform(31, 2, 2 * 4 * 5).reshape(2, 4, 5)
    C, _ = oracle.batched_gemm(A, B, 1.0, 0.0, None)
    assert np.all(np.isfinite(C))
    C0 = gen.uniform(31, 3, 2 * 3 * 5).reshape(2, 3, 5)
    C, _ = oracle.batched_gemm(A, B, 0.0, 2.0, C0)
    assert np.array_equal(C, 2.0 * C0)
    empty, _ = oracle.batched_gemm(np.zeros((0, 3, 4)), np.zeros((0, 4, 5)))
    assert empty.shape == (0, 3, 5)


@pytest.mark.parametrize("dtype,eps", [(np.float64, 2.0 ** -53), (np.float32, 2.0 ** -24)])
def test_agrees_with_a_library_product_within_the_summation_bound(dtype, eps):
    batch, m, n, k = 7, 9, 11, 13
    A = gen.uniform(41, 1, batch * m * k).reshape(batch, m, k).astype(dtype)
    B = gen.uniform(41, 2, batch * k * n).reshape(batch, k, n).astype(dtype)
    C, absAB = oracle.batched_gemm(A, B)
    lib = np.matmul(A.astype(np.float64), B.astype(np.float64))          # any summation order
    assert np.all(np.abs(C.astype(np.float64) - lib) <= 2 * (k + 1) * eps * absAB)
    assert np.allclose(absAB, np.matmul(np.abs(A).astype(np.float64), np.abs(B).astype(np.float64)), rtol=1e-12)
