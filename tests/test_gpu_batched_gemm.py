"""Parity of lapis_batched_gemm (through the C ABI) with the CPU oracle, element by element."""
import numpy as np
import pytest
import torch

import gen
import oracle
import paper_2509_25605_amd as L

pytestmark = pytest.mark.gpu

EPS = {np.float64: 2.0 ** -53, np.float32: 2.0 ** -24}


def say(msg):
    """Names the case before the GPU step (flushed: a faulting run leaves it in the log)."""
    print(f"[case] {msg}", flush=True)


def _run(A, B, alpha=1.0, beta=0.0, C0=None):
    batch, m, k = A.shape
    n = B.shape[2]
    dt = torch.float64 if A.dtype == np.float64 else torch.float32
    dA = torch.from_numpy(np.ascontiguousarray(A)).cuda()
    dB = torch.from_numpy(np.ascontiguousarray(B)).cuda()
    if C0 is None:
        dC = torch.full((batch, m, n), float("nan"), dtype=dt, device="cuda")     # beta == 0: never read
    else:
        dC = torch.from_numpy(np.ascontiguousarray(C0)).cuda()
    code = L.LAPIS_F64 if A.dtype == np.float64 else L.LAPIS_F32
    L.lapis_batched_gemm(batch, m, n, k, alpha, dA, dB, beta, dC, code, torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    return dC.cpu().numpy()


def _check(A, B, alpha=1.0, beta=0.0, C0=None, what=""):
    got = _run(A, B, alpha, beta, C0)
    ref, absAB = oracle.batched_gemm(A, B, alpha, beta, C0)
    k = A.shape[2]
    eps = EPS[A.dtype.type]
    # both sides sum k products (the oracle in double): |difference| <= 8 (k + 2) eps (|alpha| |A||B| + |beta||C0|)
    bound = 8.0 * (k + 2) * eps * (abs(alpha) * absAB + (abs(beta) * np.abs(C0) if C0 is not None else 0.0))
    err = np.abs(got.astype(np.float64) - ref.astype(np.float64))
    bad = np.argwhere(~(err <= bound))
    assert bad.size == 0, f"{what}: {bad.shape[0]} elements off, first {bad[0]}: {got[tuple(bad[0])]} vs {ref[tuple(bad[0])]}"


SHAPES = [(1, 1, 1), (2, 3, 4), (3, 3, 3), (4, 4, 4), (5, 7, 6), (8, 8, 8), (7, 1, 9), (1, 13, 2), (12, 12, 12),
          (16, 16, 16), (10, 20, 5), (17, 5, 31), (32, 32, 32), (32, 1, 32), (2, 32, 2),
          # whole matrix-core tiles in m and n, k in whole steps (8 doubles / 16 floats) and not
          (16, 32, 8), (32, 16, 24), (16, 16, 32), (32, 32, 16), (32, 32, 8), (16, 32, 12), (32, 32, 20)]


@pytest.mark.parametrize("dtype", [np.float64, np.float32])
@pytest.mark.parametrize("m,n,k", SHAPES)
def test_batched_gemm_shapes(m, n, k, dtype):
    say(f"batched gemm {m}x{n}x{k} {np.dtype(dtype).name}")
    batch = 1000 + 37                                   # several tiles and a ragged last one
    A = gen.uniform(51, 1, batch * m * k).reshape(batch, m, k).astype(dtype)
    B = gen.uniform(51, 2, batch * k * n).reshape(batch, k, n).astype(dtype)
    C0 = gen.uniform(51, 3, batch * m * n).reshape(batch, m, n).astype(dtype)
    _check(A, B, what="alpha=1 beta=0")
    _check(A, B, -0.5, 1.25, C0, what="alpha=-0.5 beta=1.25")


@pytest.mark.parametrize("dtype", [np.float64, np.float32])
@pytest.mark.parametrize("m,n,k", [(8, 8, 8), (12, 12, 12), (16, 16, 16), (24, 20, 32), (32, 32, 32)])
def test_batched_gemm_operands_one_element_off_alignment(m, n, k, dtype):
    """Operands that start one element into their allocations: aligned to the element only, so neither
    kernel may use its 16-byte accesses."""
    say(f"batched gemm {m}x{n}x{k} {np.dtype(dtype).name}, operands one element past 16-byte alignment")
    batch = 301
    A = gen.uniform(53, 1, batch * m * k).reshape(batch, m, k).astype(dtype)
    B = gen.uniform(53, 2, batch * k * n).reshape(batch, k, n).astype(dtype)
    C0 = gen.uniform(53, 3, batch * m * n).reshape(batch, m, n).astype(dtype)

    def shifted(a):
        buf = torch.empty(a.size + 1, dtype=torch.from_numpy(a).dtype, device="cuda")
        view = buf[1:].view(a.shape)
        view.copy_(torch.from_numpy(a))
        assert view.data_ptr() % 16 != 0
        return view

    dA, dB, dC = shifted(A), shifted(B), shifted(C0)
    code = L.LAPIS_F64 if dtype == np.float64 else L.LAPIS_F32
    L.lapis_batched_gemm(batch, m, n, k, 0.75, dA, dB, -1.5, dC, code, torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    got = dC.cpu().numpy()
    ref, absAB = oracle.batched_gemm(A, B, 0.75, -1.5, C0)
    bound = 8.0 * (k + 2) * EPS[dtype] * (0.75 * absAB + 1.5 * np.abs(C0))
    assert np.all(np.abs(got.astype(np.float64) - ref.astype(np.float64)) <= bound)


def test_batched_gemm_small_integers_exact_and_batch_sizes():
    for batch in (1, 2, 63, 64, 65, 4097):
        say(f"batched gemm integers batch={batch}")
        m, n, k = 6, 5, 7
        u = gen.uniform(61, 1, batch * (m * k + k * n))
        A = np.floor(u[: batch * m * k] * 9 - 4).reshape(batch, m, k)
        B = np.floor(u[batch * m * k:] * 9 - 4).reshape(batch, k, n)
        got = _run(A, B)
        ref, _ = oracle.batched_gemm(A, B)
        assert np.array_equal(got, ref)                 # integers: every order of summation is exact


def test_batched_gemm_errors_and_empty_batch():
    s = torch.cuda.current_stream().cuda_stream
    t = torch.zeros(16, dtype=torch.float64, device="cuda")
    L.lapis_batched_gemm(0, 2, 2, 2, 1.0, None, None, 0.0, None, L.LAPIS_F64, s)       # nothing to do
    for args in [(-1, 2, 2, 2), (1, 0, 2, 2), (1, 2, 33, 2), (1, 2, 2, 40)]:
        with pytest.raises(L.LapisError) as e:
            L.lapis_batched_gemm(*args, 1.0, t, t, 0.0, t, L.LAPIS_F64, s)
        assert e.value.code == L.LAPIS_ERR_INVALID_ARG
    with pytest.raises(L.LapisError) as e:
        L.lapis_batched_gemm(1, 2, 2, 2, 1.0, t, None, 0.0, t, L.LAPIS_F64, s)
    assert e.value.code == L.LAPIS_ERR_INVALID_ARG
    with pytest.raises(L.LapisError) as e:
        L.lapis_batched_gemm(1, 2, 2, 2, 1.0, t, t, 0.0, t, 7, s)
    assert e.value.code == L.LAPIS_ERR_UNSUPPORTED


def test_batched_gemm_non_finite_values():
    A = np.ones((3, 2, 2))
    B = np.ones((3, 2, 2))
    A[1, 0, 1] = np.inf
    B[2, 1, 0] = np.nan
    got = _run(A, B)
    ref, _ = oracle.batched_gemm(A, B)
    assert np.array_equal(np.isnan(got), np.isnan(ref)) and np.array_equal(np.isinf(got), np.isinf(ref))
    assert np.array_equal(got[0], ref[0])


def test_batched_gemm_large_batch_sampled():
    """The size the bench times (2^20 products of 8 x 8 doubles), checked on sampled entries."""
    say("batched gemm 2^20 x 8x8x8 sampled")
    batch, m = 1 << 20, 8
    A = gen.uniform(71, 1, batch * m * m).reshape(batch, m, m)
    B = gen.uniform(71, 2, batch * m * m).reshape(batch, m, m)
    got = _run(A, B)
    pick = np.unique(np.concatenate([[0, 1, batch - 1, batch - 2], (gen.uniform(72, 1, 4000, 0.0, 1.0) * batch).astype(np.int64)]))
    ref, absAB = oracle.batched_gemm(A[pick], B[pick])
    assert np.all(np.abs(got[pick] - ref) <= 8.0 * (m + 2) * EPS[np.float64] * absAB)
