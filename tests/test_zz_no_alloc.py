"""lapis_spmv_static_scratch (the product for callers that cannot allocate: its intermediate sums
live in a buffer inside the library's code object) against lapis_spmv and the oracle: two calls
in a row, the second on a smaller matrix, so the second finds the first call's leftovers in the
shared buffer."""
import sys

import numpy as np
import pytest

import gen
import oracle
from helpers import DeviceCsr, assert_close, general_bound

pytestmark = pytest.mark.gpu


def say(msg):
    print(f"[case] {msg}", file=sys.stderr, flush=True)


def run_both(w, alpha, beta):
    import torch
    import paper_2509_25605_amd as L

    dev = DeviceCsr(w.nrows, w.ncols, w.rowptr, w.colidx, w.vals)
    try:
        need = L.lapis_spmv_scratch_bytes(dev.mat.handle)
        x = torch.from_numpy(w.x).cuda()
        y0 = gen.uniform(5, gen.STREAM_Y0, w.nrows).astype(w.vals.dtype)
        y_ref = torch.from_numpy(y0).cuda()
        y_new = torch.from_numpy(y0).cuda()
        L.lapis_spmv(dev.mat.handle, alpha, x, beta, y_ref)
        L.lapis_spmv_static_scratch(dev.mat.handle, alpha, x, beta, y_new)
        torch.cuda.synchronize()
        got, same = y_new.cpu().numpy(), y_ref.cpu().numpy()
    finally:
        dev.close()
    ref, absAx = oracle.spmv(w.rowptr, w.colidx, w.vals, w.x, alpha, beta, y0)
    assert_close(got, ref, general_bound(np.diff(w.rowptr), absAx, w.vals.dtype, alpha, beta, y0),
                 "static scratch vs oracle")
    assert np.array_equal(got, same), "the two entry points run the same kernels in the same order"
    return need


def test_two_calls_in_a_row_the_second_smaller():
    # column split with virtual rows, tiles and LDS blocks (x far larger than an L2), then a
    # smaller matrix of the same kind, then one with bin-9 rows but no split
    say("static scratch: wide power-law matrix, n = 1.5 M")
    big = run_both(gen.workload(4, {"n": 1_500_000, "cap": 60_000}), 1.0, 0.0)
    say("static scratch: smaller power-law matrix, n = 0.7 M")
    small = run_both(gen.workload(4, {"n": 700_000, "cap": 20_000}), 1.5, -0.5)
    assert 0 < small < big <= 32 << 20
    say("static scratch: narrow matrix with long rows (tiles, no split)")
    n = 3000
    lengths = np.full(n, 5, dtype=np.int64)
    lengths[[7, 900, 2500]] = [5000, 9000, 4097]
    rowptr, colidx, vals = gen.random_csr(n, 20000, lengths, 77, np.float64)

    class W:
        pass
    w = W()
    w.nrows, w.ncols, w.rowptr, w.colidx, w.vals = n, 20000, rowptr, colidx, vals
    w.x = gen.uniform(78, gen.STREAM_X, 20000)
    tiles_only = run_both(w, 1.0, 0.0)
    assert 0 < tiles_only < small
    say("static scratch: no scratch at all (a stencil)")
    assert run_both(gen.workload(2, {"nx": 24, "ny": 20, "nz": 9}), 1.0, 0.0) == 0


def test_a_matrix_beyond_the_buffer_is_refused():
    import torch
    import paper_2509_25605_amd as L

    say("static scratch: refusal")
    # 300 000 rows of 80 entries over 2^24 columns in doubles: 32 column blocks x 300 000 virtual
    # rows x 8 bytes = 77 MB of sums
    n, ncols, per = 300_000, 1 << 24, 80
    rowptr = torch.arange(0, (n + 1) * per, per, dtype=torch.int32, device="cuda:0")
    step = ncols // per
    colidx = ((torch.arange(n * per, dtype=torch.int64, device="cuda:0") % per) * step
              + (torch.arange(n * per, dtype=torch.int64, device="cuda:0") // per) % step).to(torch.int32)
    vals = torch.ones(n * per, dtype=torch.float64, device="cuda:0")
    x = torch.ones(ncols, dtype=torch.float64, device="cuda:0")
    y = torch.zeros(n, dtype=torch.float64, device="cuda:0")
    with L.CsrMatrix(n, ncols, rowptr, colidx, vals) as A:
        assert L.lapis_spmv_scratch_bytes(A.handle) > 32 << 20
        with pytest.raises(L.LapisError) as e:
            L.lapis_spmv_static_scratch(A.handle, 1.0, x, 0.0, y)
        assert e.value.code == L.LAPIS_ERR_INVALID_ARG and "scratch" in str(e.value)
        L.lapis_spmv(A.handle, 1.0, x, 0.0, y)          # the ordinary entry point takes it
        torch.cuda.synchronize()
        assert torch.all(y == per).item()
