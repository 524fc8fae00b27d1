"""lapis_spmv / lapis_spmm enqueue kernels only (no allocation, no copy, no memset), so a caller can
record them into a HIP graph; replays must reproduce the eager result."""
import numpy as np
import pytest
import torch

import gen
import oracle
import paper_2509_25605_amd as L

pytestmark = pytest.mark.gpu


def _say(msg):
    print(f"[case] {msg}", flush=True)


@pytest.mark.parametrize("cfg,scale", [(1, None), (2, {"nx": 40, "ny": 12, "nz": 9}), (4, {"n": 30000, "cap": 20000})])
def test_spmv_in_a_graph_replays_like_eager(cfg, scale):
    _say(f"graph capture workload {cfg}")
    w = gen.workload(cfg, scale)
    dt = torch.float64 if w.dtype == np.float64 else torch.float32
    rowptr, colidx, vals = (torch.from_numpy(a).cuda() for a in (w.rowptr, w.colidx, w.vals))
    x = torch.from_numpy(np.ascontiguousarray(w.x)).cuda()
    y = torch.zeros(w.nrows, dtype=dt, device="cuda")
    eps = 2.0 ** -53 if w.dtype == np.float64 else 2.0 ** -24
    with L.CsrMatrix(w.nrows, w.ncols, rowptr, colidx, vals) as A:
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            A.spmv(x, y, 1.0, 0.0)                      # warm-up outside the capture
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            A.spmv(x, y, 1.0, 0.0)
        for rep in range(3):
            xh = gen.uniform(700 + rep, gen.STREAM_X, w.ncols).astype(w.dtype)
            x.copy_(torch.from_numpy(xh))               # eager work between the replays
            y.fill_(float("nan"))
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            got = y.cpu().numpy().astype(np.float64)
            ref, absAx = oracle.spmv(w.rowptr, w.colidx, w.vals, xh)
            tol = 8.0 * np.diff(w.rowptr) * eps * absAx
            assert np.all(np.abs(got - ref.astype(np.float64)) <= tol), f"replay {rep} differs"
            eager = torch.empty_like(y)
            A.spmv(x, eager, 1.0, 0.0)
            torch.cuda.synchronize()
            assert torch.equal(eager, y), f"replay {rep} is not bitwise the eager result"


def test_spmm_and_batched_gemm_in_a_graph():
    _say("graph capture spmm + batched gemm")
    w = gen.workload(5, {"nx": 20, "ny": 12, "nz": 9, "k": 16})
    rowptr, colidx, vals = (torch.from_numpy(a).cuda() for a in (w.rowptr, w.colidx, w.vals))
    X = torch.from_numpy(np.ascontiguousarray(w.x)).cuda()
    Y = torch.zeros(w.nrows, 16, dtype=torch.float64, device="cuda")
    batch, m = 300, 6
    A = gen.uniform(81, 1, batch * m * m).reshape(batch, m, m)
    B = gen.uniform(81, 2, batch * m * m).reshape(batch, m, m)
    dA, dB = torch.from_numpy(A).cuda(), torch.from_numpy(B).cuda()
    dC = torch.zeros(batch, m, m, dtype=torch.float64, device="cuda")
    with L.CsrMatrix(w.nrows, w.ncols, rowptr, colidx, vals) as M:
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            M.spmm(X, Y)
            L.lapis_batched_gemm(batch, m, m, m, 1.0, dA, dB, 0.0, dC, L.LAPIS_F64)
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            M.spmm(X, Y)
            L.lapis_batched_gemm(batch, m, m, m, 1.0, dA, dB, 0.0, dC, L.LAPIS_F64)
        for rep in range(3):
            Xh = gen.uniform(800 + rep, gen.STREAM_X, w.ncols * 16).reshape(w.ncols, 16)
            X.copy_(torch.from_numpy(Xh))
            Ah = gen.uniform(810 + rep, 1, batch * m * m).reshape(batch, m, m)
            dA.copy_(torch.from_numpy(Ah))
            Y.fill_(float("nan"))
            dC.fill_(float("nan"))
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            ref, absAX = oracle.spmm(w.rowptr, w.colidx, w.vals, Xh)
            tol = 8.0 * np.diff(w.rowptr)[:, None] * 2.0 ** -53 * absAX
            assert np.all(np.abs(Y.cpu().numpy() - ref) <= tol), f"spmm replay {rep} differs"
            refC, absAB = oracle.batched_gemm(Ah, B)
            assert np.all(np.abs(dC.cpu().numpy() - refC) <= 8.0 * (m + 2) * 2.0 ** -53 * absAB), f"gemm replay {rep} differs"
