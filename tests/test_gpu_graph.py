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
