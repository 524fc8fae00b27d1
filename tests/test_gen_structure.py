"""Structure of the seeded synthetic workloads (inputs only).  The counts are
derived by hand in tests/golden/stencil_structure.txt."""
import os

import numpy as np
import pytest

import gen


def _golden(golden_dir):
    out = {}
    with open(os.path.join(golden_dir, "stencil_structure.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            name, n, nnz, *pairs = line.split()
            out[name] = (int(n), int(nnz), {int(p.split(":")[0]): int(p.split(":")[1]) for p in pairs})
    return out


def test_counter_based_generator_is_pure():
    a = gen.uniform(5, 2, 1000)
    b = gen.uniform(5, 2, 2000)
    assert np.array_equal(a, b[:1000])                      # index addressed, not sequential state
    assert not np.array_equal(a, gen.uniform(6, 2, 1000))
    assert not np.array_equal(a, gen.uniform(5, 3, 1000))
    assert a.min() >= -1.0 and a.max() < 1.0
    assert abs(a.mean()) < 0.1 and abs(np.var(b) - 1 / 3) < 0.03
    f = gen.uniform(5, 2, 100000, dtype=np.float32)
    assert f.dtype == np.float32 and f.min() >= -1.0 and f.max() < 1.0
    z = gen.normal(5, 1, 200000)
    assert abs(z.mean()) < 0.01 and abs(z.std() - 1) < 0.01


def test_workload1_structure(golden_dir):
    n, nnz, hist = _golden(golden_dir)["poisson2d_64x64"]
    w = gen.workload(1)
    assert (w.nrows, w.nnz) == (n, nnz) and w.dtype == np.float64
    lens, counts = np.unique(np.diff(w.rowptr), return_counts=True)
    assert dict(zip(lens.tolist(), counts.tolist())) == hist
    for i in (0, 63, 64, 2080, 4095):
        cols = w.colidx[w.rowptr[i]:w.rowptr[i + 1]]
        v = w.vals[w.rowptr[i]:w.rowptr[i + 1]]
        assert np.all(np.diff(cols) > 0)
        assert set((cols - i).tolist()) <= {-64, -1, 0, 1, 64}
        assert np.array_equal(v, np.where(cols == i, 4.0, -1.0))
    assert (w.alpha, w.beta) == (1.0, 0.0)


@pytest.mark.parametrize("dims", [(128, 128, 128), (5, 4, 3), (1, 1, 1), (2, 1, 7)])
def test_workload2_structure(golden_dir, dims):
    nx, ny, nz = dims
    w = gen.workload(2, {"nx": nx, "ny": ny, "nz": nz})
    if dims == (128, 128, 128):
        n, nnz, hist = _golden(golden_dir)["stencil27_128"]
        assert (w.nrows, w.nnz) == (n, nnz)
        lens, counts = np.unique(np.diff(w.rowptr), return_counts=True)
        assert dict(zip(lens.tolist(), counts.tolist())) == hist
    span = lambda m: np.minimum(np.arange(m) + 1, m - 1) - np.maximum(np.arange(m) - 1, 0) + 1
    expect = (span(nz)[:, None, None] * span(ny)[None, :, None] * span(nx)[None, None, :]).ravel()
    assert np.array_equal(np.diff(w.rowptr), expect)
    rows = np.repeat(np.arange(w.nrows), np.diff(w.rowptr))
    c = w.colidx.astype(np.int64)
    for div, mod in ((1, nx), (nx, ny), (nx * ny, nz)):              # x, y, z grid coordinates
        assert np.all(np.abs((c // div) % mod - (rows // div) % mod) <= 1)
    inner = np.ones(w.nnz, dtype=bool)
    inner[w.rowptr[1:-1]] = False
    assert np.all(np.diff(w.colidx)[inner[1:]] > 0)          # strictly ascending inside each row
    diag = w.colidx == rows
    assert diag.sum() == w.nrows
    assert np.all((w.vals[diag] >= 26.0) & (w.vals[diag] < 27.0))
    assert np.all((w.vals[~diag] >= -1.0) & (w.vals[~diag] < 0.0))
    # one independent draw per stored entry, indexed by its CSR position
    u = gen.uniform(gen.BASE_SEED + 2, gen.STREAM_VALUES, w.nnz, 0.0, 1.0)
    assert np.array_equal(w.vals, np.where(diag, 26.0 + u, -1.0 + u))


def test_workload3_structure():
    w = gen.workload(3, {"n": 1 << 16})
    assert np.array_equal(w.rowptr, 16 * np.arange((1 << 16) + 1))
    c = w.colidx.reshape(-1, 16)
    assert np.all(np.diff(c, axis=1) > 0) and c.min() >= 0 and c.max() < (1 << 16)
    assert (w.alpha, w.beta) == (1.5, 0.5) and w.y0 is not None
    # columns are uniform: mean close to n/2, and rows differ
    assert abs(c.mean() / (1 << 16) - 0.5) < 0.01
    assert abs(w.vals.std() - 1) < 0.01


def test_workload4_structure():
    n, cap = 1 << 18, 20000
    w = gen.workload(4, {"n": n, "cap": cap})
    L = np.diff(w.rowptr)
    assert w.dtype == np.float32 and w.x.dtype == np.float32
    assert L.min() == 1 and L.max() == cap
    # P(L = 1) = 1/zeta(1.8) = 0.5313..., P(L = 2) = 2^-1.8 of that
    p1 = (L == 1).mean()
    assert abs(p1 - 0.5313) < 0.01
    assert abs((L == 2).mean() / p1 - 2.0 ** -1.8) < 0.01
    # clipping puts the whole tail on the cap: P(L >= cap) ~ cap^-0.8 / (0.8 zeta)
    tail = cap ** -0.8 / (0.8 * 1.8822)
    assert abs((L == cap).mean() - tail) < 0.5 * tail
    rows = np.repeat(np.arange(n), L)
    inner = np.ones(w.nnz, dtype=bool)
    inner[w.rowptr[1:-1]] = False
    assert np.all(np.diff(w.colidx)[inner[1:]] > 0)          # sorted and distinct per row
    assert w.colidx.min() >= 0 and w.colidx.max() < n
    assert w.vals.min() >= -1.0 and w.vals.max() < 1.0


def test_table3_standins_have_the_papers_shapes(golden_dir):
    """Rows, mean and maximum entries per row as printed in the paper's Table 3."""
    for line in open(os.path.join(golden_dir, "paper_table3.txt")):
        if line.startswith("#") or not line.strip():
            continue
        name, rows, mean, mx, _ = line.split()
        w = gen.table3_standin(name)
        L = np.diff(w.rowptr)
        assert w.nrows == int(rows) and L.max() == int(mx) and L.min() >= 1
        assert abs(L.mean() - float(mean)) < 0.01 * float(mean)
        inner = np.ones(w.nnz, dtype=bool)
        inner[w.rowptr[1:-1]] = False
        assert np.all(np.diff(w.colidx)[inner[1:]] > 0)
        assert w.colidx.min() >= 0 and w.colidx.max() < w.ncols
    # Elasticity3D_60 is exactly the 60^3 x 3-dof block stencil: nnz = 9 * 178^3
    w = gen.table3_standin("Elasticity3D_60")
    assert w.nnz == 9 * 178 ** 3
    rows = np.repeat(np.arange(w.nrows), np.diff(w.rowptr))
    assert np.all(np.abs(w.colidx // 3 % 60 - rows // 3 % 60) <= 1)
