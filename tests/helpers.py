"""Shared helpers of the GPU parity tests: upload a workload, call the library
through its C ABI (via the ctypes binding), bring results back, and state the
tolerance."""
import numpy as np

EPS = {np.dtype(np.float64): 2.0 ** -53, np.dtype(np.float32): 2.0 ** -24}


def literal_bound(nnz_row, absAx, dtype):
    """|y - y_ref| <= 8 * nnz_row * eps * (|A||x|)_i, eps = 2^-53 (double) or 2^-24 (float):
    the tolerance the five workloads are held to."""
    return 8.0 * nnz_row * EPS[np.dtype(dtype)] * absAx


def general_bound(nnz_row, absAx, dtype, alpha, beta, y0):
    """The same bound extended to alpha, beta: the two extra roundings of the
    scaling step and the beta*y0 term enter the magnitude."""
    extra = 0.0 if (y0 is None or beta == 0.0) else abs(beta) * np.abs(y0.astype(np.float64))
    return 8.0 * (nnz_row + 2) * EPS[np.dtype(dtype)] * (abs(alpha) * absAx + extra)


def assert_close(got, ref, tol, what=""):
    got = got.astype(np.float64)
    ref = ref.astype(np.float64)
    err = np.abs(got - ref)
    bad = ~(err <= tol)          # also catches NaN
    if bad.any():
        i = np.flatnonzero(bad.ravel())[:5]
        raise AssertionError(
            f"{what}: {bad.sum()} of {bad.size} elements out of tolerance; first at {i.tolist()}: "
            f"got {got.ravel()[i]}, ref {ref.ravel()[i]}, err {err.ravel()[i]}, tol {np.broadcast_to(tol, got.shape).ravel()[i]}")


class DeviceCsr:
    """Uploads CSR arrays and creates the library handle."""

    def __init__(self, nrows, ncols, rowptr, colidx, vals):
        import torch
        import paper_2509_25605_amd as L

        self.L = L
        self.torch = torch
        dev = torch.device("cuda:0")
        self.nrows, self.ncols = nrows, ncols
        self.np_dtype = vals.dtype
        self.h_rowptr, self.h_colidx = rowptr, colidx
        self.rowptr = torch.from_numpy(rowptr).to(dev)
        self.colidx = torch.from_numpy(colidx).to(dev) if colidx.size else torch.empty(0, dtype=torch.int32, device=dev)
        self.vals = torch.from_numpy(vals).to(dev) if vals.size else torch.empty(
            0, dtype=torch.float64 if vals.dtype == np.float64 else torch.float32, device=dev)
        self.mat = L.CsrMatrix(nrows, ncols, self.rowptr, self.colidx, self.vals)

    def spmv(self, x, alpha=1.0, beta=0.0, y0=None, y_fill=None, paper_shape=False):
        torch = self.torch
        dx = torch.from_numpy(np.ascontiguousarray(x, dtype=self.np_dtype)).cuda()
        if y0 is not None:
            dy = torch.from_numpy(np.ascontiguousarray(y0, dtype=self.np_dtype)).cuda()
        else:
            dy = torch.full((self.nrows,), float("nan") if y_fill is None else y_fill,
                            dtype=dx.dtype, device="cuda:0")
        if paper_shape:
            self.L.lapis_spmv_paper_shape(self.mat.handle, alpha, dx, beta, dy)
        else:
            self.mat.spmv(dx, dy, alpha, beta)
        torch.cuda.synchronize()
        return dy.cpu().numpy()

    def spmv_transpose(self, x, alpha=1.0, beta=0.0, y0=None):
        torch = self.torch
        dx = torch.from_numpy(np.ascontiguousarray(x, dtype=self.np_dtype)).cuda()
        if y0 is not None:
            dy = torch.from_numpy(np.ascontiguousarray(y0, dtype=self.np_dtype)).cuda()
        else:
            dy = torch.full((self.ncols,), float("nan"), dtype=dx.dtype, device="cuda:0")
        self.mat.spmv_transpose(dx, dy, alpha, beta)
        torch.cuda.synchronize()
        return dy.cpu().numpy()

    def spmm(self, X, alpha=1.0, beta=0.0, Y0=None, ldx=None, ldy=None):
        torch = self.torch
        k = X.shape[1]
        ldx = ldx or k
        ldy = ldy or k
        dt = torch.float64 if self.np_dtype == np.float64 else torch.float32
        dX = torch.full((max(self.ncols, 1), ldx), float("nan"), dtype=dt, device="cuda:0")
        dX[: self.ncols, :k] = torch.from_numpy(np.ascontiguousarray(X, dtype=self.np_dtype)).cuda()
        dY = torch.full((max(self.nrows, 1), ldy), float("nan"), dtype=dt, device="cuda:0")
        if Y0 is not None:
            dY[: self.nrows, :k] = torch.from_numpy(np.ascontiguousarray(Y0, dtype=self.np_dtype)).cuda()
        self.L.lapis_spmm(self.mat.handle, k, alpha, dX, ldx, beta, dY, ldy)
        torch.cuda.synchronize()
        out = dY.cpu().numpy()
        if ldy > k and self.nrows > 0:
            assert np.all(np.isnan(out[: self.nrows, k:])), "padding columns of Y were written"
        return out[: self.nrows, :k]

    def partition(self):
        return self.mat.partition()

    def index16(self):
        return self.mat.index16()

    def patterns(self):
        return self.mat.patterns()

    def share_classes(self):
        return self.mat.share_classes()

    def split(self):
        return self.mat.split()

    def close(self):
        self.mat.close()
