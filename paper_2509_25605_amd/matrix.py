"""A small owner object around the C handle: keeps the borrowed device arrays
alive for as long as the handle exists and frees the handle on close()."""
from __future__ import annotations

from . import binding as B


class CsrMatrix:
    def __init__(self, nrows, ncols, rowptr, colidx, vals, stream=None):
        import torch

        if not (rowptr.is_cuda and colidx.is_cuda and vals.is_cuda):
            raise ValueError("rowptr, colidx and vals must be GPU tensors")
        if rowptr.dtype != torch.int32 or colidx.dtype != torch.int32:
            raise TypeError("rowptr and colidx must be int32")
        if vals.dtype not in (torch.float32, torch.float64):
            raise TypeError("vals must be float32 or float64")
        if not (rowptr.is_contiguous() and colidx.is_contiguous() and vals.is_contiguous()):
            raise ValueError("CSR arrays must be contiguous")
        self.nrows, self.ncols, self.nnz = int(nrows), int(ncols), int(vals.numel())
        self.rowptr, self.colidx, self.vals = rowptr, colidx, vals  # borrowed by the handle
        self.dtype = vals.dtype
        code = B.LAPIS_F64 if vals.dtype == torch.float64 else B.LAPIS_F32
        self.handle = B.lapis_csr_create(self.nrows, self.ncols, self.nnz, rowptr, colidx, vals,
                                         code, stream)

    def _check_vec(self, t, numel, name):
        if not t.is_cuda or t.dtype != self.dtype or not t.is_contiguous() or t.numel() < numel:
            raise ValueError(f"{name}: need a contiguous GPU tensor of {self.dtype} with >= {numel} elements")

    def spmv(self, x, y, alpha=1.0, beta=0.0, stream=None):
        """y = alpha*A*x + beta*y, in place on y; returns y."""
        self._check_vec(x, self.ncols, "x")
        self._check_vec(y, self.nrows, "y")
        B.lapis_spmv(self.handle, alpha, x, beta, y, stream)
        return y

    def spmv_transpose(self, x, y, alpha=1.0, beta=0.0, stream=None):
        """y = alpha*A^T*x + beta*y for x of nrows and y of ncols values, in place on y; returns y."""
        self._check_vec(x, self.nrows, "x")
        self._check_vec(y, self.ncols, "y")
        B.lapis_spmv_transpose(self.handle, alpha, x, beta, y, stream)
        return y

    def spmm(self, X, Y, alpha=1.0, beta=0.0, stream=None):
        """Y = alpha*A*X + beta*Y for row-major X (ncols x k) and Y (nrows x k)."""
        k = X.shape[1]
        if X.dim() != 2 or Y.dim() != 2 or Y.shape[1] != k or X.stride(1) != 1 or Y.stride(1) != 1:
            raise ValueError("X and Y must be row-major 2-D with the same number of columns")
        if X.shape[0] < self.ncols or Y.shape[0] < self.nrows or X.dtype != self.dtype or Y.dtype != self.dtype:
            raise ValueError("X / Y shape or dtype does not match the matrix")
        ldx = X.stride(0) if X.shape[0] > 1 else k
        ldy = Y.stride(0) if Y.shape[0] > 1 else k
        B.lapis_spmm(self.handle, k, alpha, X, ldx, beta, Y, ldy, stream)
        return Y

    def transposed(self, stream=None):
        """A CsrMatrix for A^T whose handle owns its arrays (built on the device)."""
        t = object.__new__(CsrMatrix)
        t.handle = B.lapis_csr_create_transpose(self.handle, stream)
        t.nrows, t.ncols, t.nnz = self.ncols, self.nrows, self.nnz
        t.rowptr = t.colidx = t.vals = None
        t.dtype = self.dtype
        return t

    def arrays(self):
        """Host copies (rowptr, colidx, vals) of the handle's CSR arrays."""
        return B.lapis_csr_copy_arrays(self.handle)

    def index16(self):
        """The 16-bit column offsets of the narrow stream chunks (see lapis_csr_copy_index16)."""
        return B.lapis_csr_copy_index16(self.handle)

    def patterns(self):
        """The row patterns of the stream chunks (see lapis_csr_copy_patterns)."""
        return B.lapis_csr_copy_patterns(self.handle)

    def share_classes(self):
        """How lapis_spmm treats every chunk (see lapis_csr_copy_share_classes); None when not computed."""
        return B.lapis_csr_copy_share_classes(self.handle)

    def partition(self):
        return B.lapis_csr_copy_partition(self.handle)

    def split(self):
        return B.lapis_csr_copy_split(self.handle)

    def close(self):
        if self.handle is not None:
            B.lapis_csr_destroy(self.handle)
            self.handle = None

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.close()
