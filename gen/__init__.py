"""Seeded synthetic inputs for the CSR SpMV / SpMM workloads.

Inputs only: sparsity structure, matrix values, dense vectors.  None of the
method's arithmetic lives here, so the CPU oracle's tests and the GPU
library's tests may both draw from this module without sharing any of the
code under test.

The five workloads stand in for the SuiteSparse / Galeri matrices the paper
times in Section 6.2 (Table 3), which are not available offline.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass, field
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "lapis_gen.c")
_LIB = os.path.join(_HERE, "liblapis_gen.so")

BASE_SEED = 20250925  # workload c uses BASE_SEED + c
STREAM_STRUCTURE, STREAM_VALUES, STREAM_X, STREAM_Y0 = 0, 1, 2, 3


def build(force: bool = False) -> str:
    """Compile the generator library with gcc; returns its path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-o", _LIB, _SRC, "-lm"]
        )
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        u64, i64, f64, i32 = ctypes.c_uint64, ctypes.c_int64, ctypes.c_double, ctypes.c_int
        p = ctypes.c_void_p
        lib.lapis_gen_bits.restype = u64
        lib.lapis_gen_bits.argtypes = [u64, u64, u64]
        lib.lapis_gen_uniform_f64.argtypes = [u64, u64, f64, f64, p, i64]
        lib.lapis_gen_uniform_f32.argtypes = [u64, u64, f64, f64, p, i64]
        lib.lapis_gen_normal_f64.argtypes = [u64, u64, p, i64]
        lib.lapis_gen_poisson2d.restype = i64
        lib.lapis_gen_poisson2d.argtypes = [i64, i64, p, p, p]
        lib.lapis_gen_stencil27_rowptr.restype = i64
        lib.lapis_gen_stencil27_rowptr.argtypes = [i64, i64, i64, p]
        lib.lapis_gen_stencil27_fill.argtypes = [i64, i64, i64, u64, p, p, p]
        lib.lapis_gen_fixed_rows.restype = i32
        lib.lapis_gen_fixed_rows.argtypes = [i64, i64, i32, u64, p, p]
        lib.lapis_gen_zipf_lengths.restype = i32
        lib.lapis_gen_zipf_lengths.argtypes = [i64, f64, i64, u64, p]
        lib.lapis_gen_rowptr_from_lengths.restype = i64
        lib.lapis_gen_rowptr_from_lengths.argtypes = [i64, p, p]
        lib.lapis_gen_stratified_cols.restype = i32
        lib.lapis_gen_stratified_cols.argtypes = [i64, i64, p, u64, p]
        lib.lapis_gen_block_stencil_rowptr.restype = i64
        lib.lapis_gen_block_stencil_rowptr.argtypes = [i64, i64, i64, i64, p]
        lib.lapis_gen_block_stencil_fill.argtypes = [i64, i64, i64, i64, u64, p, p, p]
        lib.lapis_gen_gamma_lengths.argtypes = [i64, f64, i64, u64, p]
        lib.lapis_gen_banded_cols.restype = i32
        lib.lapis_gen_banded_cols.argtypes = [i64, i64, p, i64, u64, p]
        _lib = lib
    return _lib


def _ptr(a: np.ndarray):
    return a.ctypes.data_as(ctypes.c_void_p)


# --------------------------------------------------------------------------
# element generators
# --------------------------------------------------------------------------
def bits(seed: int, stream: int, index: int) -> int:
    return int(_load().lapis_gen_bits(seed, stream, index))


def uniform(seed: int, stream: int, n: int, lo: float = -1.0, hi: float = 1.0,
            dtype=np.float64) -> np.ndarray:
    """n draws from U[lo, hi)."""
    out = np.empty(n, dtype=dtype)
    if dtype == np.float64:
        _load().lapis_gen_uniform_f64(seed, stream, lo, hi, _ptr(out), n)
    elif dtype == np.float32:
        _load().lapis_gen_uniform_f32(seed, stream, lo, hi, _ptr(out), n)
    else:
        raise TypeError(dtype)
    return out


def normal(seed: int, stream: int, n: int) -> np.ndarray:
    out = np.empty(n, dtype=np.float64)
    _load().lapis_gen_normal_f64(seed, stream, _ptr(out), n)
    return out


# --------------------------------------------------------------------------
# structures
# --------------------------------------------------------------------------
def poisson2d(nx: int, ny: int):
    """5-point Laplacian, diag 4, off-diag -1, Dirichlet; returns (rowptr, colidx, vals)."""
    n = nx * ny
    rowptr = np.empty(n + 1, dtype=np.int32)
    nnz = _load().lapis_gen_poisson2d(nx, ny, _ptr(rowptr), None, None)
    colidx = np.empty(nnz, dtype=np.int32)
    vals = np.empty(nnz, dtype=np.float64)
    _load().lapis_gen_poisson2d(nx, ny, _ptr(rowptr), _ptr(colidx), _ptr(vals))
    return rowptr, colidx, vals


def stencil27(nx: int, ny: int, nz: int, seed: int):
    """27-point stencil, off-diag U[-1,0), diag 26 + U[0,1); returns (rowptr, colidx, vals)."""
    n = nx * ny * nz
    rowptr = np.empty(n + 1, dtype=np.int32)
    nnz = _load().lapis_gen_stencil27_rowptr(nx, ny, nz, _ptr(rowptr))
    colidx = np.empty(nnz, dtype=np.int32)
    vals = np.empty(nnz, dtype=np.float64)
    _load().lapis_gen_stencil27_fill(nx, ny, nz, seed, _ptr(rowptr), _ptr(colidx), _ptr(vals))
    return rowptr, colidx, vals


def fixed_rows(nrows: int, ncols: int, per_row: int, seed: int):
    """per_row distinct uniform columns per row, sorted; returns (rowptr, colidx)."""
    rowptr = np.empty(nrows + 1, dtype=np.int32)
    colidx = np.empty(nrows * per_row, dtype=np.int32)
    if _load().lapis_gen_fixed_rows(nrows, ncols, per_row, seed, _ptr(rowptr), _ptr(colidx)):
        raise ValueError("fixed_rows: bad arguments")
    return rowptr, colidx


def zipf_rows(nrows: int, ncols: int, s: float, cap: int, seed: int):
    """Row lengths ~ Zipf(s) clipped to [1, cap]; stratified distinct sorted columns."""
    length = np.empty(nrows, dtype=np.int32)
    if _load().lapis_gen_zipf_lengths(nrows, s, cap, seed, _ptr(length)):
        raise ValueError("zipf_rows: bad arguments")
    rowptr = np.empty(nrows + 1, dtype=np.int32)
    nnz = _load().lapis_gen_rowptr_from_lengths(nrows, _ptr(length), _ptr(rowptr))
    if nnz < 0:
        raise ValueError("zipf_rows: nnz exceeds int32")
    colidx = np.empty(nnz, dtype=np.int32)
    if _load().lapis_gen_stratified_cols(nrows, ncols, _ptr(rowptr), seed, _ptr(colidx)):
        raise ValueError("zipf_rows: a row is longer than ncols")
    return rowptr, colidx


def rows_from_lengths(length: np.ndarray, ncols: int, seed: int):
    """Arbitrary row lengths (each <= ncols); stratified distinct sorted columns."""
    length = np.ascontiguousarray(length, dtype=np.int32)
    nrows = length.size
    rowptr = np.empty(nrows + 1, dtype=np.int32)
    nnz = _load().lapis_gen_rowptr_from_lengths(nrows, _ptr(length), _ptr(rowptr))
    if nnz < 0:
        raise ValueError("nnz exceeds int32")
    colidx = np.empty(nnz, dtype=np.int32)
    if _load().lapis_gen_stratified_cols(nrows, ncols, _ptr(rowptr), seed, _ptr(colidx)):
        raise ValueError("a row is longer than ncols")
    return rowptr, colidx


def block_stencil(nx: int, ny: int, nz: int, dof: int, seed: int):
    """27-point stencil with dof unknowns per grid point; returns (rowptr, colidx, vals)."""
    n = nx * ny * nz * dof
    rowptr = np.empty(n + 1, dtype=np.int32)
    nnz = _load().lapis_gen_block_stencil_rowptr(nx, ny, nz, dof, _ptr(rowptr))
    colidx = np.empty(nnz, dtype=np.int32)
    vals = np.empty(nnz, dtype=np.float64)
    _load().lapis_gen_block_stencil_fill(nx, ny, nz, dof, seed, _ptr(rowptr), _ptr(colidx), _ptr(vals))
    return rowptr, colidx, vals


def banded_rows(nrows: int, mean: float, max_len: int, seed: int, band_factor: int = 40):
    """Row lengths with the given mean (approximately) and maximum (exactly), columns in a band
    around the diagonal, sorted and distinct; returns (rowptr, colidx)."""
    length = np.empty(nrows, dtype=np.int32)
    _load().lapis_gen_gamma_lengths(nrows, mean, max_len, seed, _ptr(length))
    rowptr = np.empty(nrows + 1, dtype=np.int32)
    nnz = _load().lapis_gen_rowptr_from_lengths(nrows, _ptr(length), _ptr(rowptr))
    if nnz < 0:
        raise ValueError("banded_rows: nnz exceeds int32")
    colidx = np.empty(nnz, dtype=np.int32)
    if _load().lapis_gen_banded_cols(nrows, nrows, _ptr(rowptr), band_factor, seed, _ptr(colidx)):
        raise ValueError("banded_rows: a row is longer than the matrix is wide")
    return rowptr, colidx


# Shapes of the four matrices of the paper's Table 3 (rows, mean and maximum entries per row).
# The matrices themselves are not available offline; these are synthetic stand-ins of the same shape.
TABLE3_SHAPES = {
    "StocF-1465": (1465137, 14.34, 189),
    "PFlow_742": (742793, 50.0, 137),
    "Elasticity3D_60": (648000, 78.33, 81),
    "audikw_1": (943695, 82.28, 345),
}


def table3_standin(name: str, scale: float = 1.0) -> "Workload":
    """Synthetic f64 matrix with the row count, mean and maximum row length of a Table 3 matrix.
    Elasticity3D_60 is a 60^3 grid with 3 unknowns per point and a 27-point block stencil (the
    construction the paper describes for it); the others get gamma-distributed row lengths and
    banded columns.  `scale` < 1 shrinks the row count (and the grid) for tests."""
    rows, mean, mx = TABLE3_SHAPES[name]
    seed = BASE_SEED + 100 + sorted(TABLE3_SHAPES).index(name)
    if name == "Elasticity3D_60":
        g = max(2, int(round(60 * scale ** (1.0 / 3.0))))
        rowptr, colidx, vals = block_stencil(g, g, g, 3, seed)
    else:
        n = max(mx + 1, int(rows * scale))
        rowptr, colidx = banded_rows(n, mean, mx, seed)
        vals = uniform(seed, STREAM_VALUES, int(rowptr[-1]))
    n = rowptr.size - 1
    return Workload(f"table3_{name}_n{n}_f64", n, n, rowptr, colidx, vals,
                    uniform(seed, STREAM_X, n), 1.0, 0.0, meta={"stands_in_for": name})


# --------------------------------------------------------------------------
# the five workloads
# --------------------------------------------------------------------------
@dataclass
class Workload:
    """One problem instance: y = alpha*A*x + beta*y0 (k == 0) or Y = alpha*A*X + beta*Y0."""
    name: str
    nrows: int
    ncols: int
    rowptr: np.ndarray
    colidx: np.ndarray
    vals: np.ndarray
    x: np.ndarray            # shape (ncols,) for SpMV, (ncols, k) row-major for SpMM
    alpha: float = 1.0
    beta: float = 0.0
    y0: Optional[np.ndarray] = None
    k: int = 0               # 0: SpMV; > 0: SpMM with k columns
    meta: dict = field(default_factory=dict)

    @property
    def nnz(self) -> int:
        return int(self.rowptr[-1])

    @property
    def dtype(self):
        return self.vals.dtype


def workload(cfg: int, scale: Optional[dict] = None) -> Workload:
    """Build workload cfg in 1..5.  `scale` overrides the size parameters so
    that tests can build reduced instances of the same recipe:
      cfg 1: nx, ny          (default 64, 64)
      cfg 2, 5: nx, ny, nz   (default 128^3); cfg 5 also k (default 16)
      cfg 3: n, per_row      (default 2^22, 16)
      cfg 4: n, s, cap       (default 2^23, 1.8, 200000)
      cfg 6..9: scale        (default 1.0; stand-ins for the four matrices of the paper's Table 3)
    """
    sc = dict(scale or {})
    seed = BASE_SEED + cfg
    if cfg == 1:
        nx, ny = sc.get("nx", 64), sc.get("ny", 64)
        rowptr, colidx, vals = poisson2d(nx, ny)
        n = nx * ny
        return Workload(f"poisson2d_{nx}x{ny}_f64", n, n, rowptr, colidx, vals,
                        uniform(seed, STREAM_X, n), 1.0, 0.0)
    if cfg in (2, 5):
        nx, ny, nz = sc.get("nx", 128), sc.get("ny", 128), sc.get("nz", 128)
        mseed = BASE_SEED + 2  # workload 5 reuses workload 2's matrix
        rowptr, colidx, vals = stencil27(nx, ny, nz, mseed)
        n = nx * ny * nz
        if cfg == 2:
            return Workload(f"stencil27_{nx}x{ny}x{nz}_f64", n, n, rowptr, colidx, vals,
                            uniform(seed, STREAM_X, n), 1.0, 0.0)
        k = sc.get("k", 16)
        X = uniform(seed, STREAM_X, n * k).reshape(n, k)
        return Workload(f"stencil27_{nx}x{ny}x{nz}_f64_spmm_k{k}", n, n, rowptr, colidx, vals,
                        X, 1.0, 0.0, k=k)
    if cfg == 3:
        n, per_row = sc.get("n", 1 << 22), sc.get("per_row", 16)
        rowptr, colidx = fixed_rows(n, n, per_row, seed)
        vals = normal(seed, STREAM_VALUES, n * per_row)
        return Workload(f"uniform{per_row}_n{n}_f64", n, n, rowptr, colidx, vals,
                        uniform(seed, STREAM_X, n), 1.5, 0.5,
                        y0=uniform(seed, STREAM_Y0, n))
    if cfg == 4:
        n, s, cap = sc.get("n", 1 << 23), sc.get("s", 1.8), sc.get("cap", 200000)
        rowptr, colidx = zipf_rows(n, n, s, min(cap, n), seed)
        vals = uniform(seed, STREAM_VALUES, int(rowptr[-1]), dtype=np.float32)
        return Workload(f"zipf{s}_cap{cap}_n{n}_f32", n, n, rowptr, colidx, vals,
                        uniform(seed, STREAM_X, n, dtype=np.float32), 1.0, 0.0,
                        meta={"s": s, "cap": cap})
    if cfg in (6, 7, 8, 9):   # stand-ins for the paper's Table 3, in the table's order
        name = ["StocF-1465", "PFlow_742", "Elasticity3D_60", "audikw_1"][cfg - 6]
        return table3_standin(name, sc.get("scale", 1.0))
    raise ValueError(f"unknown workload {cfg}")


def random_csr(nrows: int, ncols: int, lengths: np.ndarray, seed: int, dtype=np.float64,
               sorted_cols: bool = True, allow_duplicates: bool = False, small_ints: bool = False):
    """Small general CSR for unit tests.  With allow_duplicates the columns are
    independent uniform draws (may repeat, not sorted unless sorted_cols)."""
    lengths = np.ascontiguousarray(lengths, dtype=np.int32)
    assert lengths.size == nrows
    if allow_duplicates:
        rowptr = np.zeros(nrows + 1, dtype=np.int32)
        np.cumsum(lengths, out=rowptr[1:])
        nnz = int(rowptr[-1])
        colidx = np.floor(uniform(seed, STREAM_STRUCTURE, nnz, 0.0, float(ncols))).astype(np.int32)
        colidx = np.minimum(colidx, ncols - 1)
        if sorted_cols:
            for i in range(nrows):
                colidx[rowptr[i]:rowptr[i + 1]].sort()
    else:
        rowptr, colidx = rows_from_lengths(lengths, ncols, seed)
        if not sorted_cols:
            key = uniform(seed, STREAM_STRUCTURE + 16, colidx.size, 0.0, 1.0)
            for i in range(nrows):
                b, e = rowptr[i], rowptr[i + 1]
                colidx[b:e] = colidx[b:e][np.argsort(key[b:e], kind="stable")]
    nnz = int(rowptr[-1])
    if small_ints:
        vals = np.floor(uniform(seed, STREAM_VALUES, nnz, -4.0, 5.0)).astype(dtype)
    else:
        vals = uniform(seed, STREAM_VALUES, nnz, dtype=np.float64).astype(dtype)
    return rowptr, colidx, vals
