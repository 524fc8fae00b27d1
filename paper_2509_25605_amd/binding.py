"""ctypes binding of liblapis_mi355x.so: argument marshalling only.

The functions carry the names of the C entry points (include/lapis.h).  Array
arguments are torch tensors on the GPU (their data_ptr() is passed) or plain
integer device addresses; PyTorch serves for device memory and streams only.
There is no CPU fallback: if the library is not built, loading it raises.
"""
from __future__ import annotations

import ctypes
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "liblapis_mi355x.so")

LAPIS_OK, LAPIS_ERR_INVALID_ARG, LAPIS_ERR_UNSUPPORTED, LAPIS_ERR_ALLOC, LAPIS_ERR_DEVICE = range(5)
LAPIS_F32, LAPIS_F64 = 0, 1

EXPORTS = [
    "lapis_csr_create", "lapis_spmv", "lapis_spmv_paper_shape", "lapis_paper_vector_length", "lapis_spmm", "lapis_csr_destroy",
    "lapis_csr_partition_sizes", "lapis_csr_copy_partition", "lapis_csr_split_sizes",
    "lapis_csr_copy_split", "lapis_csr_half_bandwidth", "lapis_partition_constants",
    "lapis_csr_copy_index16", "lapis_csr_copy_patterns", "lapis_csr_copy_share_classes", "lapis_csr_huge_sizes", "lapis_csr_copy_huge",
    "lapis_spmv_transpose", "lapis_csr_create_transpose", "lapis_csr_shape", "lapis_csr_copy_arrays",
    "lapis_dualview_create", "lapis_dualview_subview", "lapis_dualview_host", "lapis_dualview_device",
    "lapis_dualview_modify_host", "lapis_dualview_modify_device", "lapis_dualview_sync_device",
    "lapis_dualview_sync_host", "lapis_dualview_copy_counts", "lapis_dualview_destroy",
    "lapis_spmv_dualview",
    "lapis_batched_gemm",
    "lapis_spmv_static_scratch", "lapis_spmv_scratch_bytes",
    "lapis_last_error",
]


class LapisError(RuntimeError):
    def __init__(self, code: int, text: str):
        super().__init__(f"lapis error {code}: {text}")
        self.code = code


_lib = None


def load() -> ctypes.CDLL:
    """Load the built library (build with `python -m paper_2509_25605_amd.build`)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                f"{LIB_PATH} is not built; run paper_2509_25605_amd.build.build() first")
        # One HIP runtime per process: PyTorch (which owns the streams and the device memory the
        # callers pass in) ships its own, so it is loaded first and this library binds to it.
        import torch  # noqa: F401

        lib = ctypes.CDLL(LIB_PATH)
        i64, f64, p, i32 = ctypes.c_int64, ctypes.c_double, ctypes.c_void_p, ctypes.c_int
        lib.lapis_csr_create.argtypes = [ctypes.POINTER(p), i64, i64, i64, p, p, p, i32, p]
        lib.lapis_spmv.argtypes = [p, f64, p, f64, p, p]
        lib.lapis_spmv_paper_shape.argtypes = [p, f64, p, f64, p, p]
        lib.lapis_spmv_static_scratch.argtypes = [p, f64, p, f64, p, p]
        lib.lapis_spmv_scratch_bytes.argtypes = [p]
        lib.lapis_spmv_transpose.argtypes = [p, f64, p, f64, p, p]
        lib.lapis_csr_huge_sizes.argtypes = [p] + [ctypes.POINTER(i64)] * 3
        lib.lapis_csr_copy_huge.argtypes = [p, p, p, p]
        lib.lapis_csr_copy_index16.argtypes = [p, ctypes.POINTER(i32), ctypes.POINTER(i64), ctypes.POINTER(i64), p, p, p]
        lib.lapis_csr_copy_patterns.argtypes = [p, ctypes.POINTER(i32), ctypes.POINTER(i64), ctypes.POINTER(i64), p, p, p]
        lib.lapis_csr_copy_share_classes.argtypes = [p, ctypes.POINTER(i32), p]
        lib.lapis_csr_create_transpose.argtypes = [ctypes.POINTER(p), p, p]
        lib.lapis_csr_shape.argtypes = [p] + [ctypes.POINTER(i64)] * 3 + [ctypes.POINTER(i32)]
        lib.lapis_csr_copy_arrays.argtypes = [p, p, p, p]
        lib.lapis_paper_vector_length.argtypes = [i64, i64]
        lib.lapis_spmm.argtypes = [p, i64, f64, p, i64, f64, p, i64, p]
        lib.lapis_csr_destroy.argtypes = [p]
        lib.lapis_csr_partition_sizes.argtypes = [p] + [ctypes.POINTER(i64)] * 4
        lib.lapis_csr_copy_partition.argtypes = [p, p, p, p, p, p, p, p]
        lib.lapis_csr_split_sizes.argtypes = [p] + [ctypes.POINTER(i64)] * 6
        lib.lapis_csr_copy_split.argtypes = [p, p, p, p, p, p, p]
        lib.lapis_csr_half_bandwidth.argtypes = [p, ctypes.POINTER(i64)]
        lib.lapis_partition_constants.argtypes = [ctypes.POINTER(i64)]
        lib.lapis_dualview_create.argtypes = [ctypes.POINTER(p), i64]
        lib.lapis_dualview_subview.argtypes = [ctypes.POINTER(p), p, i64, i64]
        for name in ("lapis_dualview_host", "lapis_dualview_device"):
            getattr(lib, name).argtypes = [p]
        for name in ("lapis_dualview_modify_host", "lapis_dualview_modify_device", "lapis_dualview_destroy"):
            getattr(lib, name).argtypes = [p]
        for name in ("lapis_dualview_sync_device", "lapis_dualview_sync_host"):
            getattr(lib, name).argtypes = [p, p]
        lib.lapis_dualview_copy_counts.argtypes = [p, ctypes.POINTER(i64), ctypes.POINTER(i64)]
        lib.lapis_spmv_dualview.argtypes = [p, f64, p, f64, p, p]
        lib.lapis_batched_gemm.argtypes = [i64, i32, i32, i32, f64, p, p, f64, p, i32, p]
        for name in EXPORTS[:-1]:
            getattr(lib, name).restype = i32
        lib.lapis_spmv_scratch_bytes.restype = i64
        lib.lapis_dualview_host.restype = p
        lib.lapis_dualview_device.restype = p
        lib.lapis_last_error.restype = ctypes.c_char_p
        lib.lapis_last_error.argtypes = []
        _lib = lib
    return _lib


def _addr(a):
    """Device address of a torch tensor, or the integer / None given."""
    if a is None:
        return None
    if isinstance(a, int):
        return a
    return a.data_ptr()


def _stream(stream):
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


def _check(rc: int):
    if rc != LAPIS_OK:
        raise LapisError(rc, load().lapis_last_error().decode())


def lapis_last_error() -> str:
    return load().lapis_last_error().decode()


def lapis_csr_create(nrows, ncols, nnz, d_rowptr, d_colidx, d_vals, dtype, stream=None):
    """Returns the opaque handle (a ctypes.c_void_p).  The three arrays are borrowed."""
    out = ctypes.c_void_p()
    _check(load().lapis_csr_create(ctypes.byref(out), nrows, ncols, nnz, _addr(d_rowptr),
                                   _addr(d_colidx), _addr(d_vals), dtype, _stream(stream)))
    return out


def lapis_spmv(A, alpha, d_x, beta, d_y, stream=None):
    _check(load().lapis_spmv(A, float(alpha), _addr(d_x), float(beta), _addr(d_y), _stream(stream)))


def lapis_spmv_static_scratch(A, alpha, d_x, beta, d_y, stream=None):
    _check(load().lapis_spmv_static_scratch(A, float(alpha), _addr(d_x), float(beta), _addr(d_y), _stream(stream)))


def lapis_spmv_scratch_bytes(A) -> int:
    return int(load().lapis_spmv_scratch_bytes(A))


def lapis_csr_copy_index16(A):
    """dict(enabled, narrow_entries, framed_entries, chunk_base, frame_table, col16) of a handle
    (arrays None when not enabled)."""
    n, _, z, _ = lapis_csr_shape(A)
    on, narrow, framed = ctypes.c_int(), ctypes.c_int64(), ctypes.c_int64()
    _check(load().lapis_csr_copy_index16(A, ctypes.byref(on), ctypes.byref(narrow), ctypes.byref(framed), None, None, None))
    out = {"enabled": bool(on.value), "narrow_entries": narrow.value, "framed_entries": framed.value,
           "chunk_base": None, "frame_table": None, "col16": None}
    if on.value:
        rows = lapis_partition_constants()["stream_rows"]
        chunks = (n + rows - 1) // rows
        out["chunk_base"] = np.empty(chunks, dtype=np.int32)
        out["frame_table"] = np.empty(32 * chunks, dtype=np.int32)
        out["col16"] = np.empty(z, dtype=np.uint16)
        _check(load().lapis_csr_copy_index16(A, None, None, None, out["chunk_base"].ctypes.data,
                                             out["frame_table"].ctypes.data, out["col16"].ctypes.data))
    return out


def lapis_csr_copy_share_classes(A):
    """int32 array of the share class of every chunk of a handle, or None when the classes were not computed."""
    n, _, _, _ = lapis_csr_shape(A)
    on = ctypes.c_int()
    _check(load().lapis_csr_copy_share_classes(A, ctypes.byref(on), None))
    if not on.value:
        return None
    out = np.zeros((n + 31) // 32, dtype=np.int32)
    _check(load().lapis_csr_copy_share_classes(A, ctypes.byref(on), out.ctypes.data_as(ctypes.c_void_p)))
    return out


def lapis_csr_copy_patterns(A):
    """dict(enabled, entries, pat_off, row_pat, pool) of a handle (arrays None when not enabled)."""
    n, _, _, _ = lapis_csr_shape(A)
    on, entries, pool = ctypes.c_int(), ctypes.c_int64(), ctypes.c_int64()
    _check(load().lapis_csr_copy_patterns(A, ctypes.byref(on), ctypes.byref(entries), ctypes.byref(pool), None, None, None))
    out = {"enabled": bool(on.value), "entries": entries.value, "pool_size": pool.value,
           "pat_off": None, "row_pat": None, "pool": None}
    if on.value:
        rows = lapis_partition_constants()["stream_rows"]
        out["pat_off"] = np.empty((n + rows - 1) // rows + 1, dtype=np.int32)
        out["row_pat"] = np.empty(n, dtype=np.uint16)
        out["pool"] = np.empty(pool.value, dtype=np.int32)
        _check(load().lapis_csr_copy_patterns(A, None, None, None, out["pat_off"].ctypes.data,
                                              out["row_pat"].ctypes.data, out["pool"].ctypes.data))
    return out


def lapis_csr_create_transpose(A, stream=None):
    """Returns the handle of A^T (it owns its arrays)."""
    h = ctypes.c_void_p()
    _check(load().lapis_csr_create_transpose(ctypes.byref(h), A, _stream(stream)))
    return h


def lapis_csr_shape(A):
    """(nrows, ncols, nnz, dtype code) of a handle."""
    n, m, z, d = ctypes.c_int64(), ctypes.c_int64(), ctypes.c_int64(), ctypes.c_int()
    _check(load().lapis_csr_shape(A, ctypes.byref(n), ctypes.byref(m), ctypes.byref(z), ctypes.byref(d)))
    return n.value, m.value, z.value, d.value


def lapis_csr_copy_arrays(A):
    """Host copies (rowptr, colidx, vals) of a handle's CSR arrays."""
    n, _, z, d = lapis_csr_shape(A)
    rowptr = np.empty(n + 1, dtype=np.int32)
    colidx = np.empty(z, dtype=np.int32)
    vals = np.empty(z, dtype=np.float64 if d == LAPIS_F64 else np.float32)
    _check(load().lapis_csr_copy_arrays(A, rowptr.ctypes.data, colidx.ctypes.data, vals.ctypes.data))
    return rowptr, colidx, vals


def lapis_spmv_transpose(A, alpha, d_x, beta, d_y, stream=None):
    _check(load().lapis_spmv_transpose(A, float(alpha), _addr(d_x), float(beta), _addr(d_y), _stream(stream)))


def lapis_spmv_paper_shape(A, alpha, d_x, beta, d_y, stream=None):
    _check(load().lapis_spmv_paper_shape(A, float(alpha), _addr(d_x), float(beta), _addr(d_y),
                                         _stream(stream)))


def lapis_paper_vector_length(nrows, nnz):
    return load().lapis_paper_vector_length(nrows, nnz)


def lapis_spmm(A, k, alpha, d_X, ldx, beta, d_Y, ldy, stream=None):
    _check(load().lapis_spmm(A, k, float(alpha), _addr(d_X), ldx, float(beta), _addr(d_Y), ldy,
                             _stream(stream)))


def lapis_batched_gemm(batch, m, n, k, alpha, d_A, d_B, beta, d_C, dtype, stream=None):
    """C[b] = alpha*A[b]@B[b] + beta*C[b] on contiguous device tensors (batch, m, k), (batch, k, n),
    (batch, m, n); dtype is LAPIS_F32 or LAPIS_F64."""
    _check(load().lapis_batched_gemm(batch, m, n, k, float(alpha), _addr(d_A), _addr(d_B), float(beta),
                                     _addr(d_C), dtype, _stream(stream)))


def lapis_csr_destroy(A):
    _check(load().lapis_csr_destroy(A))


def lapis_csr_partition_sizes(A):
    """(num_stream_chunks, num_binned_rows, num_long_rows, num_tiles)"""
    v = [ctypes.c_int64() for _ in range(4)]
    _check(load().lapis_csr_partition_sizes(A, *[ctypes.byref(x) for x in v]))
    return tuple(x.value for x in v)


def lapis_partition_constants():
    out = (ctypes.c_int64 * 10)()
    _check(load().lapis_partition_constants(out))
    return {"num_bins": out[0], "wave": out[1], "long_threshold": out[2], "tile_nnz": out[3],
            "stream_rows": out[4], "stream_min_nnz": out[5], "split_block_bytes": out[6],
            "split_max_blocks": out[7], "huge_row": out[8], "lds_block_bytes": out[9]}


def lapis_csr_copy_partition(A):
    """Host copies of the row partition as NumPy int32 arrays."""
    ns, nb_rows, m, t = lapis_csr_partition_sizes(A)
    nb = lapis_partition_constants()["num_bins"]
    res = {
        "stream_chunks": np.empty(ns, dtype=np.int32),
        "stream_offset": np.empty(5, dtype=np.int32),
        "bin_offset": np.empty(nb + 1, dtype=np.int32),
        "row_perm": np.empty(nb_rows, dtype=np.int32),
        "long_off": np.empty(m + 1, dtype=np.int32),
        "tile_row": np.empty(t + 1, dtype=np.int32),
        "tile_nz": np.empty(t + 1, dtype=np.int32),
    }
    ptr = lambda a: a.ctypes.data_as(ctypes.c_void_p)
    _check(load().lapis_csr_copy_partition(A, ptr(res["stream_chunks"]), ptr(res["stream_offset"]),
                                           ptr(res["bin_offset"]),
                                           ptr(res["row_perm"]), ptr(res["long_off"]),
                                           ptr(res["tile_row"]), ptr(res["tile_nz"])))
    return res


def lapis_csr_split_sizes(A):
    """(num_blocks, block_width, num_split_rows, num_virtual_rows, num_long, num_tiles)"""
    v = [ctypes.c_int64() for _ in range(6)]
    _check(load().lapis_csr_split_sizes(A, *[ctypes.byref(x) for x in v]))
    return tuple(x.value for x in v)


def lapis_csr_copy_split(A):
    """Host copies of the column split; {'num_blocks': 0, ...} when the split is off."""
    nb, W, S, nv, m, t = lapis_csr_split_sizes(A)
    if nb == 0:
        return {"num_blocks": 0, "block_width": 0, "num_split_rows": 0, "num_huge_rows": 0}
    nbins = lapis_partition_constants()["num_bins"]
    H, nbf, fW = (ctypes.c_int64(), ctypes.c_int64(), ctypes.c_int64())
    _check(load().lapis_csr_huge_sizes(A, ctypes.byref(H), ctypes.byref(nbf), ctypes.byref(fW)))
    H, nbf, fW = H.value, nbf.value, fW.value
    res = {
        "num_blocks": nb, "block_width": W, "num_split_rows": S,
        "num_huge_rows": H, "num_fblocks": nbf, "fblock_width": fW,
        "split_rows": np.empty(S, dtype=np.int32), "huge_rows": np.empty(H, dtype=np.int32),
        "fcut": np.empty((nbf + 1) * H, dtype=np.int32),
        "cut": np.empty((nb + 1) * S, dtype=np.int32),
        "bin_offset": np.empty(nbins + 1, dtype=np.int32),
        "row_perm": np.empty(nv, dtype=np.int32),
        "long_off": np.empty(m + 1, dtype=np.int32),
        "tile_row": np.empty(t + 1, dtype=np.int32),
        "tile_nz": np.empty(t + 1, dtype=np.int32),
    }
    ptr = lambda a: a.ctypes.data_as(ctypes.c_void_p)
    _check(load().lapis_csr_copy_split(A, ptr(res["cut"]), ptr(res["bin_offset"]), ptr(res["row_perm"]),
                                       ptr(res["long_off"]), ptr(res["tile_row"]), ptr(res["tile_nz"])))
    _check(load().lapis_csr_copy_huge(A, ptr(res["split_rows"]), ptr(res["huge_rows"]), ptr(res["fcut"])))
    return res


def lapis_csr_half_bandwidth(A):
    v = ctypes.c_int64()
    _check(load().lapis_csr_half_bandwidth(A, ctypes.byref(v)))
    return v.value


class DualView:
    """Thin owner of a lapis_dualview_t: a pinned host buffer (exposed as a NumPy array) paired
    with a device buffer, synchronised lazily."""

    def __init__(self, count=None, dtype=np.float64, _handle=None, _count=None):
        self.dtype = np.dtype(dtype)
        if _handle is None:
            h = ctypes.c_void_p()
            _check(load().lapis_dualview_create(ctypes.byref(h), int(count) * self.dtype.itemsize))
            self.handle, self.count = h, int(count)
        else:
            self.handle, self.count = _handle, _count

    def subview(self, first, count):
        h = ctypes.c_void_p()
        _check(load().lapis_dualview_subview(ctypes.byref(h), self.handle, first * self.dtype.itemsize,
                                             count * self.dtype.itemsize))
        return DualView(dtype=self.dtype, _handle=h, _count=count)

    @property
    def host(self):
        """NumPy view of the host buffer (call modify_host() after writing to it)."""
        addr = load().lapis_dualview_host(self.handle)
        buf = (ctypes.c_char * (self.count * self.dtype.itemsize)).from_address(addr)
        return np.frombuffer(buf, dtype=self.dtype, count=self.count)

    @property
    def device_ptr(self):
        return load().lapis_dualview_device(self.handle)

    def modify_host(self):
        _check(load().lapis_dualview_modify_host(self.handle))

    def modify_device(self):
        _check(load().lapis_dualview_modify_device(self.handle))

    def sync_device(self, stream=None):
        _check(load().lapis_dualview_sync_device(self.handle, _stream(stream)))

    def sync_host(self, stream=None):
        _check(load().lapis_dualview_sync_host(self.handle, _stream(stream)))

    def copy_counts(self):
        a, b = ctypes.c_int64(), ctypes.c_int64()
        _check(load().lapis_dualview_copy_counts(self.handle, ctypes.byref(a), ctypes.byref(b)))
        return a.value, b.value

    def close(self):
        if self.handle is not None:
            _check(load().lapis_dualview_destroy(self.handle))
            self.handle = None


def lapis_spmv_dualview(A, alpha, x: "DualView", beta, y: "DualView", stream=None):
    _check(load().lapis_spmv_dualview(A, float(alpha), x.handle, float(beta), y.handle, _stream(stream)))
