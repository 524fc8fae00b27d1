"""ctypes binding of libceilings_mi355x.so (include/lapis_ceilings.h): the measurement kernels
bench.py times beside the products.  Argument marshalling only."""
from __future__ import annotations

import ctypes
import os

from .binding import _addr, _stream

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libceilings_mi355x.so")
EXPORTS = ["lapis_ceiling_read", "lapis_ceiling_gather", "lapis_ceiling_rows"]

_lib = None


def load() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(f"{LIB_PATH} is not built; run paper_2509_25605_amd.build.build() first")
        import torch  # noqa: F401  (one HIP runtime per process: PyTorch's is loaded first)

        lib = ctypes.CDLL(LIB_PATH)
        i64, p, i32 = ctypes.c_int64, ctypes.c_void_p, ctypes.c_int
        lib.lapis_ceiling_read.argtypes = [p, i64, i32, p, p]
        lib.lapis_ceiling_gather.argtypes = [p, i64, p, i64, p, p]
        lib.lapis_ceiling_rows.argtypes = [p, i64, i32, i32, i32, p, p]
        for name in EXPORTS:
            getattr(lib, name).restype = i32
        _lib = lib
    return _lib


def _check(rc, what):
    if rc != 0:
        raise ValueError(f"{what}: argument out of range")


def lapis_ceiling_read(d_buf, nbytes, nontemporal, d_sink, stream=None):
    _check(load().lapis_ceiling_read(_addr(d_buf), int(nbytes), int(bool(nontemporal)), _addr(d_sink), _stream(stream)),
           "lapis_ceiling_read")


def lapis_ceiling_gather(d_table, table_len, d_idx, n, d_sink, stream=None):
    _check(load().lapis_ceiling_gather(_addr(d_table), int(table_len), _addr(d_idx), int(n), _addr(d_sink),
                                       _stream(stream)), "lapis_ceiling_gather")


def lapis_ceiling_rows(d_table, table_rows, iters, num_waves, random, d_sink, stream=None):
    _check(load().lapis_ceiling_rows(_addr(d_table), int(table_rows), int(iters), int(num_waves), int(bool(random)),
                                     _addr(d_sink), _stream(stream)), "lapis_ceiling_rows")
