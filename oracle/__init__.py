"""Python face of the CPU oracle (oracle/lapis_oracle.c).

TEST INFRASTRUCTURE ONLY.  Tests, the smoke check and the bench's
cpu_baseline leg may import this package; the product package never does.
It builds the C file with gcc (-O2 -ffp-contract=off, no OpenMP: the oracle is
serial) and marshals NumPy arrays.  Every product, sum and index structure is computed in the
C file; what this module adds in Python is the geometry of the column split (split_geometry:
two integer divisions), the choice of the rows that are split (split_partition: rows of the
last two bins by length, the lengths of the virtual rows as differences of the cut table) and
the "enabled" rules (a structure is kept when its chunks hold at least half of the entries) and
share_classes (which kernel family the product with a block of vectors may use for a chunk: a
decision about speed that no result depends on, read off the partition and the row patterns).
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "lapis_oracle.c")
_LIB = os.path.join(_HERE, "liblapis_oracle.so")

# The partition definition's parameters as the oracle states them (wavefront width,
# long-row threshold, tile size, bin count, rows and minimum entries of a stream chunk).  A test checks that the GPU
# library reports the same values.
WAVE = 64
LONG_THRESHOLD = 4096
TILE_NNZ = 4096
NUM_BINS = 10
STREAM_ROWS = 32
STREAM_MIN_NNZ = 64
SPLIT_BLOCK_BYTES = 1 << 21   # target size of one column block of x
SPLIT_MAX_BLOCKS = 32
HUGE_ROW = 16384            # rows with more entries are cut at LDS-sized column blocks
LDS_BLOCK_BYTES = 65536     # bytes of x one such block holds
PATTERN_MAX_ROW = 128        # longest row a patterned chunk may have
PATTERN_SLOTS = 8            # distinct row patterns per chunk at most
PATTERN_TABLE = 512          # diagonals in a chunk's pattern table at most


def build(force: bool = False) -> str:
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-ffp-contract=off", "-shared", "-fPIC", "-o", _LIB, _SRC, "-lm"]
        )
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        i64, f64, p = ctypes.c_int64, ctypes.c_double, ctypes.c_void_p
        for name in ("oracle_spmv_f64", "oracle_spmv_f32"):
            getattr(lib, name).argtypes = [i64, p, p, p, p, f64, f64, p, p, p]
            getattr(lib, name).restype = None
        for name in ("oracle_spmv_transpose_f64", "oracle_spmv_transpose_f32"):
            getattr(lib, name).argtypes = [i64, i64, p, p, p, p, f64, f64, p, p, p, p]
            getattr(lib, name).restype = None
        lib.oracle_transpose.argtypes = [i64, i64, p, p, p, i64, p, p, p]
        lib.oracle_transpose.restype = None
        for name in ("oracle_spmm_f64", "oracle_spmm_f32"):
            getattr(lib, name).argtypes = [i64, i64, p, p, p, p, i64, f64, f64, p, p, i64, p]
            getattr(lib, name).restype = None
        lib.oracle_partition_num_bins.argtypes = [i64]
        lib.oracle_partition_num_bins.restype = ctypes.c_int
        lib.oracle_partition_stream_chunks.argtypes = [i64, p, i64, i64, p, p, p]
        lib.oracle_demoted_chunks.argtypes = [i64, p, i64, i64, i64, p, p]
        lib.oracle_demoted_chunks.restype = None
        lib.oracle_partition_stream_chunks.restype = i64
        lib.oracle_index16.argtypes = [i64, p, p, i64, i64, p, p, p, p, p]
        lib.oracle_index16.restype = None
        for name in ("oracle_batched_gemm_f64", "oracle_batched_gemm_f32"):
            getattr(lib, name).argtypes = [i64, i64, i64, i64, ctypes.c_double, p, p, ctypes.c_double, p, p, p]
            getattr(lib, name).restype = None
        lib.oracle_row_patterns.argtypes = [i64, p, p, i64, i64, p, i64, i64, i64, p, p, p, p]
        lib.oracle_row_patterns.restype = None
        lib.oracle_partition_rows.argtypes = [i64, p, i64, i64, i64, i64, i64, p, p, p, p, p]
        lib.oracle_partition_rows.restype = None
        lib.oracle_partition_tiles.argtypes = [p, i64, p, i64, i64, p, p, p]
        lib.oracle_partition_tiles.restype = None
        lib.oracle_split_cuts.argtypes = [p, p, p, i64, i64, i64, p, p]
        lib.oracle_split_cuts.restype = None
        _lib = lib
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _check_csr(rowptr, colidx, vals):
    assert rowptr.dtype == np.int32 and colidx.dtype == np.int32
    assert rowptr.flags.c_contiguous and colidx.flags.c_contiguous and vals.flags.c_contiguous
    assert vals.dtype in (np.float32, np.float64)


def spmv(rowptr, colidx, vals, x, alpha=1.0, beta=0.0, y0=None):
    """Returns (y, absAx): y = alpha*A*x + beta*y0 in vals.dtype, absAx = |A||x| in float64."""
    _check_csr(rowptr, colidx, vals)
    n = rowptr.size - 1
    dt = vals.dtype
    x = np.ascontiguousarray(x, dtype=dt)
    if beta != 0.0:
        assert y0 is not None
        y0 = np.ascontiguousarray(y0, dtype=dt)
    y = np.empty(n, dtype=dt)
    absAx = np.empty(n, dtype=np.float64)
    fn = _load().oracle_spmv_f64 if dt == np.float64 else _load().oracle_spmv_f32
    fn(n, _p(rowptr), _p(colidx), _p(vals), _p(x), float(alpha), float(beta),
       _p(y0) if beta != 0.0 else None, _p(y), _p(absAx))
    return y, absAx


def spmv_transpose(rowptr, colidx, vals, ncols, x, alpha=1.0, beta=0.0, y0=None):
    """Returns (y, absATx): y = alpha*A^T*x + beta*y0 (ncols values, vals.dtype) for x of nrows
    values, and |A^T||x| in float64."""
    _check_csr(rowptr, colidx, vals)
    n = rowptr.size - 1
    dt = vals.dtype
    x = np.ascontiguousarray(x, dtype=dt)
    assert x.size == n
    if beta != 0.0:
        assert y0 is not None
        y0 = np.ascontiguousarray(y0, dtype=dt)
        assert y0.size == ncols
    y = np.empty(ncols, dtype=dt)
    absATx = np.empty(ncols, dtype=np.float64)
    acc = np.empty(2 * max(ncols, 1), dtype=np.float64)
    fn = _load().oracle_spmv_transpose_f64 if dt == np.float64 else _load().oracle_spmv_transpose_f32
    fn(n, ncols, _p(rowptr), _p(colidx), _p(vals), _p(x), float(alpha), float(beta),
       _p(y0) if beta != 0.0 else None, _p(y), _p(absATx), _p(acc))
    return y, absATx


def transpose(rowptr, colidx, vals, ncols):
    """CSR arrays (tptr, tidx, tvals) of A^T; entries of a row of A^T ordered by (row of A,
    position in that row)."""
    _check_csr(rowptr, colidx, vals)
    n = rowptr.size - 1
    tptr = np.empty(ncols + 1, dtype=np.int32)
    tidx = np.empty(colidx.size, dtype=np.int32)
    tvals = np.empty(vals.size, dtype=vals.dtype)
    _load().oracle_transpose(n, ncols, _p(rowptr), _p(colidx), _p(vals), vals.itemsize, _p(tptr), _p(tidx), _p(tvals))
    return tptr, tidx, tvals


def spmm(rowptr, colidx, vals, X, alpha=1.0, beta=0.0, Y0=None):
    """Returns (Y, absAX) for row-major X (ncols x k); Y is nrows x k contiguous."""
    _check_csr(rowptr, colidx, vals)
    n = rowptr.size - 1
    dt = vals.dtype
    assert X.ndim == 2 and X.dtype == dt and X.strides[1] == X.itemsize
    k = X.shape[1]
    ldx = X.strides[0] // X.itemsize if X.shape[0] > 1 else k
    if beta != 0.0:
        assert Y0 is not None
        Y0 = np.ascontiguousarray(Y0, dtype=dt)
        assert Y0.shape == (n, k)
    Y = np.empty((n, k), dtype=dt)
    absAX = np.empty((n, k), dtype=np.float64)
    fn = _load().oracle_spmm_f64 if dt == np.float64 else _load().oracle_spmm_f32
    fn(n, k, _p(rowptr), _p(colidx), _p(vals), _p(X), ldx, float(alpha), float(beta),
       _p(Y0) if beta != 0.0 else None, _p(Y), k, _p(absAX))
    return Y, absAX


def batched_gemm(A, B, alpha=1.0, beta=0.0, C0=None):
    """Returns (C, absAB): C[b] = alpha*A[b]@B[b] + beta*C0[b] in A.dtype for A (batch, m, k) and
    B (batch, k, n), and sum_l |A[b,i,l]||B[b,l,j]| in float64."""
    assert A.ndim == 3 and B.ndim == 3 and A.shape[0] == B.shape[0] and A.shape[2] == B.shape[1]
    assert A.dtype == B.dtype and A.dtype in (np.float32, np.float64)
    batch, m, k = A.shape
    n = B.shape[2]
    A = np.ascontiguousarray(A)
    B = np.ascontiguousarray(B)
    if beta != 0.0:
        assert C0 is not None and C0.shape == (batch, m, n)
        C0 = np.ascontiguousarray(C0, dtype=A.dtype)
    C = np.empty((batch, m, n), dtype=A.dtype)
    absAB = np.empty((batch, m, n), dtype=np.float64)
    fn = _load().oracle_batched_gemm_f64 if A.dtype == np.float64 else _load().oracle_batched_gemm_f32
    fn(batch, m, n, k, float(alpha), _p(A), _p(B), float(beta), _p(C0) if beta != 0.0 else None, _p(C), _p(absAB))
    return C, absAB


def demoted_chunks(rowptr, colidx, ncols, itemsize, wave=WAVE, stream_rows=STREAM_ROWS,
                   stream_min_nnz=STREAM_MIN_NNZ):
    """uint8 per chunk: 1 for the chunks that would stream but are demoted to the bins (x far
    larger than an L2, columns neither narrow nor framed, a row above `wave` entries)."""
    n = rowptr.size - 1
    nchunks = (n + stream_rows - 1) // stream_rows
    out = np.zeros(nchunks, dtype=np.uint8)
    if split_geometry(ncols, itemsize)[0] == 0 or nchunks == 0:
        return out
    base = index16(rowptr, colidx, stream_rows, stream_min_nnz)["chunk_base"]
    _load().oracle_demoted_chunks(n, _p(rowptr), stream_rows, stream_min_nnz, wave, _p(base), _p(out))
    return out


def partition(rowptr, wave=WAVE, long_threshold=LONG_THRESHOLD, tile_nnz=TILE_NNZ,
              stream_rows=STREAM_ROWS, stream_min_nnz=STREAM_MIN_NNZ, colidx=None, ncols=None, itemsize=None):
    """Reference row partition.  Returns a dict with stream_chunks[] (class by class),
    stream_offset[5], bin_offset[num_bins+1],
    row_perm[rows outside stream chunks], long_off[m+1], tile_row[T+1], tile_nz[T+1].
    With colidx, ncols and itemsize the chunks of demoted_chunks() do not stream (the library
    always knows the columns; without them the partition is the one of the row lengths alone)."""
    assert rowptr.dtype == np.int32 and rowptr.flags.c_contiguous
    lib = _load()
    n = rowptr.size - 1
    nb = lib.oracle_partition_num_bins(wave)
    nchunks = (n + stream_rows - 1) // stream_rows
    demoted = None
    if colidx is not None:
        demoted = demoted_chunks(rowptr, colidx, ncols, itemsize, wave, stream_rows, stream_min_nnz)
    stream_chunks = np.empty(nchunks, dtype=np.int32)
    stream_offset = np.zeros(5, dtype=np.int32)
    ns = lib.oracle_partition_stream_chunks(n, _p(rowptr), stream_rows, stream_min_nnz, _p(demoted),
                                            _p(stream_chunks), _p(stream_offset))
    stream_chunks = stream_chunks[:ns].copy()
    bin_offset = np.zeros(nb + 1, dtype=np.int32)
    row_perm = np.empty(n, dtype=np.int32)
    m = ctypes.c_int64(0)
    T = ctypes.c_int64(0)
    lib.oracle_partition_rows(n, _p(rowptr), wave, long_threshold, tile_nnz, stream_rows,
                              stream_min_nnz, _p(demoted), _p(bin_offset), _p(row_perm),
                              ctypes.addressof(m), ctypes.addressof(T))
    m, T = m.value, T.value
    row_perm = row_perm[:bin_offset[nb]].copy()
    long_rows = np.ascontiguousarray(row_perm[bin_offset[nb - 1]:bin_offset[nb]])
    long_off = np.zeros(m + 1, dtype=np.int32)
    tile_row = np.zeros(T + 1, dtype=np.int32)
    tile_nz = np.zeros(T + 1, dtype=np.int32)
    lib.oracle_partition_tiles(_p(rowptr), tile_nnz, _p(long_rows), m, T, _p(long_off),
                               _p(tile_row), _p(tile_nz))
    return {"num_bins": nb, "stream_chunks": stream_chunks, "stream_offset": stream_offset,
            "bin_offset": bin_offset,
            "row_perm": row_perm, "long_off": long_off, "tile_row": tile_row, "tile_nz": tile_nz}


def index16(rowptr, colidx, stream_rows=STREAM_ROWS, stream_min_nnz=STREAM_MIN_NNZ):
    """16-bit column codes of the stream chunks: dict(enabled, narrow_entries, framed_entries,
    chunk_base[num_chunks] (>= 0: narrow chunk, its smallest column; -2: framed; -1: neither),
    frame_table[32 * num_chunks], col16[nnz]); enabled when the narrow and framed chunks
    together hold at least half of the entries."""
    assert rowptr.dtype == np.int32 and colidx.dtype == np.int32
    n = rowptr.size - 1
    nchunks = (n + stream_rows - 1) // stream_rows
    chunk_base = np.empty(nchunks, dtype=np.int32)
    frame_table = np.empty(32 * nchunks, dtype=np.int32)
    col16 = np.empty(colidx.size, dtype=np.uint16)
    scratch = np.empty(max(16 * stream_rows * stream_rows, 1), dtype=np.int32)   # rows of at most 2^4 * stream_rows entries
    counts = np.zeros(2, dtype=np.int64)
    _load().oracle_index16(n, _p(rowptr), _p(colidx), stream_rows, stream_min_nnz, _p(chunk_base),
                           _p(frame_table), _p(col16), _p(scratch), _p(counts))
    narrow, framed = int(counts[0]), int(counts[1])
    return {"enabled": narrow + framed > 0 and 2 * (narrow + framed) >= colidx.size,
            "narrow_entries": narrow, "framed_entries": framed,
            "chunk_base": chunk_base, "frame_table": frame_table, "col16": col16}


def row_patterns(rowptr, colidx, ncols=None, itemsize=None, wave=WAVE, stream_rows=STREAM_ROWS,
                 stream_min_nnz=STREAM_MIN_NNZ, max_row=PATTERN_MAX_ROW, max_patterns=PATTERN_SLOTS,
                 max_table=PATTERN_TABLE):
    """Row patterns of the stream chunks: dict(enabled, entries, pat_off[num_chunks + 1],
    row_pat[nrows] (uint16), pool[pat_off[-1]]): row i of a patterned chunk c has the columns
    i + shift_i + pool[pat_off[c] + (row_pat[i] & 511) + k], shift_i = bits 9..15 of row_pat[i] as a
    signed 7-bit number (pattern_start_shift splits the two).  With ncols and itemsize the demoted chunks are
    left out, as in partition().  enabled when the patterned chunks hold at least half of
    the entries."""
    assert rowptr.dtype == np.int32 and colidx.dtype == np.int32
    assert max_table <= 512 and max_patterns <= 64
    n = rowptr.size - 1
    nchunks = (n + stream_rows - 1) // stream_rows
    demoted = None
    if ncols is not None:
        demoted = demoted_chunks(rowptr, colidx, ncols, itemsize, wave, stream_rows, stream_min_nnz)
    pat_off = np.zeros(nchunks + 1, dtype=np.int32)
    row_pat = np.zeros(n, dtype=np.uint16)
    entries = ctypes.c_int64(0)
    args = (n, _p(rowptr), _p(colidx), stream_rows, stream_min_nnz, _p(demoted), max_row, max_patterns,
            max_table, _p(pat_off), _p(row_pat))
    _load().oracle_row_patterns(*args, None, ctypes.addressof(entries))
    pool = np.zeros(int(pat_off[-1]), dtype=np.int32)
    _load().oracle_row_patterns(*args, _p(pool), ctypes.addressof(entries))
    e = int(entries.value)
    return {"enabled": e > 0 and 2 * e >= colidx.size, "entries": e, "pat_off": pat_off,
            "row_pat": row_pat, "pool": pool}


def pattern_start_shift(row_pat):
    """(start in the chunk's table, shift) of every row from the packed row_pat values."""
    rp = np.asarray(row_pat).astype(np.int64)
    shift = rp >> 9
    return rp & 511, np.where(shift >= 64, shift - 128, shift)


SHARE_PLAIN, SHARE_NONE, SHARE_BLOCK3, SHARE_BLOCK2 = 1, 2, 3, 4
SHARE_MAX_ODD = 4


def share_classes(rowptr, part, pats, stream_rows=STREAM_ROWS, max_odd=SHARE_MAX_ODD, window=1024, wave=WAVE,
                  only=None):
    """The class of every chunk for the product with a block of vectors: 0 not a stream chunk, SHARE_NONE,
    SHARE_PLAIN (neighbouring rows use neighbouring rows of X), SHARE_BLOCK3 / SHARE_BLOCK2 (so do the rows
    of grid points with 3 / 2 unknowns), from the partition `part` and the row patterns `pats` as the
    library's header defines them; None when the patterns are not enabled or no chunk streams.  Written out
    chunk by chunk, row by row; with `only` (chunk numbers) the other chunks are left at -1."""
    n = rowptr.size - 1
    nchunks = (n + stream_rows - 1) // stream_rows
    if not pats["enabled"] or part["stream_chunks"].size == 0:
        return None
    start, shift = pattern_start_shift(pats["row_pat"])
    out = np.zeros(nchunks, dtype=np.int32)
    streams = set(int(c) for c in part["stream_chunks"])
    if only is not None:
        out[:] = -1
        out[[c for c in only if c not in streams]] = 0
        streams &= set(int(c) for c in only)
    for c in sorted(streams):
        out[c] = SHARE_NONE
        rows = list(range(c * stream_rows, min((c + 1) * stream_rows, n)))
        table = pats["pool"][pats["pat_off"][c]:pats["pat_off"][c + 1]]
        length = [int(rowptr[i + 1] - rowptr[i]) for i in rows]
        L = max(length)
        if table.size == 0 or L == 0:
            continue
        ref = rows[length.index(L)]                                   # the first row of the greatest length
        stored = [int(d) for d in table[start[ref]:start[ref] + L]]
        if any(b <= a for a, b in zip(stored, stored[1:])):
            continue
        same_list = [length[j] == L and start[i] == start[ref] for j, i in enumerate(rows)]
        same_both = [same_list[j] and shift[i] == shift[ref] for j, i in enumerate(rows)]
        first_entry, last_entry = int(rowptr[rows[0]]), int(rowptr[rows[-1] + 1])
        if (same_both.count(False) <= max_odd and L <= wave
                and last_entry - first_entry // 8 * 8 + wave <= window):
            out[c] = SHARE_PLAIN
            continue
        if same_list.count(False) > max_odd or L > 2 * wave:
            continue
        steps = set()
        for g in range(0, stream_rows, 4):
            v = [j + int(shift[rows[j]]) for j in range(g, min(g + 4, len(rows))) if same_list[j]]
            steps |= {x - min(v) for x in v}
        steps.discard(0)
        if steps == {3}:
            out[c] = SHARE_BLOCK3
        elif steps == {2}:
            out[c] = SHARE_BLOCK2
    return out


def split_geometry(ncols, itemsize, block_bytes=SPLIT_BLOCK_BYTES, max_blocks=SPLIT_MAX_BLOCKS):
    """(number of column blocks, block width); (0, 0) when x is too small to be worth splitting."""
    target = block_bytes // itemsize
    nb = min(max_blocks, -(-ncols // target))
    if nb < 2:
        return 0, 0
    return nb, -(-ncols // nb)


def split_partition(rowptr, colidx, ncols, itemsize, part=None, wave=WAVE, long_threshold=LONG_THRESHOLD,
                    tile_nnz=TILE_NNZ, block_bytes=SPLIT_BLOCK_BYTES, max_blocks=SPLIT_MAX_BLOCKS,
                    huge_row=HUGE_ROW, lds_block_bytes=LDS_BLOCK_BYTES):
    """Reference column split of the rows of the last two bins.  Rows of more than huge_row
    entries ('huge_rows', in row_perm order) are cut at the boundaries of column blocks that hold
    lds_block_bytes of x ('fcut', num_fblocks blocks of fblock_width columns); the other rows
    ('num_split_rows' of them, in row_perm order) are cut at the coarse blocks into virtual rows,
    which get bins and tiles of their own.  Returns a dict; 'num_blocks' == 0 means the split is
    off (x small, no such rows, or one of them with unsorted columns)."""
    part = part or partition(rowptr, wave, long_threshold, tile_nnz, colidx=colidx, ncols=ncols, itemsize=itemsize)
    nb_bins = part["num_bins"]
    off = part["bin_offset"]
    rows = np.ascontiguousarray(part["row_perm"][off[nb_bins - 2]:off[nb_bins]])
    nb, W = split_geometry(ncols, itemsize, block_bytes, max_blocks)
    none = {"num_blocks": 0, "block_width": 0, "num_split_rows": 0, "num_huge_rows": 0}
    if nb == 0 or rows.size == 0:
        return none
    lengths = (rowptr[rows + 1] - rowptr[rows]).astype(np.int64)
    split_rows = np.ascontiguousarray(rows[lengths <= huge_row])
    huge_rows = np.ascontiguousarray(rows[lengths > huge_row])
    S, H = split_rows.size, huge_rows.size
    fW = lds_block_bytes // itemsize
    nbf = -(-ncols // fW)
    if (nb + 1) * S > 2 ** 31 - 1 or (nbf + 1) * H > 2 ** 31 - 1:
        return none

    def cuts(row_list, blocks, width):
        out = np.empty((blocks + 1) * row_list.size, dtype=np.int32)
        ok = ctypes.c_int32(1)
        _load().oracle_split_cuts(_p(rowptr), _p(colidx), _p(row_list), row_list.size, blocks, width, _p(out),
                                  ctypes.addressof(ok))
        return out, bool(ok.value)

    cut, ok1 = cuts(split_rows, nb, W)
    fcut, ok2 = cuts(huge_rows, nbf, fW)
    if not (ok1 and ok2):
        return none
    vlen = (cut[S:] - cut[:-S]).astype(np.int64) if S else np.zeros(0, dtype=np.int64)
    fake = np.zeros(vlen.size + 1, dtype=np.int32)      # only row lengths enter bins and tiles
    np.cumsum(vlen, out=fake[1:])
    vp = partition(fake, wave, long_threshold, tile_nnz, stream_rows=STREAM_ROWS, stream_min_nnz=2 ** 31 - 1)
    assert vp["stream_chunks"].size == 0
    return {"num_blocks": nb, "block_width": W, "num_split_rows": S, "split_rows": split_rows, "cut": cut,
            "bin_offset": vp["bin_offset"], "row_perm": vp["row_perm"], "long_off": vp["long_off"],
            "tile_row": vp["tile_row"], "tile_nz": vp["tile_nz"],
            "num_huge_rows": H, "huge_rows": huge_rows, "num_fblocks": nbf, "fblock_width": fW, "fcut": fcut}
