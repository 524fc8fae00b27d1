"""Host-side checks of the C ABI that need no GPU: the library loads, exports
every function include/lapis.h declares, and rejects bad arguments before it
touches the device."""
import ctypes
import os
import re

import pytest

import paper_2509_25605_amd as L
from paper_2509_25605_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(binding.LIB_PATH):
        from paper_2509_25605_amd.build import build
        build()
    return binding.load()


def declared_functions():
    text = open(os.path.join(ROOT, "include", "lapis.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(lapis_\w+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = declared_functions()
    assert set(names) == set(binding.EXPORTS)
    for name in names:
        assert getattr(lib, name) is not None


def test_header_constants_match_library_and_oracle(lib):
    import oracle
    c = L.lapis_partition_constants()
    text = open(os.path.join(ROOT, "include", "lapis.h")).read()
    macro = lambda n: int(re.search(rf"#define\s+{n}\s+(\d+)", text).group(1))
    assert c == {"num_bins": macro("LAPIS_NUM_BINS"), "wave": macro("LAPIS_WAVE"),
                 "long_threshold": macro("LAPIS_LONG_THRESHOLD"), "tile_nnz": macro("LAPIS_TILE_NNZ"),
                 "stream_rows": macro("LAPIS_STREAM_ROWS"), "stream_min_nnz": macro("LAPIS_STREAM_MIN_NNZ"),
                 "split_block_bytes": macro("LAPIS_SPLIT_BLOCK_BYTES"),
                 "split_max_blocks": macro("LAPIS_SPLIT_MAX_BLOCKS"), "huge_row": macro("LAPIS_HUGE_ROW"),
                 "lds_block_bytes": macro("LAPIS_LDS_BLOCK_BYTES")}
    assert (c["huge_row"], c["lds_block_bytes"]) == (oracle.HUGE_ROW, oracle.LDS_BLOCK_BYTES)
    assert (c["split_block_bytes"], c["split_max_blocks"]) == (oracle.SPLIT_BLOCK_BYTES, oracle.SPLIT_MAX_BLOCKS)
    assert (c["num_bins"], c["wave"], c["long_threshold"], c["tile_nnz"], c["stream_rows"],
            c["stream_min_nnz"]) == (oracle.NUM_BINS, oracle.WAVE, oracle.LONG_THRESHOLD, oracle.TILE_NNZ,
                                     oracle.STREAM_ROWS, oracle.STREAM_MIN_NNZ)
    # the row-pattern limits are compile-time constants of the library (a static_assert ties its
    # kernels to the header); the oracle keeps its own copies
    assert macro("LAPIS_PATTERN_MAX_ROW") == oracle.PATTERN_MAX_ROW
    assert macro("LAPIS_PATTERN_SLOTS") == oracle.PATTERN_SLOTS
    assert macro("LAPIS_PATTERN_TABLE") == oracle.PATTERN_TABLE


def _create(lib, nrows, ncols, nnz, rowptr, colidx, vals, dtype, out=True):
    h = ctypes.c_void_p(0xdead)
    rc = lib.lapis_csr_create(ctypes.byref(h) if out else None, nrows, ncols, nnz, rowptr, colidx,
                              vals, dtype, None)
    return rc, h


@pytest.mark.parametrize("args,code", [
    ((-1, 4, 0, 8, 8, 8, 1), L.LAPIS_ERR_INVALID_ARG),            # negative nrows
    ((4, -1, 0, 8, 8, 8, 1), L.LAPIS_ERR_INVALID_ARG),            # negative ncols
    ((4, 4, -1, 8, 8, 8, 1), L.LAPIS_ERR_INVALID_ARG),            # negative nnz
    ((4, 4, 2 ** 31, 8, 8, 8, 1), L.LAPIS_ERR_INVALID_ARG),       # nnz beyond int32
    ((2 ** 31 - 1, 4, 0, 8, 8, 8, 1), L.LAPIS_ERR_INVALID_ARG),   # nrows + 1 beyond int32
    ((4, 4, 3, None, 8, 8, 1), L.LAPIS_ERR_INVALID_ARG),          # null rowptr
    ((4, 4, 3, 8, None, 8, 1), L.LAPIS_ERR_INVALID_ARG),          # null colidx with nnz > 0
    ((4, 4, 3, 8, 8, None, 1), L.LAPIS_ERR_INVALID_ARG),          # null vals with nnz > 0
    ((0, 4, 3, 8, 8, 8, 1), L.LAPIS_ERR_INVALID_ARG),             # entries in a matrix without rows
    ((4, 4, 3, 8, 8, 8, 2), L.LAPIS_ERR_UNSUPPORTED),             # unknown dtype
    ((4, 4, 3, 8, 8, 8, -1), L.LAPIS_ERR_UNSUPPORTED),
])
def test_create_rejects_bad_arguments_on_the_host(lib, args, code):
    rc, h = _create(lib, *args)
    assert rc == code
    assert h.value is None                                          # *out = NULL on error
    assert L.lapis_last_error() != ""


def test_null_handles_and_out_pointer(lib):
    assert _create(lib, 4, 4, 0, 8, 8, 8, 1, out=False)[0] == L.LAPIS_ERR_INVALID_ARG
    assert lib.lapis_csr_destroy(None) == L.LAPIS_OK
    assert lib.lapis_spmv(None, 1.0, 8, 0.0, 8, None) == L.LAPIS_ERR_INVALID_ARG
    assert lib.lapis_spmv_paper_shape(None, 1.0, 8, 0.0, 8, None) == L.LAPIS_ERR_INVALID_ARG
    assert lib.lapis_spmm(None, 4, 1.0, 8, 4, 0.0, 8, 4, None) == L.LAPIS_ERR_INVALID_ARG
    assert lib.lapis_csr_partition_sizes(None, None, None, None, None) == L.LAPIS_ERR_INVALID_ARG
    assert lib.lapis_csr_copy_partition(None, None, None, None, None, None, None, None) == L.LAPIS_ERR_INVALID_ARG
    assert lib.lapis_csr_split_sizes(None, None, None, None, None, None, None) == L.LAPIS_ERR_INVALID_ARG
    assert lib.lapis_csr_copy_split(None, None, None, None, None, None, None) == L.LAPIS_ERR_INVALID_ARG
    assert lib.lapis_csr_half_bandwidth(None, None) == L.LAPIS_ERR_INVALID_ARG
    assert lib.lapis_partition_constants(None) == L.LAPIS_ERR_INVALID_ARG
    with pytest.raises(L.LapisError) as e:
        L.lapis_spmv(None, 1.0, 8, 0.0, 8, stream=0)
    assert e.value.code == L.LAPIS_ERR_INVALID_ARG


def test_paper_vector_length_on_table3(lib, golden_dir):
    """The per-matrix vector length of the paper's estimate on the matrices of its Table 3."""
    for line in open(os.path.join(golden_dir, "paper_table3.txt")):
        if line.startswith("#") or not line.strip():
            continue
        name, rows, mean, _mx, expect = line.split()
        rows, nnz = int(rows), int(round(int(rows) * float(mean)))
        assert L.lapis_paper_vector_length(rows, nnz) == int(expect), name
    assert L.lapis_paper_vector_length(10, 10) == 1
    assert L.lapis_paper_vector_length(10, 11) == 2
    assert L.lapis_paper_vector_length(10, 30) == 4
    assert L.lapis_paper_vector_length(10, 31) == 4
    assert L.lapis_paper_vector_length(10, 41) == 8
    assert L.lapis_paper_vector_length(1, 10 ** 9) == 64
    assert L.lapis_paper_vector_length(0, 0) == 1


def test_header_is_plain_c_and_declares_what_the_library_exports(tmp_path):
    """include/lapis.h compiles as C99 on its own, and a C program that takes the address of every
    declared function links against the library (no call is made: no GPU needed)."""
    import subprocess
    text = open(os.path.join(ROOT, "include", "lapis.h")).read()
    names = sorted(set(re.findall(r"\b(lapis_[a-z0-9_]+)\s*\(", text)) - {"lapis_csr_t", "lapis_dualview_t"})
    assert set(names) == set(binding.EXPORTS)
    src = tmp_path / "client.c"
    src.write_text('#include "lapis.h"\n#include <stdio.h>\ntypedef void (*fn_t)(void);\nint main(void) {\n    fn_t f[] = {'
                   + ", ".join(f"(fn_t){n}" for n in names)
                   + "};\n    printf(\"%d\\n\", (int)(sizeof f / sizeof f[0]));\n    return f[0] == 0;\n}\n")
    exe = tmp_path / "client"
    lib_dir = os.path.dirname(binding.LIB_PATH)
    cmd = ["gcc", "-std=c99", "-pedantic", "-Wall", "-Werror", "-I", os.path.join(ROOT, "include"), str(src), "-o", str(exe),
           "-L", lib_dir, "-l:" + os.path.basename(binding.LIB_PATH), "-Wl,-rpath," + lib_dir,
           "-Wl,--allow-shlib-undefined"]
    res = subprocess.run(cmd, capture_output=True, text=True)
    assert res.returncode == 0, res.stderr[-2000:]


def test_ceilings_library_exports_what_its_header_declares(tmp_path):
    """include/lapis_ceilings.h (the measurement kernels of bench.py) is plain C, and every function it
    declares is exported by libceilings_mi355x.so; argument checks answer without touching a GPU."""
    import subprocess
    from paper_2509_25605_amd import ceilings
    if not os.path.exists(ceilings.LIB_PATH):
        from paper_2509_25605_amd.build import build
        build()
    text = open(os.path.join(ROOT, "include", "lapis_ceilings.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = sorted(set(re.findall(r"\b(lapis_\w+)\s*\(", text)))
    assert set(names) == set(ceilings.EXPORTS)
    lib = ceilings.load()
    for name in names:
        assert getattr(lib, name) is not None
    src = tmp_path / "c.c"
    src.write_text('#include "lapis_ceilings.h"\nint main(void) { return 0; }\n')
    res = subprocess.run(["gcc", "-std=c99", "-pedantic", "-Wall", "-Werror", "-I", os.path.join(ROOT, "include"), "-c",
                          str(src), "-o", str(tmp_path / "c.o")], capture_output=True, text=True)
    assert res.returncode == 0, res.stderr[-2000:]
    assert lib.lapis_ceiling_read(None, 1024, 0, None, None) == 1
    assert lib.lapis_ceiling_read(16, 1000, 0, 16, None) == 1          # not a multiple of 16 bytes
    assert lib.lapis_ceiling_gather(None, 8, None, 8, None, None) == 1
    assert lib.lapis_ceiling_rows(16, 1000, 1, 1, 0, 16, None) == 1    # not a power of two
