"""The C sources that run on the host (the oracle and the input generators) built with
AddressSanitizer and UndefinedBehaviorSanitizer, and the small brute-force cases run through them in
a child process: an out-of-bounds access, an overflow or a misaligned read in either fails the test."""
import os
import subprocess
import sys
import textwrap

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

DRIVER = textwrap.dedent("""
    import ctypes, os, sys
    import numpy as np
    sys.path.insert(0, {root!r})
    import gen, oracle
    # swap in the instrumented libraries before either package loads its own
    gen._lib = None; oracle._lib = None
    gen._LIB = {gen_lib!r}; oracle._LIB = {oracle_lib!r}
    gen.build = lambda force=False: gen._LIB
    oracle.build = lambda force=False: oracle._LIB
    assert oracle._load()._name == oracle._LIB and gen._load()._name == gen._LIB      # the instrumented builds
    assert any("asan" in line for line in open("/proc/self/maps"))
    rng = np.random.default_rng(3)
    for n, ncols, dtype in ((1, 1, np.float64), (7, 5, np.float32), (33, 64, np.float64), (64, 3, np.float32)):
        lengths = rng.integers(0, min(ncols, 9) + 1, size=n)
        rowptr, colidx, vals = gen.random_csr(n, ncols, lengths, seed=5 + n, dtype=dtype, allow_duplicates=True,
                                              sorted_cols=False)
        x = gen.uniform(9, gen.STREAM_X, ncols).astype(dtype)
        y0 = gen.uniform(9, gen.STREAM_Y0, n).astype(dtype)
        dense = np.zeros((n, ncols))
        for i in range(n):
            for j in range(rowptr[i], rowptr[i + 1]):
                dense[i, colidx[j]] += float(vals[j])
        for alpha, beta in ((1.0, 0.0), (-0.5, 2.0)):
            y, absAx = oracle.spmv(rowptr, colidx, vals, x, alpha, beta, y0)
            want = alpha * dense @ x.astype(np.float64) + beta * y0
            tol = 8 * (np.diff(rowptr) + 2) * (2.0 ** -24 if dtype == np.float32 else 2.0 ** -53) * (
                abs(alpha) * absAx + abs(beta) * np.abs(y0)) + 1e-300
            assert np.all(np.abs(y - want) <= tol)
        X = gen.uniform(10, gen.STREAM_X, ncols * 3).astype(dtype).reshape(ncols, 3)
        Y, _ = oracle.spmm(rowptr, colidx, vals, X)
        for c in range(3):
            yc, _ = oracle.spmv(rowptr, colidx, vals, np.ascontiguousarray(X[:, c]))
            assert np.array_equal(Y[:, c], yc)
        t = oracle.transpose(rowptr, colidx, vals, ncols)
        assert t[0][-1] == rowptr[-1]
        oracle.spmv_transpose(rowptr, colidx, vals, ncols, y0)
        oracle.partition(rowptr, colidx=colidx, ncols=ncols, itemsize=vals.itemsize)
        oracle.index16(rowptr, colidx)
        oracle.row_patterns(rowptr, colidx, ncols, vals.itemsize)
    # structures on matrices with stream chunks, long rows and a column split
    w = gen.workload(2, {{"nx": 17, "ny": 9, "nz": 5}})
    oracle.partition(w.rowptr, colidx=w.colidx, ncols=w.ncols, itemsize=8)
    oracle.index16(w.rowptr, w.colidx); oracle.row_patterns(w.rowptr, w.colidx, w.ncols, 8)
    oracle.spmv(w.rowptr, w.colidx, w.vals, w.x)
    w = gen.workload(4, {{"n": 70000, "cap": 20000}})
    oracle.split_partition(w.rowptr, w.colidx, w.ncols, 4, block_bytes=1 << 16)
    oracle.spmv(w.rowptr, w.colidx, w.vals, w.x)
    for cfg, sc in ((1, None), (3, {{"n": 4096}}), (6, {{"scale": 0.002}}), (8, {{"grid": 5}})):
        w = gen.workload(cfg, sc)
        oracle.spmv(w.rowptr, w.colidx, w.vals, w.x, w.alpha, w.beta, w.y0)
    A = gen.uniform(1, 1, 5 * 3 * 4).reshape(5, 3, 4); B = gen.uniform(1, 2, 5 * 4 * 2).reshape(5, 4, 2)
    C, _ = oracle.batched_gemm(A, B)
    assert np.allclose(C, A @ B)
    print("sanitized run ok")
""")


def test_oracle_and_generators_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    flags = ["-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
             "-ffp-contract=off", "-shared", "-fPIC"]
    oracle_lib, gen_lib = str(tmp_path / "liboracle_san.so"), str(tmp_path / "libgen_san.so")
    subprocess.check_call(["gcc", *flags, "-o", oracle_lib, os.path.join(ROOT, "oracle", "lapis_oracle.c"), "-lm"])
    subprocess.check_call(["gcc", *flags, "-o", gen_lib, os.path.join(ROOT, "gen", "lapis_gen.c"), "-lm"])
    asan = subprocess.check_output(["gcc", "-print-file-name=libasan.so"], text=True).strip()
    env = dict(os.environ)
    # the sanitizer runtime has to come first in the process; leak checking would report the interpreter's own
    env["LD_PRELOAD"] = (asan + " " + env.get("LD_PRELOAD", "")).strip()
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=0:exitcode=97"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:exitcode=98:print_stacktrace=1"
    script = tmp_path / "driver.py"
    script.write_text(DRIVER.format(root=ROOT, gen_lib=gen_lib, oracle_lib=oracle_lib))
    res = subprocess.run([sys.executable, str(script)], capture_output=True, text=True, env=env, timeout=600)
    assert res.returncode == 0, (res.stdout[-2000:], res.stderr[-4000:])
    assert "sanitized run ok" in res.stdout
    assert "runtime error" not in res.stderr and "AddressSanitizer" not in res.stderr
