"""Host-side contract of bench.py that needs no GPU: one GPU only, and the byte count of the metric."""
import os
import subprocess
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    res = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert res.returncode != 0
    assert "one GPU" in res.stderr and res.stdout.strip() == ""


def test_algorithmic_bytes_are_the_csr_arrays_and_the_vectors_once_each():
    sys.path.insert(0, ROOT)
    import bench
    import gen
    w = gen.workload(1)                                        # 64 x 64 5-point, f64, beta = 0
    expect = w.nnz * (8 + 4) + (w.nrows + 1) * 4 + w.ncols * 8 + w.nrows * 8
    assert bench.algorithmic_bytes(w) == expect == 324612      # the figure of the scope table
    w = gen.workload(3, {"n": 1024})                           # beta != 0: y is read and written
    assert bench.algorithmic_bytes(w) == w.nnz * 12 + (w.nrows + 1) * 4 + w.ncols * 8 + 2 * w.nrows * 8
    w = gen.workload(5, {"nx": 8, "ny": 8, "nz": 8})           # SpMM, k = 16
    assert bench.algorithmic_bytes(w) == w.nnz * 12 + (w.nrows + 1) * 4 + (w.ncols + w.nrows) * 16 * 8
    assert bench.HBM_PEAK_GBS == 8000.0


def test_parity_check_of_the_bench_flags_what_it_should():
    """The in-run check of bench.py: exact results pass, an error above the bound, an error on a row
    without entries and a NaN all fail."""
    sys.path.insert(0, ROOT)
    import bench
    import gen
    import oracle
    w = gen.workload(1)
    ref, absAx = oracle.spmv(w.rowptr, w.colidx, w.vals, w.x, w.alpha, w.beta, w.y0)
    good = bench.parity_check(w, ref.copy(), ref, absAx)
    assert good["checked"] and good["ok"] and good["max_err_over_tol"] == 0.0 and good["elements"] == w.nrows
    near = ref.copy()
    near[10] += 4 * 5 * 2.0 ** -53 * absAx[10]                 # half of the bound of a 5-entry row
    res = bench.parity_check(w, near, ref, absAx)
    assert res["ok"] and 0.3 < res["max_err_over_tol"] <= 1.0
    far = ref.copy()
    far[10] += 16 * 5 * 2.0 ** -53 * absAx[10]
    res = bench.parity_check(w, far, ref, absAx)
    assert not res["ok"] and res["max_err_over_tol"] > 1.0
    nan = ref.copy()
    nan[3] = np.nan
    assert not bench.parity_check(w, nan, ref, absAx)["ok"]
    zero_tol = bench.parity_check(w, np.nextafter(ref, np.inf), ref, np.zeros_like(absAx))
    assert not zero_tol["ok"] and zero_tol["max_err_over_tol"] is None


def test_source_fingerprint_follows_the_kernel_sources():
    sys.path.insert(0, ROOT)
    import bench
    fp = bench.source_fingerprint()
    assert len(fp) == 12 and int(fp, 16) >= 0
    assert bench.source_fingerprint("spmm") != bench.source_fingerprint("spmv")      # the SpMM kernels count for SpMM only
    for m in bench.MEASURED.values():
        assert set(m) == {"traffic", "source", "kernel", "profile"}
        assert os.path.exists(os.path.join(ROOT, m["profile"]))
    # comments and layout do not count, code does
    code = 'int f(int a) { return a + 1; }  // adds one\n/* block\n comment */ const char *s = "// not a comment";\n'
    same = 'int f(int a)\n{\n    return a + 1;   // one more\n}\nconst char *s = "// not a comment";\n'
    other = 'int f(int a) { return a + 2; }\nconst char *s = "// not a comment";\n'
    assert bench.strip_comments(code) == bench.strip_comments(same)
    assert bench.strip_comments(code) != bench.strip_comments(other)
    assert '"// not a comment"' in bench.strip_comments(code) and "adds one" not in bench.strip_comments(code)
