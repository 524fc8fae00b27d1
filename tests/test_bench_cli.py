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
