#!/usr/bin/env python3
"""Benchmark of the CSR SpMV / SpMM hot path on one MI355X.

A step is one lapis_spmv call (y = alpha*A*x + beta*y) on the 128^3 27-point fp64 stencil matrix
(workload 2, the headline), inputs resident in HBM.  Timing follows the paper's protocol
(Appendix, system configuration: untimed warm-up, then the mean over the timed repetitions).
Prints ONE JSON line.  Without --config the line also carries, under "configs", the other four
synthetic workloads (1, 3, 4: SpMV; 5: SpMM with 16 columns), each timed the same way with the
CPU oracle timed beside it, and every timed product is checked element by element against the
oracle's result (per element |y - y_ref| <= 8 nnz_row eps (|A||x|)_i).

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--config C] [--no-cpu]
  python bench.py --ceiling read|gather|rows      what the GPU delivers for the access patterns
                                                  the kernels are made of (one JSON line)
"""
import argparse
import hashlib
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0  # MI355X HBM3E, published peak
EPS = {np.dtype(np.float64): 2.0 ** -53, np.dtype(np.float32): 2.0 ** -24}

# HBM bytes per step from rocprofv3 --pmc FETCH_SIZE and WRITE_SIZE runs of this script (summed over
# the kernels of one step; commands and figures in profiles/), each scaled by what the same counter
# reads for a plain 1 GiB device copy (FETCH_SIZE x2.000, WRITE_SIZE x1.000).  "source" is the
# fingerprint (see source_fingerprint) of the kernel sources the figure was measured with: when the
# sources on disk differ, the line reports the figure with "traffic_stale": true.  "profile" is the
# summary the figure is taken from.
MEASURED = {
    "poisson2d_64x64_f64": {
        "traffic": 0.44e6, "source": "5101719d3314", "profile": "profiles/spmv_stream_poisson2d_64_f64.md",
        "kernel": "spmv_stream_kernel<double, 2, true, 4, 16, 1> (4: row patterns)"},
    "stencil27_128x128x128_f64": {
        "traffic": 505.35e6, "source": "5101719d3314", "profile": "profiles/spmv_stream_stencil27_128_f64.md",
        "kernel": "spmv_stream_kernel<double, 2, true, 4, 16, 1> (4: row patterns)"},
    "uniform16_n4194304_f64": {
        "traffic": 8439.92e6, "source": "5101719d3314", "profile": "profiles/spmv_stream_uniform16_f64.md",
        "kernel": "spmv_stream_kernel<double, 2, true, 0, 16, 1> (0: 32-bit columns)"},
    "zipf1.8_cap200000_n8388608_f32": {
        "traffic": 8689.40e6, "source": "5101719d3314", "profile": "profiles/spmv_powerlaw_zipf_f32.md",
        "kernel": "spmv_short_kernel<float, true> (2 launches) + spmv_ldsblock_kernel<float> + spmv_stream_kernel<float, ...>"},
    "stencil27_128x128x128_f64_spmm_k16": {
        "traffic": 1038.58e6, "source": "536874115369", "profile": "profiles/spmm_shared_stencil27_128_k16_f64.md",
        "kernel": "spmm_shared_kernel<double, 2, 8, true> (rows of X shared by 4 consecutive rows)"},
    "table3_StocF-1465_n1465137_f64": {
        "traffic": 243.82e6, "source": "5101719d3314", "profile": "profiles/spmv_stream_stocf_standin_f64.md",
        "kernel": "spmv_stream_kernel<double, 2, true, 1, 16, 1> (1: 16-bit column offsets)"},
    "table3_PFlow_742_n742793_f64": {
        "traffic": 399.93e6, "source": "5101719d3314", "profile": "profiles/spmv_stream_pflow_standin_f64.md",
        "kernel": "spmv_stream_kernel<double, 4, true, 1, 16, 2> (1: 16-bit column offsets; 2 wavefronts per workgroup)"},
    "table3_Elasticity3D_60_n648000_f64": {
        "traffic": 430.27e6, "source": "5101719d3314", "profile": "profiles/spmv_stream_elasticity3d_60_standin_f64.md",
        "kernel": "spmv_stream_kernel<double, 8, true, 4, 16, 1> (4: row patterns, with shifts)"},
    "table3_Elasticity3D_60_n648000_f64_spmm_k16": {
        "traffic": 996.11e6, "source": "536874115369",
        "profile": "profiles/spmm_block_shared_elasticity3d_60_standin_k16_f64.md",
        "kernel": "spmm_block_shared_kernel<double, 2, true, 3, 32> (rows of X shared by the rows of a grid point) + "
                  "spmm_stream_kernel<double, 2, 8, true, true, true> (the other chunks)"},
    "table3_PFlow_742_n742793_f64_spmm_k16": {
        "traffic": 576.93e6, "source": "536874115369", "profile": "profiles/spmm_stream_pflow_standin_k16_f64.md",
        "kernel": "spmm_stream_kernel<double, 2, 8, true, true, false> (16-bit column offsets, one wavefront per chunk)"},
    "table3_audikw_1_n943695_f64": {
        "traffic": 814.08e6, "source": "5101719d3314", "profile": "profiles/spmv_stream_audikw_standin_f64.md",
        "kernel": "spmv_stream_kernel<double, 8, true, 1, 16, 4> (1: 16-bit column offsets; 4 wavefronts per workgroup)"},
}
# The sources a product is compiled from: lapis_spmv does not include the SpMM kernels.
FINGERPRINT_FILES = {
    "spmv": ["spmv_kernels.hpp", "analysis_kernels.hpp", "lapis_api.hip", "device_utils.hpp"],
    "spmm": ["spmv_kernels.hpp", "spmm_kernels.hpp", "analysis_kernels.hpp", "lapis_api.hip", "device_utils.hpp"],
}


def strip_comments(text):
    """C++ source without its comments and with every run of white space as one blank (string and
    character literals are kept as they are), so that rewording a comment is not a change of the code."""
    out, i, n = [], 0, len(text)
    while i < n:
        c = text[i]
        if c in "\"'":
            j = i + 1
            while j < n and text[j] != c:
                j += 2 if text[j] == "\\" else 1
            out.append(text[i:j + 1])
            i = j + 1
        elif text.startswith("//", i):
            j = text.find("\n", i)
            i = n if j < 0 else j
        elif text.startswith("/*", i):
            j = text.find("*/", i + 2)
            i = n if j < 0 else j + 2
            out.append(" ")
        else:
            out.append(c)
            i += 1
    return " ".join("".join(out).split())


def source_fingerprint(product="spmv"):
    """First 12 hex digits of the SHA-256 of the kernel and launch sources (csrc/) of a product ("spmv" or
    "spmm") without their comments, so that a traffic figure measured with other code is recognisable as stale."""
    h = hashlib.sha256()
    for name in FINGERPRINT_FILES[product]:
        with open(os.path.join(ROOT, "paper_2509_25605_amd", "csrc", name), "r", encoding="utf-8") as f:
            h.update(strip_comments(f.read()).encode("utf-8"))
            h.update(b"\0")
    return h.hexdigest()[:12]


def algorithmic_bytes(w):
    """vals + colidx + rowptr + x + y (y twice when beta != 0), each counted once."""
    e = w.vals.itemsize
    k = max(w.k, 1)
    y_passes = 2 if w.beta != 0.0 else 1
    return (w.nnz * (e + 4) + (w.nrows + 1) * 4 + w.ncols * k * e + y_passes * w.nrows * k * e)


VARIANT_KERNEL = {"paper-shape": "spmv_vector_kernel", "transpose": "transpose_scatter_kernel",
                  "graph": "all kernels of the step, replayed from a HIP graph",
                  "transposed-handle": "all kernels of the step",
                  "host-buffers": "all kernels and copies of the step"}


def time_steps(torch, step, warmup, steps):
    """(wall ms per step between two synchronisations, ms per step between two events recorded on the
    launch stream, which is torch's current stream)."""
    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    wall0 = time.perf_counter()
    start.record()
    for _ in range(steps):
        step()
    stop.record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - wall0) * 1e3
    return wall_ms / steps, start.elapsed_time(stop) / steps


def batched_gemm_bench(args, scale, torch, gen, L, dev):
    """One step = one lapis_batched_gemm over the whole batch; bytes = A + B + C once each."""
    batch, m = int(scale.get("batch", 1 << 20)), int(scale.get("m", 8))
    n, k = int(scale.get("n", m)), int(scale.get("k", m))
    dt = np.float32 if scale.get("f32") else np.float64
    A = gen.uniform(20250925, gen.STREAM_VALUES, batch * m * k).reshape(batch, m, k).astype(dt)
    B = gen.uniform(20250925, gen.STREAM_X, batch * k * n).reshape(batch, k, n).astype(dt)
    dA, dB = torch.from_numpy(A).to(dev), torch.from_numpy(B).to(dev)
    dC = torch.zeros((batch, m, n), dtype=dA.dtype, device=dev)
    code = L.LAPIS_F64 if dt == np.float64 else L.LAPIS_F32
    ms_per_step, kernel_ms = time_steps(torch, lambda: L.lapis_batched_gemm(batch, m, n, k, 1.0, dA, dB, 0.0, dC, code),
                                        args.warmup, args.steps)
    nbytes = batch * (m * k + k * n + m * n) * A.itemsize
    flops = 2.0 * batch * m * n * k
    cpu = None
    if not args.no_cpu:
        import oracle
        sample = min(batch, max(1, int(2e8 / (m * n * k))))      # about a second per pass
        best, spent, reps = float("inf"), 0.0, 0
        while spent < args.cpu_seconds or reps < 3:
            t = time.perf_counter()
            oracle.batched_gemm(A[:sample], B[:sample])
            d = time.perf_counter() - t
            best, spent, reps = min(best, d), spent + d, reps + 1
        cpu = {"value": round(nbytes * (sample / batch) / best / 1e9, 3), "unit": "GB/s", "cores": 1, "kind": "oracle",
               "sample": f"first {sample} of {batch} products, best of {reps} serial passes ({best * 1e3:.1f} ms each), "
                         f"1 of {os.cpu_count()} host cores"}
    achieved = nbytes / (kernel_ms * 1e-3) / 1e9
    print(json.dumps({
        "metric": "batched GEMM effective HBM GB/s (A+B+C bytes / time); gflops alongside",
        "value": round(nbytes / (ms_per_step * 1e-3) / 1e9, 2), "unit": "GB/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 6), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f64" if dt == np.float64 else "f32", "data": "synthetic",
        "config": {"workload": f"batched_gemm_{batch}x{m}x{n}x{k}_{'f64' if dt == np.float64 else 'f32'}",
                   "bytes_per_step": nbytes, "variant": "batched-gemm"},
        "gflops": round(flops / (ms_per_step * 1e-3) / 1e9, 2),
        "roofline": {"bound": "hbm", "achieved": round(achieved, 2), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(achieved / HBM_PEAK_GBS, 4),
                     # measured with rocprofv3 on the default size (profiles/): every byte moves once
                     "traffic": 1610.72e6 if (batch, m, n, k, dt) == (1 << 20, 8, 8, 8, np.float64) else None,
                     "algorithmic_bytes": nbytes,
                     "kernel": "batched_gemm_kernel", "kernel_ms": round(kernel_ms, 6)},
        "cpu_baseline": cpu}))


# ---- ceilings: what the GPU delivers for the access patterns the kernels are made of ----------------
def ceiling_read(torch, dev, nbytes=704 << 20, reps=30):
    """One pass of 16-byte streaming loads over a buffer the size of workload 2's matrix: GB/s."""
    from paper_2509_25605_amd import ceilings as C
    buf = torch.zeros(nbytes // 8, dtype=torch.float64, device=dev)
    sink = torch.zeros(8, dtype=torch.float64, device=dev)
    out = {}
    for label, nt in (("read_GBps", 0), ("read_nontemporal_GBps", 1)):
        _, ms = time_steps(torch, lambda: C.lapis_ceiling_read(buf, nbytes, nt, sink), 3, reps)
        out[label] = round(nbytes / (ms * 1e-3) / 1e9, 1)
    out["read_bytes"] = nbytes
    return out


def ceiling_gather(torch, dev, table_len=1 << 22, n=1 << 26, reps=10):
    """Random 8-byte gathers from a table far larger than an L2 (the x of workload 3), indices
    streamed: G gathers/s."""
    from paper_2509_25605_amd import ceilings as C
    table = torch.zeros(table_len, dtype=torch.float64, device=dev)
    gen_ = torch.Generator(device=dev)
    gen_.manual_seed(20250925)
    idx = torch.randint(0, table_len, (n,), dtype=torch.int32, device=dev, generator=gen_)
    sink = torch.zeros(8, dtype=torch.float64, device=dev)
    _, ms = time_steps(torch, lambda: C.lapis_ceiling_gather(table, table_len, idx, n, sink), 2, reps)
    return {"gather_G_per_s": round(n / (ms * 1e-3) / 1e9, 2), "gather_table_bytes": table_len * 8, "gathers": n}


def ceiling_rows(torch, dev, table_bytes=(1 << 20, 2 << 20, 4 << 20, 8 << 20, 32 << 20, 1 << 30), waves_per_cu=12, iters=200):
    """128-byte rows through the L1 of every CU (16 bytes per lane, 16 rows in flight): TB/s by table size."""
    from paper_2509_25605_amd import ceilings as C
    sink = torch.zeros(8, dtype=torch.float64, device=dev)
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    out = {}
    for nb in table_bytes:
        rows = nb // 128
        table = torch.zeros(nb // 8, dtype=torch.float64, device=dev)
        waves = cus * waves_per_cu
        _, ms = time_steps(torch, lambda: C.lapis_ceiling_rows(table, rows, iters, waves, 1, sink), 1, 3)
        out[f"rows_TBps_table_{nb >> 10}KiB"] = round(waves * iters * 16 * 1024 / (ms * 1e-3) / 1e12, 2)
        del table
    return out


# ---- one workload -----------------------------------------------------------------------------------
def oracle_leg(w, seconds):
    """The oracle on the full workload, on one host core: (cpu_baseline dict, y_ref, |A||x|)."""
    import oracle
    fn = (lambda: oracle.spmv(w.rowptr, w.colidx, w.vals, w.x, w.alpha, w.beta, w.y0)) if w.k == 0 else (
        lambda: oracle.spmm(w.rowptr, w.colidx, w.vals, w.x, w.alpha, w.beta, w.y0))
    ref, absAx = fn()
    reps, best, spent = 0, float("inf"), 0.0
    while spent < seconds or reps < 3:
        t = time.perf_counter()
        fn()
        d = time.perf_counter() - t
        best, spent, reps = min(best, d), spent + d, reps + 1
    nbytes = algorithmic_bytes(w)
    flops = 2.0 * w.nnz * max(w.k, 1)
    cpu = {"value": round(nbytes / best / 1e9, 3), "unit": "GB/s", "cores": 1, "kind": "oracle",
           "sample": f"full workload, best of {reps} serial passes ({best * 1e3:.2f} ms each; "
                     f"{flops / best / 1e9:.2f} GFLOP/s), 1 of {os.cpu_count()} host cores"}
    return cpu, ref, absAx


def parity_check(w, got, ref, absAx):
    """Every element of the product against the oracle's: |y - y_ref| <= 8 nnz_row eps (|A||x|)_i."""
    nnz_row = np.diff(w.rowptr).astype(np.float64)
    if w.k:
        nnz_row = nnz_row[:, None]
    tol = 8.0 * nnz_row * EPS[np.dtype(w.dtype)] * absAx
    err = np.abs(got.astype(np.float64).reshape(ref.shape) - ref.astype(np.float64))
    with np.errstate(divide="ignore", invalid="ignore"):
        ratio = np.where(err == 0.0, 0.0, err / tol)          # err > 0 with tol == 0 gives inf
    worst = float(np.nanmax(ratio)) if ratio.size else 0.0
    ok = bool(np.all(err <= tol))                              # also false for NaN
    return {"checked": True, "ok": ok, "max_err_over_tol": round(worst, 4) if np.isfinite(worst) else None,
            "elements": int(err.size), "bound": "8*nnz_row*eps*(|A||x|)_i"}


def as_spmm(w, k, gen, cfg):
    """The matrix of an SpMV workload with a block of k vectors (row-major X from the workload's own
    seed and stream, Y = A X): the shape of workload 5 on another matrix."""
    import dataclasses
    X = gen.uniform(gen.BASE_SEED + cfg, gen.STREAM_X, w.ncols * k, dtype=w.dtype).reshape(w.ncols, k)
    return dataclasses.replace(w, name=f"{w.name}_spmm_k{k}", x=X, alpha=1.0, beta=0.0, y0=None, k=k)


def run_workload(cfg, scale, variant, steps, warmup, cpu_seconds, torch, gen, L, dev, fingerprint, spmm_k=0):
    """Times one workload and returns its entry: times, rates, roofline figures, oracle baseline, parity."""
    w = gen.workload(cfg, scale or None)
    if spmm_k:
        if w.k:
            sys.exit("bench.py: --spmm-k applies to the SpMV workloads")
        w = as_spmm(w, spmm_k, gen, cfg)
    tdt = torch.float64 if w.dtype == np.float64 else torch.float32
    rowptr = torch.from_numpy(w.rowptr).to(dev)
    colidx = torch.from_numpy(w.colidx).to(dev)
    vals = torch.from_numpy(w.vals).to(dev)
    x = torch.from_numpy(np.ascontiguousarray(w.x)).to(dev)
    k = max(w.k, 1)
    y = (torch.from_numpy(w.y0).to(dev) if w.y0 is not None
         else torch.zeros(w.nrows * k, dtype=tdt, device=dev))
    L.CsrMatrix(w.nrows, w.ncols, rowptr, colidx, vals).close()   # first call also loads the code object
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    A = L.CsrMatrix(w.nrows, w.ncols, rowptr, colidx, vals)
    torch.cuda.synchronize()
    create_ms = (time.perf_counter() - t0) * 1e3                  # analysis of an already loaded library

    if variant != "tuned" and w.k != 0:
        sys.exit("bench.py: --variant applies to the SpMV workloads only")
    if variant in ("transpose", "transposed-handle", "host-buffers") and w.nrows != w.ncols:
        sys.exit("bench.py: this variant expects a square workload")
    product = None          # the call the parity check repeats on a fresh y
    if variant == "paper-shape":
        product = lambda yy: L.lapis_spmv_paper_shape(A.handle, w.alpha, x, w.beta, yy)
    elif variant == "transpose":
        step = lambda: L.lapis_spmv_transpose(A.handle, w.alpha, x, w.beta, y)
    elif variant == "transposed-handle":
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        At = A.transposed()
        torch.cuda.synchronize()
        create_ms = (time.perf_counter() - t0) * 1e3     # transposition + analysis of A^T
        step = lambda: L.lapis_spmv(At.handle, w.alpha, x, w.beta, y)
    elif variant == "host-buffers":
        xv, yv = L.DualView(w.ncols, w.dtype), L.DualView(w.nrows, w.dtype)
        xv.host[:] = w.x
        yv.host[:] = 0.0 if w.y0 is None else w.y0
        yv.modify_host()

        def step():
            xv.modify_host()                     # the caller rewrote x on the host
            L.lapis_spmv_dualview(A.handle, w.alpha, xv, w.beta, yv)
            yv.sync_host()                       # and reads y on the host
    elif variant == "graph":
        per_graph = 50
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            L.lapis_spmv(A.handle, w.alpha, x, w.beta, y)
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            for _ in range(per_graph):
                L.lapis_spmv(A.handle, w.alpha, x, w.beta, y)
        steps = max(per_graph, steps // per_graph * per_graph)
        replays = iter(range(10 ** 9))
        step = lambda: graph.replay() if next(replays) % per_graph == 0 else None
    elif w.k == 0:
        product = lambda yy: L.lapis_spmv(A.handle, w.alpha, x, w.beta, yy)
    else:
        product = lambda yy: L.lapis_spmm(A.handle, w.k, w.alpha, x, w.k, w.beta, yy, w.k)
    if product is not None:
        step = lambda: product(y)

    ms_per_step, kernel_ms = time_steps(torch, step, warmup, steps)
    nbytes = algorithmic_bytes(w)
    flops = 2.0 * w.nnz * k
    gbs = nbytes / (ms_per_step * 1e-3) / 1e9
    achieved = nbytes / (kernel_ms * 1e-3) / 1e9

    cpu = parity = None
    if cpu_seconds is not None:
        cpu, ref, absAx = oracle_leg(w, cpu_seconds)
        if product is not None:
            # the timed call once more, from the workload's own y0 (NaN where y is write-only)
            yc = (torch.from_numpy(w.y0).to(dev) if w.y0 is not None
                  else torch.full((w.nrows * k,), float("nan"), dtype=tdt, device=dev))
            product(yc)
            torch.cuda.synchronize()
            parity = parity_check(w, yc.cpu().numpy(), ref, absAx)

    m = MEASURED.get(w.name) if variant == "tuned" else None
    traffic = m["traffic"] if m else None
    entry = {
        "workload": w.name, "dtype": "f64" if w.dtype == np.float64 else "f32", "nrows": w.nrows, "nnz": w.nnz,
        "k": w.k, "alpha": w.alpha, "beta": w.beta, "steps": steps, "warmup": warmup,
        "ms_per_step": round(ms_per_step, 6), "us_per_step": round(ms_per_step * 1e3, 3),
        "kernel_ms": round(kernel_ms, 6), "create_ms": round(create_ms, 3),
        "GBps": round(gbs, 2), "gflops": round(flops / (ms_per_step * 1e-3) / 1e9, 2),
        "algorithmic_bytes": nbytes, "frac_basis": "csr_bytes",
        "frac": round(achieved / HBM_PEAK_GBS, 4),
        "traffic": traffic,
        "traffic_frac": round(traffic / (kernel_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4) if traffic else None,
        "traffic_stale": (m["source"] != source_fingerprint("spmm" if w.k else "spmv")) if m else None,
        "kernel": (m["kernel"] if m else "all kernels of the step") if variant == "tuned" else VARIANT_KERNEL[variant],
        "cpu_baseline": cpu, "parity": parity,
    }
    A.close()
    return entry, w


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=1000)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", type=int, default=None,
                    help="workload 1..5 (2 = the headline workload); 6..9 = stand-ins for the paper's Table 3.  "
                         "Without it: workload 2 as the headline plus workloads 1, 3, 4, 5 under \"configs\"")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle timing and the parity check")
    ap.add_argument("--cpu-seconds", type=float, default=10.0, help="oracle timing budget of the headline workload")
    ap.add_argument("--cpu-seconds-extra", type=float, default=4.0, help="the same for each workload under \"configs\"")
    ap.add_argument("--scale", default=None,
                    help="override size parameters of the workload's recipe, e.g. nx=288,ny=288,nz=288 "
                         "(labelled in config.workload; the default sizes are the benchmark's)")
    ap.add_argument("--spmm-k", type=int, default=0,
                    help="with --config N (an SpMV workload): time lapis_spmm on its matrix with this many columns")
    ap.add_argument("--zipf-s", type=float, default=None,
                    help="workload 4 only: Zipf exponent (default 1.8; 2.0 gives the 'mean about 8' variant)")
    ap.add_argument("--variant", choices=["tuned", "paper-shape", "transpose", "transposed-handle", "host-buffers",
                                          "batched-gemm", "graph"], default="tuned",
                    help="paper-shape: the single-vector-length kernel of the paper's loop mapping; "
                         "transpose: y = alpha*A^T*x + beta*y (column-wise traversal, atomics); transposed-handle: "
                         "the same product through a handle for A^T built on the device; host-buffers: the "
                         "product on lazily synchronised host buffers with x rewritten on the host and y "
                         "read back every step (PCIe-inclusive rate, never the headline value); batched-gemm: "
                         "lapis_batched_gemm on 2^20 products of 8 x 8 doubles (--scale batch=,m=,n=,k=,f32=1 "
                         "to change that), a workload of its own, --config is ignored; graph: the tuned product "
                         "recorded 50 times into a HIP graph and replayed (what a launch-bound caller such as "
                         "workload 1 gains; --steps is rounded to a multiple of 50)")
    ap.add_argument("--ceiling", choices=["read", "gather", "rows"], default=None,
                    help="measure what the GPU delivers for one access pattern instead (plain streaming read; "
                         "random 8-byte gathers; 128-byte rows through L1) and exit")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="run a plain device copy of known size instead (reference for the "
                         "FETCH_SIZE / WRITE_SIZE counters) and exit")
    ap.add_argument("--fingerprint", action="store_true", help="print the fingerprint of the kernel sources and exit")
    args = ap.parse_args()
    if args.fingerprint:
        print(f"spmv {source_fingerprint('spmv')} spmm {source_fingerprint('spmm')}")
        return
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on exactly one GPU (no sharding, no collectives); use --gpus 1")

    import torch
    import gen
    import paper_2509_25605_amd as L

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    L.load()  # fails loudly if the HIP library is not built
    dev = torch.device("cuda:0")

    if args.copy_calibration:
        nbytes = 1 << 30
        src = torch.ones(nbytes // 8, dtype=torch.float64, device=dev)
        dst = torch.empty_like(src)
        for _ in range(max(args.steps, 1) if args.steps < 50 else 5):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration_bytes_read": nbytes, "bytes_written": nbytes}))
        return
    if args.ceiling:
        fn = {"read": ceiling_read, "gather": ceiling_gather, "rows": ceiling_rows}[args.ceiling]
        print(json.dumps({"ceiling": args.ceiling, **fn(torch, dev)}))
        return

    scale = {}
    if args.scale:
        for item in args.scale.split(","):
            key, val = item.split("=")
            scale[key.strip()] = float(val) if "." in val else int(val)
    if args.variant == "batched-gemm":
        batched_gemm_bench(args, scale, torch, gen, L, dev)
        return
    if args.spmm_k and (args.config is None or args.variant != "tuned"):
        sys.exit("bench.py: --spmm-k needs --config N and the tuned variant")
    all_five = args.config is None and args.variant == "tuned" and not scale
    cfg = 2 if args.config is None else args.config
    if args.zipf_s is not None and cfg == 4:
        scale["s"] = args.zipf_s
    fingerprint = source_fingerprint("spmm" if (args.spmm_k or (args.config == 5)) else "spmv")
    head, w = run_workload(cfg, scale, args.variant, args.steps, args.warmup,
                           None if args.no_cpu else args.cpu_seconds, torch, gen, L, dev, fingerprint,
                           spmm_k=args.spmm_k)
    ceilings = ceiling_read(torch, dev, reps=10) if args.variant == "tuned" else {}

    configs = None
    if all_five:
        # the other four synthetic workloads, shorter timed loops for the long products
        configs = []
        cap = {1: args.steps, 3: 200, 4: 100, 5: 400}
        for c in (1, 2, 3, 4, 5):
            if c == cfg:
                configs.append(head)
                continue
            entry, _ = run_workload(c, None, "tuned", max(1, min(args.steps, cap[c])), args.warmup,
                                    None if args.no_cpu else args.cpu_seconds_extra, torch, gen, L, dev, fingerprint)
            configs.append(entry)
        ceilings.update(ceiling_gather(torch, dev, reps=5))
        for e in configs:       # workloads whose columns are random: the floor the gather rate sets
            if e["workload"].startswith(("uniform16", "zipf")):
                e["gather_floor_ms"] = round(e["nnz"] / (ceilings["gather_G_per_s"] * 1e9) * 1e3, 4)

    traffic, kernel_ms = head["traffic"], head["kernel_ms"]
    out = {
        "metric": "CSR SpMV effective HBM GB/s (vals+colidx+rowptr+x+y bytes / time); "
                  "gflops and frac_hbm_peak alongside",
        "value": head["GBps"], "unit": "GB/s", "n_gpus": 1, "steps": head["steps"], "warmup": args.warmup,
        "ms_per_step": head["ms_per_step"], "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": head["dtype"], "data": "synthetic",
        "config": {"workload": w.name, "nrows": w.nrows, "nnz": w.nnz, "k": w.k, "alpha": w.alpha,
                   "beta": w.beta, "index": "int32", "bytes_per_step": head["algorithmic_bytes"], "variant": args.variant},
        "gflops": head["gflops"],
        # value / peak: CSR's bytes over time.  The kernels move fewer bytes than CSR holds where the analysis
        # replaced column indices by 16-bit codes or row patterns: traffic_frac is the bytes really moved / peak
        "frac_hbm_peak": round(head["GBps"] / HBM_PEAK_GBS, 4),
        "traffic_frac": head["traffic_frac"],
        "create_ms": head["create_ms"],
        "roofline": {"bound": "hbm", "achieved": round(head["algorithmic_bytes"] / (kernel_ms * 1e-3) / 1e9, 2),
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": head["frac"], "frac_basis": "csr_bytes",
                     "traffic": traffic,
                     # measured HBM bytes per launch / live kernel time: what the memory system really moved
                     "traffic_rate_GBps": round(traffic / (kernel_ms * 1e-3) / 1e9, 2) if traffic else None,
                     "traffic_frac": head["traffic_frac"], "traffic_stale": head["traffic_stale"],
                     "traffic_source": (MEASURED.get(w.name) or {}).get("source") if args.variant == "tuned" else None,
                     "source_fingerprint": fingerprint,
                     "algorithmic_bytes": head["algorithmic_bytes"],
                     "practical_ceiling": ceilings or None,
                     "kernel": head["kernel"], "kernel_ms": kernel_ms},
        "cpu_baseline": head["cpu_baseline"],
        "parity": head["parity"],
    }
    if configs is not None:
        out["configs"] = configs
    print(json.dumps(out))
    checked = [e["parity"] for e in (configs or [head]) if e["parity"] is not None]
    if any(not p["ok"] for p in checked):
        sys.exit("bench.py: a timed product does not match the oracle within the bound (see \"parity\")")


if __name__ == "__main__":
    main()
