#!/usr/bin/env python3
"""Benchmark of the CSR SpMV hot path on one MI355X.

A step is one lapis_spmv call (y = alpha*A*x + beta*y) on the 128^3 27-point
fp64 stencil matrix, inputs resident in HBM.  Timing follows the paper's
protocol (Appendix, system configuration: untimed warm-up, then the mean over
the timed repetitions).  Prints one JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--config C] [--no-cpu]
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0  # MI355X HBM3E, published peak

# HBM bytes per launch of the dominant kernel, from rocprofv3 --pmc FETCH_SIZE and WRITE_SIZE runs of
# this script, each scaled by what the same counter reads for a plain 1 GiB device copy
# (FETCH_SIZE x2.000, WRITE_SIZE x1.000).  Re-measure after a kernel change.
MEASURED_TRAFFIC_BYTES = {
    "stencil27_128x128x128_f64": 505.30e6,
    "stencil27_128x128x128_f64_spmm_k16": 1036.91e6,
    "table3_Elasticity3D_60_n648000_f64": 522.18e6,
    "zipf1.8_cap200000_n8388608_f32": 9123.91e6,
}
DOMINANT_KERNEL = {
    "stencil27_128x128x128_f64": "spmv_stream_kernel<double, 2, true, 4> (4: row patterns)",
    "stencil27_128x128x128_f64_spmm_k16": "spmm_stream_kernel<double, 2, 8, true, true, true> (last: rows of X shared by 4 consecutive rows)",
    "table3_Elasticity3D_60_n648000_f64": "spmv_stream_kernel<double, 8, true, 1> (1: 16-bit column offsets)",
}


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
    step = lambda: L.lapis_batched_gemm(batch, m, n, k, 1.0, dA, dB, 0.0, dC, code)
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    wall0 = time.perf_counter()
    start.record()
    for _ in range(args.steps):
        step()
    stop.record()
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - wall0) * 1e3 / args.steps
    kernel_ms = start.elapsed_time(stop) / args.steps
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


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=1000)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", type=int, default=2, help="workload 1..5 (2 = the headline workload); 6..9 = stand-ins for the paper's Table 3")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle timing")
    ap.add_argument("--cpu-seconds", type=float, default=10.0)
    ap.add_argument("--scale", default=None,
                    help="override size parameters of the workload's recipe, e.g. nx=288,ny=288,nz=288 "
                         "(labelled in config.workload; the default sizes are the benchmark's)")
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
    ap.add_argument("--copy-calibration", action="store_true",
                    help="run a plain device copy of known size instead (reference for the "
                         "FETCH_SIZE / WRITE_SIZE counters) and exit")
    args = ap.parse_args()
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

    scale = {}
    if args.scale:
        for item in args.scale.split(","):
            key, val = item.split("=")
            scale[key.strip()] = float(val) if "." in val else int(val)
    if args.variant == "batched-gemm":
        batched_gemm_bench(args, scale, torch, gen, L, dev)
        return
    if args.zipf_s is not None and args.config == 4:
        scale["s"] = args.zipf_s
    w = gen.workload(args.config, scale or None)
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

    if args.variant != "tuned" and w.k != 0:
        sys.exit("bench.py: --variant applies to the SpMV workloads only")
    if args.variant in ("transpose", "transposed-handle", "host-buffers") and w.nrows != w.ncols:
        sys.exit("bench.py: this variant expects a square workload")
    if args.variant == "paper-shape":
        step = lambda: L.lapis_spmv_paper_shape(A.handle, w.alpha, x, w.beta, y)
    elif args.variant == "transpose":
        step = lambda: L.lapis_spmv_transpose(A.handle, w.alpha, x, w.beta, y)
    elif args.variant == "transposed-handle":
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        At = A.transposed()
        torch.cuda.synchronize()
        create_ms = (time.perf_counter() - t0) * 1e3     # transposition + analysis of A^T
        step = lambda: L.lapis_spmv(At.handle, w.alpha, x, w.beta, y)
    elif args.variant == "host-buffers":
        xv, yv = L.DualView(w.ncols, w.dtype), L.DualView(w.nrows, w.dtype)
        xv.host[:] = w.x
        yv.host[:] = 0.0 if w.y0 is None else w.y0
        yv.modify_host()

        def step():
            xv.modify_host()                     # the caller rewrote x on the host
            L.lapis_spmv_dualview(A.handle, w.alpha, xv, w.beta, yv)
            yv.sync_host()                       # and reads y on the host
    elif args.variant == "graph":
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
        args.steps = max(per_graph, args.steps // per_graph * per_graph)
        replays = iter(range(10 ** 9))
        step = lambda: graph.replay() if next(replays) % per_graph == 0 else None
    elif w.k == 0:
        step = lambda: L.lapis_spmv(A.handle, w.alpha, x, w.beta, y)
    else:
        step = lambda: L.lapis_spmm(A.handle, w.k, w.alpha, x, w.k, w.beta, y, w.k)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    wall0 = time.perf_counter()
    start.record()
    for _ in range(args.steps):
        step()
    stop.record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - wall0) * 1e3
    ev_ms = start.elapsed_time(stop)
    ms_per_step = wall_ms / args.steps          # barrier-to-barrier wall clock
    kernel_ms = ev_ms / args.steps              # events on the launch stream

    nbytes = algorithmic_bytes(w)
    flops = 2.0 * w.nnz * k
    gbs = nbytes / (ms_per_step * 1e-3) / 1e9
    achieved = nbytes / (kernel_ms * 1e-3) / 1e9

    cpu = None
    if not args.no_cpu:
        import oracle
        fn = (lambda: oracle.spmv(w.rowptr, w.colidx, w.vals, w.x, w.alpha, w.beta, w.y0)) if w.k == 0 else (
            lambda: oracle.spmm(w.rowptr, w.colidx, w.vals, w.x, w.alpha, w.beta, w.y0))
        fn()
        reps, best, spent = 0, float("inf"), 0.0
        while spent < args.cpu_seconds or reps < 3:
            t = time.perf_counter()
            fn()
            d = time.perf_counter() - t
            best, spent, reps = min(best, d), spent + d, reps + 1
        cpu = {"value": round(nbytes / best / 1e9, 3), "unit": "GB/s", "cores": 1, "kind": "oracle",
               "sample": f"full workload, best of {reps} serial passes ({best * 1e3:.1f} ms each; "
                         f"{flops / best / 1e9:.2f} GFLOP/s), 1 of {os.cpu_count()} host cores"}

    traffic = MEASURED_TRAFFIC_BYTES.get(w.name) if args.variant == "tuned" else None
    out = {
        "metric": "CSR SpMV effective HBM GB/s (vals+colidx+rowptr+x+y bytes / time); "
                  "gflops and frac_hbm_peak alongside",
        "value": round(gbs, 2), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 6), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f64" if w.dtype == np.float64 else "f32", "data": "synthetic",
        "config": {"workload": w.name, "nrows": w.nrows, "nnz": w.nnz, "k": w.k, "alpha": w.alpha,
                   "beta": w.beta, "index": "int32", "bytes_per_step": nbytes, "variant": args.variant},
        "gflops": round(flops / (ms_per_step * 1e-3) / 1e9, 2),
        "frac_hbm_peak": round(gbs / HBM_PEAK_GBS, 4),
        "create_ms": round(create_ms, 3),
        "roofline": {"bound": "hbm", "achieved": round(achieved, 2), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(achieved / HBM_PEAK_GBS, 4),
                     "traffic": traffic,
                     # measured HBM bytes per launch / live kernel time: what the memory system really moved
                     "traffic_rate_GBps": round(traffic / (kernel_ms * 1e-3) / 1e9, 2) if traffic else None,
                     # the same against the peak: frac counts CSR's bytes, this one the bytes moved (the
                     # row patterns and 16-bit column codes move fewer than CSR has)
                     "traffic_frac": round(traffic / (kernel_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4) if traffic else None,
                     "algorithmic_bytes": nbytes,
                     "kernel": (DOMINANT_KERNEL.get(w.name, "all kernels of the step") if args.variant == "tuned"
                                else VARIANT_KERNEL[args.variant]),
                     "kernel_ms": round(kernel_ms, 6)},
        "cpu_baseline": cpu,
    }
    A.close()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
