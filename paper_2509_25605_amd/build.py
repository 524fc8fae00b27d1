"""Builds the gfx950 shared library from csrc/ with hipcc (cross-compiles without a GPU)."""
from __future__ import annotations

import os
import subprocess
import tempfile
from concurrent.futures import ThreadPoolExecutor

_HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(_HERE, "csrc")
LIB_PATH = os.path.join(_HERE, "liblapis_mi355x.so")
SOURCES = ["lapis_api.hip", "dualview.hip", "batched_gemm.hip"]
# the measurement kernels bench.py times beside the products (include/lapis_ceilings.h): a library of their own
CEILINGS_LIB_PATH = os.path.join(_HERE, "libceilings_mi355x.so")
CEILINGS_SOURCES = ["ceilings.hip"]
HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    # packed-fp32 instructions are kept off for every HIP translation unit
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-command-line-argument",
]


def _run(cmd) -> str:
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in res.stdout.splitlines() if "packed-fp32-ops" not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    return out


def build(verbose: bool = False) -> str:
    """Compile every HIP source (side by side, objects in a temporary folder) and link them into
    liblapis_mi355x.so and libceilings_mi355x.so; always recompiles."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    with tempfile.TemporaryDirectory(prefix="lapis_build_") as tmp:
        sources = SOURCES + CEILINGS_SOURCES
        objects = [os.path.join(tmp, os.path.splitext(s)[0] + ".o") for s in sources]
        with ThreadPoolExecutor(max_workers=len(sources)) as pool:
            logs = list(pool.map(lambda so: _run([hipcc, *HIPCC_FLAGS, "-c", os.path.join(CSRC, so[0]), "-o", so[1]]),
                                 zip(sources, objects)))
        logs.append(_run([hipcc, *HIPCC_FLAGS, "-shared", "-o", LIB_PATH, *objects[:len(SOURCES)]]))
        logs.append(_run([hipcc, *HIPCC_FLAGS, "-shared", "-o", CEILINGS_LIB_PATH, *objects[len(SOURCES):]]))
    out = "\n".join(l for l in logs if l.strip())
    if verbose and out:
        print(out)
    return LIB_PATH


if __name__ == "__main__":
    print(build(verbose=True))
