"""Build the HIP library (gfx950) in-tree:  python -m paper_2205_09120_amd.build"""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "liblowbit_gemm.so")
OBJDIR = os.path.join(HERE, "_build")  # objects are kept: the host-sanitizer test links its own api.o against them
SOURCES = ["api.hip", "pack.hip", "gemm_popc.hip", "gemm_skinny.hip", "gemm_i8_mfma.hip", "gemm_i8_skinny.hip", "gemm_mx_mfma.hip", "im2col.hip", "calibrate.hip"]
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-fvisibility=hidden",
    # keep the compiler from forming packed-FP32 instructions
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
]


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    proc = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in proc.stdout.splitlines() if "packed-fp32-ops" not in l)
    if proc.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    if verbose and out.strip():
        print(out)


def build(verbose: bool = False) -> str:
    """Compile every HIP source into liblowbit_gemm.so.  Always recompiles (objects in parallel, then one link)."""
    import concurrent.futures
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    missing = [s for s in SOURCES if not os.path.exists(os.path.join(CSRC, s))]
    if missing:
        raise RuntimeError(f"missing sources: {missing}")
    os.makedirs(OBJDIR, exist_ok=True)
    cflags = [f for f in FLAGS if f != "-shared"]
    jobs = []
    for src in SOURCES:
        obj = object_path(src)
        jobs.append(([hipcc] + cflags + ["-I", CSRC, "-c", os.path.join(CSRC, src), "-o", obj + ".tmp"], obj))
    workers = max(1, min(8, os.cpu_count() or 1, len(jobs)))
    with concurrent.futures.ThreadPoolExecutor(max_workers=workers) as pool:
        list(pool.map(lambda j: _run(j[0], verbose), jobs))
    for _, obj in jobs:
        os.replace(obj + ".tmp", obj)
    tmp = LIB + ".tmp"
    _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp] + [j[1] for j in jobs], verbose)
    os.replace(tmp, LIB)
    return LIB


def object_path(src: str) -> str:
    """Where build() leaves the object of one source."""
    return os.path.join(OBJDIR, src.replace(".hip", ".o"))


if __name__ == "__main__":
    print(build(verbose=True))
