"""Compile the HIP sources into paper_1801_04928_amd/liblf.so for gfx950 (hipcc cross-compiles
without a GPU), and the benchmark's measurement aid (bench_probe.hip beside bench.py: plain streaming
kernels and a matrix-instruction loop, no part of the library) into libbench_probe.so.  Run as
`python -m paper_1801_04928_amd.build`."""
from __future__ import annotations

import os
import shutil
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "liblf.so")
SOURCES = ["lf_api.hip", "b1_kernels.hip", "batched_kernels.hip", "persistent_kernels.hip"]
OBJ_DIR = os.path.join(HERE, "_build")              # object files (not committed)
ROOT = os.path.dirname(HERE)
PROBE_LIB = os.path.join(ROOT, "libbench_probe.so")      # measurement aid of bench.py, not part of the library
PROBE_SOURCES = [os.path.join(ROOT, "bench_probe.hip")]

FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    # packed fp32 math is switched off for every kernel of this library
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-command-line-argument", "-Wno-unknown-warning-option",
]


def hipcc() -> str:
    exe = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(exe):
        raise RuntimeError("hipcc not found")
    return exe


def _run(cmd, verbose: bool) -> None:
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    out = "\n".join(l for l in (res.stdout + res.stderr).splitlines()
                    if "packed-fp32-ops" not in l or "error" in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    if verbose and out.strip():
        print(out)


def _compile(lib: str, sources, verbose: bool) -> None:
    """One object per source file, compiled side by side, then one link."""
    from concurrent.futures import ThreadPoolExecutor
    os.makedirs(OBJ_DIR, exist_ok=True)
    flags = [f for f in FLAGS if f != "-shared"]
    jobs = []
    for s in sources:
        obj = os.path.join(OBJ_DIR, os.path.splitext(os.path.basename(s))[0] + ".o")
        jobs.append((obj, [hipcc(), *flags, "-c", "-o", obj, os.path.join(CSRC, s)]))
    with ThreadPoolExecutor(max_workers=min(4, len(jobs))) as pool:
        list(pool.map(lambda j: _run(j[1], verbose), jobs))
    _run([hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", lib, *[j[0] for j in jobs]], verbose)


def build(verbose: bool = True) -> str:
    _compile(LIB, SOURCES, verbose)
    _compile(PROBE_LIB, PROBE_SOURCES, verbose)
    return LIB


if __name__ == "__main__":
    build()
    print("built", LIB)
    sys.exit(0)
