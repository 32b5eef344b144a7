"""Compile the HIP sources into paper_1801_04928_amd/liblf.so for gfx950 (hipcc cross-compiles
without a GPU), and the benchmark's matrix-core probe into libprobe.so.  Run as
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
PROBE_LIB = os.path.join(HERE, "libprobe.so")      # measurement aid of bench.py, not part of the library
PROBE_SOURCES = ["peak_probe.hip"]

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


def _compile(lib: str, sources, verbose: bool) -> None:
    srcs = [os.path.join(CSRC, s) for s in sources]
    cmd = [hipcc(), *FLAGS, "-o", lib, *srcs]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    out = "\n".join(l for l in (res.stdout + res.stderr).splitlines()
                    if "packed-fp32-ops" not in l or "error" in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    if verbose and out.strip():
        print(out)


def build(verbose: bool = True) -> str:
    _compile(LIB, SOURCES, verbose)
    _compile(PROBE_LIB, PROBE_SOURCES, verbose)
    return LIB


if __name__ == "__main__":
    build()
    print("built", LIB)
    sys.exit(0)
