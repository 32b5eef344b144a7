"""The host side of the library (handle, argument and state checks, workspace layout, schedule functions)
built with the undefined-behaviour sanitizer in trapping mode, and the host-only ABI tests run against that
build in a child process: any signed overflow, misaligned access, out-of-range shift or enum value, or null
dereference on those paths ends the child with a trap.  (Device code is compiled as usual; no kernel runs here.)"""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_1801_04928_amd", "csrc")
SOURCES = ["lf_api.hip", "b1_kernels.hip", "batched_kernels.hip", "persistent_kernels.hip"]
HOST_SAN = ["-Xarch_host", "-fsanitize=undefined", "-Xarch_host", "-fsanitize-trap=undefined"]

CHILD = r"""
import sys
sys.path.insert(0, {root!r})
import paper_1801_04928_amd.binding as binding
binding.library_path = lambda: {lib!r}
import pytest
sys.exit(pytest.main(["-q", "-x", "-p", "no:cacheprovider", {abi!r}]))
"""


def test_abi_tests_pass_on_a_host_sanitized_build(tmp_path):
    hipcc = "/opt/rocm/bin/hipcc"
    flags = ["--offload-arch=gfx950", "-O1", "-std=c++17", "-fPIC", "-Xclang", "-target-feature", "-Xclang",
             "-packed-fp32-ops", "-Wno-unused-command-line-argument", "-Wno-unknown-warning-option"]

    def compile_one(src):
        obj = str(tmp_path / (os.path.splitext(src)[0] + ".o"))
        res = subprocess.run([hipcc, *flags, *HOST_SAN, "-c", "-o", obj, os.path.join(CSRC, src)],
                             capture_output=True, text=True)
        assert res.returncode == 0, res.stderr[-2000:]
        return obj

    with ThreadPoolExecutor(max_workers=4) as pool:
        objs = list(pool.map(compile_one, SOURCES))
    lib = str(tmp_path / "liblf_sanitized.so")
    res = subprocess.run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", lib, *objs],
                         capture_output=True, text=True)
    assert res.returncode == 0, res.stderr[-2000:]
    child = CHILD.format(root=ROOT, lib=lib, abi=os.path.join(ROOT, "tests", "test_abi.py"))
    res = subprocess.run([sys.executable, "-c", child], capture_output=True, text=True, cwd=ROOT)
    assert res.returncode == 0, (res.stdout[-3000:] + res.stderr[-2000:])
    assert " passed" in res.stdout
