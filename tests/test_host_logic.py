"""Host-only checks of the persistent kernels' tag arithmetic (csrc/persistent_epoch.h), compiled with the
host compiler: the tags never take the value the exchange buffers are cleared to, the two backward grids'
tags never meet, and the launch count wraps without passing through 0."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

PROGRAM = r"""
#include "persistent_epoch.h"
#include <cstdio>
int main() {
    using namespace lf;
    // around the wrap: counts 2^31 - 3 .. 2^31 - 1, then 1, 2, ...
    unsigned c = 0x7ffffffdu;
    for (int i = 0; i < 8; ++i) {
        if (c == 0u || c > 0x7fffffffu) { std::printf("count out of range: %u\n", c); return 1; }
        if (forward_epoch(c) == 0u || backward_epoch(c, true) == 0u || backward_epoch(c, false) == 0u) {
            std::printf("zero tag at count %u\n", c); return 1;
        }
        if ((backward_epoch(c, true) & 1u) != 0u || (backward_epoch(c, false) & 1u) != 1u) {
            std::printf("parity broken at count %u\n", c); return 1;
        }
        const unsigned n = next_launch_count(c);
        if (n == c) { std::printf("count stuck at %u\n", c); return 1; }
        if (backward_epoch(n, true) == backward_epoch(c, true)) { std::printf("tag repeats at %u\n", c); return 1; }
        c = n;
    }
    if (next_launch_count(0x7fffffffu) != 1u) { std::printf("wrap is not to 1\n"); return 1; }
    if (next_launch_count(1u) != 2u) return 1;
    // a sample of the whole range
    for (unsigned long long v = 1; v <= 0x7fffffffull; v += 9973) {
        const unsigned x = (unsigned)v;
        if (backward_epoch(x, true) == 0u || backward_epoch(x, false) == 0u || forward_epoch(x) == 0u) return 1;
        if (backward_epoch(x, true) / 2u != x || backward_epoch(x, false) / 2u != x) return 1;   // no overflow
    }
    std::printf("ok\n");
    return 0;
}
"""


def test_epoch_tags(tmp_path):
    src = tmp_path / "epoch_test.cpp"
    src.write_text(PROGRAM)
    exe = tmp_path / "epoch_test"
    inc = os.path.join(ROOT, "paper_1801_04928_amd", "csrc")
    subprocess.run(["g++", "-std=c++17", "-O1", "-I", inc, "-o", str(exe), str(src)], check=True)
    out = subprocess.run([str(exe)], capture_output=True, text=True)
    assert out.returncode == 0 and out.stdout.strip() == "ok", out.stdout + out.stderr
