"""Host-only checks of the persistent kernels' host-evaluable arithmetic, compiled with the host compiler.
csrc/persistent_epoch.h: the tags never take the value the exchange buffers are cleared to, the two backward
grids' tags never meet, and the launch count wraps without passing through 0.
csrc/persistent_partition.h: the workers' slots are a permutation of their indices, every row of a partition's
layers is stored by exactly one of its members, and a partition laid out across XCDs has members on all 8."""
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


PARTITION_PROGRAM = r"""
#include "persistent_partition.h"
#include <cstdio>
#include <vector>
int main() {
    using namespace lf;
    const int workers[] = {1, 3, 8, 24, 64, 96, 200, 256, 512};
    const int widths[] = {4, 64, 260, 1000, 1024, 4096};
    for (int nw : workers)
        for (int k = 1; k <= 40; ++k) {
            if (k > nw) continue;
            for (int spread = 0; spread < 2; ++spread) {
                // the slot is a permutation of the workgroup index
                std::vector<int> seen((size_t)nw, 0);
                for (int wid = 0; wid < nw; ++wid) {
                    const int v = worker_slot(wid, nw, k, spread != 0);
                    if (v < 0 || v >= nw || seen[(size_t)v]++) { std::printf("slot nw=%d k=%d wid=%d\n", nw, k, wid); return 1; }
                }
                // a partition whose layout is spread has members on all 8 XCDs (workgroup index mod 8)
                if (spread && k % 4 == 0 && nw % 8 == 0 && (nw / 8) % k == 0) {
                    for (int part = 0; part < k; ++part) {
                        int xcds = 0;
                        for (int wid = 0; wid < nw; ++wid)
                            if (worker_slot(wid, nw, k, true) % k == part) xcds |= 1 << (wid % 8);
                        if (xcds != 0xff) { std::printf("partition %d of k=%d nw=%d misses an XCD\n", part, k, nw); return 1; }
                    }
                }
                // every row of a partition's layers has exactly one owner among its members
                for (int N : widths)
                    for (int part = 0; part < k; ++part) {
                        std::vector<int> owners((size_t)N, 0);
                        const int members = partition_members(part, nw, k);
                        int counted = 0;
                        for (int wid = 0; wid < nw; ++wid) {
                            const int v = worker_slot(wid, nw, k, spread != 0);
                            if (v % k != part) continue;
                            ++counted;
                            int b, e;
                            member_rows(v / k, members, N, &b, &e);
                            if (b < 0 || e > N || b > e) { std::printf("range nw=%d k=%d N=%d\n", nw, k, N); return 1; }
                            for (int r = b; r < e; ++r) ++owners[(size_t)r];
                        }
                        if (counted != members) { std::printf("members nw=%d k=%d part=%d\n", nw, k, part); return 1; }
                        for (int r = 0; r < N; ++r)
                            if (owners[(size_t)r] != 1) { std::printf("row %d of N=%d: %d owners (nw=%d k=%d part=%d)\n", r, N, owners[(size_t)r], nw, k, part); return 1; }
                    }
            }
        }
    std::printf("ok\n");
    return 0;
}
"""


def test_worker_partitions(tmp_path):
    src = tmp_path / "partition_test.cpp"
    src.write_text(PARTITION_PROGRAM)
    exe = tmp_path / "partition_test"
    inc = os.path.join(ROOT, "paper_1801_04928_amd", "csrc")
    subprocess.run(["g++", "-std=c++17", "-O2", "-I", inc, "-o", str(exe), str(src)], check=True)
    out = subprocess.run([str(exe)], capture_output=True, text=True)
    assert out.returncode == 0 and out.stdout.strip() == "ok", out.stdout + out.stderr
