"""Helpers for the GPU parity tests: run the library on a synthetic net and compare every tensor
with the CPU oracle, layer by layer."""
import sys
import time

import numpy as np

from oracle import backprop as O

TOL = {"f32": 1e-5, "bf16": 2e-2}

# A tensor whose largest oracle entry is below this is in (or next to) the fp32 subnormal range,
# where a relative 1e-5 is not representable; it is compared in units of the smallest subnormal.
SUBNORMAL_SCALE = 2.0 ** -126 * 2.0 ** 10
DENORM_ULP = 2.0 ** -149


def log(msg):
    sys.stderr.write(f"[{time.strftime('%H:%M:%S')}] {msg}\n")
    sys.stderr.flush()


def compare(name, got, want, tol, report, denorm_ulps=24.0):
    """Normwise error max|got-want| / max|want| <= tol (or an absolute bound for subnormal tensors)."""
    want = np.asarray(want, dtype=np.float64)
    got = np.asarray(got, dtype=np.float64).reshape(want.shape)
    assert np.all(np.isfinite(got)), f"{name}: non-finite values"
    scale = float(np.max(np.abs(want)))
    diff = float(np.max(np.abs(got - want)))
    err = diff / scale if scale > 0 else (0.0 if diff == 0 else float("inf"))
    if err > tol and scale < SUBNORMAL_SCALE:
        # too close to the subnormal range for a relative bound: absolute, in denormal ulps, and listed
        report.setdefault("subnormal", []).append((name, scale, diff / DENORM_ULP))
        assert diff <= denorm_ulps * DENORM_ULP, f"{name}: subnormal tensor off by {diff / DENORM_ULP:.1f} denormal ulps"
        return 0.0
    report["worst"] = max(report.get("worst", 0.0), err)
    assert err <= tol, f"{name}: normwise error {err:.3e} > {tol:.1e}"
    return err


def to_np(t):
    return t.detach().float().cpu().numpy()


def run_gpu(net, k, sched=None, poison=True):
    """Build a LeapfrogNet for the synthetic net, run forward + backward(k), return it (synchronised)."""
    import torch
    import paper_1801_04928_amd as P
    s = net.spec
    g = P.LeapfrogNet(s.L, list(s.widths) if s.widths else s.N, s.B, s.dtype)
    g.load(net)
    if sched is not None:
        g.set_schedule(sched)
    if poison:
        poison_buffers(g)
    g.forward()
    g.backward(k)
    torch.cuda.synchronize()
    return g


def poison_buffers(g, whole_workspace=True):
    """NaN in every buffer the pass must overwrite: a read before the producer has written shows up.
    whole_workspace=True (only before the first pass of a handle) also covers the library's internal
    exchange buffers; afterwards only the activations and errors are poisoned, because the tagged
    words of the persistent path must keep the tags of the previous pass."""
    if whole_workspace:
        g.workspace.view(g.torch.float32)[: g.workspace.numel() // 4].fill_(float("nan"))
    else:
        for l in range(2, g.L + 1):
            g.activation(l).fill_(float("nan"))
            g.delta(l).fill_(float("nan"))
    for t in g.nabla_w + g.nabla_b:
        t.fill_(float("nan"))


def tile_origins(rows, cols, count, size, rng, boundary=256):
    """Upper-left corners of the sampled tiles of one rows x cols matrix: the four corner tiles, one tile
    straddling every multiple of `boundary` (the largest kernel tile) in each dimension -- row boundary m is
    paired with a column boundary drawn from a random permutation -- and random tiles up to `count`."""
    rmax, cmax = max(0, rows - size), max(0, cols - size)
    picks = [(0, 0), (0, cmax), (rmax, 0), (rmax, cmax)]
    rb = [min(rmax, max(0, m - size // 2)) for m in range(boundary, rows, boundary)]
    cb = [min(cmax, max(0, m - size // 2)) for m in range(boundary, cols, boundary)]
    n = max(len(rb), len(cb))
    if n:
        rb = rb or [0]
        cb = cb or [0]
        perm = rng.permutation(n)
        picks += [(rb[i % len(rb)], cb[int(perm[i]) % len(cb)]) for i in range(n)]
    while len(picks) < count:
        picks.append((int(rng.integers(0, rmax + 1)), int(rng.integers(0, cmax + 1))))
    return picks


def check_against_oracle(net, g, tol=None, sample_tiles=None, rng=None):
    """Compare a^l, delta^l, nabla_b^l and nabla_w^l for every layer.  With sample_tiles = (count, size)
    nabla_w is compared on at least that many size x size tiles per layer (see tile_origins), formed one by
    one from the oracle's delta and a via eq. (bp4)."""
    s = net.spec
    tol = TOL[s.dtype] if tol is None else tol
    report = {}
    w, b = net.w_by_layer, net.b_by_layer
    a = O.forward(w, b, net.x(), s.L)
    for l in range(2, s.L + 1):
        compare(f"a^{l}", to_np(g.activation(l)), a[l], tol, report)
    for l, delta, nb, nw in O.backward_layers(w, a, net.y(), s.L, want_nabla_w=sample_tiles is None):
        compare(f"delta^{l}", to_np(g.delta(l)), delta, tol, report)
        gw, gb = g.grads(l)
        compare(f"nabla_b^{l}", to_np(gb), nb, tol, report)
        if sample_tiles is None:
            compare(f"nabla_w^{l}", to_np(gw), nw, tol, report)
        else:
            count, size = sample_tiles
            origins = tile_origins(s.width(l), s.width(l - 1), count, size, rng)
            want_all = np.stack([delta[:, j0:j0 + size].T @ a[l - 1][:, k0:k0 + size] for j0, k0 in origins])
            got_all = to_np(g.torch.stack([gw[j0:j0 + size, k0:k0 + size] for j0, k0 in origins]))
            report["tiles_per_layer"] = len(origins)
            compare(f"nabla_w^{l}[tiles]", got_all, want_all, tol, report)
            assert bool(g.torch.isfinite(gw).all()), f"nabla_w^{l}: non-finite values"
        if l % 8 == 0:
            log(f"  layer {l} checked, worst so far {report.get('worst', 0.0):.2e}")
    return report
