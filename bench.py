"""Benchmark: full backpropagation passes per second on one MI355X.

A step is one pass of the whole hot path -- forward (x),(z),(a), then the leapfrogged backward pass
(bp1)-(bp4) with k workers -- over one seeded synthetic input that is already resident in HBM.
Prints ONE JSON line.  Without --config the five benchmark configurations run one after another in this
process: the top level of the line is the largest one (configuration 5, bf16 minibatch), and `per_config`
carries the same figures for each.  The roofline objects price the backward pass against the HBM peak
(B = 1) or the MFMA peak (minibatch); the cpu_baseline objects are the CPU oracle timed on this machine's
cores.  The timed steps run a configuration's largest worker count k; `cost_model` times the other configured
worker counts, the chain alone and the sequential pass as well, and the fastest configured k is quoted under
`roofline.fastest_configured_k`.
"""
from __future__ import annotations

import argparse
import ctypes
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
MFMA_PEAK_TFLOPS = {"f32": 157.3, "bf16": 2500.0}
ALL_CONFIGS = ["cfg1", "cfg2", "cfg3", "cfg4", "cfg5"]
SCHED_NAMES = ["auto", "streams", "persistent", "redundant", "fused"]


def matrix_sizes(spec):
    """Entries of w^l, l = 2..L: n_l * n_{l-1} (N^2 when every layer has N neurons)."""
    return [spec.width(l) * spec.width(l - 1) for l in range(2, spec.L + 1)]


def algorithmic_work(spec, sgd=False):
    """Per backward pass.  B = 1: bytes the method must move, 4 bytes per entry of a matrix read or written:
    the chain reads w^{l+1} for l = L-1..2, the workers write nabla_w^l for l = 2..L (vectors are O(N),
    ignored).  Minibatch: 2 B flops per matrix entry for each chain and each gradient contraction.
    sgd: the descent step fused into the workers reads and rewrites w^l instead of writing nabla_w^l."""
    sizes = matrix_sizes(spec)
    every, chain = sum(sizes), sum(sizes[1:])        # the chain never reads w^2
    if spec.B == 1:
        es = 4 if spec.dtype == "f32" else 2
        return {"bound": "hbm", "bwd": es * chain + (8 if sgd else 4) * every, "chain": es * chain,
                "fwd": es * every, "unit": "GB/s", "peak": HBM_PEAK_GBS, "scale": 1e9}
    f = 2.0 * spec.B
    return {"bound": "mfma", "bwd": f * (chain + every), "chain": f * chain, "fwd": f * every, "unit": "TFLOP/s",
            "peak": MFMA_PEAK_TFLOPS[spec.dtype], "scale": 1e12}


def measured_traffic(cfg_name, k):
    """HBM bytes per launch of the backward kernel as stored by the committed rocprofv3 counter runs
    (profiles/traffic.json) -- not a counter read in this run -- or None when the kernel source has changed
    since they were taken."""
    import hashlib
    path = os.path.join(ROOT, "profiles", "traffic.json")

    def source_hash(names):
        h = hashlib.sha256()
        for name in names:
            h.update(open(os.path.join(ROOT, "paper_1801_04928_amd", "csrc", name), "rb").read())
        return h.hexdigest()
    try:
        rec = json.load(open(path))
        e = rec.get(f"{cfg_name}_k{k}")
        if e is None:
            return None
        if "source_sha256" in e:          # a minibatch pass: the sum over its kernels, hashed with their sources
            if e["source_sha256"] != source_hash(e["sources"]):
                return None
        elif rec.get("kernel_source_sha256") != source_hash(("persistent_kernels.hip", "persistent.h", "persistent_partition.h", "device_helpers.h")):
            return None
        return e["fetch_bytes"] + e["write_bytes"]
    except Exception:
        return None


# ------------------------------------------------------------------------------------------ CPU oracle
def _blas_threads():
    try:
        from threadpoolctl import threadpool_info
        return max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        return os.cpu_count() or 1


class _one_thread:
    """Limits the BLAS behind numpy to one thread (threadpoolctl); a no-op if that module is missing."""

    def __enter__(self):
        try:
            from threadpoolctl import threadpool_limits
            self._ctx = threadpool_limits(limits=1)
            self._ctx.__enter__()
            self.ok = True
        except Exception:
            self._ctx, self.ok = None, False
        return self

    def __exit__(self, *exc):
        if self._ctx is not None:
            self._ctx.__exit__(*exc)


def cpu_baseline(net, gpu_net=None, budget_s=8.0):
    """The oracle as it stands, timed on the host twice: on all the cores its BLAS takes by default and on one
    thread.  Whole passes for the nets whose pass takes seconds; for the others a three-layer net at full
    width (two weight layers: forward + chain + gradient each), scaled to the whole net, and on one thread
    with an eighth of the samples as well.  Where a whole oracle pass is run, the gradients still in the
    GPU's buffers from the timed passes are compared with it (normwise error per tensor, worst over the
    layers)."""
    import numpy as np
    from oracle import backprop as O
    cores = _blas_threads()
    s = net.spec
    M = s.L - 1
    flops_pass = 6.0 * s.B * sum(matrix_sizes(s))
    if flops_pass < 5e10 or s.widths:
        w = {l: net.w(l) for l in range(2, s.L + 1)}
        b = {l: net.b(l) for l in range(2, s.L + 1)}
        x, y = net.x(), net.y()
        ref = O.full_pass(w, b, x, y, s.L)

        def timed(limit):
            n, t0 = 0, time.perf_counter()
            while True:
                O.full_pass(w, b, x, y, s.L)
                n += 1
                dt = time.perf_counter() - t0
                if dt > limit or n >= 100:
                    return n, dt
        n, dt = timed(budget_s)
        out = {"value": n / dt, "unit": "passes/s", "cores": cores, "kind": "oracle",
               "sample": f"{n} full forward+backward passes of the same net"}
        with _one_thread() as one:
            if one.ok:
                n1, dt1 = timed(budget_s)
                out["single_thread"] = {"value": n1 / dt1, "unit": "passes/s", "cores": 1,
                                        "sample": f"{n1} full passes, BLAS limited to one thread"}
        if gpu_net is not None:
            _, _, nb, nw, _ = ref
            worst, tiny = 0.0, 0
            for l in range(2, s.L + 1):
                gw, gb = gpu_net.grads(l)
                for got, want in ((gw, nw[l]), (gb, nb[l])):
                    if float(np.max(np.abs(want))) < 2.0 ** -116:
                        tiny += 1              # fp32 leaves its normal range here; the tests bound these absolutely
                        continue
                    worst = max(worst, O.normwise_error(got.detach().float().cpu().numpy().reshape(want.shape), want))
            out["parity"] = {"worst_normwise_error": worst, "tensors_below_fp32_normal_range": tiny,
                             "what": "gradients of the last timed pass against the oracle, all layers"}
        return out
    # two weight layers at full width, scaled by M / 2
    w = {l: net.w(l) for l in (2, 3)}
    b = {l: net.b(l) for l in (2, 3)}
    x, y = net.x(), net.y()
    t0 = time.perf_counter()
    O.full_pass(w, b, x, y, 3)
    dt = time.perf_counter() - t0
    out = {"value": 1.0 / (dt * M / 2.0), "unit": "passes/s", "cores": cores, "kind": "oracle",
           "sample": f"extrapolated from 2 of {M} layers at full N, B (one pass of a 3-layer net, x{M / 2:.1f})"}
    with _one_thread() as one:
        if one.ok:
            frac = 8
            xs, ys = x[: max(1, s.B // frac)], y[: max(1, s.B // frac)]
            t0 = time.perf_counter()
            O.full_pass(w, b, xs, ys, 3)
            dt1 = time.perf_counter() - t0
            scale = (M / 2.0) * (s.B / xs.shape[0])
            out["single_thread"] = {"value": 1.0 / (dt1 * scale), "unit": "passes/s", "cores": 1,
                                    "sample": f"extrapolated from 2 of {M} layers at full N with {xs.shape[0]} of "
                                              f"{s.B} samples (x{scale:.1f}), BLAS limited to one thread"}
    return out


# ------------------------------------------------------------------------------------------ machine rates
class MachineRates:
    """What plain kernels reach on this machine, measured once per process and quoted beside the rooflines:
    a 1 GiB device copy and plain streaming kernels for HBM, the vendor library's 8192^3 product and a
    register-resident matrix-instruction loop for the matrix cores."""

    def __init__(self, torch):
        self.torch = torch
        self._hbm = None
        self._mfma = {}
        self._probe = None

    def _lib(self):
        if self._probe is None:
            import ctypes
            p = ctypes.CDLL(os.path.join(ROOT, "libbench_probe.so"))
            p.probe_stream.restype = ctypes.c_double
            p.probe_stream.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p,
                                       ctypes.c_size_t, ctypes.c_void_p, ctypes.c_void_p]
            p.probe_mfma_loop.restype = ctypes.c_double
            p.probe_mfma_loop.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p]
            self._probe = p
        return self._probe

    def hbm(self):
        if self._hbm is not None:
            return self._hbm
        torch = self.torch
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        best = 1e9
        for _ in range(5):
            e0.record(); dst.copy_(src); e1.record(); torch.cuda.synchronize()
            best = min(best, e0.elapsed_time(e1))
        out = {"value": 2.0 * src.numel() * 4 / (best * 1e-3) / 1e9, "unit": "GB/s",
               "what": "1 GiB device copy (torch), bytes read + written, best of 5"}
        try:
            probe = self._lib()
            src.zero_()
            sink = torch.zeros(1, device="cuda")
            cus = torch.cuda.get_device_properties(0).multi_processor_count
            stream = torch.cuda.current_stream().cuda_stream
            nbytes = src.numel() * 4
            for mode, name in ((0, "read"), (1, "write"), (2, "read_and_write")):
                best, moved = 1e9, 0.0
                for per_cu in (2, 4, 8, 16, 32):            # workgroups per compute unit: the best is reported
                    for _ in range(3):
                        e0.record()
                        moved = probe.probe_stream(mode, per_cu * cus, src.data_ptr(), dst.data_ptr(), nbytes,
                                                   sink.data_ptr(), stream)
                        e1.record()
                        torch.cuda.synchronize()
                        best = min(best, e0.elapsed_time(e1))
                out["stream_" + name] = {
                    "value": moved / (best * 1e-3) / 1e9 if moved > 0 else None, "unit": "GB/s",
                    "what": "plain 128-bit streaming kernel over 1 GiB per buffer, best launch shape of 5, best of 3"}
            # the single-sample backward pass's own access patterns (N = 4096) as plain kernels
            probe.probe_strips_beside_rows.restype = ctypes.c_double
            probe.probe_strips_beside_rows.argtypes = [ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int,
                                                       ctypes.c_int, ctypes.c_void_p]
            mats, passes = nbytes // (4096 * 4096 * 4), 62
            for mode, name in ((0, "strips_read"), (1, "rows_written"), (2, "strips_read_beside_rows_written")):
                ms = min(probe.probe_strips_beside_rows(mode, src.data_ptr(), dst.data_ptr(), mats, passes,
                                                        sink.data_ptr()) for _ in range(3))
                moved = passes * 4096 * 4096 * 4 * (2 if mode == 2 else 1)
                out[name] = {
                    "value": moved / (ms * 1e-3) / 1e9 if ms > 0 else None, "unit": "GB/s",
                    "what": "plain kernels with the N = 4096 backward pass's access patterns (256-byte column strips in "
                            "four row blocks read by 256 workgroups, rows written by 256 workgroups, 62 matrices each), "
                            "best of 3"}
        except OSError as ex:
            out["stream_read"] = {"value": None, "what": f"not measured: {str(ex)[:80]}"}
        del src, dst
        torch.cuda.empty_cache()
        self._hbm = out
        return out

    def mfma(self, dtype):
        if dtype in self._mfma:
            return self._mfma[dtype]
        torch = self.torch
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        dt = torch.bfloat16 if dtype == "bf16" else torch.float32
        a_ = torch.randn(8192, 8192, device="cuda", dtype=dt)
        b_ = torch.randn(8192, 8192, device="cuda", dtype=dt)
        c_ = a_ @ b_
        best = 1e9
        for _ in range(5):
            e0.record(); c_ = a_ @ b_; e1.record(); torch.cuda.synchronize()
            best = min(best, e0.elapsed_time(e1))
        out = {"value": 2.0 * 8192 ** 3 / (best * 1e-3) / 1e12, "unit": "TFLOP/s",
               "what": f"torch.matmul 8192^3 {dtype} (vendor library), best of 5"}
        del a_, b_, c_
        try:
            probe = self._lib()
            sink = torch.zeros(1, device="cuda")
            cus = torch.cuda.get_device_properties(0).multi_processor_count
            stream = torch.cuda.current_stream().cuda_stream
            is_bf = 1 if dtype == "bf16" else 0
            probe.probe_mfma_loop(is_bf, 2 * cus, 2000, sink.data_ptr(), stream)
            torch.cuda.synchronize()
            best, flops = 1e9, 0.0
            for _ in range(3):
                e0.record()
                flops = probe.probe_mfma_loop(is_bf, 2 * cus, 10000, sink.data_ptr(), stream)
                e1.record()
                torch.cuda.synchronize()
                best = min(best, e0.elapsed_time(e1))
            out["mfma_loop"] = {
                "value": flops / (best * 1e-3) / 1e12 if flops > 0 else None, "unit": "TFLOP/s",
                "what": f"register-resident loop of 32x32 {dtype} matrix instructions on {cus} compute units, best of 3"}
        except OSError as ex:
            out["mfma_loop"] = {"value": None, "what": f"not measured: {str(ex)[:80]}"}
        torch.cuda.empty_cache()
        self._mfma[dtype] = out
        return out

    def vendor_same_shapes(self, spec):
        """The vendor library on this net's own two backward products (widest layer): the chain's D W
        (B x N x N) and the gradient's D^T A (N x N x B, fp32 result), one after the other."""
        torch = self.torch
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        dt = torch.bfloat16 if spec.dtype == "bf16" else torch.float32
        n_ = spec.N
        d_ = torch.randn(spec.B, n_, device="cuda", dtype=dt)
        w_ = torch.randn(n_, n_, device="cuda", dtype=dt)
        x_ = torch.rand(spec.B, n_, device="cuda", dtype=dt)

        def both():
            d_ @ w_
            if dt == torch.float32:
                d_.t() @ x_
            else:
                torch.mm(d_.t(), x_, out_dtype=torch.float32)
        try:
            both()
            best = 1e9
            for _ in range(5):
                e0.record(); both(); e1.record(); torch.cuda.synchronize()
                best = min(best, e0.elapsed_time(e1))
            return {"value": 4.0 * spec.B * n_ * n_ / (best * 1e-3) / 1e12, "unit": "TFLOP/s",
                    "what": f"torch: (B x N)(N x N) then (N x B)(B x N) -> fp32, B={spec.B} N={n_} {spec.dtype}, "
                            "the two products of one backward layer without their epilogues, best of 5"}
        except Exception as ex:      # an older torch without out_dtype
            return {"value": None, "what": f"not measured: {str(ex)[:80]}"}


# ------------------------------------------------------------------------------------------ one configuration
def time_backward_only(torch, g, k, reps, warm=2):
    """Median and minimum time (ms) of the backward pass alone, HIP events on the launch stream around every
    one of `reps` passes (each after a forward pass of its own)."""
    for _ in range(warm):
        g.forward()
        g.backward(k)
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
    torch.cuda.synchronize()
    for e0, e1 in evs:
        g.forward()
        e0.record()
        g.backward(k)
        e1.record()
    torch.cuda.synchronize()
    ts = sorted(e0.elapsed_time(e1) for e0, e1 in evs)
    return ts[len(ts) // 2], ts[0]


def load_net(net, g, torch):
    """Draw the net's tensors on the host (layers side by side on a few threads: every tensor has a random
    stream of its own) and copy them to the device."""
    from concurrent.futures import ThreadPoolExecutor
    L = net.spec.L
    with ThreadPoolExecutor(max_workers=min(8, os.cpu_count() or 1)) as pool:
        for l, w in zip(range(2, L + 1), pool.map(net.w, range(2, L + 1))):
            g.w[l - 2].copy_(torch.from_numpy(w))
            g.b[l - 2].copy_(torch.from_numpy(net.b(l)))
            if g.master_w is not None:
                g.master_w[l - 2].copy_(torch.from_numpy(w))
    g.x.copy_(torch.from_numpy(net.x()))
    g.y.copy_(torch.from_numpy(net.y()))


def run_config(net, name, args, steps, warmup, rates, P, torch, extras=True):
    s = net.spec
    # small: a pass takes well under a millisecond, so an event record is a visible share of it
    small = name in ("cfg1", "cfg2") if name else 6.0 * s.B * sum(matrix_sizes(s)) < 2e9
    k = args.k or (max(s.ks) if name else min(8, s.L - 1))
    sched = args.sched
    g = P.LeapfrogNet(s.L, list(s.widths) if s.widths else s.N, s.B, s.dtype)
    fused_sgd = args.sgd > 0.0 and not args.sgd_unfused
    if fused_sgd:
        g.set_sgd(args.sgd)
    load_net(net, g, torch)
    g.set_schedule(getattr(P, "LF_SCHED_" + sched.upper()))
    torch.cuda.synchronize()
    masters = [t.float() for t in g.w] if (args.sgd > 0.0 and not fused_sgd and s.dtype == "bf16") else None

    def backward():
        g.backward(k)
        if args.sgd > 0.0 and not fused_sgd:  # the plain alternative: gradients through memory, then one update per tensor
            if masters is None:
                torch._foreach_add_(g.w, g.nabla_w, alpha=-args.sgd)
            else:                             # bf16 storage: fp32 masters stepped, the bf16 weights rewritten from them
                torch._foreach_add_(masters, g.nabla_w, alpha=-args.sgd)
                torch._foreach_copy_(g.w, masters)
            torch._foreach_add_(g.b, g.nabla_b, alpha=-args.sgd)

    for _ in range(warmup):
        g.forward()
        backward()
    torch.cuda.synchronize()

    # Timed region: exactly `steps` passes.  Events on the stream the passes are enqueued on (torch's current
    # stream, handed to the library) bracket the forward and the backward pass of every `every`-th step: an
    # event record costs a few microseconds of stream time, which is 7 % of a pass of the small nets, so only
    # a sample of the steps carries them there (at least 8; all steps of the large nets, where they cost nothing).
    every = max(1, min(args.event_every, steps // 8)) if small else 1
    marked = [i for i in range(steps) if i % every == every - 1] or [steps - 1]
    ev = {i: (torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True),
              torch.cuda.Event(enable_timing=True)) for i in marked}
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        e = ev.get(i)
        if e is None:
            g.forward()
            backward()
        else:
            e[0].record()
            g.forward()
            e[1].record()
            backward()
            e[2].record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    fwd_ms = sum(e[0].elapsed_time(e[1]) for e in ev.values()) / len(ev)
    bwd_ms = sum(e[1].elapsed_time(e[2]) for e in ev.values()) / len(ev)
    bwd_list = sorted(e[1].elapsed_time(e[2]) for e in ev.values())

    if args.calibrate_copy:
        src = torch.empty(1 << 28, dtype=torch.float32, device="cuda")
        src.fill_(1.0)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)          # reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del src, dst

    work = algorithmic_work(s, sgd=args.sgd > 0.0)
    achieved = work["bwd"] / (bwd_ms * 1e-3) / work["scale"]
    persistent = (s.B == 1 and s.dtype == "f32" and s.N <= 4096 and sched in ("auto", "persistent", "fused")
                  and not s.widths)
    kernel = "k_bwd_persistent (one launch = the whole backward pass)" if persistent else \
        "backward pass (bp1)-(bp4), all kernels"
    achievable = None
    if not args.no_achievable:
        achievable = dict(rates.hbm() if work["bound"] == "hbm" else rates.mfma(s.dtype))
        if work["bound"] == "mfma":
            achievable["same_shapes"] = rates.vendor_same_shapes(s)
    traffic = measured_traffic(s.name, k) if (persistent or (s.B > 1 and sched == "auto" and not s.widths
                                                            and args.sgd <= 0.0)) else None
    entry = {
        "config": name or s.name,
        "workload": f"{s.name}: sigmoid MLP L={s.L} N={s.N} B={s.B} {s.dtype}, k={k}, seed {s.seed}",
        "k": k, "schedule": sched, "weight_matrices": s.L - 1, "dtype": s.dtype,
        "descent_step": None if args.sgd <= 0.0 else
        {"eta": args.sgd, "how": "fused into the workers" if fused_sgd else "separate torch update after the pass"},
        "value": steps / wall, "unit": "passes/s", "steps": steps, "warmup": warmup,
        "ms_per_step": wall / steps * 1e3,
        "fwd_ms": fwd_ms, "bwd_ms": bwd_ms, "bwd_ms_median": bwd_list[len(bwd_list) // 2],
        "bwd_ms_min": bwd_list[0], "bwd_passes_per_s": 1e3 / bwd_ms, "steps_with_events": len(ev),
        "weights_cache_warm": bool(4 * sum(matrix_sizes(s)) * (1 if s.dtype == "f32" else 0.5) < 256e6),
        "roofline": {"bound": work["bound"], "kernel": kernel, "achieved": achieved,
                     "peak": work["peak"], "unit": work["unit"], "frac": achieved / work["peak"],
                     "traffic": traffic,
                     "traffic_source": "profiles/traffic.json: rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this "
                                       "kernel source, stored; not counters of this run" if traffic else None,
                     "algorithmic_per_launch": work["bwd"],
                     "fwd_achieved": work["fwd"] / (fwd_ms * 1e-3) / work["scale"],
                     "fwd_bwd_frac": (work["fwd"] + work["bwd"]) / ((fwd_ms + bwd_ms) * 1e-3) / work["scale"] / work["peak"],
                     "achievable": achievable,
                     "frac_of_achievable": None if achievable is None else achieved / achievable["value"]},
    }
    if work["bound"] == "hbm" and small:
        chain_steps = s.L - 2
        entry["latency_bound"] = {"dependent_chain_steps": chain_steps,
                                  "us_per_step": bwd_ms * 1e3 / max(1, chain_steps),
                                  "what": "backward time / dependent delta-chain steps: the weights sit in the 256 MB "
                                          "cache, so the pass is bound by the per-step exchange, not by HBM"}

    # The paper's cost model on this machine (section 4): f2 = the delta chain alone, T_bwd(1) = f2 + f3 in line,
    # T_bwd(k) with the gradients on k workers; "hidden" = T_bwd(k_max) <= 1.05 max(f2, work / measured rate).
    if extras and args.sgd <= 0.0 and sched in ("auto", "streams", "persistent"):
        reps = 40 if small else 8
        model = {"reps": reps}
        if k > 1:
            model["bwd_ms_k1"] = time_backward_only(torch, g, 1, reps)[0]
        model[f"bwd_ms_k{k}"] = time_backward_only(torch, g, k, reps)[0]
        for kk in (s.ks if name else ()):              # the configuration's other worker counts
            if f"bwd_ms_k{kk}" not in model:
                model[f"bwd_ms_k{kk}"] = time_backward_only(torch, g, kk, reps)[0]
        timed = {int(key[8:]): v for key, v in model.items() if key.startswith("bwd_ms_k")}
        best_k = min(timed, key=timed.get)
        model["fastest_configured_k"] = {"k": best_k, "bwd_ms": timed[best_k],
                                         "roofline_frac": work["bwd"] / (timed[best_k] * 1e-3) / work["scale"] / work["peak"]}
        # (beside the figures of the timed steps, which run the configuration's largest k)
        entry["roofline"]["fastest_configured_k"] = dict(model["fastest_configured_k"],
                                                         what="backward-only passes, mean of %d" % reps)
        g.set_debug_flags(P.LF_DEBUG_CHAIN_ONLY)
        model["chain_alone_ms"] = time_backward_only(torch, g, k, reps)[0]
        g.set_debug_flags(0)
        if persistent:
            g.set_schedule(P.LF_SCHED_FUSED)
            model["bwd_ms_fused_on_chain"] = time_backward_only(torch, g, 1, reps)[0]
            g.set_schedule(getattr(P, "LF_SCHED_" + sched.upper()))
        floor_ms = None
        if achievable is not None:
            if work["bound"] == "hbm":
                rate = (achievable.get("stream_read_and_write") or {}).get("value") or achievable["value"]
                floor_ms = work["bwd"] / (rate * 1e9) * 1e3
                model["floor_what"] = "backward bytes / measured rate of plain kernels reading and writing at once"
                same = (achievable.get("strips_read_beside_rows_written") or {}).get("value")
                if same and not small:
                    # the same bytes at the rate plain kernels with this pass's own access patterns reach side by side
                    model["floor_same_patterns_ms"] = work["bwd"] / (same * 1e9) * 1e3
                    model["frac_of_same_patterns_rate"] = achieved / same
            else:
                rate = (achievable.get("mfma_loop") or {}).get("value") or achievable["value"]
                floor_ms = work["bwd"] / (rate * 1e12) * 1e3
                model["floor_what"] = "backward flops / measured rate of a register-resident matrix-instruction loop"
            model["floor_ms"] = floor_ms
        bound = max(model["chain_alone_ms"], floor_ms or 0.0)
        model["hidden_bound_ms"] = 1.05 * bound
        model["gradients_hidden_behind_chain"] = bool(model[f"bwd_ms_k{k}"] <= 1.05 * bound) if k > 1 else None
        if "floor_same_patterns_ms" in model and k > 1:
            model["within_5_percent_of_same_patterns_floor"] = bool(
                model[f"bwd_ms_k{k}"] <= 1.05 * max(model["chain_alone_ms"], model["floor_same_patterns_ms"]))
        # restore the full pass's gradients for the parity leg
        g.forward()
        g.backward(k)
        torch.cuda.synchronize()
        entry["cost_model"] = model

    if not args.no_cpu_baseline:
        # (after descent steps the GPU's weights are no longer the oracle's: no parity figure then)
        entry["cpu_baseline"] = cpu_baseline(net, g if args.sgd <= 0.0 else None, budget_s=args.cpu_budget)
    g.close()
    del g
    torch.cuda.empty_cache()
    return entry


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", default="", choices=[""] + ALL_CONFIGS,
                    help="run this configuration alone (default: all five, configuration 5 as the headline)")
    ap.add_argument("--widths", default="",
                    help="instead of --config: neurons of layers 1..L, comma-separated (with --batch, --dtype)")
    ap.add_argument("--batch", type=int, default=1)
    ap.add_argument("--dtype", default="f32", choices=["f32", "bf16"])
    ap.add_argument("--sgd", type=float, default=0.0,
                    help="eta > 0: every backward pass applies the descent step")
    ap.add_argument("--sgd-unfused", action="store_true",
                    help="with --sgd: store the gradients and apply the step with a separate plain torch update, for comparison")
    ap.add_argument("--k", type=int, default=0, help="workers (0 = the configuration's largest k)")
    ap.add_argument("--sched", default="auto", choices=SCHED_NAMES,
                    help="redundant = Algorithm 1 as printed: every worker recomputes its own delta chain (B = 1, k <= 8); "
                         "fused = the on-chain fusion (B = 1, persistent kernel)")
    ap.add_argument("--event-every", type=int, default=8,
                    help="small nets: bracket every n-th timed step with HIP events (phase times, roofline)")
    ap.add_argument("--small-steps-factor", type=int, default=10,
                    help="all-configurations run: the two small nets time this many times --steps")
    ap.add_argument("--cpu-budget", type=float, default=6.0, help="seconds per oracle timing leg")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-achievable", action="store_true",
                    help="skip the measurement of the rate plain library kernels reach on this machine")
    ap.add_argument("--no-cost-model", action="store_true",
                    help="skip the chain-alone / k = 1 / on-chain-fusion timings")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 1 GiB device copy (for scaling rocprofv3 byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: the library runs on one GPU only; --gpus must be 1", file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_1801_04928_amd as P
    from lf_inputs import config_net, make_net

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    torch.cuda.set_device(0)
    rates = MachineRates(torch)
    entries = []
    if args.widths:
        widths = [int(v) for v in args.widths.split(",")]
        net = make_net(len(widths), widths, args.batch, dtype=args.dtype, seed=0, cache=True,
                       name="widths " + "-".join(str(v) for v in widths))
        entries.append(run_config(net, "", args, args.steps, args.warmup, rates, P, torch,
                                  extras=not args.no_cost_model))
    else:
        names = [args.config] if args.config else ALL_CONFIGS
        for name in names:
            net = config_net(name, cache=name in ("cfg1", "cfg2", "cfg3"))
            # the headline configuration times exactly --steps passes after exactly --warmup; in the run over all
            # five the two small nets, whose pass takes 0.03-0.2 ms, time more passes for a steadier figure
            factor = args.small_steps_factor if (not args.config and name in ("cfg1", "cfg2")) else 1
            t0 = time.perf_counter()
            entries.append(run_config(net, name, args, args.steps * factor, args.warmup, rates, P, torch,
                                      extras=not args.no_cost_model))
            entries[-1]["bench_wall_s"] = time.perf_counter() - t0
            print(f"bench.py: {name} done in {entries[-1]['bench_wall_s']:.1f} s", file=sys.stderr, flush=True)
            del net
    head = entries[-1]                 # the largest configuration that was run
    out = {
        "metric": "full backprop passes/sec at 1 GPU",
        "value": head["value"],
        "unit": "passes/s",
        "n_gpus": 1,
        "steps": head["steps"],
        "warmup": head["warmup"],
        "ms_per_step": head["ms_per_step"],
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": head["dtype"],
        "data": "synthetic",
        "config": {"workload": head["workload"], "k": head["k"], "schedule": head["schedule"],
                   "weight_matrices": head["weight_matrices"], "descent_step": head["descent_step"]},
    }
    for key in ("fwd_ms", "bwd_ms", "bwd_ms_median", "bwd_ms_min", "bwd_passes_per_s", "steps_with_events",
                "weights_cache_warm", "roofline", "latency_bound", "cost_model", "cpu_baseline"):
        if key in head:
            out[key] = head[key]
    if len(entries) > 1:
        out["per_config"] = entries
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
