"""Benchmark: full backpropagation passes per second on one MI355X.

A step is one pass of the whole hot path -- forward (x),(z),(a), then the leapfrogged backward pass
(bp1)-(bp4) with k workers -- over one seeded synthetic input that is already resident in HBM.
Prints ONE JSON line.  The roofline object prices the backward pass against the HBM peak (B = 1) or
the MFMA peak (minibatch); the cpu_baseline object is the CPU oracle timed on this machine's cores.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
MFMA_PEAK_TFLOPS = {"f32": 157.3, "bf16": 2500.0}


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
        return {"bound": "hbm", "bwd": es * chain + (8 if sgd else 4) * every,
                "fwd": es * every, "unit": "GB/s", "peak": HBM_PEAK_GBS, "scale": 1e9}
    f = 2.0 * spec.B
    return {"bound": "mfma", "bwd": f * (chain + every), "fwd": f * every, "unit": "TFLOP/s",
            "peak": MFMA_PEAK_TFLOPS[spec.dtype], "scale": 1e12}


def measured_traffic(cfg_name, k):
    """HBM bytes per launch of the backward kernel from the committed rocprofv3 counter runs
    (profiles/traffic.json), or None when the kernel source has changed since they were taken."""
    import hashlib
    path = os.path.join(ROOT, "profiles", "traffic.json")
    try:
        rec = json.load(open(path))
        h = hashlib.sha256()
        for name in ("persistent_kernels.hip", "persistent.h", "device_helpers.h"):
            h.update(open(os.path.join(ROOT, "paper_1801_04928_amd", "csrc", name), "rb").read())
        if rec.get("kernel_source_sha256") != h.hexdigest():
            return None
        e = rec.get(f"{cfg_name}_k{k}")
        return None if e is None else e["fetch_bytes"] + e["write_bytes"]
    except Exception:
        return None


def cpu_baseline(net, gpu_net=None, budget_s=12.0):
    """The oracle as it stands, timed on the host: whole passes for the small nets; for nets whose
    pass takes minutes, two full layers (forward + chain + gradient) scaled to the whole net.
    Where a whole oracle pass is run, the gradients still in the GPU's buffers from the timed passes
    are compared with it (normwise error per tensor, worst over the layers)."""
    import numpy as np
    from oracle import backprop as O
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count() or 1
    s = net.spec
    M = s.L - 1
    flops_pass = 6.0 * s.B * sum(matrix_sizes(s))
    if flops_pass < 5e10 or s.widths:
        w = {l: net.w(l) for l in range(2, s.L + 1)}
        b = {l: net.b(l) for l in range(2, s.L + 1)}
        x, y = net.x(), net.y()
        ref = O.full_pass(w, b, x, y, s.L)
        n, t0 = 0, time.perf_counter()
        while True:
            O.full_pass(w, b, x, y, s.L)
            n += 1
            dt = time.perf_counter() - t0
            if dt > budget_s or n >= 200:
                break
        out = {"value": n / dt, "unit": "passes/s", "cores": cores, "kind": "oracle",
               "sample": f"{n} full forward+backward passes of the same net"}
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
    # two layers at full width, scaled by M / 2
    sub_L = 3
    w = {l: net.w(l) for l in (2, 3)}
    b = {l: net.b(l) for l in (2, 3)}
    x, y = net.x(), net.y()
    t0 = time.perf_counter()
    O.full_pass(w, b, x, y, sub_L)
    dt = time.perf_counter() - t0
    return {"value": 1.0 / (dt * M / 2.0), "unit": "passes/s", "cores": cores, "kind": "oracle",
            "sample": f"extrapolated from 2 of {M} layers at full N, B (one pass of a 3-layer net, x{M / 2:.1f})"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", default="cfg2", choices=["cfg1", "cfg2", "cfg3", "cfg4", "cfg5"])
    ap.add_argument("--widths", default="",
                    help="instead of --config: neurons of layers 1..L, comma-separated (with --batch, --dtype)")
    ap.add_argument("--batch", type=int, default=1)
    ap.add_argument("--dtype", default="f32", choices=["f32", "bf16"])
    ap.add_argument("--sgd", type=float, default=0.0,
                    help="eta > 0: every backward pass applies the descent step (fp32 nets, stream schedule)")
    ap.add_argument("--sgd-unfused", action="store_true",
                    help="with --sgd: store the gradients and apply the step with a separate plain torch update, for comparison")
    ap.add_argument("--k", type=int, default=0, help="workers (0 = the configuration's largest k)")
    ap.add_argument("--sched", default="auto", choices=["auto", "streams", "persistent", "redundant"],
                    help="redundant = Algorithm 1 as printed: every worker recomputes its own delta chain (B = 1, k <= 8)")
    ap.add_argument("--event-every", type=int, default=8,
                    help="small nets: bracket every n-th timed step with HIP events (phase times, roofline)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-achievable", action="store_true",
                    help="skip the measurement of the rate plain library kernels reach on this machine")
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
    if args.widths:
        widths = [int(v) for v in args.widths.split(",")]
        net = make_net(len(widths), widths, args.batch, dtype=args.dtype, seed=0, cache=True,
                       name="widths " + "-".join(str(v) for v in widths))
        s = net.spec
        k = args.k or min(8, s.L - 1)
        small = 6.0 * s.B * sum(matrix_sizes(s)) < 1e10
    else:
        net = config_net(args.config, cache=args.config in ("cfg1", "cfg2"))
        s = net.spec
        k = args.k or max(s.ks)
        small = args.config in ("cfg1", "cfg2")
    steps = args.steps if small else min(args.steps, 20)
    warmup = args.warmup if small else min(args.warmup, 3)

    g = P.LeapfrogNet(s.L, list(s.widths) if s.widths else s.N, s.B, s.dtype)
    g.load(net)
    g.set_schedule({"auto": P.LF_SCHED_AUTO, "streams": P.LF_SCHED_STREAMS,
                    "persistent": P.LF_SCHED_PERSISTENT, "redundant": P.LF_SCHED_REDUNDANT}[args.sched])
    fused = args.sgd > 0.0 and not args.sgd_unfused
    if fused:
        g.set_sgd(args.sgd)
    torch.cuda.synchronize()

    masters = [t.float() for t in g.w] if (args.sgd > 0.0 and not fused and s.dtype == "bf16") else None

    def backward():
        g.backward(k)
        if args.sgd > 0.0 and not fused:      # the plain alternative: gradients through memory, then one update per tensor
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
    # a sample of the steps carries them (all steps of the large nets, where they cost nothing).
    every = max(1, args.event_every) if small else 1
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
    t1 = time.perf_counter()
    wall = t1 - t0
    fwd_ms = sum(e[0].elapsed_time(e[1]) for e in ev.values()) / len(ev)
    bwd_ms = sum(e[1].elapsed_time(e[2]) for e in ev.values()) / len(ev)

    if args.calibrate_copy:
        src = torch.empty(1 << 28, dtype=torch.float32, device="cuda")
        src.fill_(1.0)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)          # reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()

    work = algorithmic_work(s, sgd=args.sgd > 0.0)
    achieved = work["bwd"] / (bwd_ms * 1e-3) / work["scale"]
    bwd_list = sorted(e[1].elapsed_time(e[2]) for e in ev.values())

    # What plain library kernels reach on this machine, for scale (outside the timed region): a 1 GiB
    # device copy for the HBM-bound nets, an 8192^3 torch.matmul in the net's type for the MFMA-bound ones.
    achievable = None
    if not args.no_achievable:
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        if work["bound"] == "hbm":
            src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")
            dst = torch.empty_like(src)
            best = 1e9
            for _ in range(5):
                e0.record(); dst.copy_(src); e1.record(); torch.cuda.synchronize()
                best = min(best, e0.elapsed_time(e1))
            achievable = {"value": 2.0 * src.numel() * 4 / (best * 1e-3) / 1e9, "unit": "GB/s",
                          "what": "1 GiB device copy (torch), bytes read + written, best of 5"}
            # plain streaming kernels of this repository (csrc/peak_probe.hip): read only, write only, both at once
            try:
                import ctypes
                probe = ctypes.CDLL(os.path.join(ROOT, "paper_1801_04928_amd", "libprobe.so"))
                probe.probe_stream.restype = ctypes.c_double
                probe.probe_stream.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p,
                                               ctypes.c_size_t, ctypes.c_void_p, ctypes.c_void_p]
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
                    achievable["stream_" + name] = {
                        "value": moved / (best * 1e-3) / 1e9 if moved > 0 else None, "unit": "GB/s",
                        "what": "plain 128-bit streaming kernel over 1 GiB per buffer, best launch shape of 5, best of 3"}
            except OSError as ex:
                achievable["stream_read"] = {"value": None, "what": f"not measured: {str(ex)[:80]}"}
            del src, dst
        else:
            dt = torch.bfloat16 if s.dtype == "bf16" else torch.float32
            a_ = torch.randn(8192, 8192, device="cuda", dtype=dt)
            b_ = torch.randn(8192, 8192, device="cuda", dtype=dt)
            c_ = a_ @ b_
            best = 1e9
            for _ in range(5):
                e0.record(); c_ = a_ @ b_; e1.record(); torch.cuda.synchronize()
                best = min(best, e0.elapsed_time(e1))
            achievable = {"value": 2.0 * 8192 ** 3 / (best * 1e-3) / 1e12, "unit": "TFLOP/s",
                          "what": f"torch.matmul 8192^3 {s.dtype} (vendor library), best of 5"}
            del a_, b_, c_
            # the vendor library on this net's own two backward products (widest layer): the chain's
            # D W (B x N x N) and the gradient's D^T A (N x N x B, fp32 result), one after the other
            n_ = s.N
            d_ = torch.randn(s.B, n_, device="cuda", dtype=dt)
            w_ = torch.randn(n_, n_, device="cuda", dtype=dt)
            x_ = torch.rand(s.B, n_, device="cuda", dtype=dt)

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
                achievable["same_shapes"] = {
                    "value": 4.0 * s.B * n_ * n_ / (best * 1e-3) / 1e12, "unit": "TFLOP/s",
                    "what": f"torch: (B x N)(N x N) then (N x B)(B x N) -> fp32, B={s.B} N={n_} {s.dtype}, "
                            "the two products of one backward layer without their epilogues, best of 5"}
            except Exception as ex:      # an older torch without out_dtype
                achievable["same_shapes"] = {"value": None, "what": f"not measured: {str(ex)[:80]}"}
            del d_, w_, x_
            # and what the matrix cores sustain when nothing else limits them: a loop of matrix instructions
            # that never leaves the registers, two waves per SIMD on every compute unit
            try:
                import ctypes
                probe = ctypes.CDLL(os.path.join(ROOT, "paper_1801_04928_amd", "libprobe.so"))
                probe.probe_mfma_loop.restype = ctypes.c_double
                probe.probe_mfma_loop.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_void_p,
                                                  ctypes.c_void_p]
                sink = torch.zeros(1, device="cuda")
                cus = torch.cuda.get_device_properties(0).multi_processor_count
                stream = torch.cuda.current_stream().cuda_stream
                is_bf = 1 if s.dtype == "bf16" else 0
                probe.probe_mfma_loop(is_bf, 2 * cus, 2000, sink.data_ptr(), stream)
                torch.cuda.synchronize()
                best, flops = 1e9, 0.0
                for _ in range(3):
                    e0.record()
                    flops = probe.probe_mfma_loop(is_bf, 2 * cus, 10000, sink.data_ptr(), stream)
                    e1.record()
                    torch.cuda.synchronize()
                    best = min(best, e0.elapsed_time(e1))
                achievable["mfma_loop"] = {
                    "value": flops / (best * 1e-3) / 1e12 if flops > 0 else None, "unit": "TFLOP/s",
                    "what": f"register-resident loop of 32x32 {s.dtype} matrix instructions on {cus} compute units, best of 3"}
            except OSError as ex:
                achievable["mfma_loop"] = {"value": None, "what": f"not measured: {str(ex)[:80]}"}
    persistent = (s.B == 1 and s.dtype == "f32" and s.N <= 4096 and args.sched in ("auto", "persistent")
                  and not s.widths)
    kernel = "k_bwd_persistent (one launch = the whole backward pass)" if persistent else \
        "backward pass (bp1)-(bp4), all kernels"
    out = {
        "metric": "full backprop passes/sec at 1 GPU",
        "value": steps / wall,
        "unit": "passes/s",
        "n_gpus": 1,
        "steps": steps,
        "warmup": warmup,
        "ms_per_step": wall / steps * 1e3,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": s.dtype,
        "data": "synthetic",
        "config": {"workload": f"{s.name}: sigmoid MLP L={s.L} N={s.N} B={s.B} {s.dtype}, k={k}, seed {s.seed}",
                   "k": k, "schedule": args.sched, "weight_matrices": s.L - 1,
                   "descent_step": None if args.sgd <= 0.0 else
                   {"eta": args.sgd, "how": "fused into the workers" if fused else "separate torch update after the pass"}},
        "fwd_ms": fwd_ms,
        "bwd_ms": bwd_ms,
        "bwd_ms_median": bwd_list[len(bwd_list) // 2],
        "bwd_ms_min": bwd_list[0],
        "bwd_passes_per_s": 1e3 / bwd_ms,
        "steps_with_events": len(ev),
        "weights_cache_warm": bool(4 * sum(matrix_sizes(s)) * (1 if s.dtype == "f32" else 0.5) < 256e6),
        "roofline": {"bound": work["bound"], "kernel": kernel, "achieved": achieved,
                     "peak": work["peak"], "unit": work["unit"], "frac": achieved / work["peak"],
                     "traffic": measured_traffic(s.name, k) if persistent else None,
                     "algorithmic_per_launch": work["bwd"],
                     "fwd_achieved": work["fwd"] / (fwd_ms * 1e-3) / work["scale"],
                     "fwd_bwd_frac": (work["fwd"] + work["bwd"]) / ((fwd_ms + bwd_ms) * 1e-3) / work["scale"] / work["peak"],
                     "achievable": achievable,
                     "frac_of_achievable": None if achievable is None else achieved / achievable["value"]},
    }
    if not args.no_cpu_baseline:
        # (after descent steps the GPU's weights are no longer the oracle's: no parity figure then)
        out["cpu_baseline"] = cpu_baseline(net, g if args.sgd <= 0.0 else None)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
