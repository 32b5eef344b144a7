"""Writes profiles/traffic.json, the stored HBM-traffic figures that bench.py quotes as `roofline.traffic`,
from two rocprofv3 counter runs per configuration:

    rocprofv3 --pmc FETCH_SIZE --output-format csv -d <dir>/FETCH_SIZE_<cfg> -o p -- python3 bench.py --config <cfg> \
        --steps 20 --warmup 5 --no-cpu-baseline --no-achievable --no-cost-model --calibrate-copy
    (and the same with WRITE_SIZE)

usage: python bench_traffic_record.py <dir>        (cfg2 .. cfg5, k = their largest; cfg4 and cfg5 with
                                                     --steps 2 --warmup 1)

Both counters are in KiB per dispatch; each is scaled by what the same counter reads for the plain 1 GiB device
copy that --calibrate-copy adds to the run.  cfg2, cfg3: one launch is the whole backward pass.  cfg4, cfg5: the
backward pass is many launches; the record adds up, per pass, the kernels of the backward pass (the output
error, the chain products and their split finishes, the gradient products, the bias sums).  Every entry carries a
hash of the sources of its kernels, and bench.py reports the figures only while that hash matches."""
import collections
import csv
import hashlib
import json
import os
import re
import sys

ROOT = os.path.dirname(os.path.abspath(__file__))


def counter(path, name):
    d = collections.defaultdict(list)
    for r in csv.DictReader(open(path)):
        if r["Counter_Name"] == name:
            d[r["Kernel_Name"]].append(float(r["Counter_Value"]))
    return d


PERSISTENT_SOURCES = ("persistent_kernels.hip", "persistent.h", "persistent_partition.h", "device_helpers.h")
MINIBATCH_SOURCES = ("batched_kernels.hip", "b1_kernels.hip", "lf_internal.h", "device_helpers.h")


def source_hash(names):
    h = hashlib.sha256()
    for name in names:
        h.update(open(os.path.join(ROOT, "paper_1801_04928_amd", "csrc", name), "rb").read())
    return h.hexdigest()


def backward_part(kernel_name):
    """Which part of the minibatch backward pass a kernel is (None: a forward kernel, or not ours)."""
    if "k_output_error" in kernel_name:
        return "output error (bp1)"
    if "k_bias_grad" in kernel_name:
        return "bias sums (bp3)"
    if "k_grad_stream" in kernel_name:
        return "gradient product (bp4)"
    if "k_split_finish" in kernel_name:        # the chain's instance has epilogue 2 (sigma'), the forward's 1
        return "chain split finish (bp2)" if re.search(r"Li2E|, 2>|,2>", kernel_name) else None
    m = re.search(r"k_gemm\w*(<|I)", kernel_name)
    if m:
        demangled = re.search(r"<(?:float, |__bf16, )?(true|false), (true|false)", kernel_name)
        mangled = re.search(r"k_gemm\w*I(?:f|DF16b)?Lb([01])ELb([01])E", kernel_name)
        if demangled:
            p_ic, q_ic = demangled.group(1) == "true", demangled.group(2) == "true"
        elif mangled:
            p_ic, q_ic = mangled.group(1) == "1", mangled.group(2) == "1"
        else:
            return None
        if p_ic and q_ic:
            return "gradient product (bp4)"
        if q_ic:
            return "chain product (bp2)"
    return None


def minibatch_pass(src, cfg):
    f = counter(os.path.join(src, f"FETCH_SIZE_{cfg}", "p_counter_collection.csv"), "FETCH_SIZE")
    w = counter(os.path.join(src, f"WRITE_SIZE_{cfg}", "p_counter_collection.csv"), "WRITE_SIZE")
    cal_f = max(v for kk, vv in f.items() if "copyBuffer" in kk for v in vv)
    cal_w = max(v for kk, vv in w.items() if "copyBuffer" in kk for v in vv)
    fs, ws = round(1048576.0 / cal_f, 3), round(1048576.0 / cal_w, 3)
    passes = sum(len(v) for kk, v in f.items() if "k_output_error" in kk)
    parts = collections.OrderedDict()
    for kk in f:
        part = backward_part(kk)
        if part is None:
            continue
        e = parts.setdefault(part, {"dispatches_per_pass": 0.0, "fetch_bytes": 0, "write_bytes": 0})
        e["dispatches_per_pass"] += len(f[kk]) / passes
        e["fetch_bytes"] += int(sum(f[kk]) * 1024 * fs / passes)
        e["write_bytes"] += int(sum(w[kk]) * 1024 * ws / passes)
    return {"kernel": "backward pass, all kernels", "passes_in_run": passes, "fetch_scale": fs, "write_scale": ws,
            "parts": parts, "fetch_bytes": sum(e["fetch_bytes"] for e in parts.values()),
            "write_bytes": sum(e["write_bytes"] for e in parts.values()),
            "source_sha256": source_hash(MINIBATCH_SOURCES), "sources": list(MINIBATCH_SOURCES),
            "copy_fetch_kib_raw": cal_f, "copy_write_kib_raw": cal_w}


def main(src):
    rec = {"kernel_source_sha256": source_hash(PERSISTENT_SOURCES),
           "note": "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (KiB per dispatch, mean over the dispatches of one bench.py "
                   "run), each scaled by the factor the same counter shows for a plain 1 GiB device copy in the same "
                   "run.  The top-level hash covers persistent_kernels.hip, persistent.h and device_helpers.h (cfg2, cfg3); "
                   "the minibatch entries carry the hash of their own sources."}
    for cfg, k in (("cfg2", 8), ("cfg3", 8)):
        f = counter(os.path.join(src, f"FETCH_SIZE_{cfg}", "p_counter_collection.csv"), "FETCH_SIZE")
        w = counter(os.path.join(src, f"WRITE_SIZE_{cfg}", "p_counter_collection.csv"), "WRITE_SIZE")
        cal_f = max(v for kk, vv in f.items() if "copyBuffer" in kk for v in vv)
        cal_w = max(v for kk, vv in w.items() if "copyBuffer" in kk for v in vv)
        fs, ws = round(1048576.0 / cal_f, 3), round(1048576.0 / cal_w, 3)
        e = {}
        for kk in f:
            m = re.search(r"k_(bwd|fwd)_persistent<[^>]*>", kk)
            if not m:
                continue
            fr, wr = sum(f[kk]) / len(f[kk]), sum(w[kk]) / len(w[kk])
            e[m.group(1)] = {"kernel": m.group(0), "dispatches": len(f[kk]), "fetch_kib_raw": round(fr, 1),
                             "fetch_scale": fs, "write_kib_raw": round(wr, 1), "write_scale": ws,
                             "fetch_bytes": int(fr * 1024 * fs), "write_bytes": int(wr * 1024 * ws)}
        rec[f"{cfg}_k{k}"] = dict(e["bwd"], forward=e["fwd"], copy_fetch_kib_raw=cal_f, copy_write_kib_raw=cal_w)
    for cfg, k in (("cfg4", 4), ("cfg5", 8)):
        if os.path.exists(os.path.join(src, f"FETCH_SIZE_{cfg}", "p_counter_collection.csv")):
            rec[f"{cfg}_k{k}"] = minibatch_pass(src, cfg)
    json.dump(rec, open(os.path.join(ROOT, "profiles", "traffic.json"), "w"), indent=1)
    print(json.dumps(rec, indent=1))


if __name__ == "__main__":
    main(sys.argv[1])
