"""Writes profiles/traffic.json, the stored HBM-traffic figures that bench.py quotes as `roofline.traffic`,
from two rocprofv3 counter runs per configuration:

    rocprofv3 --pmc FETCH_SIZE --output-format csv -d <dir>/FETCH_SIZE_<cfg> -o p -- python3 bench.py --config <cfg> \
        --steps 20 --warmup 5 --no-cpu-baseline --no-achievable --no-cost-model --calibrate-copy
    (and the same with WRITE_SIZE)

usage: python bench_traffic_record.py <dir>        (configurations cfg2 and cfg3, k = their largest)

Both counters are in KiB per dispatch; each is scaled by what the same counter reads for the plain 1 GiB device
copy that --calibrate-copy adds to the run.  The record carries a hash of the persistent kernels' sources, and
bench.py reports the figures only while that hash matches."""
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


def main(src):
    h = hashlib.sha256()
    for name in ("persistent_kernels.hip", "persistent.h", "device_helpers.h"):
        h.update(open(os.path.join(ROOT, "paper_1801_04928_amd", "csrc", name), "rb").read())
    rec = {"kernel_source_sha256": h.hexdigest(),
           "note": "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (KiB per dispatch, mean over the dispatches of one bench.py "
                   "run), each scaled by the factor the same counter shows for a plain 1 GiB device copy in the same "
                   "run.  The hash covers persistent_kernels.hip, persistent.h and device_helpers.h."}
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
    json.dump(rec, open(os.path.join(ROOT, "profiles", "traffic.json"), "w"), indent=1)
    print(json.dumps(rec, indent=1))


if __name__ == "__main__":
    main(sys.argv[1])
