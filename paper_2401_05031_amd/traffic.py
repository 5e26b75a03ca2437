"""Turns two rocprofv3 --pmc runs of bench.py (FETCH_SIZE, then WRITE_SIZE; both with --calibrate)
into per-launch HBM traffic per kernel family, scaled by what the same counters read for the
256 MiB device copy that --calibrate adds, and stores the figures bench.py reports as `traffic`.

    python -m paper_2401_05031_amd.traffic FETCH.csv WRITE.csv WORKLOAD [out.json]
"""
from __future__ import annotations

import csv
import json
import os
import sys
from collections import defaultdict

CAL_BYTES = 256 << 20
FAMILIES = {
    "gemm": ("gemm_mfma", "gemm_valu"),
    "attention": ("attention_",),
    "merge_apply": ("merge_apply_ln_kernel", "merge_apply_kernel"),
    "splitk_reduce_ln": ("splitk_reduce_ln_kernel",),
    "merge_plan": ("merge_plan_kernel",),
    "layer_norm": ("layer_norm_kernel",),
}
DEFAULT_OUT = os.path.join(os.path.dirname(os.path.abspath(__file__)), "hbm_traffic.json")


def _load(path: str, counter: str):
    per = defaultdict(lambda: [0, 0.0])
    cal = 0.0
    for r in csv.DictReader(open(path)):
        if r["Counter_Name"] != counter:
            continue
        name, val = r["Kernel_Name"], float(r["Counter_Value"])
        if "copyBuffer" in name:
            cal = max(cal, val)                      # the 256 MiB copy is by far the largest copy
        for fam, keys in FAMILIES.items():
            if any(k in name for k in keys):
                per[fam][0] += 1
                per[fam][1] += val
    return per, cal


def main(argv):
    fetch_csv, write_csv, workload = argv[1], argv[2], argv[3]
    out = argv[4] if len(argv) > 4 else DEFAULT_OUT
    f, fcal = _load(fetch_csv, "FETCH_SIZE")
    w, wcal = _load(write_csv, "WRITE_SIZE")
    fscale = CAL_BYTES / (fcal * 1024.0)             # counters are in KiB per dispatch
    wscale = CAL_BYTES / (wcal * 1024.0)
    res = {"workload": workload, "unit": "bytes per launch (fetch + write), averaged over the launches of one forward",
           "fetch_scale": round(fscale, 4), "write_scale": round(wscale, 4),
           "source": "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE over `bench.py --steps 2 --warmup 1 --no-cpu --no-clock --others '' "
                     "--calibrate`, each scaled by the counter's reading for the 256 MiB device copy in the same run",
           "families": {}}
    for fam in FAMILIES:
        if f[fam][0] == 0:
            continue
        fb = f[fam][1] / f[fam][0] * 1024.0 * fscale
        wb = w[fam][1] / max(w[fam][0], 1) * 1024.0 * wscale
        res["families"][fam] = {"launches": f[fam][0], "fetch_bytes": round(fb), "write_bytes": round(wb),
                                "bytes": round(fb + wb)}
    json.dump(res, open(out, "w"), indent=1)
    print(json.dumps(res, indent=1))


if __name__ == "__main__":
    main(sys.argv)
