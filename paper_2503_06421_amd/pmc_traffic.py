"""HBM traffic of the LoRA read-modify-write kernels from two rocprofv3 counter runs of bench.py.

    python -m paper_2503_06421_amd.pmc_traffic --fetch DIR --write DIR --key WORKLOAD --command "..." [--out profiles/hbm_traffic.json]

DIR are the output directories of

    rocprofv3 --pmc FETCH_SIZE --output-format csv -d DIR -o p -- python3 bench.py --only ... --kernel-level-only --cpu-seconds 0
    rocprofv3 --pmc WRITE_SIZE --output-format csv -d DIR -o p -- python3 bench.py --only ... --kernel-level-only --cpu-seconds 0

(each counter in a run of its own).  Both counters are reported in KiB per dispatch; what one KiB
of a counter stands for is calibrated on launches of known traffic in the same run: the stand-alone
conversions bench.py always makes (1 GiB of fp16 read, 1 GiB of bf16 written per launch).  The result
-- mean HBM bytes per launch over all launches of the LoRA kernels -- is stored under WORKLOAD in
the JSON file bench.py reads its `roofline.traffic` from.  Only this arithmetic on counter values
happens here; nothing touches the GPU.
"""
from __future__ import annotations

import argparse
import csv
import glob
import json
import os

CAL_BYTES = 1 << 30          # bench.py's stand-alone convert launches: this much read and this much written


def rows_of(d):
    files = glob.glob(os.path.join(d, "**", "*counter_collection.csv"), recursive=True)
    if not files:
        raise SystemExit("no counter_collection.csv under %s" % d)
    out = []
    for f in files:
        with open(f) as fh:
            out.extend(csv.DictReader(fh))
    return out


def per_kernel(rows, counter):
    """{kind: [value per dispatch]} for kind in ("lora", "cal")."""
    vals = {"lora": [], "cal": []}
    for r in rows:
        if r["Counter_Name"] != counter:
            continue
        k = r["Kernel_Name"]
        if "lora_mfma" in k or "lora_ordered" in k:
            vals["lora"].append(float(r["Counter_Value"]))
        elif "convert_segments_kernel" in k and int(r["Grid_Size"]) == (CAL_BYTES // 2 // 8):   # one lane per 8 elements
            vals["cal"].append(float(r["Counter_Value"]))
    return vals


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--fetch", required=True)
    ap.add_argument("--write", required=True)
    ap.add_argument("--key", required=True, help="workload name, e.g. llama3_70b_shaped")
    ap.add_argument("--command", required=True, help="the profiled command, recorded with the figures")
    ap.add_argument("--out", default=os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "profiles", "hbm_traffic.json"))
    a = ap.parse_args()
    f = per_kernel(rows_of(a.fetch), "FETCH_SIZE")
    w = per_kernel(rows_of(a.write), "WRITE_SIZE")
    if not f["cal"] or not w["cal"] or not f["lora"] or not w["lora"]:
        raise SystemExit("calibration or LoRA launches missing: %s / %s" % ({k: len(v) for k, v in f.items()}, {k: len(v) for k, v in w.items()}))
    if len(f["lora"]) != len(w["lora"]):
        raise SystemExit("the two runs differ in their number of LoRA launches: %d / %d" % (len(f["lora"]), len(w["lora"])))
    mean = lambda x: sum(x) / len(x)
    fetch_scale = CAL_BYTES / 1024.0 / mean(f["cal"])        # true KiB per counted KiB
    write_scale = CAL_BYTES / 1024.0 / mean(w["cal"])
    fetch_bytes = mean(f["lora"]) * 1024.0 * fetch_scale
    write_bytes = mean(w["lora"]) * 1024.0 * write_scale
    rec = {"kernel": "lora_mfma_kernel / lora_mfma_lds_kernel", "launches": len(f["lora"]),
           "hbm_bytes_per_launch": round(fetch_bytes + write_bytes), "fetch_bytes_per_launch": round(fetch_bytes),
           "write_bytes_per_launch": round(write_bytes), "fetch_scale": round(fetch_scale, 4), "write_scale": round(write_scale, 4),
           "calibration": "%d stand-alone convert launches of 1 GiB in + 1 GiB out in the same runs" % len(f["cal"]),
           "command": a.command}
    try:
        with open(a.out) as fh:
            data = json.load(fh)
    except (OSError, ValueError):
        data = {}
    data[a.key] = rec
    with open(a.out, "w") as fh:
        json.dump(data, fh, indent=1, sort_keys=True)
        fh.write("\n")
    print(json.dumps({a.key: rec}))


if __name__ == "__main__":
    main()
