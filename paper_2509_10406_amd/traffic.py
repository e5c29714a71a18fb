"""HBM traffic per kernel launch from two rocprofv3 counter runs of bench.py.

    rocprofv3 --pmc FETCH_SIZE --kernel-trace --output-format csv -d DIR_F -o f -- python3 bench.py ...
    rocprofv3 --pmc WRITE_SIZE --kernel-trace --output-format csv -d DIR_W -o w -- python3 bench.py ...
    python -m paper_2509_10406_amd.traffic DIR_F/f_counter_collection.csv DIR_W/w_counter_collection.csv \
        --workload cfg3 --out profiles/hbm_traffic_cfg3.json

Both counters are in KiB per dispatch.  Each is scaled by what it reads for a plain copy kernel of known
size in the same run: bench.py casts the bf16 output O to fp32 once (B*Hq*N*D elements: 2 bytes read and
4 bytes written per element), a streaming elementwise kernel of torch's.
"""
from __future__ import annotations

import argparse
import collections
import csv
import json
import re

from .inputs import CONFIGS

_NAME = re.compile(r"\b(k_[a-z0-9_]+)")


def _load(path: str, counter: str):
    agg = collections.defaultdict(lambda: [0, 0.0])
    for row in csv.DictReader(open(path)):
        if row["Counter_Name"] != counter:
            continue
        full = row["Kernel_Name"]
        if "bfloat16tofloat32" in full.replace("_", "").lower() or ("BFloat16" in full and "float" in full and "copy" in full.lower()):
            name = "calibration_copy"
        else:
            m = _NAME.search(full)
            name = m.group(1) if m else full[:40]
        agg[name][0] += 1
        agg[name][1] += float(row["Counter_Value"]) * 1024.0
    return agg


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("fetch_csv")
    ap.add_argument("write_csv")
    ap.add_argument("--workload", default="cfg3")
    ap.add_argument("--out", required=True)
    a = ap.parse_args()
    w = CONFIGS[a.workload]
    elems = w.B * w.Hq * w.N * w.D
    f, wr = _load(a.fetch_csv, "FETCH_SIZE"), _load(a.write_csv, "WRITE_SIZE")
    if "calibration_copy" not in f or "calibration_copy" not in wr:
        raise SystemExit("the bf16 -> fp32 cast of O was not found in the counter files")
    kf = 2.0 * elems / (f["calibration_copy"][1] / f["calibration_copy"][0])
    kw = 4.0 * elems / (wr["calibration_copy"][1] / wr["calibration_copy"][0])
    flags = "" if a.workload == "cfg3" else f" --workload {a.workload}"
    out = {"workload": a.workload, "unit": "bytes per launch",
           "commands": [
               "rocprofv3 --pmc FETCH_SIZE --kernel-trace --output-format csv -d DIR_F -o f -- python3 bench.py"
               f"{flags} --steps 1 --warmup 0 --no-cpu-baseline --no-variants --serial-streams",
               "rocprofv3 --pmc WRITE_SIZE --kernel-trace --output-format csv -d DIR_W -o w -- python3 bench.py"
               f"{flags} --steps 1 --warmup 0 --no-cpu-baseline --no-variants --serial-streams",
               f"python -m paper_2509_10406_amd.traffic DIR_F/f_counter_collection.csv DIR_W/w_counter_collection.csv"
               f" --workload {a.workload} --out profiles/hbm_traffic_{a.workload}.json"],
           "calibration": {"kernel": "torch bf16 -> fp32 cast of O", "elements": elems,
                           "fetch_factor": kf, "write_factor": kw},
           "kernels": {}}
    for k in sorted(f):
        if not k.startswith("k_"):
            continue
        out["kernels"][k] = {"launches": f[k][0],
                             "fetch_bytes": kf * f[k][1] / f[k][0],
                             "write_bytes": kw * wr[k][1] / wr[k][0] if k in wr else 0.0}
    with open(a.out, "w") as fh:
        json.dump(out, fh, indent=1)
    print(f"fetch factor {kf:.3f}, write factor {kw:.3f}; {len(out['kernels'])} kernels -> {a.out}")


if __name__ == "__main__":
    main()
