"""Per-kernel summary of rocprofv3 SQ counter runs of bench.py (matrix-core, vector-unit and LDS activity).

    rocprofv3 --pmc SQ_BUSY_CU_CYCLES SQ_WAVE_CYCLES SQ_VALU_MFMA_BUSY_CYCLES SQ_INSTS_MFMA SQ_INSTS_VALU \
              SQ_INSTS_LDS SQ_ACTIVE_INST_VALU SQ_ACTIVE_INST_LDS --kernel-include-regex 'k_flash|k_assign' \
              --kernel-trace --output-format csv -d DIR_A -o a -- python3 bench.py --steps 1 --warmup 0 \
              --no-cpu-baseline --no-variants --serial-streams
    rocprofv3 --pmc SQ_WAIT_ANY SQ_WAIT_INST_ANY SQ_WAIT_INST_LDS SQ_ACTIVE_INST_ANY SQ_INSTS_VALU_TRANS_F32 \
              SQ_INSTS_VALU_CVT SQ_LDS_BANK_CONFLICT SQ_BUSY_CYCLES (same options) -d DIR_B -o b -- python3 bench.py ...
    python -m paper_2509_10406_amd.counters DIR_A/a_counter_collection.csv DIR_B/b_counter_collection.csv \
        --out profiles/mfma_counters_cfg3.txt

One hardware pass holds at most 8 SQ counters, hence two runs.  bench.py launches the flash kernels twice over:
for MuSe's block diagonal (block = N / 8: the short launches) and for the in-house exact attention (block = N: the
long launches); the assignment kernel (k_assign_res, or k_assign_bf16 for the largest C x D) runs for the query side (Cq centroids: short) and the key side (Ck centroids: long).
The launches of one kernel are split into these two classes by their duration.

Derived columns (per launch averages):
  mfma_busy   SQ_VALU_MFMA_BUSY_CYCLES / (4 SQ_BUSY_CU_CYCLES): share of the busy cycles of a CU's four SIMDs in which
              the matrix pipe works (an MFMA 32x32x16 bf16 holds it 32 cycles; 100 % would be the bf16 peak at the
              clock the kernel ran at)
  valu/mfma   vector instructions other than MFMA per MFMA instruction
  trans/mfma  transcendental (exp) instructions per MFMA;  cvt/mfma  conversions per MFMA
  lds/mfma    LDS instructions per MFMA
  w_lds, w_any   wave cycles waiting for LDS / for anything, over all wave cycles
  bank_cf     LDS bank-conflict cycles over LDS-active cycles

With --mode vector the same two-run scheme summarises the kernels that are NOT contractions (far-field streaming,
per-query and per-chain kernels), from
    run A: SQ_BUSY_CU_CYCLES SQ_WAVE_CYCLES SQ_VALU_MFMA_BUSY_CYCLES SQ_INSTS_MFMA SQ_INSTS_VALU SQ_INSTS_LDS
           SQ_ACTIVE_INST_VALU SQ_INSTS_VMEM_WR
    run B: SQ_WAIT_ANY SQ_WAIT_INST_ANY SQ_WAIT_INST_LDS SQ_ACTIVE_INST_ANY SQ_INSTS_VMEM_RD SQ_INSTS_SALU
           SQ_ACTIVE_INST_VMEM SQ_WAVES
    (--kernel-include-regex 'k_summaries|k_farfield_fwd|k_block_summaries|k_comp2|k_chain_grads|k_cell_grads|k_cells_to_keys_mx|k_ff_bwd|k_hit_lists|k_merge_ret|k_ret_|k_c3_pairs|k_update')
    python -m paper_2509_10406_amd.counters DIR_A/a_counter_collection.csv DIR_B/b_counter_collection.csv \
        --mode vector --out profiles/vector_counters_cfg3.txt
Columns of that mode (per launch averages):
  waves        wavefronts of the launch;  valu/wave, lds/wave, rd/wave, wr/wave, mfma/wave  instructions per wavefront
  valu_busy    SQ_ACTIVE_INST_VALU / SQ_BUSY_CU_CYCLES: share of the busy cycles in which a SIMD's vector pipe issues
               (the counter is in units of four cycles per wave, a CU has four SIMDs: the factors cancel)
  mfma_busy    as above
  w_any        wave cycles waiting for anything over all wave cycles
A kernel with valu_busy near 0.7 is bound by vector instructions whatever its memory traffic; one with a low valu_busy
and a high w_any waits for memory.
"""
from __future__ import annotations

import argparse
import collections
import csv
import math
import re

_NAME = re.compile(r"\b(k_[a-z0-9_]+)")


def _load(path):
    rows = collections.defaultdict(dict)   # dispatch id -> {counter: value, "_k": kernel, "_t": duration}
    for r in csv.DictReader(open(path)):
        m = _NAME.search(r["Kernel_Name"])
        if not m:
            continue
        d = rows[(path, r["Dispatch_Id"])]
        d["_k"] = m.group(1)
        d["_t"] = float(r["End_Timestamp"]) - float(r["Start_Timestamp"])
        d[r["Counter_Name"]] = float(r["Counter_Value"])
    return list(rows.values())


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("csv", nargs="+")
    ap.add_argument("--out", required=True)
    ap.add_argument("--mode", choices=["mfma", "vector"], default="mfma")
    a = ap.parse_args()
    disp = [d for p in a.csv for d in _load(p)]
    by_kernel = collections.defaultdict(list)
    for d in disp:
        by_kernel[d["_k"]].append(d)
    if a.mode == "vector":
        return _vector(by_kernel, a.out)
    lines = []
    hdr = f"{'kernel':18s} {'class':14s} {'launches':>8s} {'avg_us':>9s} {'mfma_busy':>9s} {'valu/mfma':>9s} {'trans/mfma':>10s} " \
          f"{'cvt/mfma':>8s} {'lds/mfma':>8s} {'w_lds':>6s} {'w_any':>6s} {'bank_cf':>7s}"
    lines.append(hdr)
    for k in sorted(by_kernel):
        ds = by_kernel[k]
        tmin, tmax = min(d["_t"] for d in ds), max(d["_t"] for d in ds)
        split = math.sqrt(tmin * tmax) if tmax > 3 * tmin else None
        classes = {"all": ds} if split is None else {
            "short launches": [d for d in ds if d["_t"] < split], "long launches": [d for d in ds if d["_t"] >= split]}
        for cname, cds in classes.items():
            def avg(c):
                v = [d[c] for d in cds if c in d]
                return sum(v) / len(v) if v else float("nan")
            n_a = sum(1 for d in cds if "SQ_INSTS_MFMA" in d)
            mf = avg("SQ_INSTS_MFMA")
            f = lambda x: "   -" if x != x else f"{x:.3f}"
            lines.append(
                f"{k:18s} {cname:14s} {n_a:8d} {sum(d['_t'] for d in cds) / len(cds) / 1e3:9.1f} "
                f"{f(avg('SQ_VALU_MFMA_BUSY_CYCLES') / (4 * avg('SQ_BUSY_CU_CYCLES'))):>9s} "
                f"{f((avg('SQ_INSTS_VALU') - mf) / mf):>9s} {f(avg('SQ_INSTS_VALU_TRANS_F32') / mf):>10s} "
                f"{f(avg('SQ_INSTS_VALU_CVT') / mf):>8s} {f(avg('SQ_INSTS_LDS') / mf):>8s} "
                f"{f(avg('SQ_WAIT_INST_LDS') / avg('SQ_WAVE_CYCLES')):>6s} {f(avg('SQ_WAIT_ANY') / avg('SQ_WAVE_CYCLES')):>6s} "
                f"{f(avg('SQ_LDS_BANK_CONFLICT') / avg('SQ_ACTIVE_INST_LDS')):>7s}")
    with open(a.out, "w") as fh:
        fh.write(__doc__.split("Derived columns")[0].rstrip() + "\n\n")
        fh.write("Derived columns" + __doc__.split("Derived columns")[1].rstrip() + "\n\n")
        fh.write("\n".join(lines) + "\n")
    print("\n".join(lines))


def _vector(by_kernel, out):
    lines = [f"{'kernel':20s} {'launches':>8s} {'avg_us':>9s} {'waves':>8s} {'valu/wave':>9s} {'lds/wave':>8s} {'rd/wave':>8s} "
             f"{'wr/wave':>8s} {'mfma/wave':>9s} {'valu_busy':>9s} {'mfma_busy':>9s} {'w_any':>6s}"]
    for k in sorted(by_kernel):
        ds = by_kernel[k]

        def avg(c):
            v = [d[c] for d in ds if c in d]
            return sum(v) / len(v) if v else float("nan")
        wv = avg("SQ_WAVES")
        f = lambda x, nd=3: "   -" if x != x else f"{x:.{nd}f}"
        lines.append(
            f"{k:20s} {sum(1 for d in ds if 'SQ_WAVES' in d):8d} {sum(d['_t'] for d in ds) / len(ds) / 1e3:9.1f} {f(wv, 0):>8s} "
            f"{f(avg('SQ_INSTS_VALU') / wv, 0):>9s} {f(avg('SQ_INSTS_LDS') / wv, 0):>8s} {f(avg('SQ_INSTS_VMEM_RD') / wv, 0):>8s} "
            f"{f(avg('SQ_INSTS_VMEM_WR') / wv, 0):>8s} {f(avg('SQ_INSTS_MFMA') / wv, 0):>9s} "
            f"{f(avg('SQ_ACTIVE_INST_VALU') / avg('SQ_BUSY_CU_CYCLES')):>9s} "
            f"{f(avg('SQ_VALU_MFMA_BUSY_CYCLES') / (4 * avg('SQ_BUSY_CU_CYCLES'))):>9s} "
            f"{f(avg('SQ_WAIT_ANY') / avg('SQ_WAVE_CYCLES')):>6s}")
    with open(out, "w") as fh:
        fh.write(__doc__.split("Derived columns")[0].rstrip() + "\n\n")
        fh.write("With --mode vector" + __doc__.split("With --mode vector")[1].rstrip() + "\n\n")
        fh.write("\n".join(lines) + "\n")
    print("\n".join(lines))


if __name__ == "__main__":
    main()
