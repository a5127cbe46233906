"""Summarise rocprofv3 CSV output of `bench.py --workload W --no-secondary` into profiles/measured.json.

bench.py reads that file for the figures it cannot measure in its own run: the HBM-side bytes of one attention
launch (FETCH_SIZE and WRITE_SIZE, each scaled by what the same counter reads for the plain 512 MiB copy that
`--copy-calibration` runs in the same process) and the clock the box sustained under the kernel
(GRBM_GUI_ACTIVE cycles of all eight XCDs / 8 / the launch's duration).  One entry per workload, stamped with the
commit the profile was taken at.  Host-side text processing only.

    python -m paper_2405_07719_amd.profile_summary --workload hybrid_u8r2_L212992 \\
        --fetch <dir>/FETCH_SIZE/bench_counter_collection.csv --write <dir>/WRITE_SIZE/bench_counter_collection.csv \\
        --clock-counters <dir>/clk/bench_counter_collection.csv --clock-trace <dir>/clk/bench_kernel_trace.csv \\
        --kernel-stats <dir>/kt/bench_kernel_stats.csv --git-head $(git rev-parse --short HEAD)
"""
from __future__ import annotations

import argparse
import collections
import csv
import json
import os

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
COPY_KIB = 524288.0                       # the calibration copy: 512 MiB read, 512 MiB written
KERNELS = {"attention_fwd": "block_attn_fwd_mfma", "bwd_dq": "bwd_dq_kernel", "bwd_dkdv": "bwd_dkdv_kernel",
           "bwd_dq_ds": "bwd_dq_ds_kernel", "layout_a2a": "layout_a2a_kernel", "lse_merge": "lse_merge_kernel",
           "attention_fwd_fp32_out": "block_attn_fwd_mfma<.., float>", "attention_fwd_state": "block_attn_fwd_mfma<.., STATE>", "calib_pure_mfma": "calib_pure_mfma", "calib_attention_mix": "calib_attention_mix", "copy": "copyBuffer"}


def _short(name):
    for key, pat in KERNELS.items():
        if pat in name and not (key == "bwd_dq" and "bwd_dq_ds" in name):
            if key == "attention_fwd":
                # instances of the forward kernel (the profiler prints some names mangled, some demangled): bf16 out
                # without the ring state = the launch of the one-launch ring loop; fp32 out = partial results of a
                # step-by-step ring or of a key split; the rest = the state-carrying step kernel
                if "DF16bLb0E" in name:
                    return "attention_fwd"
                if "float" in name or "EfLb" in name:
                    return "attention_fwd_fp32_out"
                return "attention_fwd_state"
            return key
    return None


def counter_means(path, counter):
    """{kernel key: (mean, max, dispatches)} of one counter (KiB per dispatch for FETCH_SIZE / WRITE_SIZE)."""
    agg = collections.defaultdict(list)
    with open(path) as f:
        for r in csv.DictReader(f):
            if r["Counter_Name"] != counter:
                continue
            k = _short(r["Kernel_Name"])
            if k:
                agg[k].append(float(r["Counter_Value"]))
    if "copy" in agg:   # the calibration copy is the largest one; a workload's own (smaller) buffer copies are not it
        agg["copy"] = [x for x in agg["copy"] if x >= 0.9 * max(agg["copy"])]
    return {k: (sum(v) / len(v), max(v), len(v)) for k, v in agg.items()}


def clocks(counter_csv, trace_csv):
    """{kernel key: (cycles per XCD, duration ns, GHz, dispatches)} over the second half of each kernel's dispatches."""
    dur = {}
    with open(trace_csv) as f:
        for r in csv.DictReader(f):
            dur[r["Dispatch_Id"]] = int(r["End_Timestamp"]) - int(r["Start_Timestamp"])
    agg = collections.defaultdict(list)
    with open(counter_csv) as f:
        for r in csv.DictReader(f):
            if r["Counter_Name"] != "GRBM_GUI_ACTIVE" or r["Dispatch_Id"] not in dur:
                continue
            k = _short(r["Kernel_Name"])
            if k:
                agg[k].append((float(r["Counter_Value"]), dur[r["Dispatch_Id"]]))
    out = {}
    for k, v in agg.items():
        tail = v[len(v) // 2:]
        cyc = sum(a for a, _ in tail) / len(tail) / 8.0          # the counter sums the eight XCDs
        d = sum(b for _, b in tail) / len(tail)
        out[k] = (cyc, d, cyc / d, len(tail))
    return out


def counter_table(paths):
    """Every counter of the given collection files as a table: one row per counter, one column per kernel (mean per
    dispatch, summed over the chip by the profiler).  bwd_dkdv is split by its template flag (plain / writes dS)."""
    table = collections.defaultdict(lambda: collections.defaultdict(list))
    for path in paths:
        with open(path) as f:
            for r in csv.DictReader(f):
                k = _short(r["Kernel_Name"])
                if not k or k == "copy":
                    continue
                if k == "bwd_dkdv":
                    k = "bwd_dkdv (writes dS)" if "true" in r["Kernel_Name"] else "bwd_dkdv"
                table[r["Counter_Name"]][k].append(float(r["Counter_Value"]))
    cols = sorted({k for c in table.values() for k in c})
    print("| counter | " + " | ".join(cols) + " |")
    print("|---|" + "---|" * len(cols))
    for c in table:
        print(f"| {c} | " + " | ".join(f"{sum(table[c][k]) / len(table[c][k]):.4g}" if table[c][k] else "" for k in cols) + " |")
    mf = table.get("SQ_INSTS_MFMA")
    if mf:
        print("\nper MFMA instruction:\n")
        print("| counter | " + " | ".join(cols) + " |")
        print("|---|" + "---|" * len(cols))
        for c in table:
            if c.startswith("SQ_INSTS_") and c != "SQ_INSTS_MFMA":
                print(f"| {c} | " + " | ".join(
                    f"{(sum(table[c][k]) / len(table[c][k])) / (sum(mf[k]) / len(mf[k])):.3f}" if table[c][k] and mf.get(k) and sum(mf[k]) else ""
                    for k in cols) + " |")


def kernel_stats(path):
    rows = []
    with open(path) as f:
        for r in csv.DictReader(f):
            rows.append((r["Name"], int(r["Calls"]), float(r["AverageNs"]), float(r["MinNs"]), float(r["MaxNs"]), float(r["Percentage"])))
    return rows


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", required=True)
    ap.add_argument("--fetch")
    ap.add_argument("--write")
    ap.add_argument("--clock-counters")
    ap.add_argument("--clock-trace")
    ap.add_argument("--kernel-stats")
    ap.add_argument("--counter-table", nargs="*", default=[], help="counter collection files to print as one table")
    ap.add_argument("--git-head", required=True)
    ap.add_argument("--out", default=os.path.join(ROOT, "profiles", "measured.json"))
    a = ap.parse_args()
    entry = {"git_head": a.git_head}
    if a.fetch and a.write:
        fe, wr = counter_means(a.fetch, "FETCH_SIZE"), counter_means(a.write, "WRITE_SIZE")
        f_scale, w_scale = COPY_KIB / fe["copy"][0], COPY_KIB / wr["copy"][0]
        entry["fetch_scale"], entry["write_scale"] = round(f_scale, 4), round(w_scale, 4)
        print(f"copy calibration: FETCH_SIZE {fe['copy'][0]:.0f} KiB -> x{f_scale:.3f}, WRITE_SIZE {wr['copy'][0]:.0f} KiB -> x{w_scale:.3f}")
        print("| kernel | dispatches | FETCH_SIZE KiB mean (max) | WRITE_SIZE KiB mean (max) | bytes per launch (scaled, mean) |")
        print("|---|---|---|---|---|")
        per = {}
        for k in fe:
            if k == "copy" or k not in wr:
                continue
            b = (fe[k][0] * f_scale + wr[k][0] * w_scale) * 1024.0
            per[k] = round(b)
            print(f"| {KERNELS[k]} | {fe[k][2]} | {fe[k][0]:.0f} ({fe[k][1]:.0f}) | {wr[k][0]:.0f} ({wr[k][1]:.0f}) | {b:.4g} |")
        entry["traffic_bytes"] = per.get("attention_fwd")
        entry["traffic_bytes_by_kernel"] = per
    if a.clock_counters and a.clock_trace:
        ck = clocks(a.clock_counters, a.clock_trace)
        print("| kernel | dispatches | cycles per XCD (M) | duration us | clock GHz |")
        print("|---|---|---|---|---|")
        for k, (cyc, d, ghz, n) in ck.items():
            if k == "copy":   # buffer copies of a few microseconds: no clock to read from them
                continue
            print(f"| {KERNELS[k]} | {n} | {cyc / 1e6:.3f} | {d / 1e3:.1f} | {ghz:.3f} |")
        if "attention_fwd" in ck:
            entry["clock_ghz"] = round(ck["attention_fwd"][2], 3)
            entry["attention_cycles"] = round(ck["attention_fwd"][0])
    if a.kernel_stats:
        print("| kernel | calls | avg us | min us | max us | % |")
        print("|---|---|---|---|---|---|")
        for name, calls, avg, mn, mx, pct in kernel_stats(a.kernel_stats)[:14]:
            print(f"| {name[:90]} | {calls} | {avg / 1e3:.1f} | {mn / 1e3:.1f} | {mx / 1e3:.1f} | {pct:.1f} |")
            if "block_attn_fwd_mfma" in name and "attention_avg_us" not in entry:
                entry["attention_avg_us"] = round(avg / 1e3, 1)
    if a.counter_table:
        counter_table(a.counter_table)
    data = {}
    if os.path.exists(a.out):
        with open(a.out) as f:
            data = json.load(f)
    data[a.workload] = {**data.get(a.workload, {}), **entry}
    with open(a.out, "w") as f:
        json.dump(data, f, indent=1, sort_keys=True)
        f.write("\n")
    print(f"wrote {a.out}: {a.workload} -> {entry}")


if __name__ == "__main__":
    main()
