"""Turns rocprofv3 output of a bench.py run into the short summaries kept under profiles/.

    python -m paper_2603_27156_amd.profile_summary --workload cfg2-1M --title "..." \
        --stats <dir>/<name>_kernel_stats.csv --pmc <dir>/..._counter_collection.csv [--pmc ...] \
        --command "<the rocprofv3 command lines>" --copy-bytes <bytes one k_copy_planes launch reads> \
        --md profiles/<kernel-and-workload>.md [--json profiles/gsr_step_counters.json]

--stats: the per-kernel table of `rocprofv3 --kernel-trace --stats` (average launch durations).
--pmc:   `rocprofv3 --pmc <counters>` passes (one file per pass); counters are averaged per launch and kernel.
         FETCH_SIZE / WRITE_SIZE (KiB per dispatch) are scaled by what the same counter reads for the plain
         layout-copy kernel of known size (--copy-bytes read and written per launch), which calibrates the counter's
         unit on this machine; the factors are stated in the summary.
--json:  the file bench.py reads its `roofline.traffic` and `roofline.pipes` from: per workload and kernel class the
         counted HBM bytes per launch and the share of a SIMD's cycles its vector / matrix pipes are busy, with the
         commit the passes were taken at.
Nothing here runs on the GPU; the tool only reads CSV files.
"""
from __future__ import annotations

import argparse
import collections
import csv
import json
import os
import re
import subprocess


def kernel_class(name: str):
    """bench.py's kernel class of a kernel name, or None."""
    m = re.search(r"k_block<\d+, [\w:]+, (-?\d+), (true|false), (true|false)[,>]", name)
    if m:
        if m.group(1) == "1":
            return "block_forward"
        return "block_backward" if m.group(2) == "true" else "block_inverse"
    if "k_grad<" in name:
        return "grad"
    if "k_dw<" in name:
        return "weight_gradient"
    if "k_sum<" in name:
        return "group_sum"
    if "k_copy_planes<" in name:
        return "layout_copy"
    if "k_hub_" in name:
        return "hub_first_pass"
    if "k_tie_fixup<" in name:
        return "tie_fixup"
    if "k_head" in name:
        return "head"
    if "k_spmm_tile<" in name:
        return "gsr_spmm"
    if "k_gs_tile<" in name:
        return "gsr_group_sparse"
    if "k_aggregate_tile<" in name:
        return "gsr_spmm_compressed"
    if "k_slot_tile<" in name:
        return "slot_block"
    return None


def short(name: str) -> str:
    name = re.sub(r"^void ", "", name)
    return re.sub(r"\(.*", "", name).replace("gsr::", "")


def read_stats(path):
    rows = []
    with open(path) as f:
        for r in csv.DictReader(f):
            rows.append(dict(name=r["Name"], calls=int(r["Calls"]), total_ms=float(r["TotalDurationNs"]) / 1e6,
                             avg_us=float(r["AverageNs"]) / 1e3, pct=float(r["Percentage"]),
                             min_us=float(r["MinNs"]) / 1e3, max_us=float(r["MaxNs"]) / 1e3))
    return rows


def read_pmc(paths):
    """{kernel name: {counter: average per launch}} and {kernel name: launches in one pass}, over all passes (a
    counter collected in several passes is averaged over all of them)."""
    total = collections.defaultdict(lambda: collections.defaultdict(float))
    rows = collections.defaultdict(lambda: collections.defaultdict(int))
    for p in paths:
        with open(p) as f:
            for r in csv.DictReader(f):
                k = r["Kernel_Name"]
                total[k][r["Counter_Name"]] += float(r["Counter_Value"])
                rows[k][r["Counter_Name"]] += 1
    avg = {k: {c: v / rows[k][c] for c, v in cs.items()} for k, cs in total.items()}
    count = {k: min(rows[k].values()) for k in rows}
    return avg, count


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", required=True)
    ap.add_argument("--title", required=True)
    ap.add_argument("--stats")
    ap.add_argument("--pmc", action="append", default=[])
    ap.add_argument("--command", action="append", default=[])
    ap.add_argument("--copy-bytes", type=float, default=0.0)
    ap.add_argument("--md", required=True)
    ap.add_argument("--json")
    ap.add_argument("--note", action="append", default=[])
    ap.add_argument("--min-pct", type=float, default=0.05)
    args = ap.parse_args()

    try:
        commit = subprocess.check_output(["git", "rev-parse", "--short", "HEAD"], text=True,
                                         cwd=os.path.dirname(os.path.abspath(__file__))).strip()
    except Exception:
        commit = "unknown"
    out = [f"# {args.title}", "", f"Library sources at commit {commit}.  Commands (from /tmp with TMPDIR=/tmp, one MI355X):", ""]
    out += [f"    {c}" for c in args.command] + [""]

    classes = {}
    if args.stats:
        rows = [r for r in read_stats(args.stats) if "gsr::" in r["name"]]
        tot = sum(r["total_ms"] for r in rows)
        out += ["| kernel | calls | total ms | avg us | % of the library's GPU time | min us | max us |", "|---|---:|---:|---:|---:|---:|---:|"]
        for r in sorted(rows, key=lambda r: -r["total_ms"]):
            share = 100.0 * r["total_ms"] / tot
            if share < args.min_pct:
                continue
            out.append(f"| `{short(r['name'])}` | {r['calls']} | {r['total_ms']:.1f} | {r['avg_us']:.1f} | {share:.2f} | {r['min_us']:.1f} | {r['max_us']:.1f} |")
            kc = kernel_class(r["name"])
            if kc:
                e = classes.setdefault(kc, {"calls": 0, "total_us": 0.0})
                e["calls"] += r["calls"]
                e["total_us"] += r["total_ms"] * 1e3
        out.append("")
        for e in classes.values():
            e["avg_launch_us"] = e.pop("total_us") / e["calls"]

    if args.pmc:
        avg, count = read_pmc(args.pmc)
        by_class = collections.defaultdict(lambda: collections.defaultdict(float))
        n_class = collections.defaultdict(int)
        for k, cs in avg.items():
            kc = kernel_class(k)
            if not kc:
                continue
            for c, v in cs.items():
                by_class[kc][c] += v * count[k]
            n_class[kc] += count[k]
        for kc in by_class:
            for c in by_class[kc]:
                by_class[kc][c] /= n_class[kc]
        f_fetch = f_write = None
        copy = by_class.get("layout_copy", {})
        if args.copy_bytes and "FETCH_SIZE" in copy:
            f_fetch = args.copy_bytes / (copy["FETCH_SIZE"] * 1024.0)
        if args.copy_bytes and "WRITE_SIZE" in copy:
            f_write = args.copy_bytes / (copy["WRITE_SIZE"] * 1024.0)
        if f_fetch or f_write:
            out += [f"Calibration on `k_copy_planes` ({args.copy_bytes / 1e6:.0f} MB read and written per launch): "
                    f"FETCH_SIZE reads {copy.get('FETCH_SIZE', 0):.0f} KiB (factor {f_fetch:.2f}), "
                    f"WRITE_SIZE {copy.get('WRITE_SIZE', 0):.0f} KiB (factor {f_write:.2f}).", ""]
        counters = sorted({c for cs in by_class.values() for c in cs})
        out += ["| kernel class | launches | " + " | ".join(counters) + " |", "|---|---:|" + "---:|" * len(counters)]
        for kc in sorted(by_class, key=lambda k: -n_class[k]):
            out.append(f"| {kc} | {n_class[kc]} | " + " | ".join(f"{by_class[kc].get(c, float('nan')):.4g}" for c in counters) + " |")
        out.append("")
        derived = []
        for kc, cs in by_class.items():
            e = classes.setdefault(kc, {})
            if f_fetch and f_write and "FETCH_SIZE" in cs and "WRITE_SIZE" in cs:
                e["hbm_bytes_per_launch"] = cs["FETCH_SIZE"] * 1024.0 * f_fetch + cs["WRITE_SIZE"] * 1024.0 * f_write
                e["fetch_kib_raw"], e["write_kib_raw"] = cs["FETCH_SIZE"], cs["WRITE_SIZE"]
            pipes = {}
            # SQ_BUSY_CYCLES is summed over the 32 shader engines; SQ_ACTIVE_INST_* and SQ_WAVE_CYCLES count in units
            # of 4 cycles; SQ_VALU_MFMA_BUSY_CYCLES is summed over the 1,024 SIMDs (4,096 wave slots)
            kcyc = cs.get("SQ_BUSY_CYCLES", 0.0) / 32.0
            if kcyc > 0:
                pipes["kernel_cycles"] = kcyc
                if "SQ_ACTIVE_INST_VALU" in cs:
                    pipes["valu_busy"] = 4.0 * cs["SQ_ACTIVE_INST_VALU"] / (1024.0 * kcyc)
                if "SQ_VALU_MFMA_BUSY_CYCLES" in cs:
                    pipes["mfma_busy"] = cs["SQ_VALU_MFMA_BUSY_CYCLES"] / (1024.0 * kcyc)
                if "SQ_WAVE_CYCLES" in cs:
                    pipes["residency"] = 4.0 * cs["SQ_WAVE_CYCLES"] / (4096.0 * kcyc)
            if "SQ_INSTS_VALU" in cs:
                pipes["valu_insts_per_launch"] = cs["SQ_INSTS_VALU"]
            if "SQ_INSTS_MFMA" in cs:
                pipes["mfma_insts_per_launch"] = cs["SQ_INSTS_MFMA"]
            if pipes:
                e["pipes"] = pipes
            if "hbm_bytes_per_launch" in e:
                derived.append(f"| {kc} | {e['hbm_bytes_per_launch'] / 1e6:.1f} | {cs['FETCH_SIZE'] * 1024 / 1e6:.1f} | {cs['WRITE_SIZE'] * 1024 / 1e6:.1f} |")
        if derived:
            out += ["| kernel class | HBM MB per launch (calibrated) | FETCH_SIZE MB raw | WRITE_SIZE MB raw |", "|---|---:|---:|---:|"] + derived + [""]
    out += args.note
    with open(args.md, "w") as f:
        f.write("\n".join(out) + "\n")
    if args.json:
        try:
            with open(args.json) as f:
                rec = json.load(f)
        except (OSError, ValueError):
            rec = {"workloads": {}}
        rec["commit"] = commit
        rec["written_by"] = "python -m paper_2603_27156_amd.profile_summary"
        rec["workloads"][args.workload] = {"summary": os.path.relpath(args.md, os.path.dirname(os.path.abspath(args.json)) + "/.."),
                                           "commit": commit, "kernels": classes}
        with open(args.json, "w") as f:
            json.dump(rec, f, indent=1, sort_keys=True)
            f.write("\n")
    print("\n".join(out))


if __name__ == "__main__":
    main()
