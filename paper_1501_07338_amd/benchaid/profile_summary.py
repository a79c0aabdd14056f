"""Turns the raw CSV output of rocprofv3 runs of `bench.py --markers` into the short text summaries and the
traffic table kept under profiles/.

The benchmark, run with --markers, launches an empty marker kernel ahead of each per-layer timing phase (grid
size = 64 x phase number; the numbering is in the detail file it writes).  Walking a run's dispatches in order,
everything between a marker and the next one belongs to that phase, so each convolution pass gets rows of its
own even where one kernel name serves several layers.

    python -m paper_1501_07338_amd.benchaid.profile_summary --name cfg5_f32_bf16 --detail <dir>/detail.json \\
        --trace <dir>/trace --fetch <dir>/fetch --write <dir>/write \\
        --mfma <dir>/mfma --cmd "<the bench.py arguments of the runs>" [--out profiles]

Counter calibration: the phase "copy of 1 GiB" is a plain streaming copy (2^30 bytes read, 2^30 written); the
factor bytes / (counter KiB x 1024) it gives for FETCH_SIZE and for WRITE_SIZE scales every other reading.
"""
from __future__ import annotations

import argparse
import collections
import csv
import glob
import json
import os
import statistics
import subprocess

NAME_W = 96


def short(name: str) -> str:
    name = name.replace("void vcnn::", "").replace("vcnn::", "")
    return name[:NAME_W]


def find(dirname, pattern):
    hits = sorted(glob.glob(os.path.join(dirname, "**", pattern), recursive=True))
    if not hits:
        raise SystemExit(f"no {pattern} under {dirname}")
    return hits[0]


def phases_of(rows, markers, name_key, grid_key, id_key="Dispatch_Id"):
    """rows: dispatch records in any order -> {phase: [records]} using the marker kernels."""
    rows = sorted(rows, key=lambda r: int(r[id_key]))
    out = collections.OrderedDict()
    cur = None
    for r in rows:
        if "benchaid_marker_kernel" in r[name_key]:
            cur = markers.get(str(int(r[grid_key]) // 64))
            if cur == "-":
                cur = None
            continue
        if cur is not None:
            out.setdefault(cur, []).append(r)
    return out


def load_trace(dirname):
    rows = list(csv.DictReader(open(find(dirname, "*kernel_trace.csv"))))
    for r in rows:
        r["us"] = (int(r["End_Timestamp"]) - int(r["Start_Timestamp"])) / 1e3
        r["grid"] = int(r["Grid_Size_X"]) * int(r["Grid_Size_Y"]) * int(r["Grid_Size_Z"])
    return rows


def load_counters(dirname):
    """-> list of dispatch records {Dispatch_Id, Kernel_Name, Grid_Size, us, counters{name: value}}"""
    by_id = {}
    for r in csv.DictReader(open(find(dirname, "*counter_collection.csv"))):
        d = by_id.setdefault(r["Dispatch_Id"], {"Dispatch_Id": r["Dispatch_Id"], "Kernel_Name": r["Kernel_Name"],
                                               "Grid_Size": r["Grid_Size"], "counters": {},
                                               "us": (int(r["End_Timestamp"]) - int(r["Start_Timestamp"])) / 1e3})
        d["counters"][r["Counter_Name"]] = d["counters"].get(r["Counter_Name"], 0.0) + float(r["Counter_Value"])
    return list(by_id.values())


def group(records, name_key, grid_of):
    g = collections.OrderedDict()
    for r in records:
        g.setdefault((short(r[name_key]), grid_of(r)), []).append(r)
    return g


def git_head():
    try:
        return subprocess.run(["git", "rev-parse", "--short", "HEAD"], capture_output=True, text=True).stdout.strip()
    except OSError:
        return "unknown"


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--name", required=True, help="what the runs cover; prefix of the files written")
    ap.add_argument("--detail", required=True)
    ap.add_argument("--trace")
    ap.add_argument("--fetch")
    ap.add_argument("--write")
    ap.add_argument("--mfma")
    ap.add_argument("--cmd", required=True, help="the bench.py arguments the profiled runs used")
    ap.add_argument("--out", default="profiles")
    args = ap.parse_args()
    detail = json.load(open(args.detail))
    markers = detail["markers"]
    os.makedirs(args.out, exist_ok=True)
    head = git_head()

    if args.trace:
        rows = load_trace(args.trace)
        ph = phases_of(rows, markers, "Kernel_Name", "grid")
        out = [f"rocprofv3 kernel trace by benchmark phase: {args.name}, one MI355X (source tree at commit {head})", "",
               "command (from the repository root on the GPU box):",
               f"  rocprofv3 --kernel-trace --stats --output-format csv -d <dir> -o p -- python3 bench.py {args.cmd}",
               "Each phase is one convolution pass called back to back (one untimed call, then the timed ones); durations in",
               "microseconds per dispatch.  'per call' = sum over the pass's kernels of their dispatches per call x average.", ""]
        for phase, recs in ph.items():
            g = group(recs, "Kernel_Name", lambda r: r["grid"])
            calls = min(len(v) for v in g.values())
            out.append(f"== {phase}  ({calls} calls)")
            out.append("   %-*s %10s %6s %10s %10s %10s" % (NAME_W, "kernel", "grid", "disp.", "avg_us", "min_us", "max_us"))
            total = 0.0
            for (name, grid), v in g.items():
                us = [r["us"] for r in v]
                total += sum(us) / calls
                out.append("   %-*s %10d %6d %10.2f %10.2f %10.2f" % (NAME_W, name, grid, len(v), statistics.mean(us), min(us), max(us)))
            out.append("   per call: %.2f us" % total)
            out.append("")
        stats = list(csv.DictReader(open(find(args.trace, "*kernel_stats.csv"))))
        out.append("== whole run, kernels by total time (rocprofv3 --stats)")
        out.append("   %-*s %6s %12s %10s %6s" % (NAME_W, "kernel", "calls", "total_us", "avg_us", "pct"))
        for r in stats[:40]:
            out.append("   %-*s %6s %12.1f %10.2f %6.2f" % (NAME_W, short(r["Name"]), r["Calls"], float(r["TotalDurationNs"]) / 1e3,
                                                          float(r["AverageNs"]) / 1e3, float(r["Percentage"])))
        open(os.path.join(args.out, f"{args.name}_kernel_trace_by_pass.txt"), "w").write("\n".join(out) + "\n")

    traffic = {"commit": head, "command": f"bench.py {args.cmd}", "passes": {}}
    if args.fetch and args.write:
        f_ph = phases_of(load_counters(args.fetch), markers, "Kernel_Name", "Grid_Size")
        w_ph = phases_of(load_counters(args.write), markers, "Kernel_Name", "Grid_Size")

        def avg_counter(recs, counter):
            g = group(recs, "Kernel_Name", lambda r: int(r["Grid_Size"]))
            return {k: (statistics.mean(r["counters"].get(counter, 0.0) for r in v), statistics.mean(r["us"] for r in v), len(v))
                    for k, v in g.items()}

        cal_f = avg_counter(f_ph.get("copy of 1 GiB", []), "FETCH_SIZE")
        cal_w = avg_counter(w_ph.get("copy of 1 GiB", []), "WRITE_SIZE")
        gib = float(1 << 30)
        kf = next((k for k in cal_f if "benchaid_copy" in k[0]), None)
        kw = next((k for k in cal_w if "benchaid_copy" in k[0]), None)
        scale_f = gib / (cal_f[kf][0] * 1024.0) if kf else 1.0
        scale_w = gib / (cal_w[kw][0] * 1024.0) if kw else 1.0
        traffic["calibration"] = {"kernel": "benchaid_copy_kernel, 2^30 bytes read and 2^30 written",
                                  "FETCH_SIZE_KiB": cal_f[kf][0] if kf else None, "WRITE_SIZE_KiB": cal_w[kw][0] if kw else None,
                                  "fetch_scale": scale_f, "write_scale": scale_w}
        out = [f"rocprofv3 HBM traffic counters by benchmark phase: {args.name}, one MI355X (source tree at commit {head})", "",
               "commands (two runs, one counter each):",
               f"  rocprofv3 --pmc FETCH_SIZE --kernel-trace --output-format csv -d <dir> -o f -- python3 bench.py {args.cmd}",
               f"  rocprofv3 --pmc WRITE_SIZE --kernel-trace --output-format csv -d <dir> -o w -- python3 bench.py {args.cmd}",
               "counter unit: KiB per dispatch, averaged over the phase's dispatches of that kernel.",
               "calibration on the plain copy of 2^30 bytes (benchaid_copy_kernel): FETCH_SIZE reads %s KiB, WRITE_SIZE %s KiB" %
               ("%.0f" % cal_f[kf][0] if kf else "n/a", "%.0f" % cal_w[kw][0] if kw else "n/a"),
               "  => bytes = FETCH_SIZE x 1024 x %.3f + WRITE_SIZE x 1024 x %.3f" % (scale_f, scale_w), ""]
        for phase in f_ph:
            if phase not in w_ph:
                continue
            af, aw = avg_counter(f_ph[phase], "FETCH_SIZE"), avg_counter(w_ph[phase], "WRITE_SIZE")
            out.append(f"== {phase}")
            out.append("   %-*s %10s %12s %12s %12s %10s" % (NAME_W, "kernel", "grid", "FETCH KiB", "WRITE KiB", "HBM MB", "dur us"))
            calls = min(v[2] for v in af.values())
            pass_bytes, top = 0.0, None
            for k, (fv, us, cnt) in af.items():
                wv = aw.get(k, (0.0, 0.0, 0))[0]
                nbytes = fv * 1024.0 * scale_f + wv * 1024.0 * scale_w
                pass_bytes += nbytes * cnt / calls
                if top is None or us * cnt > top[1]:
                    top = (k, us * cnt, nbytes, fv, wv)
                out.append("   %-*s %10d %12.0f %12.0f %12.1f %10.1f" % (NAME_W, k[0], k[1], fv, wv, nbytes / 1e6, us))
            out.append("   whole pass per call: %.1f MB" % (pass_bytes / 1e6))
            out.append("")
            if ".conv" in phase and top:
                traffic["passes"][phase] = {"kernel": top[0][0], "grid": top[0][1], "fetch_kib": top[3], "write_kib": top[4],
                                            "hbm_bytes": top[2], "pass_hbm_bytes": pass_bytes}
        open(os.path.join(args.out, f"{args.name}_hbm_traffic_pmc.txt"), "w").write("\n".join(out) + "\n")
        # one table for every summarised set of runs: passes of other sets stay, those of this set are replaced
        path = os.path.join(args.out, "traffic.json")
        table = {"runs": {}, "passes": {}}
        if os.path.exists(path):
            try:
                kept = json.load(open(path))
                if "runs" in kept:
                    table = kept
            except ValueError:
                pass
        table["passes"] = {k: v for k, v in table["passes"].items() if v.get("run") != args.name}
        for k, v in traffic["passes"].items():
            table["passes"][k] = dict(v, run=args.name)
        table["runs"][args.name] = {"commit": traffic["commit"], "command": traffic["command"],
                                    "calibration": traffic.get("calibration")}
        json.dump(table, open(path, "w"), indent=1, sort_keys=True)

    if args.mfma:
        m_ph = phases_of(load_counters(args.mfma), markers, "Kernel_Name", "Grid_Size")
        out = [f"rocprofv3 matrix-core counters by benchmark phase: {args.name}, one MI355X (source tree at commit {head})", "",
               "command:",
               "  rocprofv3 --pmc SQ_VALU_MFMA_BUSY_CYCLES SQ_BUSY_CU_CYCLES SQ_INSTS_VALU_MFMA_MOPS_F32 SQ_INSTS_VALU_MFMA_MOPS_BF16 "
               f"GRBM_GUI_ACTIVE --kernel-trace --output-format csv -d <dir> -o m -- python3 bench.py {args.cmd}",
               "MfmaUtil = SQ_VALU_MFMA_BUSY_CYCLES / (4 SIMDs x SQ_BUSY_CU_CYCLES); executed MFMA flop = 512 x (MOPS_F32 + MOPS_BF16)",
               "per dispatch (it includes tile padding and any zero border a kernel multiplies); durations under counter",
               "collection run a few % longer than in the timed runs.", ""]
        for phase, recs in m_ph.items():
            g = group(recs, "Kernel_Name", lambda r: int(r["Grid_Size"]))
            rows = []
            for k, v in g.items():
                mops = statistics.mean(r["counters"].get("SQ_INSTS_VALU_MFMA_MOPS_F32", 0) + r["counters"].get("SQ_INSTS_VALU_MFMA_MOPS_BF16", 0) for r in v)
                if mops <= 0:
                    continue
                busy = statistics.mean(r["counters"].get("SQ_VALU_MFMA_BUSY_CYCLES", 0) for r in v)
                cu = statistics.mean(r["counters"].get("SQ_BUSY_CU_CYCLES", 0) for r in v)
                us = statistics.mean(r["us"] for r in v)
                rows.append((k, us, mops * 512 / 1e9, busy / (4 * cu) if cu else float("nan"), mops * 512 / us / 1e6))
            if not rows:
                continue
            out.append(f"== {phase}")
            out.append("   %-*s %10s %10s %12s %10s %10s" % (NAME_W, "kernel", "grid", "dur us", "MFMA GFLOP", "MfmaUtil", "TFLOP/s"))
            for k, us, gf, util, tf in rows:
                out.append("   %-*s %10d %10.1f %12.2f %10.3f %10.1f" % (NAME_W, k[0], k[1], us, gf, util, tf))
            out.append("")
        open(os.path.join(args.out, f"{args.name}_mfma_util_pmc.txt"), "w").write("\n".join(out) + "\n")


if __name__ == "__main__":
    main()
