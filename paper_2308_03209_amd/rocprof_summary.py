"""Profile a command with rocprofv3 and condense the result into the short text summary and the per-kernel
traffic table that are kept under profiles/.

    python -m paper_2308_03209_amd.rocprof_summary --tag cfg1 --title "cfg1 (...)" [--out DIR] \\
        -- python3 bench.py --no-cpu-baseline --no-also --config 1 --steps 5 --warmup 2

Four runs of the command, each a child process of its own with the program right after `--`:
  rocprofv3 --kernel-trace --stats        per-kernel durations
  rocprofv3 --pmc FETCH_SIZE              bytes fetched past L2 (KiB per dispatch)
  rocprofv3 --pmc WRITE_SIZE              bytes written past L2
  rocprofv3 --pmc TCC_HIT_sum TCC_MISS_sum
The byte counters are scaled by what the same counters read for a plain device copy of known size inside the
same run (bench.py issues a 1 GiB copy before the workload).  Written into --out: summary.txt and traffic.json
({kernel template instance: mean bytes per launch}, stamped with a hash of the kernel sources so that bench.py
quotes it only for the kernels it was measured on).  This script itself never touches the GPU.
"""
from __future__ import annotations

import argparse
import hashlib
import json
import os
import re
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)


def kernel_source_hash() -> str:
    h = hashlib.sha256()
    csrc = os.path.join(HERE, "csrc")
    for name in sorted(os.listdir(csrc)):
        # the library's sources; gather_ceiling.hip is a stand-alone program and not part of any profiled kernel
        if name.endswith((".hip", ".cpp", ".h")) and name != "gather_ceiling.hip":
            h.update(name.encode())
            h.update(open(os.path.join(csrc, name), "rb").read())
    return h.hexdigest()[:16]


def instance_name(kernel: str) -> str:
    """'void cofree::aggregate_group_kernel<float, 8, 8, false>(cofree::AggK<float>)' ->
    'aggregate_group_kernel<float,8,8,false>' (the form the library's own timing records use)."""
    k = re.sub(r"\(.*", "", kernel)
    k = k.replace("void ", "").replace("cofree::", "").replace("unsigned short", "bf16").replace(" ", "")
    return k


def find_csv(directory: str, suffix: str) -> str:
    for base, _, files in os.walk(directory):
        for f in files:
            if f.endswith(suffix):
                return os.path.join(base, f)
    raise FileNotFoundError(f"no *{suffix} under {directory}")


def run(out: str, name: str, prof_args, cmd, limit: int) -> str:
    d = os.path.join(out, name)
    os.makedirs(d, exist_ok=True)
    full = ["timeout", "-s", "KILL", str(limit), "rocprofv3", *prof_args, "--output-format", "csv", "-d", d, "-o", "p",
            "--", *cmd]
    print("[rocprof_summary]", " ".join(full), flush=True)
    with open(os.path.join(out, name + ".log"), "w") as log:
        rc = subprocess.call(full, stdout=log, stderr=subprocess.STDOUT, env=dict(os.environ, TMPDIR="/tmp"))
    if rc != 0:
        sys.stderr.write(open(os.path.join(out, name + ".log")).read()[-3000:])
        raise SystemExit(f"rocprofv3 run '{name}' failed with status {rc}")
    return " ".join(full[4:])


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--tag", required=True)
    ap.add_argument("--title", default="")
    ap.add_argument("--out", default=None)
    ap.add_argument("--limit", type=int, default=600, help="seconds per profiled run")
    ap.add_argument("--no-counters", action="store_true", help="kernel trace only")
    ap.add_argument("--kernels", default="cofree::", help="regular expression selecting the kernels of the traffic table")
    ap.add_argument("--fetch-scale", type=float, default=None,
                    help="scale of FETCH_SIZE, for a program that issues no calibration copy (take it from a run that does)")
    ap.add_argument("--write-scale", type=float, default=None)
    ap.add_argument("--append-stdout", action="store_true",
                    help="append what the program itself printed during the kernel-trace run (its own result table)")
    ap.add_argument("cmd", nargs=argparse.REMAINDER)
    args = ap.parse_args()
    cmd = args.cmd[1:] if args.cmd and args.cmd[0] == "--" else args.cmd
    if not cmd:
        raise SystemExit("give the command to profile after --")
    out = args.out or os.path.join("gpurun_out", f"prof_{args.tag}")   # default output folder, relative to the repository root
    os.makedirs(out, exist_ok=True)
    import pandas as pd
    pd.set_option("display.width", 250)
    pd.set_option("display.max_colwidth", 90)

    commands = [run(out, "stats", ["--kernel-trace", "--stats"], cmd, args.limit)]
    lines = [f"rocprofv3 summary: {args.title or args.tag}, MI355X",
             f"kernel sources: hash {kernel_source_hash()} (paper_2308_03209_amd/csrc)",
             "commands (run from the repository root with TMPDIR=/tmp; this file is written by",
             "python -m paper_2308_03209_amd.rocprof_summary, which issues them one after the other):"]
    st = pd.read_csv(find_csv(os.path.join(out, "stats"), "kernel_stats.csv"))
    st["Name"] = st["Name"].map(lambda k: instance_name(k)[:80])
    t = st[["Name", "Calls", "TotalDurationNs", "AverageNs", "Percentage", "MinNs", "MaxNs"]].head(18).copy()
    t["Total_ms"] = t.pop("TotalDurationNs") / 1e6
    t["Avg_us"] = t.pop("AverageNs") / 1e3
    t["Min_us"] = t.pop("MinNs") / 1e3
    t["Max_us"] = t.pop("MaxNs") / 1e3
    body = ["== rocprofv3 --kernel-trace --stats: per-kernel time (all launches of the run, warm-up included) ==",
            t.to_string(index=False, float_format=lambda x: f"{x:.2f}"), ""]
    traffic = {}
    if not args.no_counters:
        commands.append(run(out, "fetch", ["--pmc", "FETCH_SIZE"], cmd, args.limit))
        commands.append(run(out, "write", ["--pmc", "WRITE_SIZE"], cmd, args.limit))
        commands.append(run(out, "tcc", ["--pmc", "TCC_HIT_sum", "TCC_MISS_sum"], cmd, args.limit))

        def counters(name):
            df = pd.read_csv(find_csv(os.path.join(out, name), "counter_collection.csv"))
            df["k"] = df["Kernel_Name"].map(instance_name)
            return df

        f, w, h = counters("fetch"), counters("write"), counters("tcc")
        if args.fetch_scale is not None and args.write_scale is not None:
            sf, sw = args.fetch_scale, args.write_scale
            body += ["== rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (KiB per dispatch) ==",
                     f"scale factors given on the command line (from the calibration copy of another run): "
                     f"fetch x{sf:.3f}, write x{sw:.3f}", ""]
        else:
            is_copy = lambda df: df.k.str.contains("copyBuffer|direct_copy|elementwise_kernel")
            cf = f[is_copy(f)]["Counter_Value"].max()
            cw = w[is_copy(w)]["Counter_Value"].max()
            sf, sw = 1048576.0 / cf, 1048576.0 / cw
            body += ["== rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (KiB per dispatch), calibration ==",
                     f"plain 1 GiB device copy (1,048,576 KiB read, 1,048,576 KiB written): FETCH_SIZE = {cf:.0f}, "
                     f"WRITE_SIZE = {cw:.0f}", f"scale factors: fetch x{sf:.3f}, write x{sw:.3f}", ""]
        ours = lambda df: df[df["Kernel_Name"].str.contains(args.kernels)]
        gf = ours(f).groupby("k")["Counter_Value"].agg(["mean", "max", "count"])
        gw = ours(w).groupby("k")["Counter_Value"].agg(["mean", "max"])
        gh = ours(h).pivot_table(index="k", columns="Counter_Name", values="Counter_Value", aggfunc="mean")
        tab = pd.DataFrame({"dispatches": gf["count"], "fetch_GB_mean": gf["mean"] * 1024 * sf / 1e9,
                            "fetch_GB_max": gf["max"] * 1024 * sf / 1e9,
                            "write_GB_mean": gw["mean"] * 1024 * sw / 1e9, "write_GB_max": gw["max"] * 1024 * sw / 1e9})
        tab["L2_hit_rate"] = gh["TCC_HIT_sum"] / (gh["TCC_HIT_sum"] + gh["TCC_MISS_sum"])
        body += ["== HBM-side traffic per dispatch of the library's kernels (scaled, GB = 1e9 bytes; per template "
                 "instance, mean over its dispatches) ==",
                 tab.sort_values("fetch_GB_mean", ascending=False).to_string(float_format=lambda x: f"{x:.3f}"), ""]
        for k in gf.index:
            traffic[k] = float(gf.loc[k, "mean"] * 1024 * sf + (gw.loc[k, "mean"] * 1024 * sw if k in gw.index else 0.0))
        json.dump({"source": "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, scaled by a plain 1 GiB copy (see the summary "
                             "next to this file)", "kernel_source_hash": kernel_source_hash(),
                   "fetch_scale": sf, "write_scale": sw, "bytes_per_launch": traffic},
                  open(os.path.join(out, "traffic.json"), "w"), indent=1)
    if args.append_stdout:
        own = [l.rstrip() for l in open(os.path.join(out, "stats.log")) if not re.match(r"^[WEI]\d{8} ", l)]
        body += ["== what the program printed during the --kernel-trace run ==", *own, ""]
    lines += ["  " + c for c in commands] + [""] + body
    text = "\n".join(lines) + "\n"
    open(os.path.join(out, "summary.txt"), "w").write(text)
    print(text)
    return 0


if __name__ == "__main__":
    sys.exit(main())
