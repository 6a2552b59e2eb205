"""Turn the CSV output of three rocprofv3 runs of bench.py into the short text
summaries kept under profiles/.

Expected in <in_dir> (see the commands echoed into the summaries):
  kt_kernel_stats.csv            rocprofv3 --kernel-trace --stats -f csv -o kt
  fetch_counter_collection.csv   rocprofv3 --pmc FETCH_SIZE -f csv -o fetch
  write_counter_collection.csv   rocprofv3 --pmc WRITE_SIZE -f csv -o write

The counters are scaled by what they read for the one plain 256 MiB device
copy that bench.py issues before its timed region (__amd_rocclr_copyBuffer).

usage: python profile_summary.py <in_dir> <out_dir> [tag]
(the digits in the tag name the bench.py --config the runs were made with)
"""
from __future__ import annotations

import collections
import csv
import json
import os
import sys

CAL_BYTES = 256 << 20
CMD_KT = ("rocprofv3 --kernel-trace --stats -f csv -d <dir> -o kt -- "
          "python3 bench.py --config {cfg} --steps 5 --warmup 1 --no-cpu-baseline --no-extra")
CMD_PMC = ("rocprofv3 --pmc {c} -f csv -d <dir> -o {o} -- "
           "python3 bench.py --config {cfg} --steps 2 --warmup 1 --no-cpu-baseline --no-extra --no-graph")


def _short(name: str) -> str:
    name = name.replace("void ", "").replace("qspec::", "")
    return name.split("(")[0][:70]


def _family(name: str) -> str:
    if name.startswith("gemm_stream_kernel<"):
        return "gemm_stream_kernel<" + ",".join(name.split("<")[1].split(",")[:2]) + ", *>"
    return name.split("<")[0] + ("<*>" if "<" in name else "")


def _counter_means(path):
    agg = collections.defaultdict(list)
    with open(path) as f:
        for r in csv.DictReader(f):
            agg[_short(r["Kernel_Name"])].append(float(r["Counter_Value"]))
    return {k: (len(v), sum(v) / len(v), max(v)) for k, v in agg.items()}


def main(in_dir: str, out_dir: str, tag: str = "bench_config2") -> None:
    os.makedirs(out_dir, exist_ok=True)
    cfg = "".join(ch for ch in tag if ch.isdigit()) or "2"
    ours = ("gemm_", "quant_act", "pack_", "unpack_", "transpose_", "argmax_", "accept_", "kv_overwrite")
    lines = [f"# rocprofv3 kernel statistics, {tag}", f"# command: {CMD_KT.format(cfg=cfg)}",
             f"# {'kernel':68s} {'calls':>6s} {'avg_us':>9s} {'min_us':>9s} {'max_us':>9s} {'pct':>6s}"]
    fam = collections.OrderedDict()
    with open(os.path.join(in_dir, "kt_kernel_stats.csv")) as f:
        for r in csv.DictReader(f):
            n = _short(r["Name"])
            if n.startswith(ours):
                lines.append(f"  {n:68s} {int(r['Calls']):6d} {float(r['AverageNs'])/1e3:9.2f} "
                             f"{float(r['MinNs'])/1e3:9.2f} {float(r['MaxNs'])/1e3:9.2f} {float(r['Percentage']):6.2f}")
                if n.startswith("gemm_"):
                    e = fam.setdefault(_family(n), [0, 0.0, 0.0])
                    e[0] += int(r["Calls"]); e[1] += float(r["TotalDurationNs"]); e[2] += float(r["Percentage"])
    lines.append("# the same, summed over the instances of one kernel template and mode (the unit bench.py's")
    lines.append("# roofline object is about)")
    for n, (calls, tot, pct) in fam.items():
        lines.append(f"  {n:68s} {calls:6d} {tot/calls/1e3:9.2f} {'':9s} {'':9s} {pct:6.2f}")
    with open(os.path.join(out_dir, f"{tag}_kernel_stats.txt"), "w") as f:
        f.write("\n".join(lines) + "\n")

    fetch = _counter_means(os.path.join(in_dir, "fetch_counter_collection.csv"))
    write = _counter_means(os.path.join(in_dir, "write_counter_collection.csv"))
    cal = "__amd_rocclr_copyBuffer"
    # the largest reading among the runtime's copy dispatches is the 256 MiB copy (torch
    # issues the same copy kernel for a few tiny tensors as well)
    f_scale = CAL_BYTES / 1024.0 / fetch[cal][2]
    w_scale = CAL_BYTES / 1024.0 / write[cal][2]
    lines = [f"# HBM traffic per dispatch from rocprofv3 counters, {tag}",
             f"# commands: {CMD_PMC.format(c='FETCH_SIZE', o='fetch', cfg=cfg)}",
             f"#           {CMD_PMC.format(c='WRITE_SIZE', o='write', cfg=cfg)}",
             f"# calibration: one 256 MiB device copy reads FETCH_SIZE = {fetch[cal][2]:.1f} KiB, "
             f"WRITE_SIZE = {write[cal][2]:.1f} KiB",
             f"#   -> scale factors {f_scale:.3f} (fetch), {w_scale:.3f} (write)",
             f"# {'kernel':68s} {'n':>6s} {'fetch_MB':>10s} {'write_MB':>10s} {'total_MB':>10s}"]
    per_launch = {}
    for k in sorted(fetch):
        if not k.startswith(ours):
            continue
        fb = fetch[k][1] * f_scale * 1024
        wb = write.get(k, (0, 0.0, 0.0))[1] * w_scale * 1024
        per_launch[k] = int(fb + wb)
        lines.append(f"  {k:68s} {fetch[k][0]:6d} {fb/1e6:10.2f} {wb/1e6:10.2f} {(fb+wb)/1e6:10.2f}")
    with open(os.path.join(out_dir, f"{tag}_hbm_counters.txt"), "w") as f:
        f.write("\n".join(lines) + "\n")
    # one table for bench.py, keyed by configuration and then by kernel symbol (the same
    # symbol moves different byte counts in different configurations)
    path = os.path.join(out_dir, "hbm_traffic.json")
    by_config, sources = {}, []
    try:
        with open(path) as f:
            old = json.load(f)
        by_config, sources = old.get("by_config", {}), old.get("sources", [])
    except (OSError, ValueError):
        pass
    by_config[cfg] = per_launch
    src = f"{tag}_hbm_counters.txt"
    if src not in sources:
        sources.append(src)
    with open(path, "w") as f:
        json.dump({"sources": sources, "fetch_scale": round(f_scale, 4),
                   "write_scale": round(w_scale, 4), "by_config": by_config}, f, indent=1)
        f.write("\n")


if __name__ == "__main__":
    if len(sys.argv) < 3:
        sys.exit(__doc__)
    main(*sys.argv[1:4])
