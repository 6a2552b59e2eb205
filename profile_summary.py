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

If <in_dir> also holds sqa_counter_collection.csv / sqb_counter_collection.csv (two more
--pmc runs, see CMD_SQ), a table of those counters per GEMM kernel is written as
<tag>_sq_counters.txt: instruction counts per wave, matrix-unit and vector-ALU share of
the SIMD cycles, LDS bank conflicts.
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


SQ_A = "SQ_WAVES SQ_BUSY_CYCLES SQ_WAVE_CYCLES SQ_INSTS_VALU SQ_INSTS_MFMA SQ_VALU_MFMA_BUSY_CYCLES SQ_INSTS_LDS SQ_LDS_BANK_CONFLICT"
SQ_B = "SQ_ACTIVE_INST_VALU SQ_ACTIVE_INST_LDS SQ_WAIT_INST_ANY SQ_WAIT_ANY SQ_ACTIVE_INST_ANY SQ_INSTS_SALU SQ_INSTS_VMEM GRBM_GUI_ACTIVE"
CMD_SQ = ("rocprofv3 --pmc {c} -f csv -d <dir> -o {o} -- "
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


def sq_table(in_dir: str, out_dir: str, tag: str) -> None:
    """Mean per dispatch of the SQ counters of the two optional runs, per GEMM kernel, with
    the ratios that read directly: vector / matrix instructions per wave, share of SIMD
    cycles the matrix unit is busy (MFMA busy cycles / (4 SIMDs x 256 CUs x GUI-active cycles
    per XCD)), wave time spent issuing / waiting."""
    paths = [os.path.join(in_dir, f"{o}_counter_collection.csv") for o in ("sqa", "sqb")]
    if not all(os.path.exists(q) for q in paths):
        return
    cfg = "".join(ch for ch in tag if ch.isdigit()) or "2"
    agg = collections.defaultdict(lambda: collections.defaultdict(list))
    for q in paths:
        with open(q) as f:
            for r in csv.DictReader(f):
                agg[_short(r["Kernel_Name"])][r["Counter_Name"]].append(float(r["Counter_Value"]))
    lines = [f"# SQ counters per dispatch (mean), {tag}",
             f"# commands: {CMD_SQ.format(c=SQ_A, o='sqa', cfg=cfg)}",
             f"#           {CMD_SQ.format(c=SQ_B, o='sqb', cfg=cfg)}"]
    for k in sorted(agg):
        if not k.startswith("gemm_"):
            continue
        m = {c: sum(v) / len(v) for c, v in agg[k].items()}
        lines.append(f"  {k}  ({len(next(iter(agg[k].values())))} dispatches)")
        for c in sorted(m):
            lines.append(f"      {c:28s} {m[c]:16.1f}")
        w = m.get("SQ_WAVES", 0.0)
        if w > 0 and "GRBM_GUI_ACTIVE" in m:
            simd_cycles = m["GRBM_GUI_ACTIVE"] / 8.0 * 4 * 256        # the counter adds the 8 XCDs
            lines.append(f"      -> per wave: {m.get('SQ_INSTS_VALU', 0) / w:.0f} vector, {m.get('SQ_INSTS_MFMA', 0) / w:.0f} matrix, "
                         f"{m.get('SQ_INSTS_LDS', 0) / w:.0f} LDS, {m.get('SQ_INSTS_VMEM', 0) / w:.0f} vector-memory instructions")
            lines.append(f"      -> matrix unit busy {100 * m.get('SQ_VALU_MFMA_BUSY_CYCLES', 0) / simd_cycles:.1f} % of SIMD cycles, "
                         f"vector ALU issuing {100 * 4 * m.get('SQ_ACTIVE_INST_VALU', 0) / simd_cycles:.1f} %; "
                         f"LDS bank-conflict cycles {m.get('SQ_LDS_BANK_CONFLICT', 0):.0f}")
            if m.get("SQ_WAVE_CYCLES"):
                lines.append(f"      -> of a wave's lifetime: issuing {100 * m.get('SQ_ACTIVE_INST_ANY', 0) / m['SQ_WAVE_CYCLES']:.0f} %, "
                             f"waiting on a counter {100 * m.get('SQ_WAIT_INST_ANY', 0) / m['SQ_WAVE_CYCLES']:.0f} %")
    with open(os.path.join(out_dir, f"{tag}_sq_counters.txt"), "w") as f:
        f.write("\n".join(lines) + "\n")


if __name__ == "__main__":
    if len(sys.argv) < 3:
        sys.exit(__doc__)
    main(*sys.argv[1:4])
    sq_table(sys.argv[1], sys.argv[2], sys.argv[3] if len(sys.argv) > 3 else "bench_config2")
