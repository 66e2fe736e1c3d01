"""Turns rocprofv3 CSV output of `bench.py` runs into the short text summaries kept
under profiles/ and into the per-launch HBM traffic figures bench.py reports.

Three runs of the same bench command are expected (commands printed in the summary):
  trace : rocprofv3 --kernel-trace --stats --output-format csv -d <dir>/trace -o t -- python3 bench.py ...
  fetch : rocprofv3 --pmc FETCH_SIZE       --output-format csv -d <dir>/fetch -o f -- python3 bench.py ...
  write : rocprofv3 --pmc WRITE_SIZE       --output-format csv -d <dir>/write -o w -- python3 bench.py ...

FETCH_SIZE / WRITE_SIZE are read in KiB per dispatch and scaled by what the same
counter reads for the plain device-to-device copy of known size that bench.py
performs (hipMemcpy D2D of one arena, kernel __amd_rocclr_copyBuffer).

The bench line each run printed is expected next to its output (<dir>/bench_trace.json, the
JSON line of the trace run): the command's own arguments are taken from its "argv" field, so a
summary cannot name another command than the one that was profiled.

  python -m paper_2508_15706_amd.rocprof_summary <dir> <arena_bytes | auto> <out.md> [<traffic.json>]
  (auto: the arena size the bench line reports)
"""
from __future__ import annotations

import collections
import csv
import glob
import json
import os
import re
import sys

COPY_KERNEL = "__amd_rocclr_copyBuffer"


def short_name(name: str):
    n = name.replace("(anonymous namespace)::", "")
    if n.startswith("void "):
        n = n[5:]
    if n.startswith("k_"):
        return n.split("(")[0]
    if COPY_KERNEL in n:
        return COPY_KERNEL
    return None


def _find(d, pattern):
    hits = glob.glob(os.path.join(d, "**", pattern), recursive=True)
    return hits[0] if hits else None


def read_counter(d, sub, counter):
    path = _find(os.path.join(d, sub), "*counter_collection.csv")
    vals = collections.defaultdict(list)
    if not path:
        return vals
    for r in csv.DictReader(open(path)):
        s = short_name(r["Kernel_Name"])
        if s and r["Counter_Name"] == counter:
            vals[s].append(float(r["Counter_Value"]))
    return vals


def read_stats(d):
    path = _find(os.path.join(d, "trace"), "*kernel_stats.csv")
    out = {}
    if not path:
        return out
    for r in csv.DictReader(open(path)):
        s = short_name(r["Name"])
        if s:
            out[s] = (int(r["Calls"]), float(r["AverageNs"]), float(r["MinNs"]), float(r["MaxNs"]))
    return out


def read_last_calls(d, last_n):
    """Mean duration (us) of the last `last_n` dispatches of each kernel: the timed
    steps of bench.py come last, after set-up and the other residual mode."""
    path = _find(os.path.join(d, "trace"), "*kernel_trace.csv")
    durs = collections.defaultdict(list)
    if not path:
        return {}
    for r in csv.DictReader(open(path)):
        s = short_name(r["Kernel_Name"])
        if s:
            durs[s].append((int(r["Start_Timestamp"]), (int(r["End_Timestamp"]) - int(r["Start_Timestamp"])) / 1e3))
    out = {}
    for k, v in durs.items():
        v.sort()
        tail = [x[1] for x in v[-last_n:]]
        out[k] = sum(tail) / len(tail)
    return out


def summarize(d, arena_bytes):
    fetch = read_counter(d, "fetch", "FETCH_SIZE")
    write = read_counter(d, "write", "WRITE_SIZE")
    stats = read_stats(d)
    last = read_last_calls(d, int(os.environ.get("SL_LAST_N", "8")))
    known_kib = arena_bytes / 1024.0
    # the largest copies are the whole-arena ones
    f_copy = max(fetch.get(COPY_KERNEL, [0.0]) or [0.0])
    w_copy = max(write.get(COPY_KERNEL, [0.0]) or [0.0])
    f_scale = known_kib / f_copy if f_copy else float("nan")
    w_scale = known_kib / w_copy if w_copy else float("nan")
    kernels = {}
    for k in sorted(set(fetch) | set(write) | set(stats)):
        if k == COPY_KERNEL:
            continue
        f = sum(fetch[k]) / len(fetch[k]) if fetch.get(k) else None
        w = sum(write[k]) / len(write[k]) if write.get(k) else None
        kernels[k] = {
            "calls": stats.get(k, (0, 0, 0, 0))[0],
            "avg_us": stats.get(k, (0, 0, 0, 0))[1] / 1e3,
            "min_us": stats.get(k, (0, 0, 0, 0))[2] / 1e3,
            "max_us": stats.get(k, (0, 0, 0, 0))[3] / 1e3,
            "timed_us": last.get(k),
            "fetch_bytes": None if f is None else f * 1024.0 * f_scale,
            "write_bytes": None if w is None else w * 1024.0 * w_scale,
        }
    return {"fetch_scale": f_scale, "write_scale": w_scale, "copy_fetch_KiB": f_copy,
            "copy_write_KiB": w_copy, "copy_known_KiB": known_kib, "kernels": kernels}


def render(summary, bench_args, title):
    s = summary
    lines = [f"# {title}", "",
             "Commands (each from /tmp with TMPDIR=/tmp; repository at $R, profiler output under $OUT):", "",
             f"    rocprofv3 --kernel-trace --stats --output-format csv -d $OUT/trace -o t -- python3 $R/bench.py {bench_args}",
             f"    rocprofv3 --pmc FETCH_SIZE --output-format csv -d $OUT/fetch -o f -- python3 $R/bench.py {bench_args}",
             f"    rocprofv3 --pmc WRITE_SIZE --output-format csv -d $OUT/write -o w -- python3 $R/bench.py {bench_args}",
             f"    python3 -m paper_2508_15706_amd.rocprof_summary $OUT auto <this file>     (with the trace run's bench line in $OUT/bench_trace.json)", "",
             "(The two counter runs may take fewer steps, e.g. --steps 2 --warmup 1: the counters are read per dispatch.)", "",
             "Counter scaling: the whole-arena device copy bench.py performs (`__amd_rocclr_copyBuffer`, "
             f"{s['copy_known_KiB']:.0f} KiB read and written) reads FETCH_SIZE = {s['copy_fetch_KiB']:.1f} KiB "
             f"(scale {s['fetch_scale']:.4f}) and WRITE_SIZE = {s['copy_write_KiB']:.1f} KiB "
             f"(scale {s['write_scale']:.4f}).", "",
             "`timed us` = mean over the last dispatches of the kernel, i.e. the timed steps of the bench "
             "(the earlier calls are set-up from e = 0 and the other residual mode).", "",
             "| kernel | calls | avg us | min us | max us | timed us | HBM read / launch (GB) | HBM write / launch (GB) |",
             "|---|---|---|---|---|---|---|---|"]
    for k, v in s["kernels"].items():
        fb = "-" if v["fetch_bytes"] is None else f"{v['fetch_bytes'] / 1e9:.4f}"
        wb = "-" if v["write_bytes"] is None else f"{v['write_bytes'] / 1e9:.4f}"
        tu = "-" if v.get("timed_us") is None else f"{v['timed_us']:.1f}"
        lines.append(f"| {k} | {v['calls']} | {v['avg_us']:.1f} | {v['min_us']:.1f} | {v['max_us']:.1f} | {tu} | {fb} | {wb} |")
    lines.append("")
    return "\n".join(lines)


def main(argv):
    if len(argv) < 4:
        print(__doc__)
        return 2
    d, out_md = argv[1], argv[3]
    bench_args, arena_bytes = None, None
    line_path = os.path.join(d, "bench_trace.json")
    if os.path.exists(line_path):
        for line in open(line_path):
            if line.startswith("{"):
                rec = json.loads(line)
                bench_args = rec.get("argv")
                arena_bytes = rec.get("config", {}).get("arena_bytes")
    if bench_args is None:
        print(f"{line_path} holds no bench line with an argv field: the profiled command is unknown", file=sys.stderr)
        return 2
    if argv[2] != "auto":
        arena_bytes = float(argv[2])
    summary = summarize(d, float(arena_bytes))
    title = os.environ.get("SL_PROFILE_TITLE", "rocprofv3 summary")
    with open(out_md, "w") as f:
        f.write(render(summary, bench_args, title))
    if len(argv) > 4:
        traffic = {k: {"fetch_bytes": v["fetch_bytes"], "write_bytes": v["write_bytes"], "avg_us": v["avg_us"],
                       "timed_us": v.get("timed_us")}
                   for k, v in summary["kernels"].items()}
        import hashlib
        h = hashlib.sha256()
        csrc = os.path.join(os.path.dirname(os.path.abspath(__file__)), "csrc")
        for name in sorted(os.listdir(csrc)):       # the same hash bench.py checks before it quotes the file
            if name.endswith((".hip", ".h")):
                h.update(name.encode())
                h.update(open(os.path.join(csrc, name), "rb").read())
        with open(argv[4], "w") as f:
            json.dump({"bench_args": bench_args, "sources_sha": h.hexdigest()[:16],
                       "fetch_scale": summary["fetch_scale"],
                       "write_scale": summary["write_scale"], "kernels": traffic}, f, indent=1)
    return 0


if __name__ == "__main__":
    sys.exit(main(sys.argv))
