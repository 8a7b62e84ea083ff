"""Turn rocprofv3 CSV output into the short text summaries kept under profiles/.

    python -m paper_2304_11277_amd.profile_summary stats  <dir>/<prefix>  <out.md>  "<command>"
    python -m paper_2304_11277_amd.profile_summary traffic <fetch> <write> <fetch_probe> <write_probe> \
            <out.md> <traffic.json> <workload:mode> "<commands>"

`stats` condenses --kernel-trace --stats output (per kernel and grid size:
calls, min / median / mean duration).  `traffic` converts FETCH_SIZE and
WRITE_SIZE (KiB per dispatch) of the library's kernels into HBM bytes per
launch, scaling each counter by what it reads for the plain copy kernel of
known size (bench.py --probe-copy).
"""
from __future__ import annotations

import collections
import csv
import json
import sys

LIB_KERNELS = (("batch_kernel", "batch"), ("reduce_adam_unshard_kernel", "reduce_adam+unshard"),
               ("unshard_lp_kernel", "unshard"), ("gather_lp_kernel", "unshard_lp"), ("accumulate_kernel", "grad_accumulate"), ("unshard", "unshard"),
               ("reduce_kernel", "reduce_adam"), ("adam_kernel", "adam"),
               ("pack_kernel", "pack"), ("fsdp_probe_copy", "probe_copy"))


def short_name(kernel_name: str):
    for key, short in LIB_KERNELS:
        if key in kernel_name:
            return short
    return None


def stats(prefix: str, out_md: str, command: str) -> None:
    rows = list(csv.DictReader(open(prefix + "_kernel_trace.csv")))
    per = collections.defaultdict(list)
    for r in rows:
        s = short_name(r["Kernel_Name"])
        if s:
            per[(s, r["Kernel_Name"].split("(")[0][-60:], int(r["Grid_Size_X"]), int(r["Workgroup_Size_X"]),
                 int(r["VGPR_Count"]))].append(int(r["End_Timestamp"]) - int(r["Start_Timestamp"]))
    lines = ["# rocprofv3 kernel trace summary", "", "Command:", "", "    " + command, "",
             "Durations in microseconds, per kernel and grid size (threads).", "",
             "| kernel | grid threads | block | VGPRs | calls | min | median | mean |", "|---|---|---|---|---|---|---|---|"]
    for (s, _full, grid, wg, vgpr), v in sorted(per.items()):
        v.sort()
        lines.append(f"| {s} | {grid} | {wg} | {vgpr} | {len(v)} | {v[0] / 1e3:.2f} | {v[len(v) // 2] / 1e3:.2f} | "
                     f"{sum(v) / len(v) / 1e3:.2f} |")
    tot = collections.defaultdict(lambda: [0, 0])
    for (s, *_), v in per.items():
        tot[s][0] += len(v)
        tot[s][1] += sum(v)
    lines += ["", "| kernel | calls | average over all launches (us) |", "|---|---|---|"]
    for s, (n, t) in sorted(tot.items()):
        lines.append(f"| {s} | {n} | {t / n / 1e3:.2f} |")
    lines += ["", "rocprofv3 --stats (top rows of *_kernel_stats.csv):", ""]
    with open(prefix + "_kernel_stats.csv") as fh:
        for i, r in enumerate(csv.DictReader(fh)):
            if i >= 6:
                break
            lines.append(f"    {r['Name'][:90]:90s} calls={r['Calls']} avg_ns={float(r['AverageNs']):.0f} pct={r['Percentage']}")
    open(out_md, "w").write("\n".join(lines) + "\n")


def _counters(prefix: str, counter: str):
    per = collections.defaultdict(list)
    for r in csv.DictReader(open(prefix + "_counter_collection.csv")):
        s = short_name(r["Kernel_Name"])
        if s and r["Counter_Name"] == counter:
            per[(s, int(r["Grid_Size"]))].append(float(r["Counter_Value"]))
    return {k: sum(v) / len(v) for k, v in per.items()}, {k: len(v) for k, v in per.items()}


def traffic(fetch, write, fetch_probe, write_probe, out_md, out_json, key_prefix, commands) -> None:
    probe_kib = 256 * 1024.0
    f_probe, _ = _counters(fetch_probe, "FETCH_SIZE")
    w_probe, _ = _counters(write_probe, "WRITE_SIZE")
    f_scale = probe_kib / [v for k, v in f_probe.items() if k[0] == "probe_copy"][0]
    w_scale = probe_kib / [v for k, v in w_probe.items() if k[0] == "probe_copy"][0]
    f, fn = _counters(fetch, "FETCH_SIZE")
    w, _ = _counters(write, "WRITE_SIZE")
    lines = ["# HBM traffic per launch from rocprofv3 --pmc", "", "Commands (one counter per run):", ""]
    lines += ["    " + c for c in commands.split(" ;; ")]
    lines += ["", f"Calibration: the plain copy kernel moves 262144 KiB each way; FETCH_SIZE reads "
              f"{probe_kib / f_scale:.1f}, WRITE_SIZE reads {probe_kib / w_scale:.1f}, so the scale factors are "
              f"{f_scale:.5f} (fetch) and {w_scale:.5f} (write).", "",
              "| kernel | grid threads | launches | FETCH_SIZE KiB | WRITE_SIZE KiB | read MB | written MB | total MB |",
              "|---|---|---|---|---|---|---|---|"]
    per_kernel = collections.defaultdict(lambda: [0, 0.0])
    for k in sorted(f):
        rd = f[k] * f_scale * 1024 / 1e6
        wr = w.get(k, 0.0) * w_scale * 1024 / 1e6
        lines.append(f"| {k[0]} | {k[1]} | {fn[k]} | {f[k]:.1f} | {w.get(k, 0.0):.1f} | {rd:.2f} | {wr:.2f} | {rd + wr:.2f} |")
        per_kernel[k[0]][0] += fn[k]
        per_kernel[k[0]][1] += fn[k] * (rd + wr) * 1e6
    out = {}
    lines += ["", "Launch-weighted average HBM bytes per launch:", ""]
    for s, (n, b) in sorted(per_kernel.items()):
        if s in ("probe_copy", "pack"):
            continue
        out[f"{key_prefix}:{s}"] = round(b / n)
        lines.append(f"- {s}: {b / n / 1e6:.2f} MB")
    open(out_md, "w").write("\n".join(lines) + "\n")
    try:
        cur = json.load(open(out_json))
    except (OSError, ValueError):
        cur = {}
    cur.update(out)
    json.dump(cur, open(out_json, "w"), indent=1, sort_keys=True)


if __name__ == "__main__":
    if sys.argv[1] == "stats":
        stats(*sys.argv[2:5])
    elif sys.argv[1] == "traffic":
        traffic(*sys.argv[2:10])
    else:
        raise SystemExit(__doc__)
