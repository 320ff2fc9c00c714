"""Turns rocprofv3 CSV output of ``bench.py`` into the short text summaries kept under
``profiles/``.

    python -m paper_2307_12983_amd.profile_tools stats   <kernel_stats.csv> <bench.json> <out.md> <title> [bench.py arguments]
    python -m paper_2307_12983_amd.profile_tools traffic <fetch_counter_collection.csv> <write_counter_collection.csv> \
                                                         <kernel name> <out.txt> [bench.py arguments]
    python -m paper_2307_12983_amd.profile_tools counters <counter_collection.csv> <out.txt> <counters of the pass> [bench.py arguments]

``counters`` averages one pass of shader counters (at most 8 ``SQ_`` counters fit one pass) per
launch for every kernel of the library and relates them to the busy cycles of the compute units.

``traffic`` scales the FETCH_SIZE / WRITE_SIZE readings (KiB per dispatch) of the named kernel by
what the same counters read for bench.py's calibration copy (one ``copy_kernel`` launch that
moves CAL_COPY_FLOATS floats: the dispatch of that kernel with the largest grid), and records the
SHA-256 of the kernel sources so that ``bench.py`` drops the figure once a kernel changes.
"""
from __future__ import annotations

import csv
import glob
import hashlib
import json
import os
import re
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CAL_COPY_FLOATS = 64 * 1024 * 1024          # floats moved by bench.py's calibration copy

GEMM_MODES = {"0": "nn", "1": "nt", "2": "tn"}
GEMM_TILES = {("2", "2", "2", "2"): "128x128", ("2", "2", "1", "1"): "64x64", ("4", "1", "1", "1"): "128x32",
              ("2", "2", "2", "1"): "128x64"}


def source_hash() -> str:
    """SHA-256 over the kernel sources (any edit invalidates stored traffic figures)."""
    h = hashlib.sha256()
    for f in sorted(glob.glob(os.path.join(HERE, "csrc", "*"))):
        h.update(os.path.basename(f).encode())
        h.update(open(f, "rb").read())
    return h.hexdigest()


def short_name(profiler_name: str) -> str:
    """Maps a demangled kernel name to the name bench.py / pql_profile_end use."""
    m = re.search(r"gemm_grouped_kernel<(\d), (\d), (\d), (\d), (\d), (true|false)(?:, \d+)?>", profiler_name)
    if m:
        tile = GEMM_TILES.get(m.group(2, 3, 4, 5), "?")
        return "gemm_grouped_%s_%s%s" % (GEMM_MODES.get(m.group(1), "?"), tile, "_noise" if m.group(6) == "true" else "")
    m = re.search(r"head_kernel<\d+, (true|false)>", profiler_name)
    if m:
        return "head_kernel_policy" if m.group(1) == "true" else "head_kernel_critic"
    m = re.search(r"pql::(\w+)", profiler_name)
    return m.group(1) if m else profiler_name


def stats_summary(stats_csv, bench_json, out, title, bench_args=""):
    st = list(csv.DictReader(open(stats_csv)))
    b = json.loads(open(bench_json).read().strip().splitlines()[-1])
    with open(out, "w") as f:
        f.write("# %s\n\n" % title)
        f.write("Command (from the repository root, on one MI355X):\n\n")
        f.write("    rocprofv3 --kernel-trace --stats --output-format csv -d <out>/prof_bench -o bench -- python3 bench.py%s\n" % ((" " + bench_args) if bench_args else ""))
        f.write("    python -m paper_2307_12983_amd.profile_tools stats <out>/prof_bench/bench_kernel_stats.csv <bench line> <this file> <title>\n\n")
        f.write("Kernel summary (`bench_kernel_stats.csv`), all launches of the process (ring fill, calibration copy, "
                "warm-up, timed steps, Actor loop, event pass):\n\n")
        f.write("| kernel (name in bench.py) | calls | avg us | min us | max us | % of GPU time |\n|---|---|---|---|---|---|\n")
        for r in st:
            if float(r["Percentage"]) < 0.05:
                continue
            f.write("| `%s` (%s) | %s | %.2f | %.2f | %.2f | %s |\n" % (
                r["Name"].replace("|", "/")[:100], short_name(r["Name"]), r["Calls"], float(r["AverageNs"]) / 1e3,
                float(r["MinNs"]) / 1e3, float(r["MaxNs"]) / 1e3, r["Percentage"]))
        f.write("\nbench.py line of the same run (its per-kernel averages come from HIP events attached to each "
                "dispatch; with the profiler attached they can read a few us high, in a plain run they match the "
                "table):\n\n")
        f.write("    value = %.1f %s, ms_per_step = %.4f\n    roofline = %s\n" % (
            b["value"], b["unit"], b["ms_per_step"], json.dumps(b["roofline"])))
        f.write("    kernels = %s\n" % json.dumps([{k: (round(v, 2) if isinstance(v, float) else v) for k, v in e.items()}
                                                   for e in b["kernels"]]))


def _per_dispatch(counter_csv, counter):
    rows = [r for r in csv.DictReader(open(counter_csv)) if r["Counter_Name"] == counter]
    return [(r["Kernel_Name"], int(r["Grid_Size"]), float(r["Counter_Value"])) for r in rows]


def traffic_summary(fetch_csv, write_csv, kernel, out, bench_args="--steps 96 --warmup 16 --no-cpu-baseline --no-secondary"):
    res = {}
    for label, path, counter in (("fetch", fetch_csv, "FETCH_SIZE"), ("write", write_csv, "WRITE_SIZE")):
        d = _per_dispatch(path, counter)
        cal = max((x for x in d if "copy_kernel" in x[0]), key=lambda x: x[1])
        mine = [x[2] for x in d if short_name(x[0]) == kernel]
        if not mine:
            raise SystemExit("kernel %s not found in %s" % (kernel, path))
        mine = mine[len(mine) // 4:]                       # skip warm-up launches
        avg_kib = sum(mine) / len(mine)
        scale = (CAL_COPY_FLOATS * 4.0) / (cal[2] * 1024.0)
        res[label] = dict(avg_kib=avg_kib, cal_kib=cal[2], scale=scale, bytes=avg_kib * 1024.0 * scale, n=len(mine))
    total = res["fetch"]["bytes"] + res["write"]["bytes"]
    with open(out, "w") as f:
        f.write("# HBM traffic per launch of %s (bench.py %s)\n" % (kernel, bench_args))
        f.write("# Commands (two counter passes, each its own run; from the repository root on one MI355X):\n")
        f.write("#   rocprofv3 --pmc FETCH_SIZE --output-format csv -d <out>/pmc_fetch -o b -- python3 bench.py %s\n" % bench_args)
        f.write("#   rocprofv3 --pmc WRITE_SIZE --output-format csv -d <out>/pmc_write -o b -- python3 bench.py %s\n" % bench_args)
        f.write("#   python -m paper_2307_12983_amd.profile_tools traffic <out>/pmc_fetch/b_counter_collection.csv <out>/pmc_write/b_counter_collection.csv %s <this file>\n" % kernel)
        f.write("# Each counter (KiB per dispatch) is scaled by what it reads for the calibration copy of %d floats\n" % CAL_COPY_FLOATS)
        f.write("# (%d bytes read, as many written).\n" % (CAL_COPY_FLOATS * 4))
        f.write("kernel=%s\n" % kernel)
        f.write("source_sha256=%s\n" % source_hash())
        for label in ("fetch", "write"):
            r = res[label]
            f.write("%s_kib_per_launch=%.1f\n%s_calibration_kib=%.1f\n%s_scale=%.4f\n%s_bytes_per_launch=%.0f\n" % (
                label, r["avg_kib"], label, r["cal_kib"], label, r["scale"], label, r["bytes"]))
        f.write("traffic_bytes_per_launch=%.0f\n" % total)
        # the other kernels of the library in the same two passes (same scaling, launches after the first quarter)
        f.write("# Other kernels of the same passes, bytes per launch (fetch, write), launches averaged:\n")
        per = {}
        for label, path, counter in (("fetch", fetch_csv, "FETCH_SIZE"), ("write", write_csv, "WRITE_SIZE")):
            for name, _, val in _per_dispatch(path, counter):
                if "pql::" in name and short_name(name) != kernel and "copy_kernel" not in name and "mfma_probe" not in name:
                    per.setdefault(short_name(name), {}).setdefault(label, []).append(val)
        for name in sorted(per):
            vals = {}
            for label in ("fetch", "write"):
                v = per[name].get(label, [])
                v = v[len(v) // 4:]
                vals[label] = (sum(v) / len(v) * 1024.0 * res[label]["scale"], len(v)) if v else (0.0, 0)
            f.write("other.%s=%.0f,%.0f,%d\n" % (name, vals["fetch"][0], vals["write"][0], vals["fetch"][1]))


def stored_traffic(path, kernel):
    """The stored per-launch traffic for `kernel`, or None if absent or the sources changed."""
    if not os.path.exists(path):
        return None
    kv = dict(l.strip().split("=", 1) for l in open(path) if "=" in l and not l.startswith("#"))
    if kv.get("kernel") != kernel or kv.get("source_sha256") != source_hash():
        return None
    return float(kv["traffic_bytes_per_launch"])


def counters_summary(counter_csv, out, counters, bench_args=""):
    """Per-kernel averages per launch of one --pmc pass (warm-up launches skipped)."""
    names = counters.split()
    per = {}                                   # kernel -> dispatch -> counter -> value
    for r in csv.DictReader(open(counter_csv)):
        if "pql::" not in r["Kernel_Name"]:
            continue
        per.setdefault(short_name(r["Kernel_Name"]), {}).setdefault(r["Dispatch_Id"], {})[r["Counter_Name"]] = float(r["Counter_Value"])
    with open(out, "w") as f:
        f.write("# Shader counters per launch (bench.py, one --pmc pass)\n")
        f.write("# Command (from the repository root, on one MI355X):\n")
        f.write("#   rocprofv3 --pmc %s --output-format csv -d <out>/pmc_sq -o s -- python3 bench.py%s\n" % (
            " ".join(names), (" " + bench_args) if bench_args else ""))
        f.write("#   python -m paper_2307_12983_amd.profile_tools counters <out>/pmc_sq/s_counter_collection.csv <this file> \"<counters>\"\n")
        f.write("# Values are sums over all compute units / wavefronts of a launch, averaged over the launches after the\n")
        f.write("# first quarter; `/busy` divides by SQ_BUSY_CU_CYCLES (cycles x compute units with work).\n")
        f.write("source_sha256=%s\n" % source_hash())
        order = sorted(per, key=lambda k: -sum(d.get("SQ_BUSY_CU_CYCLES", 0.0) for d in per[k].values()))
        for k in order:
            disp = [per[k][d] for d in sorted(per[k], key=int)]
            disp = disp[len(disp) // 4:]
            f.write("\n%s  (%d launches)\n" % (k, len(disp)))
            busy = sum(d.get("SQ_BUSY_CU_CYCLES", 0.0) for d in disp) / len(disp)
            for c in names:
                v = sum(d.get(c, 0.0) for d in disp) / len(disp)
                f.write("    %-28s %16.0f" % (c, v))
                if busy > 0 and c != "SQ_BUSY_CU_CYCLES":
                    f.write("   /busy %.4f" % (v / busy))
                f.write("\n")


if __name__ == "__main__":
    if len(sys.argv) >= 6 and sys.argv[1] == "stats":
        stats_summary(*sys.argv[2:7])
    elif len(sys.argv) >= 6 and sys.argv[1] == "traffic":
        traffic_summary(*sys.argv[2:7])
    elif len(sys.argv) >= 5 and sys.argv[1] == "counters":
        counters_summary(*sys.argv[2:6])
    else:
        raise SystemExit(__doc__)
