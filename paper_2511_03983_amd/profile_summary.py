"""Condense rocprofv3 output of a run of this library into the short text summaries kept under profiles/.

    python -m paper_2511_03983_amd.profile_summary stats <x_kernel_stats.csv> <out.txt> "<command that was profiled>"
    python -m paper_2511_03983_amd.profile_summary trace <x_kernel_trace.csv> <out.txt> "<command that was profiled>"
    python -m paper_2511_03983_amd.profile_summary pmc   <x_counter_collection.csv> <out.txt> "<command that was profiled>"
    python -m paper_2511_03983_amd.profile_summary mfma  <x_counter_collection.csv> <out.txt> "<command that was profiled>"

`stats` takes the per-kernel table of `rocprofv3 --kernel-trace --stats --output-format csv`; `trace` takes the
per-dispatch table of the same run and gives one row per (kernel, grid size), so that launches of one kernel on
different shapes or layouts (the movers in the two storage layouts, each projection shape) keep their own durations;
`pmc` takes the
per-dispatch counter table of `rocprofv3 --pmc <counter> --output-format csv`, sums the rows of each dispatch and
averages per (kernel, grid size); `mfma` takes a run with SQ_VALU_MFMA_BUSY_CYCLES, SQ_BUSY_CYCLES and
SQ_INSTS_VALU_MFMA_MOPS_BF16 and prints one row per kernel with the matrix-pipe utilisation derived from them.
Kernel names are shortened; rows of other libraries' kernels are kept but
marked.  FETCH_SIZE / WRITE_SIZE are reported by the tool in KiB per dispatch.
"""
from __future__ import annotations

import collections
import csv
import re
import sys


def short(name: str) -> str:
    name = re.sub(r"\(anonymous namespace\)::", "", name)
    name = re.sub(r"^void ", "", name)
    return ("other: " + name[:64]) if name.startswith("at::") or name.startswith("__amd") else name.split("(")[0][:76]


def stats(src: str, out: str, cmd: str) -> None:
    rows = list(csv.DictReader(open(src, newline="")))
    with open(out, "w") as f:
        f.write("# rocprofv3 --kernel-trace --stats summary (durations in microseconds)\n# command: %s\n" % cmd)
        f.write("# 'other:' rows are the benchmark's own weight generation / perturbation kernels, outside the timed regions\n")
        f.write(f"{'kernel':78s} {'calls':>7s} {'total_us':>12s} {'avg_us':>10s} {'%':>6s}\n")
        for r in rows:
            pct = float(r["Percentage"])
            if pct < 0.005:
                continue
            f.write(f"{short(r['Name']):78s} {int(r['Calls']):7d} {float(r['TotalDurationNs']) / 1e3:12.1f} "
                    f"{float(r['AverageNs']) / 1e3:10.2f} {pct:6.2f}\n")


def trace(src: str, out: str, cmd: str) -> None:
    agg = collections.defaultdict(lambda: [0, 0.0, float("inf"), 0.0])
    with open(src, newline="") as f:
        for r in csv.DictReader(f):
            dur = (float(r["End_Timestamp"]) - float(r["Start_Timestamp"])) / 1e3
            grid = "x".join(str(r.get(k, "")) for k in ("Grid_Size_X", "Grid_Size_Y", "Grid_Size_Z")) if "Grid_Size_X" in r else str(r.get("Grid_Size", ""))
            a = agg[(short(r["Kernel_Name"]), grid)]
            a[0] += 1
            a[1] += dur
            a[2] = min(a[2], dur)
            a[3] = max(a[3], dur)
    total = sum(a[1] for a in agg.values())
    with open(out, "w") as f:
        f.write("# rocprofv3 --kernel-trace summary per (kernel, grid size in threads): durations in microseconds\n# command: %s\n" % cmd)
        f.write("# 'other:' rows (the benchmark's own weight generation / perturbation kernels) and rows under 0.02 % of the total are left out\n")
        f.write(f"{'kernel':72s} {'grid':>14s} {'calls':>7s} {'total_us':>12s} {'avg_us':>10s} {'min_us':>10s} {'max_us':>10s} {'%':>6s}\n")
        for (kn, grid), (n, tot, lo, hi) in sorted(agg.items(), key=lambda x: -x[1][1]):
            if kn.startswith("other:") or tot < 2e-4 * total:
                continue
            f.write(f"{kn[:72]:72s} {grid:>14s} {n:7d} {tot:12.1f} {tot / n:10.2f} {lo:10.2f} {hi:10.2f} {100.0 * tot / total:6.2f}\n")


def pmc(src: str, out: str, cmd: str) -> None:
    disp = collections.OrderedDict()
    with open(src, newline="") as f:
        for r in csv.DictReader(f):
            key = (r["Dispatch_Id"], r["Counter_Name"])
            if key not in disp:
                disp[key] = [short(r["Kernel_Name"]), r.get("Grid_Size", ""), 0.0]
            disp[key][2] += float(r["Counter_Value"])
    agg = collections.defaultdict(lambda: [0, 0.0])
    for (_, cname), (kn, grid, val) in disp.items():
        a = agg[(kn, grid, cname)]
        a[0] += 1
        a[1] += val
    with open(out, "w") as f:
        f.write("# rocprofv3 --pmc summary: average counter value per dispatch, by kernel and grid size (threads)\n# command: %s\n" % cmd)
        f.write(f"{'kernel':78s} {'grid':>10s} {'counter':>12s} {'dispatches':>10s} {'avg_per_dispatch':>18s}\n")
        for (kn, grid, cname), (n, tot) in sorted(agg.items(), key=lambda x: -x[1][1]):
            if kn.startswith("other:") and "copyBuffer" not in kn:
                continue
            f.write(f"{kn:78s} {grid:>10s} {cname:>12s} {n:10d} {tot / n:18.1f}\n")


def mfma(src: str, out: str, cmd: str) -> None:
    """MFMA_BUSY counts, summed over the chip's 1024 SIMDs, the cycles a SIMD's matrix pipe is occupied (32 per
    32x32x16 bf16 instruction); SQ_BUSY_CYCLES counts the kernel's cycles once per shader engine (32 of them).
    Utilisation = MFMA_BUSY / (32 x SQ_BUSY_CYCLES): the fraction of all SIMD-cycles with the matrix pipe busy."""
    disp = collections.OrderedDict()
    with open(src, newline="") as f:
        for r in csv.DictReader(f):
            key = r["Dispatch_Id"]
            d = disp.setdefault(key, {"k": short(r["Kernel_Name"])})
            d[r["Counter_Name"]] = d.get(r["Counter_Name"], 0.0) + float(r["Counter_Value"])
    agg = collections.defaultdict(lambda: collections.defaultdict(float))
    for d in disp.values():
        a = agg[d["k"]]
        a["n"] += 1
        for c in ("SQ_VALU_MFMA_BUSY_CYCLES", "SQ_BUSY_CYCLES", "SQ_INSTS_VALU_MFMA_MOPS_BF16"):
            a[c] += d.get(c, 0.0)
    with open(out, "w") as f:
        f.write("# matrix-pipe utilisation per kernel from one rocprofv3 --pmc run (sums over all dispatches of the kernel)\n# command: %s\n" % cmd)
        f.write("# utilisation = SQ_VALU_MFMA_BUSY_CYCLES / (32 x SQ_BUSY_CYCLES): MFMA_BUSY is summed over the 1024 SIMDs, BUSY_CYCLES over 32 shader engines\n")
        f.write(f"{'kernel':60s} {'dispatches':>10s} {'mfma_busy_cycles':>18s} {'busy_cycles':>14s} {'mfma_mops_bf16':>16s} {'utilisation':>12s}\n")
        for k, a in sorted(agg.items(), key=lambda x: -x[1]["SQ_VALU_MFMA_BUSY_CYCLES"]):
            if k.startswith("other:") or a["SQ_BUSY_CYCLES"] <= 0:
                continue
            f.write(f"{k[:60]:60s} {int(a['n']):10d} {a['SQ_VALU_MFMA_BUSY_CYCLES']:18.0f} {a['SQ_BUSY_CYCLES']:14.0f} "
                    f"{a['SQ_INSTS_VALU_MFMA_MOPS_BF16']:16.0f} {a['SQ_VALU_MFMA_BUSY_CYCLES'] / (32.0 * a['SQ_BUSY_CYCLES']):12.3f}\n")


if __name__ == "__main__":
    modes = {"stats": stats, "trace": trace, "pmc": pmc, "mfma": mfma}
    if len(sys.argv) != 5 or sys.argv[1] not in modes:
        sys.exit(__doc__)
    modes[sys.argv[1]](sys.argv[2], sys.argv[3], sys.argv[4])
