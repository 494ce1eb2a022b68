"""Condense rocprofv3 CSV output of `bench.py` into the short text summaries kept under profiles/.

    python3 -m paper_2603_02188_amd.profile_summary trace   <dir>            # --kernel-trace --stats run
    python3 -m paper_2603_02188_amd.profile_summary trace   <dir> <kernel> <first> <count>
                      # ... and the mean over launches first .. first+count-1 (in start order, from 0) of the
                      # kernels whose name contains <kernel>: the launches that bench.py's own events timed
    python3 -m paper_2603_02188_amd.profile_summary counters <fetch_dir> <write_dir> [<sq_dir>]

`<dir>` is the `-d` directory given to rocprofv3 (searched recursively for the CSV files).

The byte counters are calibrated against the plain device-to-device copies that
`bench.py --copy-calibration` issues (2^30 bytes read and 2^30 bytes written per dispatch): the
scale of FETCH_SIZE (WRITE_SIZE) is 2^20 KiB divided by what the counter reads for such a copy.
"""
from __future__ import annotations

import collections
import csv
import glob
import os
import sys

COPY_KERNEL = "__amd_rocclr_copyBuffer"
COPY_KIB = float(1 << 20)


def _find(root, suffix):
    hits = sorted(glob.glob(os.path.join(root, "**", "*" + suffix), recursive=True), key=os.path.getmtime)
    if not hits:
        raise SystemExit(f"no *{suffix} under {root}")
    return hits[-1]   # the newest run, if the directory was reused


def _short(name):
    name = name.replace("mlra::(anonymous namespace)::", "").replace("mlra::", "")
    name = name.replace("void ", "")
    cut = name.find("(")
    return name if cut < 0 else name[:cut]


def trace_summary(root):
    rows = list(csv.DictReader(open(_find(root, "_kernel_stats.csv"))))
    out = ["| kernel | calls | avg us | min us | max us | % of GPU time |", "|---|---|---|---|---|---|"]
    for r in rows:
        out.append(f"| {_short(r['Name'])} | {r['Calls']} | {float(r['AverageNs']) / 1e3:.1f} | "
                   f"{float(r['MinNs']) / 1e3:.1f} | {float(r['MaxNs']) / 1e3:.1f} | {r['Percentage']} |")
    return "\n".join(out)


def window_mean(root, kernel, first, count):
    rows = [r for r in csv.DictReader(open(_find(root, "_kernel_trace.csv"))) if kernel in r["Kernel_Name"]]
    rows.sort(key=lambda r: int(r["Start_Timestamp"]))
    sel = rows[first:first + count]
    if len(sel) < count:
        raise SystemExit(f"only {len(rows)} launches of {kernel}")
    us = [(int(r["End_Timestamp"]) - int(r["Start_Timestamp"])) / 1e3 for r in sel]
    return (f"launches {first}..{first + count - 1} of {len(rows)} of {_short(sel[0]['Kernel_Name'])}: "
            f"mean {sum(us) / len(us):.1f} us (min {min(us):.1f}, max {max(us):.1f})")


def _per_kernel(root):
    acc = collections.defaultdict(lambda: collections.defaultdict(list))
    for r in csv.DictReader(open(_find(root, "_counter_collection.csv"))):
        acc[_short(r["Kernel_Name"])][r["Counter_Name"]].append(float(r["Counter_Value"]))
    return acc


def _copy_scale(acc, counter):
    """KiB per counter unit, from the largest plain copies (the 1 GiB calibration dispatches)."""
    vals = sorted(acc.get(COPY_KERNEL, {}).get(counter, []))
    big = [v for v in vals if v > 0.9 * vals[-1]] if vals else []
    if not big:
        return None
    return COPY_KIB / (sum(big) / len(big))


N_SIMD = 1024   # MI355X: 256 compute units x 4 SIMDs; SQ_VALU_MFMA_BUSY_CYCLES is summed over them
N_SQ = 32       # ... and SQ_BUSY_CYCLES over the 32 shader engines (8 XCDs x 4), each counting the kernel's cycles


def mfma_busy_fraction(mfma_busy_cycles: float, sq_busy_cycles: float) -> float:
    """Share of the kernel's cycles in which a SIMD's matrix pipe is busy (chip average), from the two
    counters as rocprofv3 reports them per dispatch."""
    if sq_busy_cycles <= 0:
        return 0.0
    return (mfma_busy_cycles / N_SIMD) / (sq_busy_cycles / N_SQ)


def counters_summary(fetch_root, write_root, sq_root=None):
    fetch, write = _per_kernel(fetch_root), _per_kernel(write_root)
    fs, ws = _copy_scale(fetch, "FETCH_SIZE"), _copy_scale(write, "WRITE_SIZE")
    out = [f"copy calibration: a 2^30-byte copy reads FETCH_SIZE = {COPY_KIB / fs:.0f} and WRITE_SIZE = "
           f"{COPY_KIB / ws:.0f}  ->  scale {fs:.4f} KiB per FETCH_SIZE unit, {ws:.4f} KiB per WRITE_SIZE unit",
           "",
           "| kernel | dispatches | FETCH_SIZE | WRITE_SIZE | HBM read MB | HBM write MB | traffic bytes/launch |",
           "|---|---|---|---|---|---|---|"]
    traffic = {}
    for k in fetch:
        if k == COPY_KERNEL or "FETCH_SIZE" not in fetch[k] or k not in write:
            continue
        f = sum(fetch[k]["FETCH_SIZE"]) / len(fetch[k]["FETCH_SIZE"])
        w = sum(write[k]["WRITE_SIZE"]) / len(write[k]["WRITE_SIZE"])
        rb, wb = f * fs * 1024.0, w * ws * 1024.0
        traffic[k] = rb + wb
        out.append(f"| {k} | {len(fetch[k]['FETCH_SIZE'])} | {f:.0f} | {w:.0f} | {rb / 1e6:.1f} | {wb / 1e6:.1f} | "
                   f"{rb + wb:.0f} |")
    if sq_root:
        sq = _per_kernel(sq_root)
        names = sorted({c for k in sq for c in sq[k]})
        derived = "SQ_VALU_MFMA_BUSY_CYCLES" in names and "SQ_BUSY_CYCLES" in names
        head = names + (["matrix pipe busy (derived)"] if derived else [])
        out += ["", "| kernel | " + " | ".join(head) + " |", "|---|" + "---|" * len(head)]
        for k in sq:
            if k == COPY_KERNEL or k.startswith("at::"):
                continue
            mean = {c: sum(sq[k][c]) / max(1, len(sq[k][c])) for c in names if sq[k][c]}
            cells = [f"{mean[c]:.4g}" if c in mean else "-" for c in names]
            if derived:
                cells.append(f"{mfma_busy_fraction(mean.get('SQ_VALU_MFMA_BUSY_CYCLES', 0.0), mean.get('SQ_BUSY_CYCLES', 0.0)):.2f}")
            out.append(f"| {k} | " + " | ".join(cells) + " |")
        if derived:
            out += ["", f"matrix pipe busy = (SQ_VALU_MFMA_BUSY_CYCLES / {N_SIMD} SIMDs) / (SQ_BUSY_CYCLES / {N_SQ} "
                        "shader engines): the share of the kernel's cycles during which a SIMD's matrix pipe is busy, "
                        "averaged over the chip."]
    return "\n".join(out), traffic


def main(argv):
    if len(argv) >= 2 and argv[0] == "trace":
        print(trace_summary(argv[1]))
        if len(argv) >= 5:
            print()
            print(window_mean(argv[1], argv[2], int(argv[3]), int(argv[4])))
    elif len(argv) >= 3 and argv[0] == "counters":
        print(counters_summary(argv[1], argv[2], argv[3] if len(argv) > 3 else None)[0])
    else:
        raise SystemExit(__doc__)


if __name__ == "__main__":
    main(sys.argv[1:])
