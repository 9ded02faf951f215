"""Turns rocprofv3 output folders into the short text summaries kept under ``profiles/``.

    python -m paper_1802_04450_amd.profile_summary --trace DIR [--fetch DIR --write DIR --copy-fetch DIR --copy-write DIR]
        [--mfma DIR] --title TEXT --command TEXT [--command TEXT ...] --out profiles/NAME_kernels.txt
        [--traffic-out profiles/NAME_traffic.txt] [--note TEXT]

DIR are the ``-d`` folders of separate rocprofv3 runs of the same command: ``--kernel-trace --stats`` (trace),
``--pmc FETCH_SIZE`` (fetch), ``--pmc WRITE_SIZE`` (write), the same two counters for ``bench.py --copy-probe`` (a plain
1 GiB device copy whose traffic is known: the calibration of the two counters), and optionally
``--pmc SQ_INSTS_VALU_MFMA_MOPS_F64 SQ_VALU_MFMA_BUSY_CYCLES``.  The summary records the SHA-256 of the kernel sources it
was made from (``build.source_hash()``); ``bench.py`` reports the traffic figure only while that hash is the tree's.
Nothing here touches a GPU."""
from __future__ import annotations

import argparse
import collections
import csv
import glob
import os

from .build import source_hash

COPY_KIB = 1048576.0          # bench.py --copy-probe reads and writes 1 GiB


def short(name: str) -> str:
    name = name.replace("void ", "").replace("sceig::(anonymous namespace)::", "")
    name = name.split("(")[0]
    if name.startswith("rocprim::"):
        tail = name.split("detail::")[-1]
        name = "rocprim::" + tail.split("<")[0]
    return name.replace(" ", "")[:48]


def find_one(folder: str, pattern: str) -> str:
    hits = sorted(glob.glob(os.path.join(folder, "**", pattern), recursive=True))
    if not hits:
        raise FileNotFoundError(f"no {pattern} under {folder}")
    return hits[0]


def counters(folder: str):
    """(kernel, counter) -> (dispatches, average value per dispatch)"""
    acc = collections.defaultdict(lambda: [0, 0.0])
    with open(find_one(folder, "*counter_collection.csv")) as f:
        for r in csv.DictReader(f):
            key = (short(r["Kernel_Name"]), r["Counter_Name"])
            acc[key][0] += 1
            acc[key][1] += float(r["Counter_Value"])
    return {k: (c, t / c) for k, (c, t) in acc.items()}


def copy_factor(folder: str, counter: str) -> tuple:
    """The plain copy's own reading of `counter` (largest per-dispatch average among its kernels) and the factor that
    turns a reading into KiB of HBM traffic."""
    vals = [v for (k, c), (_, v) in counters(folder).items() if c == counter]
    reading = max(vals)
    return reading, COPY_KIB / reading


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--trace", required=True)
    ap.add_argument("--fetch")
    ap.add_argument("--write")
    ap.add_argument("--copy-fetch")
    ap.add_argument("--copy-write")
    ap.add_argument("--mfma")
    ap.add_argument("--title", required=True)
    ap.add_argument("--command", action="append", default=[])
    ap.add_argument("--note", action="append", default=[])
    ap.add_argument("--all-kernels", action="store_true", help="keep kernels that are not the library's or rocprim's")
    ap.add_argument("--top", type=int, default=40)
    ap.add_argument("--out", required=True)
    ap.add_argument("--traffic-out")
    a = ap.parse_args()

    with open(find_one(a.trace, "*kernel_stats.csv")) as f:
        rows = list(csv.DictReader(f))
    if not a.all_kernels:
        rows = [r for r in rows if "sceig" in r["Name"] or "rocprim" in r["Name"]]
    rows = rows[: a.top]
    have_traffic = all([a.fetch, a.write, a.copy_fetch, a.copy_write])
    fetch = write = mf = {}
    ff = wf = 1.0
    lines = [a.title, f"csrc_sha256: {source_hash()}",
             "commands (from /tmp with TMPDIR=/tmp, R = repository root, each in a run of its own):"]
    lines += ["  " + c for c in a.command]
    lines += a.note
    if have_traffic:
        fetch, write = counters(a.fetch), counters(a.write)
        fr, ff = copy_factor(a.copy_fetch, "FETCH_SIZE")
        wr, wf = copy_factor(a.copy_write, "WRITE_SIZE")
        lines.append(f"calibration: plain device copy of 1 GiB (1,048,576 KiB read and written): FETCH_SIZE = {fr:.1f} -> "
                     f"factor {ff:.3f}; WRITE_SIZE = {wr:.1f} -> factor {wf:.3f}.  HBM bytes = counter * 1024 * factor.")
    if a.mfma:
        mf = counters(a.mfma)
    lines.append("")
    head = "%-48s %6s %10s %9s %9s %9s" % ("kernel", "calls", "total_ms", "avg_us", "min_us", "max_us")
    if have_traffic:
        head += " | %15s %15s" % ("fetch_MB/launch", "write_MB/launch")
    if a.mfma:
        head += " | %14s %10s" % ("MFMA_F64_flops", "mfma_busy%")
    lines.append(head)
    traffic = []
    for r in rows:
        k = short(r["Name"])
        avg = float(r["AverageNs"]) / 1e3
        line = "%-48s %6d %10.3f %9.2f %9.2f %9.2f" % (k, int(r["Calls"]), int(r["TotalDurationNs"]) / 1e6, avg,
                                                      int(r["MinNs"]) / 1e3, int(r["MaxNs"]) / 1e3)
        if have_traffic:
            fb = fetch.get((k, "FETCH_SIZE"), (0, 0.0))[1] * 1024 * ff
            wb = write.get((k, "WRITE_SIZE"), (0, 0.0))[1] * 1024 * wf
            line += " | %15.1f %15.1f" % (fb / 1e6, wb / 1e6)
            traffic.append([k, fb, wb, avg, 0.0])
        if a.mfma:
            flops = mf.get((k, "SQ_INSTS_VALU_MFMA_MOPS_F64"), (0, 0.0))[1] * 512
            busy = mf.get((k, "SQ_VALU_MFMA_BUSY_CYCLES"), (0, 0.0))[1]
            # busy cycles are summed over the 1024 SIMDs of the chip; launch duration in cycles at 2.4 GHz
            util = busy / 1024.0 / (avg * 1e-6 * 2.4e9) * 100 if avg > 0 else 0.0
            line += " | %14.3e %10.1f" % (flops, util)
            if traffic and traffic[-1][0] == k:
                traffic[-1][4] = flops
        lines.append(line)
    with open(a.out, "w") as f:
        f.write("\n".join(lines) + "\n")
    if a.traffic_out and have_traffic:
        with open(a.traffic_out, "w") as f:
            f.write("# HBM traffic per launch from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (scaled by the copy calibration), "
                    f"bytes;\n# source and commands: {a.out}.  Columns: kernel fetch_bytes write_bytes avg_us "
                    f"mfma_f64_flops (per launch, SQ_INSTS_VALU_MFMA_MOPS_F64 * 512; 0 if not counted)\n"
                    f"# csrc_sha256: {source_hash()}\n")
            for k, fb, wb, avg, fl in traffic:
                f.write("%s %.0f %.0f %.2f %.4e\n" % (k, fb, wb, avg, fl))
    print("\n".join(lines))


if __name__ == "__main__":
    main()
