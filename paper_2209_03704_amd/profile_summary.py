"""Turn rocprofv3 output folders into the short text summaries kept under profiles/.

    python -m paper_2209_03704_amd.profile_summary trace  <label>=<dir> [<label>=<dir> ...]
    python -m paper_2209_03704_amd.profile_summary hbm    copy=<fetch_dir>,<write_dir> <layer>=<fetch_dir>,<write_dir> ...
    python -m paper_2209_03704_amd.profile_summary mfma   <layer>=<dir> ...

`trace`: per-kernel launch statistics of each folder written by
`rocprofv3 --kernel-trace --output-format csv -d <dir> -- python3 bench.py --only <layer> [--what <pass>]`.
`hbm`: HBM bytes per launch from two counter runs per layer (`--pmc FETCH_SIZE`, `--pmc WRITE_SIZE`,
both in KiB per dispatch), each scaled by what the same counter reads for `bench.py --only copy`, a
device copy of 256 MiB read + 256 MiB written; the rows are the ones bench.py reads back.
`mfma`: matrix-core busy share from `--pmc SQ_VALU_MFMA_BUSY_CYCLES SQ_INSTS_MFMA GRBM_GUI_ACTIVE`.
Only kernels of this library (and the copy yardstick) are listed.  Host-side text processing only.
"""
from __future__ import annotations

import csv
import glob
import os
import sys

from . import metrics
from . import workloads as wl

COPY_KIB = 262144.0          # bench.py --only copy: KiB read and KiB written per launch


def _rows(folder, suffix):
    files = glob.glob(os.path.join(folder, "**", "*" + suffix), recursive=True)
    if not files:
        raise SystemExit("no *%s under %s" % (suffix, folder))
    out = []
    for f in files:
        with open(f, newline="") as fh:
            out.extend(csv.DictReader(fh))
    return out


def _short(name, width=86):
    name = name.replace("(anonymous namespace)::", "").replace("void ", "")
    cut = name.find("(")
    if cut > 0:
        name = name[:cut]
    return name[:width]


def _ours(name):
    return "kst::" in name or "copyBuffer" in name


def trace(pairs):
    print("%-34s %-70s %7s %10s %10s %10s" % ("run", "kernel", "calls", "avg_us", "min_us", "max_us"))
    for label, folder in pairs:
        per = {}
        for r in _rows(folder, "kernel_trace.csv"):
            if _ours(r["Kernel_Name"]):
                per.setdefault(_short(r["Kernel_Name"], 70), []).append(
                    (int(r["End_Timestamp"]) - int(r["Start_Timestamp"])) / 1e3)
        for k, v in sorted(per.items(), key=lambda kv: -sum(kv[1])):
            print("%-34s %-70s %7d %10.2f %10.2f %10.2f" % (label, k, len(v), sum(v) / len(v), min(v), max(v)))


def _counter(folder, counter):
    per = {}
    for r in _rows(folder, "counter_collection.csv"):
        if r["Counter_Name"] == counter and _ours(r["Kernel_Name"]):
            per.setdefault(_short(r["Kernel_Name"]), []).append(float(r["Counter_Value"]))
    return {k: sum(v) / len(v) for k, v in per.items()}, {k: len(v) for k, v in per.items()}


def hbm(pairs):
    scale = {}
    table = []
    for label, folders in pairs:
        fdir, wdir = folders.split(",")
        fetch, _ = _counter(fdir, "FETCH_SIZE")
        write, _ = _counter(wdir, "WRITE_SIZE")
        if label == "copy":
            k = next(k for k in fetch if "copyBuffer" in k)
            scale = {"FETCH": COPY_KIB / fetch[k], "WRITE": COPY_KIB / write[k]}
            print("yardstick: bench.py --only copy = %s, %d KiB read + %d KiB written per launch" % (k, COPY_KIB, COPY_KIB))
            print("  FETCH_SIZE reads %.1f KiB -> scale %.4f ;  WRITE_SIZE reads %.1f KiB -> scale %.4f"
                  % (fetch[k], scale["FETCH"], write[k], scale["WRITE"]))
            print()
            print("layer | kernel | FETCH KiB raw | WRITE KiB raw | HBM bytes | algorithmic B | ratio (all kernels of the layer)")
            continue
        if not scale:
            raise SystemExit("give copy=<fetch_dir>,<write_dir> first")
        layer = wl.layer_by_name(label)
        alg = metrics.algorithmic_bytes(layer)
        rows = []
        for k in fetch:
            if "segregate" in k or "copyBuffer" in k:
                continue
            b = int(round((fetch[k] * scale["FETCH"] + write.get(k, 0.0) * scale["WRITE"]) * 1024))
            rows.append((k, fetch[k], write.get(k, 0.0), b))
        total = sum(r[3] for r in rows)
        for k, f, w, b in rows:
            print("%s | %s | %.1f | %.1f | %d | %d | %.3f" % (layer.name, k, f, w, b, alg, total / alg))
        table.append((layer.name, total, alg))


def mfma(pairs):
    print("%-6s %-60s %18s %14s %14s %7s" % ("layer", "kernel", "MFMA busy cycles", "MFMA instrs", "GUI active", "busy"))
    for label, folder in pairs:
        busy, _ = _counter(folder, "SQ_VALU_MFMA_BUSY_CYCLES")
        inst, _ = _counter(folder, "SQ_INSTS_MFMA")
        gui, _ = _counter(folder, "GRBM_GUI_ACTIVE")
        for k in busy:
            if inst.get(k, 0.0) <= 0:
                continue
            print("%-6s %-60s %18.0f %14.0f %14.0f %7.3f"
                  % (label, k[:60], busy[k], inst[k], gui[k], (busy[k] / 1024.0) / (gui[k] / 8.0)))


def main(argv):
    if len(argv) < 2 or argv[0] not in ("trace", "hbm", "mfma"):
        raise SystemExit(__doc__)
    pairs = [tuple(a.split("=", 1)) for a in argv[1:]]
    {"trace": trace, "hbm": hbm, "mfma": mfma}[argv[0]](pairs)


if __name__ == "__main__":
    main(sys.argv[1:])
