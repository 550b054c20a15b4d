"""Turns the counter files of `rocprofv3 --pmc ... -- python3 bench.py --eager ... --calib-copy` runs into the
short text table kept with the profiles.

    python -m paper_2209_06979_amd.counters_summary <dir with one sub-directory per counter pass> [name,name,...]  > summary.txt

(the optional second argument keeps only the kernels whose name contains one of the given pieces)

Every `*_counter_collection.csv` below the directory is read; counters are averaged over the dispatches of a
kernel.  FETCH_SIZE and WRITE_SIZE (KiB per dispatch) are scaled by what the same counter reads for the plain
64 MiB device copy of `--calib-copy`.  The lines starting with `library:` and `traffic` are what bench.py parses
(it drops the figures when the library it runs is another build than the one named here).
"""
from __future__ import annotations

import collections
import csv
import os
import re
import sys

COPY_BYTES = 64 * 1024 * 1024


def bench_name(kernel: str):
    """Name of the bench.py step row a device kernel belongs to (None: not a row of the step)."""
    m = re.search(r"spmm_kernel<\s*\d+,\s*\d+,\s*(\d+),\s*(\d+)", kernel)
    if m:
        return f"spmm_L{m.group(1)}R{m.group(2)}"
    m = re.search(r"spmm_slab_kernel<\s*\d+,\s*(\d+),\s*(true|false|0|1)", kernel)
    if m:
        return f"spmm_L{m.group(1)}R{'4' if m.group(2) in ('true', '1') else '8'}"
    m = re.search(r"sddmm_\w*kernel<\s*(\d+)", kernel)
    if m:
        return f"sddmm_L{m.group(1)}R{m.group(1)}"
    if "attention_fused_kernel" in kernel:
        return "attention"
    return None


def short(kernel: str) -> str:
    m = re.search(r"(\w+_kernel<[^>]*>)", kernel) or re.search(r"(\w+)\(", kernel)
    return m.group(1) if m else kernel[-48:]


def read(directory: str):
    """{kernel name: {counter: [values per dispatch]}} and the copy's {counter: value}."""
    per = collections.defaultdict(lambda: collections.defaultdict(list))
    copy = {}
    for root, _, files in os.walk(directory):
        for f in files:
            if not f.endswith("counter_collection.csv"):
                continue
            with open(os.path.join(root, f), newline="") as fh:
                for r in csv.DictReader(fh):
                    name, c, v = r["Kernel_Name"], r["Counter_Name"], float(r["Counter_Value"])
                    if "copyBuffer" in name:
                        # the calibration copy is the largest one (the others move a few KB of arguments)
                        copy[c] = max(copy.get(c, 0.0), v)
                    else:
                        per[name][c].append(v)
    return per, copy


def main(argv):
    if len(argv) not in (2, 3):
        print(__doc__, file=sys.stderr)
        return 2
    from . import binding as mc
    per, copy = read(argv[1])
    if len(argv) == 3:          # keep only kernels whose name contains one of these comma-separated pieces
        keep = argv[2].split(",")
        per = {k: v for k, v in per.items() if any(piece in k for piece in keep)}
    fs = COPY_BYTES / 1024.0 / copy["FETCH_SIZE"] if copy.get("FETCH_SIZE") else None
    wsf = COPY_BYTES / 1024.0 / copy["WRITE_SIZE"] if copy.get("WRITE_SIZE") else None
    print(f"library: {mc.lib.mc_version().decode()}")
    if fs and wsf:
        print(f"calibration: a plain 64 MiB device copy reads FETCH_SIZE = {copy['FETCH_SIZE']:.0f} KiB, WRITE_SIZE = "
              f"{copy['WRITE_SIZE']:.0f} KiB -> scale factors {fs:.3f} (fetch) and {wsf:.3f} (write)")
    counters = sorted({c for cs in per.values() for c in cs})
    print()
    print("averages per dispatch (n = dispatches seen):")
    for k in sorted(per, key=short):
        avg = {c: sum(v) / len(v) for c, v in per[k].items()}
        n = max(len(v) for v in per[k].values())
        print(f"  {short(k)}  (n={n})")
        have = [f"{c}={avg[c]:.0f}" for c in counters if c in avg]
        for i in range(0, len(have), 4):
            print("      " + "  ".join(have[i:i + 4]))
    if fs and wsf:
        print()
        print("HBM-side bytes per launch (counter x 1024 x scale factor):")
        for k in sorted(per, key=short):
            cs = per[k]
            if "FETCH_SIZE" not in cs or "WRITE_SIZE" not in cs:
                continue
            fb = sum(cs["FETCH_SIZE"]) / len(cs["FETCH_SIZE"]) * 1024 * fs
            wb = sum(cs["WRITE_SIZE"]) / len(cs["WRITE_SIZE"]) * 1024 * wsf
            row = bench_name(k)
            print(f"traffic {row or '-'} fetch_bytes={fb:.0f} write_bytes={wb:.0f} kernel={short(k)}")
    return 0


if __name__ == "__main__":
    sys.exit(main(sys.argv))
