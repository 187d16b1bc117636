"""Hardware-counter figures of the benchmark's dominant kernels, kept beside the
profiles so that bench.py does not carry pasted constants.

``python -m paper_1711_00244_amd.counters --from <dir> [<dir> ...]`` reads the
``*_counter_collection.csv`` files rocprofv3 ``--pmc`` runs of ``bench.py`` left in the
given directories, averages each counter over the dispatches of each kernel of
interest, scales FETCH_SIZE / WRITE_SIZE to bytes (factors below) and writes
``profiles/counters.json``: per kernel and workload the bytes fetched and written and
the wavefront instruction counts, plus a hash of the kernel sources they were measured
on.  ``bench.py`` reads the file and marks its ``traffic`` fields stale when the hash
no longer matches the sources it runs.
"""
from __future__ import annotations

import argparse
import csv
import glob
import hashlib
import json
import os
import re

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OUT = os.path.join(ROOT, "profiles", "counters.json")

# What the counters read for a reference copy kernel of known size on this machine
# (256 MiB device-to-device copy, bench.py --copy-calibration): FETCH_SIZE counts
# units of 64 bytes where the documentation says KiB-scaled 32-byte units (a factor
# of two on the reading in KiB), WRITE_SIZE reads KiB.
FETCH_KIB_FACTOR = 2.0
WRITE_KIB_FACTOR = 1.0

KERNELS = {"wide_mul_kernel": "wide", "wide_expand_kernel": "wide_expand", "fc_mfma_kernel": "mfma", "fc_sparse_kernel": "sparse",
           "mfma_reduce_kernel": "mfma_reduce", "wide_reduce_kernel": "wide_reduce", "fc_reduce_kernel": "sparse_reduce"}


def source_hash() -> str:
    """sha256 over the kernel and host sources of the library, in name order."""
    h = hashlib.sha256()
    for name in sorted(os.listdir(CSRC)):
        if name.endswith((".hip", ".hpp", ".cpp")):
            h.update(name.encode())
            with open(os.path.join(CSRC, name), "rb") as f:
                h.update(f.read())
    return h.hexdigest()[:16]


def load() -> dict | None:
    try:
        with open(OUT) as f:
            return json.load(f)
    except (OSError, ValueError):
        return None


def lookup(key: str) -> tuple[dict | None, bool]:
    """-> (figures of a kernel/workload key such as 'wide/fc6/256', stale?)."""
    d = load()
    if not d or key not in d.get("kernels", {}):
        return None, True
    return d["kernels"][key], d.get("source_hash") != source_hash()


def _kernel_key(name: str) -> str | None:
    for k, short in KERNELS.items():
        if re.search(r"\b" + k + r"\b", name) or ("cl::" + k) in name or k in name:
            return short
    return None


def collect(dirs, layer_of_grid) -> dict:
    """Average each counter per (kernel, grid size) over the dispatches in the csv files."""
    acc: dict = {}
    for d in dirs:
        for path in glob.glob(os.path.join(d, "**", "*counter_collection.csv"), recursive=True):
            with open(path, newline="") as f:
                for row in csv.DictReader(f):
                    short = _kernel_key(row.get("Kernel_Name", ""))
                    if short is None:
                        continue
                    grid = int(row.get("Grid_Size", 0) or 0)
                    wg = int(row.get("Workgroup_Size", 1) or 1)
                    key = (short, grid // max(wg, 1))
                    acc.setdefault(key, {}).setdefault(row["Counter_Name"], []).append(float(row["Counter_Value"]))
    out = {}
    for (short, wgs), counters in acc.items():
        label = layer_of_grid(short, wgs)
        if label is None:
            continue
        fig = {"workgroups": wgs, "dispatches": max(len(v) for v in counters.values())}
        for name, vals in counters.items():
            mean = sum(vals) / len(vals)
            if name == "FETCH_SIZE":
                fig["fetch_bytes"] = mean * 1024.0 * FETCH_KIB_FACTOR
            elif name == "WRITE_SIZE":
                fig["write_bytes"] = mean * 1024.0 * WRITE_KIB_FACTOR
            else:
                fig[name] = mean
        out[f"{short}/{label}"] = fig
    return out


def main(argv=None):
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--from", dest="dirs", nargs="+", required=True, help="rocprofv3 output directories")
    ap.add_argument("--label", action="append", default=[],
                    help="kernel:workgroups=label, e.g. wide:256=fc6/256 (which dispatches belong to which layer and batch)")
    ap.add_argument("--command", default="", help="the profiled command, recorded in the file")
    args = ap.parse_args(argv)
    labels = {}
    for item in args.label:
        k, v = item.split("=", 1)
        short, wgs = k.split(":")
        labels[(short, int(wgs))] = v
    figures = collect(args.dirs, lambda short, wgs: labels.get((short, wgs)))
    prev = load() or {}
    kernels = dict(prev.get("kernels", {})) if prev.get("source_hash") == source_hash() else {}
    kernels.update(figures)
    doc = {"source_hash": source_hash(), "fetch_kib_factor": FETCH_KIB_FACTOR, "write_kib_factor": WRITE_KIB_FACTOR,
           "command": args.command or prev.get("command", ""), "kernels": kernels}
    os.makedirs(os.path.dirname(OUT), exist_ok=True)
    with open(OUT, "w") as f:
        json.dump(doc, f, indent=1, sort_keys=True)
        f.write("\n")
    print(json.dumps({k: {n: round(v) if isinstance(v, float) else v for n, v in fig.items()} for k, fig in figures.items()}, indent=1))


if __name__ == "__main__":
    main()
