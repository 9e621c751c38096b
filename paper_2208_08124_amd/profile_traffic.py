"""Turns rocprofv3 counter runs into profiles/traffic.json: HBM bytes per launch of each
attention kernel on one workload, for the benchmark's `roofline.traffic`.

Four counter runs feed it (each its own rocprofv3 call, `cd /tmp && export TMPDIR=/tmp` first):

    rocprofv3 --pmc FETCH_SIZE --output-format csv -d <fetch> -o p -- \\
        python3 bench.py --steps 5 --warmup 2 --no-cpu-baseline --no-padded
    rocprofv3 --pmc WRITE_SIZE --output-format csv -d <write> -o p -- (same)
    rocprofv3 --pmc FETCH_SIZE --output-format csv -d <copy_fetch> -o p -- \\
        python3 bench.py --copy-calibration 1024
    rocprofv3 --pmc WRITE_SIZE --output-format csv -d <copy_write> -o p -- (same)

then

    python3 -m paper_2208_08124_amd.profile_traffic --fetch <fetch> --write <write> \\
        --copy-fetch <copy_fetch> --copy-write <copy_write> --copy-mib 1024

The counters read in KiB per dispatch up to a factor that depends on the counter; the plain
device-to-device copy of known size gives that factor (bytes moved / counter reading), which
is stored beside the results.  The file also stores build.source_id() of the tree it was
measured on; the benchmark quotes the figures only while that still matches.
"""
from __future__ import annotations

import argparse
import csv
import glob
import json
import os
import re

from . import build

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
DEFAULT_OUT = os.path.join(ROOT, "profiles", "traffic.json")


def _rows(directory):
    files = glob.glob(os.path.join(directory, "**", "*counter_collection.csv"), recursive=True)
    if not files:
        raise SystemExit("no *counter_collection.csv under " + directory)
    out = []
    for f in files:
        with open(f, newline="") as fh:
            out.extend(csv.DictReader(fh))
    return out


def short_name(kernel_name):
    """'bwd_dkv_kernel' from the profiler's name of one of this library's kernels, which is
    mangled for templates (_ZN4fmha14bwd_dkv_kernelIDF16_Lb0EEEv...) and plain otherwise;
    the instances compiled for dropout (template argument true) get ' (dropout)' appended."""
    m = re.match(r"_ZN4fmha(\d+)", kernel_name)
    if m:
        start = m.end()
        name = kernel_name[start:start + int(m.group(1))]
        return name + (" (dropout)" if "Lb1E" in kernel_name else "")
    m = re.search(r"fmha::(\w+)", kernel_name)
    return m.group(1) if m else None


def kernel_means(directory, counter):
    """{short kernel name: mean counter value per dispatch} for our kernels."""
    acc = {}
    for r in _rows(directory):
        if r["Counter_Name"] != counter:
            continue
        name = short_name(r["Kernel_Name"])
        if name:
            acc.setdefault(name, []).append(float(r["Counter_Value"]))
    return {k: sum(v) / len(v) for k, v in acc.items()}


def copy_factor(directory, counter, nbytes):
    """bytes per counter unit, from the dispatches of the runtime's copy kernel that moved nbytes."""
    vals = [float(r["Counter_Value"]) for r in _rows(directory)
            if r["Counter_Name"] == counter and "copyBuffer" in r["Kernel_Name"]]
    big = [v for v in vals if v > 0.5 * max(vals)]
    return nbytes / (sum(big) / len(big))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--fetch", required=True)
    ap.add_argument("--write", required=True)
    ap.add_argument("--copy-fetch", required=True)
    ap.add_argument("--copy-write", required=True)
    ap.add_argument("--copy-mib", type=int, default=1024)
    ap.add_argument("--workload", default="bert_large_fwd_bwd")
    ap.add_argument("--out", default=DEFAULT_OUT)
    a = ap.parse_args()
    n = a.copy_mib << 20
    ff, wf = copy_factor(a.copy_fetch, "FETCH_SIZE", n), copy_factor(a.copy_write, "WRITE_SIZE", n)
    fetch, write = kernel_means(a.fetch, "FETCH_SIZE"), kernel_means(a.write, "WRITE_SIZE")
    kernels = {k: {"fetch_bytes": round(fetch[k] * ff), "write_bytes": round(write.get(k, 0.0) * wf)}
               for k in sorted(fetch) if k != "schedule_kernel"}
    doc = {"source_id": build.source_id(), "workload": a.workload,
           "bytes_per_counter_unit": {"FETCH_SIZE": round(ff, 2), "WRITE_SIZE": round(wf, 2)},
           "calibration": "device-to-device copy of %d MiB (bench.py --copy-calibration %d)" % (a.copy_mib, a.copy_mib),
           "kernels": kernels}
    with open(a.out, "w") as fh:
        json.dump(doc, fh, indent=1, sort_keys=True)
        fh.write("\n")
    print(json.dumps(doc))


if __name__ == "__main__":
    main()
