"""Turns the CSV files rocprofv3 writes into the short text summaries kept under profiles/.

    python -m paper_2601_20499_amd.profile_summary kernels  DIR
    python -m paper_2601_20499_amd.profile_summary counters DIR
    python -m paper_2601_20499_amd.profile_summary traffic  --fetch DIR --write DIR --calib-mb N
                                                            --workload NAME [--update profiles/traffic.json]

DIR is the -d directory of one rocprofv3 run (--output-format csv).  `kernels` prints the per-kernel
durations of a --kernel-trace --stats run as a markdown table; `counters` the median per dispatch of
every counter of a --pmc run; `traffic` scales FETCH_SIZE / WRITE_SIZE (two runs) by what the same
counters read for the one large device copy of known size in the same run, prints bytes per dispatch
of every kernel, and with --update records the bytes of one attention call (main kernel + second
kernel), with a hash of the kernel sources, in the JSON file bench.py reads its `roofline.traffic`
from.
"""
from __future__ import annotations

import argparse
import collections
import csv
import glob
import hashlib
import json
import os
import statistics

PKG = os.path.dirname(os.path.abspath(__file__))
KERNEL_SOURCES = ["df_attn.hip", "df_attn_phase.inc", "df_cache.hip", "df_internal.h"]
COPY_KERNEL = "__amd_rocclr_copyBuffer"


def kernel_source_hash() -> str:
    """Identifies the kernel sources a profile was taken with (a GPU machine has no git history)."""
    h = hashlib.sha256()
    for name in KERNEL_SOURCES:
        with open(os.path.join(PKG, "csrc", name), "rb") as f:
            h.update(f.read())
    return h.hexdigest()[:16]


def _one(directory: str, suffix: str) -> str:
    found = glob.glob(os.path.join(directory, "**", "*" + suffix), recursive=True)
    if not found:
        raise SystemExit(f"no *{suffix} under {directory}")
    return sorted(found)[0]


def kernel_table(directory: str):
    rows = list(csv.DictReader(open(_one(directory, "kernel_stats.csv"))))
    out = ["| kernel | calls | avg us | min us | max us | % |", "|---|---|---|---|---|---|"]
    for r in rows:
        out.append("| `%s` | %s | %.1f | %.1f | %.1f | %.2f |" % (
            r["Name"][:90], r["Calls"], float(r["AverageNs"]) / 1e3, float(r["MinNs"]) / 1e3,
            float(r["MaxNs"]) / 1e3, float(r["Percentage"])))
    return "\n".join(out)


def counter_medians(directory: str):
    """{kernel: {counter: (median, max, n)}} over the dispatches of a --pmc run."""
    acc = collections.defaultdict(lambda: collections.defaultdict(list))
    for r in csv.DictReader(open(_one(directory, "counter_collection.csv"))):
        acc[r["Kernel_Name"]][r["Counter_Name"]].append(float(r["Counter_Value"]))
    return {k: {c: (statistics.median(v), max(v), len(v)) for c, v in cs.items()} for k, cs in acc.items()}


def counter_table(directory: str):
    med = counter_medians(directory)
    out = ["| kernel | counter | dispatches | median | max |", "|---|---|---|---|---|"]
    for k in sorted(med):
        for c in sorted(med[k]):
            m, mx, n = med[k][c]
            out.append("| `%s` | %s | %d | %.6g | %.6g |" % (k[:90], c, n, m, mx))
    return "\n".join(out)


def traffic(fetch_dir: str, write_dir: str, calib_mb: int):
    """Scaled bytes per dispatch: {kernel: (fetched, written)}, and the two scale factors."""
    f, w = counter_medians(fetch_dir), counter_medians(write_dir)
    calib_kib = calib_mb * 1024.0
    # the calibration copy is the largest dispatch of the runtime's copy kernel
    f_scale = calib_kib / f[COPY_KERNEL]["FETCH_SIZE"][1]
    w_scale = calib_kib / w[COPY_KERNEL]["WRITE_SIZE"][1]
    table = {}
    for k in f:
        if k in w and k != COPY_KERNEL:
            table[k] = (f[k]["FETCH_SIZE"][0] * f_scale * 1024.0, w[k]["WRITE_SIZE"][0] * w_scale * 1024.0)
    return table, f_scale, w_scale, f[COPY_KERNEL]["FETCH_SIZE"][1], w[COPY_KERNEL]["WRITE_SIZE"][1]


def main():
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    sub = ap.add_subparsers(dest="cmd", required=True)
    for name in ("kernels", "counters"):
        s = sub.add_parser(name)
        s.add_argument("dir")
    t = sub.add_parser("traffic")
    t.add_argument("--fetch", required=True)
    t.add_argument("--write", required=True)
    t.add_argument("--calib-mb", type=int, required=True)
    t.add_argument("--workload", required=True)
    t.add_argument("--update", default=None, help="JSON file to record the attention call's bytes in")
    a = ap.parse_args()
    if a.cmd == "kernels":
        print(kernel_table(a.dir))
    elif a.cmd == "counters":
        print(counter_table(a.dir))
    else:
        table, fs, ws, fraw, wraw = traffic(a.fetch, a.write, a.calib_mb)
        print(f"Calibration: the {a.calib_mb} MiB device copy of the same run (`{COPY_KERNEL}`, {a.calib_mb * 1024} KiB "
              f"read and written) reads FETCH_SIZE = {fraw:.1f} and WRITE_SIZE = {wraw:.1f}: scale factors "
              f"{fs:.4f} and {ws:.4f}.\n")
        print("| kernel | fetched MB | written MB |", "|---|---|---|", sep="\n")
        call = 0.0
        for k in sorted(table):
            print("| `%s` | %.1f | %.1f |" % (k[:90], table[k][0] / 1e6, table[k][1] / 1e6))
            if "df_attn_kernel" in k and "false" in k or "df_attn_merge_kernel" in k and "false" in k:
                call += table[k][0] + table[k][1]
        print(f"\ndf_attn_fwd per call (main kernel + second kernel, fetched + written): {call / 1e6:.1f} MB; "
              f"kernel sources {kernel_source_hash()}")
        if a.update:
            try:
                with open(a.update) as fh:
                    doc = json.load(fh)
            except (OSError, ValueError):
                doc = {}
            doc[a.workload] = {"kernel_source_hash": kernel_source_hash(), "attn_call_bytes": round(call),
                               "fetch_scale": round(fs, 4), "write_scale": round(ws, 4)}
            with open(a.update, "w") as fh:
                json.dump(doc, fh, indent=1, sort_keys=True)
                fh.write("\n")


if __name__ == "__main__":
    main()
