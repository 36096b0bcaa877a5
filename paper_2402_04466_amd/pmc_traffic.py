"""Turns two rocprofv3 --pmc runs of bench.py (FETCH_SIZE, then WRITE_SIZE) into HBM traffic
per launch of the convolution kernels, scaled by what the same counters read for the
library's plain copy kernel (bench.py --calibrate-copy), and writes
profiles/conv_traffic_<tag>.json + .md.  bench.py quotes the figure only while the kernel
source still has the hash recorded there.

Usage: python -m paper_2402_04466_amd.pmc_traffic <fetch counter_collection.csv> \\
           <write counter_collection.csv> <calibration MiB> <tag> "<command line used>"
"""
from __future__ import annotations

import csv
import hashlib
import json
import os
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
KERNEL_SOURCES = ("csrc/hs_kernels.hip", "csrc/hs_kernels.h")


def kernel_source_hash() -> str:
    h = hashlib.sha256()
    for rel in KERNEL_SOURCES:
        with open(os.path.join(HERE, rel), "rb") as fh:
            h.update(fh.read())
    return h.hexdigest()


def _per_kernel(path: str, counter: str):
    """{kernel name: [counter value per dispatch]} in dispatch order."""
    out = {}
    with open(path) as fh:
        for r in csv.DictReader(fh):
            if r["Counter_Name"] != counter:
                continue
            name = r["Kernel_Name"].replace("void ", "").split("(")[0]
            out.setdefault(name, []).append(float(r["Counter_Value"]))
    return out


def main(argv):
    fetch_csv, write_csv, cal_mib, tag, cmd = argv[1], argv[2], int(argv[3]), argv[4], argv[5]
    cal_bytes = cal_mib << 20
    fetch, write = _per_kernel(fetch_csv, "FETCH_SIZE"), _per_kernel(write_csv, "WRITE_SIZE")
    copy_f = sorted(fetch["hs::k_copy"])[len(fetch["hs::k_copy"]) // 2]
    copy_w = sorted(write["hs::k_copy"])[len(write["hs::k_copy"]) // 2]
    f_scale, w_scale = cal_bytes / copy_f, cal_bytes / copy_w      # bytes per counter unit
    rows, conv_f, conv_w, conv_n = [], 0.0, 0.0, 0
    for name in sorted(set(fetch) | set(write)):
        if not name.startswith("hs::") or name == "hs::k_copy":
            continue
        fv, wv = fetch.get(name, []), write.get(name, [])
        fb = f_scale * sum(fv) / max(len(fv), 1)
        wb = w_scale * sum(wv) / max(len(wv), 1)
        rows.append((name, len(fv), fb, wb))
        if "conv" in name:
            conv_f += f_scale * sum(fv)
            conv_w += w_scale * sum(wv)
            conv_n += len(fv)
    result = {
        "kernel_source_sha256": kernel_source_hash(),
        "workload": tag,
        "command": cmd,
        "calibration": {"copy_bytes": cal_bytes, "FETCH_SIZE_per_copy": copy_f,
                        "WRITE_SIZE_per_copy": copy_w, "bytes_per_FETCH_unit": f_scale,
                        "bytes_per_WRITE_unit": w_scale},
        "conv_launches": conv_n,
        "conv_hbm_bytes_per_launch": {"fetch": conv_f / conv_n, "write": conv_w / conv_n,
                                      "total": (conv_f + conv_w) / conv_n},
        "kernels": [{"name": n, "launches": c, "fetch_bytes_per_launch": f,
                     "write_bytes_per_launch": w} for n, c, f, w in rows],
    }
    os.makedirs(os.path.join(ROOT, "profiles"), exist_ok=True)
    base = os.path.join(ROOT, "profiles", f"conv_traffic_{tag}")
    with open(base + ".json", "w") as fh:
        json.dump(result, fh, indent=1)
    with open(base + ".md", "w") as fh:
        fh.write(f"# HBM traffic per launch from rocprofv3 counters: {tag}\n\n")
        fh.write("Two runs of the same command, one per counter (from the repository root):\n\n")
        fh.write(f"    {cmd.replace('COUNTER', 'FETCH_SIZE')}\n    {cmd.replace('COUNTER', 'WRITE_SIZE')}\n\n")
        fh.write("then `python -m paper_2402_04466_amd.pmc_traffic <fetch csv> <write csv> "
                 f"{cal_mib} {tag} '<command>'`.\n\n")
        fh.write(f"Calibration: the plain copy kernel `hs::k_copy` moves {cal_bytes} B each way; the "
                 f"counters read FETCH_SIZE = {copy_f:.0f} and WRITE_SIZE = {copy_w:.0f} per copy, so "
                 f"one FETCH unit = {f_scale:.1f} B and one WRITE unit = {w_scale:.1f} B.\n\n")
        fh.write("| kernel | launches | fetched MB / launch | written MB / launch |\n|---|---|---|---|\n")
        for n, c, f, w in rows:
            fh.write(f"| `{n}` | {c} | {f / 1e6:.3f} | {w / 1e6:.3f} |\n")
        fh.write(f"\nAll convolution launches ({conv_n}): {conv_f / conv_n / 1e6:.3f} MB fetched + "
                 f"{conv_w / conv_n / 1e6:.3f} MB written per launch on average.\n")
    print(json.dumps(result["conv_hbm_bytes_per_launch"]))


if __name__ == "__main__":
    main(sys.argv)
