"""Turns two rocprofv3 --pmc runs of bench.py (FETCH_SIZE, then WRITE_SIZE) into HBM traffic per
kernel launch, calibrated against the library's plain copy kernel of known size.

  python -m paper_2101_07706_amd.pmc_traffic --fetch F.csv --write W.csv --key large \
         --json profiles/traffic.json --summary profiles/large_traffic.txt --command "<how F/W were made>"

F.csv / W.csv are the *_counter_collection.csv files rocprofv3 writes with --output-format csv.
bench.py copies 512 MiB with csgs_calib_copy, so that kernel's FETCH_SIZE (WRITE_SIZE) reading
stands for 512 MiB read (written); every other kernel's reading is scaled by the same factor.
bench.py reads the JSON file for the `traffic` entry of its roofline object.

A third run with the profiler's derived counters MfmaUtil (busy cycles of the matrix cores over
elapsed cycles x SIMDs, in percent) and MfmaFlopsF64 gives the matrix-core utilisation of every
launch of the layer GEMM (listed per template instance, i.e. per layer shape) and of the library's
back-to-back matrix-instruction kernel:

  python -m paper_2101_07706_amd.pmc_traffic --mfma M.csv --summary profiles/large_step_mfma_util.txt --command "..."
"""
from __future__ import annotations

import argparse
import collections
import csv
import json
import os

CALIB_BYTES = 512 * 2 ** 20

NAMES = [("aggregate_k", "aggregate"), ("gemm_f32_k", "layer_gemm"), ("gather_rows_k", "gather_rows"),
         ("remote_count_k", "remote_count"), ("csgs::scan_edges", "scan_edges"), ("csgs::cand_partials", "cand_partials"),
         ("csgs::cand_emit", "cand_emit"),
         ("csgs::row_prefix", "row_prefix"), ("csgs::draw", "draw"), ("csgs::hits_fused", "hits_fused"),
         ("csgs::adj_fused", "adj_fused"), ("csgs::copy_k", "copy")]


def short_name(kernel: str):
    for needle, name in NAMES:
        if needle in kernel:
            return name
    return None


def per_kernel(path: str, counter: str):
    acc = collections.defaultdict(list)
    with open(path, newline="") as f:
        for row in csv.DictReader(f):
            if row["Counter_Name"] != counter:
                continue
            name = short_name(row["Kernel_Name"])
            if name:
                acc[name].append(float(row["Counter_Value"]))
    return {k: (sum(v) / len(v), len(v)) for k, v in acc.items()}


def mfma_summary(path: str, out: str, command: str):
    """Per kernel instance that issued matrix instructions: launches, mean MfmaUtil, mean MfmaFlopsF64."""
    util, flops = collections.defaultdict(list), collections.defaultdict(list)
    with open(path, newline="") as f:
        for row in csv.DictReader(f):
            k = row["Kernel_Name"]
            if "gemm_f32_k" not in k and "mfma_f64_k" not in k:
                continue
            k = k[k.index("csgs::"):] if "csgs::" in k else k
            k = k.split("(")[0]
            if row["Counter_Name"] == "MfmaUtil":
                util[k].append(float(row["Counter_Value"]))
            elif row["Counter_Name"] == "MfmaFlopsF64":
                flops[k].append(float(row["Counter_Value"]))
    lines = ["Matrix-core utilisation per launch (rocprofv3 --pmc MfmaUtil MfmaFlopsF64): busy cycles of the matrix cores over",
             "elapsed cycles x SIMDs, and fp64 matrix flops counted by the hardware",
             f"command: {command}", "",
             f"{'kernel':48s} {'launches':>8s} {'MfmaUtil %':>11s} {'GFLOP':>9s}"]
    for k in sorted(util):
        u, fl = util[k], flops.get(k, [0.0])
        lines.append(f"{k[:48]:48s} {len(u):8d} {sum(u) / len(u):11.1f} {sum(fl) / len(fl) / 1e9:9.3f}")
    lines += ["", "gemm_f32_k<BN, mode, vector, regular shape, folded K tail, BM>: in the named workload the three instances are the",
              "three layers (256 -> 256, 100 -> 256 with the folded tail, 256 -> 47); mfma_f64_k<false / true> is the library's",
              "yardstick: the same instruction back to back from registers / with operands re-read from LDS."]
    with open(out, "w") as f:
        f.write("\n".join(lines) + "\n")
    print("\n".join(lines))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--fetch")
    ap.add_argument("--write")
    ap.add_argument("--mfma")
    ap.add_argument("--key", help="workload name as bench.py uses it, e.g. large or large_x16")
    ap.add_argument("--json")
    ap.add_argument("--summary", required=True)
    ap.add_argument("--command", default="")
    a = ap.parse_args()
    if a.mfma:
        mfma_summary(a.mfma, a.summary, a.command)
        return
    if not (a.fetch and a.write and a.key and a.json):
        ap.error("--fetch, --write, --key and --json are needed for the traffic table")
    fetch, write = per_kernel(a.fetch, "FETCH_SIZE"), per_kernel(a.write, "WRITE_SIZE")
    f_scale = CALIB_BYTES / fetch["copy"][0]      # bytes per counter unit
    w_scale = CALIB_BYTES / write["copy"][0]
    table = {}
    lines = [f"HBM traffic per kernel launch, workload '{a.key}' (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, two runs)",
             f"command: {a.command}",
             f"calibration: copy kernel of {CALIB_BYTES} bytes reads FETCH_SIZE {fetch['copy'][0]:.1f} and WRITE_SIZE "
             f"{write['copy'][0]:.1f} per launch -> {f_scale:.1f} / {w_scale:.1f} bytes per counter unit", "",
             f"{'kernel':16s} {'launches':>8s} {'fetch MB':>10s} {'write MB':>10s} {'total MB':>10s}"]
    for name in sorted(set(fetch) | set(write)):
        if name == "copy":
            continue
        fb = fetch.get(name, (0.0, 0))[0] * f_scale
        wb = write.get(name, (0.0, 0))[0] * w_scale
        table[name] = fb + wb
        lines.append(f"{name:16s} {fetch.get(name, (0, 0))[1]:8d} {fb / 1e6:10.3f} {wb / 1e6:10.3f} {(fb + wb) / 1e6:10.3f}")
    data = json.load(open(a.json)) if os.path.exists(a.json) else {}
    data[a.key] = table
    with open(a.json, "w") as f:
        json.dump(data, f, indent=1, sort_keys=True)
    with open(a.summary, "w") as f:
        f.write("\n".join(lines) + "\n")
    print("\n".join(lines))


if __name__ == "__main__":
    main()
