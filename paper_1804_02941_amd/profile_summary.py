"""Summaries of rocprofv3 runs of bench.py for profiles/ (text and one JSON file; nothing here runs on a GPU).

    python -m paper_1804_02941_amd.profile_summary --trace DIR --fetch DIR --write DIR [--out profiles]

DIR are the output folders (-d) of three runs, CSV output:
    rocprofv3 --kernel-trace --stats --output-format csv -d DIR -- python bench.py --steps 50 --warmup 5
    rocprofv3 --pmc FETCH_SIZE --output-format csv -d DIR -- python bench.py --steps 20 --warmup 3 --headline-only --cpu-batch 0 --copy-calibration
    rocprofv3 --pmc WRITE_SIZE --output-format csv -d DIR -- python bench.py --steps 20 --warmup 3 --headline-only --cpu-batch 0 --copy-calibration
Writes bench_config3_kernel_stats.md (average launch durations per kernel and grid), bench_config3_hbm_counters.md
(HBM bytes per launch, the counters scaled by what they read for the 256 MiB copies of --copy-calibration) and
hbm_traffic.json (the dominant kernel's bytes, read by bench.py; it records the commit of the tree it was measured on).
"""
from __future__ import annotations

import argparse
import collections
import csv
import glob
import json
import os
import re
import subprocess

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
COPY_BYTES = 256 << 20


def _one(folder, pattern):
    files = sorted(glob.glob(os.path.join(folder, "**", pattern), recursive=True))
    if not files:
        raise SystemExit(f"no {pattern} under {folder}")
    return files[-1]


def short(name):
    name = re.sub(r"^void ", "", name).replace("(anonymous namespace)::", "")
    name = re.sub(r"\(.*$", "", name)
    return name.replace("dab::", "")


def kernel_durations(folder):
    """{(kernel, grid, workgroup): [durations in us]} of the library's kernels, in launch order."""
    acc = collections.OrderedDict()
    with open(_one(folder, "*kernel_trace.csv")) as f:
        rows = sorted(csv.DictReader(f), key=lambda r: int(r["Start_Timestamp"]))
    for r in rows:
        if "dab::" not in r["Kernel_Name"]:
            continue
        key = (short(r["Kernel_Name"]), int(r["Grid_Size_X"]), int(r["Workgroup_Size_X"]))
        acc.setdefault(key, []).append((int(r["End_Timestamp"]) - int(r["Start_Timestamp"])) / 1e3)
    return acc


def dominant_kernel_by_neighbour(folder, kernel="binconv_direct_kernel<1, 5, false, false>", grid=131072):
    """Durations (us) of the dominant kernel's launches: those that follow another launch of it (the graphs of
    ten back-to-back launches bench.py times for `roofline`), and those inside a step (behind the sort kernel)."""
    with open(_one(folder, "*kernel_trace.csv")) as f:
        rows = sorted(csv.DictReader(f), key=lambda r: int(r["Start_Timestamp"]))
    same, in_step, prev = [], [], None
    for r in rows:
        if kernel in r["Kernel_Name"] and int(r["Grid_Size_X"]) == grid:
            d = (int(r["End_Timestamp"]) - int(r["Start_Timestamp"])) / 1e3
            if prev is not None and kernel in prev["Kernel_Name"]:
                same.append(d)
            elif prev is not None and "binarize_sort_kernel" in prev["Kernel_Name"]:
                in_step.append(d)
        prev = r
    return same, in_step


STEP_KERNELS = ["prepare_rows_kernel", "prepare_rows_kernel", "binarize_sort_kernel", "binconv_direct_kernel", "binconv_direct_kernel",
                "binconv_direct_kernel", "binconv_direct_kernel", "binconv_block_kernel", "binconv_block_kernel"]


def headline_steps(folder, conv2_grid=131072):
    """The launches of the headline step (config 3, batch 256), found in the trace by their order: per position the
    kernel (with its template arguments) and its durations, and the spans from the first start to the last end."""
    with open(_one(folder, "*kernel_trace.csv")) as f:
        rows = sorted(csv.DictReader(f), key=lambda r: int(r["Start_Timestamp"]))
    names = [short(r["Kernel_Name"]) for r in rows]
    per, spans, i, n = [[] for _ in STEP_KERNELS], [], 0, len(STEP_KERNELS)
    labels = [None] * n
    while i + n <= len(rows):
        if all(names[i + k].startswith(STEP_KERNELS[k] + "<") for k in range(n)) and int(rows[i + 3]["Grid_Size_X"]) == conv2_grid:
            for k in range(n):
                per[k].append((int(rows[i + k]["End_Timestamp"]) - int(rows[i + k]["Start_Timestamp"])) / 1e3)
                labels[k] = names[i + k]
            spans.append((int(rows[i + n - 1]["End_Timestamp"]) - int(rows[i]["Start_Timestamp"])) / 1e3)
            i += n
        else:
            i += 1
    return labels, per, spans


def counter_values(folder):
    """({(kernel, grid): [values in KiB]} of the library's kernels, [values of the 256 MiB calibration copies])."""
    acc, copies = collections.OrderedDict(), []
    with open(_one(folder, "*counter_collection.csv")) as f:
        for r in csv.DictReader(f):
            v = float(r["Counter_Value"])
            if "dab::" in r["Kernel_Name"]:
                acc.setdefault((short(r["Kernel_Name"]), int(r["Grid_Size"])), []).append(v)
            elif "copyBuffer" in r["Kernel_Name"]:                    # the runtime's device-to-device copy kernel
                copies.append(v)
    return acc, copies


def calibration(copies, name):
    """KiB of real traffic per counter unit, from the three largest copies (each moves 256 MiB each way)."""
    big = sorted(copies)[-3:]
    if len(big) < 3 or max(big) > 1.05 * min(big):
        raise SystemExit(f"{name}: the calibration copies are missing or disagree: {big}")
    return (COPY_BYTES / 1024.0) / (sum(big) / 3.0), big


def git_commit():
    try:
        head = subprocess.run(["git", "rev-parse", "HEAD"], cwd=ROOT, capture_output=True, text=True, check=True).stdout.strip()
        dirty = subprocess.run(["git", "status", "--porcelain", "--", "paper_1804_02941_amd", "bench.py", "include"], cwd=ROOT,
                               capture_output=True, text=True, check=True).stdout.strip()
        return head + (" (with uncommitted changes)" if dirty else "")
    except Exception:
        return "unknown"


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--trace", required=True)
    ap.add_argument("--fetch", required=True)
    ap.add_argument("--write", required=True)
    ap.add_argument("--out", default=os.path.join(ROOT, "profiles"))
    args = ap.parse_args()
    commit = git_commit()

    dur = kernel_durations(args.trace)
    lines = ["# Library kernels over bench.py (config 3, batch 256, and the measurements beside it): launch durations", "",
             "Command (the summary is of its kernel trace; written by `python -m paper_1804_02941_amd.profile_summary`):", "",
             "    rocprofv3 --kernel-trace --stats --output-format csv -d DIR -- python bench.py --steps 50 --warmup 5", "",
             f"Tree: {commit}", "",
             "One row per kernel, grid (threads) and workgroup size, in the order of first launch.  The headline step is",
             "prepare_rows_kernel<256,...> (five layers' weight sides + a share of all activation packing),",
             "prepare_rows_kernel<512, 26,...> (conv6's weight side + the rest of the packing), binarize_sort_kernel (the rows they flag: none here), then",
             "the six products: binconv_direct_kernel<1, 5, false, false> grid 131072 is conv2, <2, 3, true, false> conv3,",
             "<4, 3, true, false> grid 115712 conv4 and conv5, binconv_block_kernel<false, false, 8, 16, 4> grid 65536 conv6 and",
             "<false, false, 2, 4, 4> grid 16384 fc7.  The other rows belong to the measurements beside the headline: the separate",
             "calls of the stage table, the chain that hands bits on (product kernels whose BITS argument is true), the training side, the",
             "weights-only layers (wbin_prepare_kernel, binconv_mfma_kernel<8, 0, 1>), configurations 2, 4 and 5 (config 5's",
             "weight sides are the binarize_rows_kernel launches with grids 2097152 and 1048576), batch 32, and the popcount-rate probe.", "",
             "| kernel | grid | workgroup | launches | average us | min us | max us |", "|---|---|---|---|---|---|---|"]
    for (k, grid, wg), v in dur.items():
        lines.append(f"| `{k}` | {grid} | {wg} | {len(v)} | {sum(v) / len(v):.2f} | {min(v):.2f} | {max(v):.2f} |")
    same, in_step = dominant_kernel_by_neighbour(args.trace)
    if same and in_step:
        lines += ["", f"The dominant kernel, conv2's `binconv_direct_kernel<1, 5, false, false>` (grid 131072), by what ran before it:",
                  f"behind another launch of itself (the graphs of ten launches that bench.py times for `roofline`): {len(same)} launches,",
                  f"average {sum(same) / len(same):.2f} us, min {min(same):.2f}; inside a step (behind the sort kernel, caches cold for its",
                  f"operands): {len(in_step)} launches, average {sum(in_step) / len(in_step):.2f} us, min {min(in_step):.2f}.  Under the profiler",
                  "every launch is serialised and a few per cent longer than in a plain graph replay (bench.py's HIP events:",
                  "`roofline.launch_ms` of the same tree)."]
    labels, per, spans = headline_steps(args.trace)
    if spans:
        what = ["weight sides of conv2-conv5, fc7 + a share of the packing", "weight side of conv6 + the rest of the packing",
                "rows handed to the sort (none here)", "product conv2", "product conv3", "product conv4", "product conv5",
                "product conv6", "product fc7"]
        lines += ["", f"The headline step kernel by kernel ({len(spans)} steps in the trace; under the profiler a launch starts when the one",
                  f"before it ends, so the durations add up to the span of a step, {sum(spans) / len(spans):.1f} us on average):", "",
                  "| launch | kernel | average us |", "|---|---|---|"]
        for k, v in enumerate(per):
            lines.append(f"| {what[k]} | `{labels[k]}` | {sum(v) / len(v):.2f} |")
    with open(os.path.join(args.out, "bench_config3_kernel_stats.md"), "w") as f:
        f.write("\n".join(lines) + "\n")

    fetch, fcopies = counter_values(args.fetch)
    write, wcopies = counter_values(args.write)
    fscale, fbig = calibration(fcopies, "FETCH_SIZE")
    wscale, wbig = calibration(wcopies, "WRITE_SIZE")
    lines = ["# Library kernels over bench.py (config 3, batch 256): HBM bytes per launch", "",
             "Commands (one counter per run; written by `python -m paper_1804_02941_amd.profile_summary`):", "",
             "    rocprofv3 --pmc FETCH_SIZE --output-format csv -d DIR -- python bench.py --steps 20 --warmup 3 --headline-only --cpu-batch 0 --copy-calibration",
             "    rocprofv3 --pmc WRITE_SIZE --output-format csv -d DIR -- python bench.py --steps 20 --warmup 3 --headline-only --cpu-batch 0 --copy-calibration", "",
             f"Tree: {commit}", "",
             f"Calibration: the three 256 MiB device-to-device copies read FETCH_SIZE = {sum(fbig) / 3:.1f} and WRITE_SIZE = {sum(wbig) / 3:.1f}",
             f"(KiB units) for 262144 KiB each way, so a FETCH_SIZE unit is {fscale:.4f} KiB and a WRITE_SIZE unit {wscale:.4f} KiB.", "",
             "| kernel | grid | launches | read MB | written MB | total MB |", "|---|---|---|---|---|---|"]
    table = {}
    for key, v in fetch.items():
        rd = sum(v) / len(v) * fscale * 1024.0
        w = write.get(key)
        wr = sum(w) / len(w) * wscale * 1024.0 if w else float("nan")
        table[key] = (rd, wr)
        lines.append(f"| `{key[0]}` | {key[1]} | {len(v)} | {rd / 1e6:.3f} | {wr / 1e6:.3f} | {(rd + wr) / 1e6:.3f} |")
    with open(os.path.join(args.out, "bench_config3_hbm_counters.md"), "w") as f:
        f.write("\n".join(lines) + "\n")

    # the dominant kernel of the headline step: the product of conv2 (the direct kernel's launch with the largest grid)
    dom = max((k for k in table if k[0].startswith("binconv_direct_kernel")), key=lambda k: table[k][1])
    rd, wr = table[dom]
    with open(os.path.join(args.out, "hbm_traffic.json"), "w") as f:
        json.dump({"commit": commit, "layer": "conv2", "batch": 256, "kernel": dom[0], "grid": dom[1],
                   "fetch_bytes": round(rd), "write_bytes": round(wr), "traffic_bytes": round(rd + wr),
                   "fetch_size_unit_kib": round(fscale, 5), "write_size_unit_kib": round(wscale, 5),
                   "source": "profiles/bench_config3_hbm_counters.md (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE over bench.py "
                             "--headline-only --copy-calibration, scaled by the 256 MiB copies)"}, f, indent=1)
        f.write("\n")
    print("wrote", args.out)


if __name__ == "__main__":
    main()
