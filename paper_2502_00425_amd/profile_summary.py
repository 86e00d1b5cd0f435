"""Turns rocprofv3 counter output of `bench.py --prefill-only` runs into the summaries under
profiles/: HBM-side bytes per GEMM launch (profiles/gemm_hbm_traffic.json, which bench.py reads
for `roofline.traffic`) and a markdown table per run.

A counter run cannot happen inside bench.py, so the flow is: run

    rocprofv3 --pmc FETCH_SIZE -f csv -d <dir_f> -o bench -- python3 bench.py --prefill-only \\
        --configs <c> --headline <c> --steps 2 --warmup 1 --copy-calibration
    rocprofv3 --pmc WRITE_SIZE -f csv -d <dir_w> -o bench -- python3 bench.py --prefill-only \\
        --configs <c> --headline <c> --steps 2 --warmup 1 --copy-calibration

once per configuration c (each counter in a run of its own; a kernel trace of the same command,
`rocprofv3 --kernel-trace --stats -f csv -d <dir_t> ...`, is tabulated by
`python -m paper_2502_00425_amd.profile_summary trace --dir <dir_t>`; any other `--pmc` run by
`python -m paper_2502_00425_amd.profile_summary counters --dir <dir>`), then

    python -m paper_2502_00425_amd.profile_summary --config <c> --fetch <dir_f> --write <dir_w> \\
        --steps 3 --build-id <id printed by the run> [--md profiles/<name>.md]

The counters are in KiB per dispatch up to a constant factor; the factor is taken from the plain
1 GiB device copy the same run makes (--copy-calibration): 1048576 KiB read and written.
The JSON carries the build id of the library the counters were measured on; bench.py refuses
figures of another build.  Only text is parsed here: nothing of the method's arithmetic.
"""
from __future__ import annotations

import argparse
import csv
import glob
import json
import os
import re
import sys
from collections import defaultdict

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
TRAFFIC_JSON = os.path.join(ROOT, "profiles", "gemm_hbm_traffic.json")
GIB_KIB = 1048576.0


def read_counter(directory: str, counter: str):
    """-> {(kernel, grid, workgroup): [value per dispatch]} for one counter."""
    files = glob.glob(os.path.join(directory, "**", "*counter_collection.csv"), recursive=True)
    if not files:
        raise SystemExit(f"no *counter_collection.csv under {directory}")
    out = defaultdict(list)
    per_dispatch = defaultdict(float)
    meta = {}
    for f in files:
        with open(f, newline="") as fh:
            for row in csv.DictReader(fh):
                if row["Counter_Name"] != counter:
                    continue
                key = (f, row["Dispatch_Id"])
                per_dispatch[key] += float(row["Counter_Value"])
                meta[key] = (short_name(row["Kernel_Name"]), int(row["Grid_Size"]), int(row["Workgroup_Size"]))
    for key, v in per_dispatch.items():
        out[meta[key]].append(v)
    return out


def short_name(k: str) -> str:
    k = re.sub(r"^void ", "", k)
    k = re.sub(r"\(anonymous namespace\)::", "", k)
    k = re.sub(r"\(.*$", "", k)
    return k.strip()


def copy_factor(table, what: str) -> float:
    """Scale factor of a counter from the 1 GiB copies of the same run."""
    best = None
    for (name, grid, wg), vals in table.items():
        if "copyBuffer" in name or "copy" in name.lower():
            m = max(vals)
            if best is None or m > best:
                best = m
    if not best or best < 1000:
        raise SystemExit(f"no 1 GiB copy found in the {what} run (was --copy-calibration given?)")
    return GIB_KIB / best


def trace_table(directory: str, projections=None,
                only=("w4a8_", "splitk_", "hadamard_", "permute_rows", "remap_mask", "aifs_attention",
                      "vt_kernel", "rope_kernel", "w4g128_")) -> str:
    """Per (kernel, launch shape) durations of a `rocprofv3 --kernel-trace` run, from its
    *_kernel_trace.csv: dispatches, average / min / max microseconds.  With `projections`
    (the order in which a step launches its linears) the GEMM and rotate+quant dispatches of a
    one-configuration run are labelled by their position in the step, which separates shapes
    that happen to have the same number of work-groups."""
    files = glob.glob(os.path.join(directory, "**", "*kernel_trace.csv"), recursive=True)
    if not files:
        raise SystemExit(f"no *kernel_trace.csv under {directory}")
    groups = defaultdict(list)
    rows = []
    for f in files:
        with open(f, newline="") as fh:
            for row in csv.DictReader(fh):
                name = short_name(row["Kernel_Name"])
                if not name.startswith(only):
                    continue
                wg = int(row["Workgroup_Size_X"]) * int(row.get("Workgroup_Size_Y", 1) or 1) * int(row.get("Workgroup_Size_Z", 1) or 1)
                grid = int(row["Grid_Size_X"]) * int(row.get("Grid_Size_Y", 1) or 1) * int(row.get("Grid_Size_Z", 1) or 1)
                rows.append((int(row["Start_Timestamp"]), name, grid // max(wg, 1),
                             (int(row["End_Timestamp"]) - int(row["Start_Timestamp"])) / 1e3))
    rows.sort()
    seen = defaultdict(int)
    for _, name, wgs, us in rows:
        label = ""
        if projections:
            kind = "gemm" if name.startswith("w4a8_gemm_kernel") else ("quant" if name.startswith("hadamard_quant_kernel") and "false" in name else None)
            if kind:
                label = projections[seen[kind] % len(projections)]
                seen[kind] += 1
        groups[(name, wgs, label)].append(us)
    lines = ["| kernel | linear | work-groups | dispatches | avg us | median us | min us | max us |", "|---|---|---|---|---|---|---|---|"]
    for (name, wgs, label), v in sorted(groups.items()):
        med = sorted(v)[len(v) // 2]
        lines.append(f"| `{name}` | {label} | {wgs} | {len(v)} | {sum(v) / len(v):.2f} | {med:.2f} | {min(v):.2f} | {max(v):.2f} |")
    return "\n".join(lines)


def counters_table(directory: str, only=("w4a8_", "splitk_", "hadamard_", "permute_rows", "remap_mask",
                                           "aifs_attention", "w4g128_")) -> str:
    """Averages per (kernel, launch shape) of every counter a `rocprofv3 --pmc` run collected
    (each dispatch summed over the counter's instances), one column per counter."""
    files = glob.glob(os.path.join(directory, "**", "*counter_collection.csv"), recursive=True)
    if not files:
        raise SystemExit(f"no *counter_collection.csv under {directory}")
    per_dispatch = defaultdict(lambda: defaultdict(float))
    meta = {}
    names = []
    for f in files:
        with open(f, newline="") as fh:
            for row in csv.DictReader(fh):
                name = short_name(row["Kernel_Name"])
                if not name.startswith(only):
                    continue
                key = (f, row["Dispatch_Id"])
                per_dispatch[key][row["Counter_Name"]] += float(row["Counter_Value"])
                meta[key] = (name, int(row["Grid_Size"]) // max(int(row["Workgroup_Size"]), 1))
                if row["Counter_Name"] not in names:
                    names.append(row["Counter_Name"])
    groups = defaultdict(list)
    for key, c in per_dispatch.items():
        groups[meta[key]].append(c)
    lines = ["| kernel | work-groups | dispatches | " + " | ".join(names) + " |", "|---|---|---|" + "---|" * len(names)]
    for (name, wgs), cs in sorted(groups.items()):
        avg = [sum(c.get(n, 0.0) for c in cs) / len(cs) for n in names]
        lines.append(f"| `{name}` | {wgs} | {len(cs)} | " + " | ".join(f"{v:.4g}" for v in avg) + " |")
    return "\n".join(lines)


def main():
    if len(sys.argv) > 1 and sys.argv[1] == "counters":
        ap = argparse.ArgumentParser()
        ap.add_argument("mode")
        ap.add_argument("--dir", required=True, help="output directory of the --pmc run")
        ap.add_argument("--md", default=None)
        a = ap.parse_args()
        table = counters_table(a.dir)
        print(table)
        if a.md:
            with open(a.md, "a") as fh:
                fh.write("\n" + table + "\n")
        return
    if len(sys.argv) > 1 and sys.argv[1] == "trace":
        ap = argparse.ArgumentParser()
        ap.add_argument("mode")
        ap.add_argument("--dir", required=True, help="output directory of the --kernel-trace run")
        ap.add_argument("--md", default=None)
        ap.add_argument("--projections", default=None,
                        help="comma-separated linears in launch order (one-configuration runs), e.g. qkv,o,gate_up,down")
        a = ap.parse_args()
        table = trace_table(a.dir, a.projections.split(",") if a.projections else None)
        print(table)
        if a.md:
            with open(a.md, "a") as fh:
                fh.write("\n" + table + "\n")
        return
    ap = argparse.ArgumentParser()
    ap.add_argument("--config", type=int, required=True)
    ap.add_argument("--fetch", required=True, help="output directory of the FETCH_SIZE run")
    ap.add_argument("--write", required=True, help="output directory of the WRITE_SIZE run")
    ap.add_argument("--steps", type=int, required=True, help="prefill steps the run made (warm-up + timed)")
    ap.add_argument("--build-id", required=True)
    ap.add_argument("--md", default=None)
    ap.add_argument("--json", default=TRAFFIC_JSON)
    args = ap.parse_args()

    fetch = read_counter(args.fetch, "FETCH_SIZE")
    write = read_counter(args.write, "WRITE_SIZE")
    ff, wf = copy_factor(fetch, "FETCH_SIZE"), copy_factor(write, "WRITE_SIZE")

    rows = []
    gemm_bytes = 0.0
    gemm_launches = 0
    for key in sorted(set(fetch) | set(write)):
        name, grid, wg = key
        fv, wv = fetch.get(key, []), write.get(key, [])
        n = max(len(fv), len(wv))
        f_avg = sum(fv) / len(fv) * ff if fv else 0.0
        w_avg = sum(wv) / len(wv) * wf if wv else 0.0
        rows.append((name, grid // wg, n, f_avg, w_avg))
        if name.startswith("w4a8_gemm_kernel") or name.startswith("splitk_reduce_kernel"):
            gemm_bytes += (f_avg + w_avg) * 1024.0 * n
            if name.startswith("w4a8_gemm_kernel"):
                gemm_launches += n
    if gemm_launches == 0:
        raise SystemExit("no w4a8_gemm_kernel dispatch in the counter output")
    per_launch = gemm_bytes / gemm_launches
    per_step = gemm_bytes / args.steps

    data = {"build_id": args.build_id, "configs": {}}
    if os.path.exists(args.json):
        with open(args.json) as fh:
            old = json.load(fh)
        if old.get("build_id") == args.build_id:
            data = old
    data["fetch_factor"], data["write_factor"] = round(ff, 4), round(wf, 4)
    data["configs"][f"c{args.config}"] = {
        "bytes_per_gemm_launch": round(per_launch, 1), "bytes_per_step": round(per_step, 1),
        "gemm_launches_counted": gemm_launches, "steps": args.steps,
        "includes": "w4a8_gemm_kernel fetch + write, plus the split-K reduce kernel's",
    }
    os.makedirs(os.path.dirname(args.json), exist_ok=True)
    with open(args.json, "w") as fh:
        json.dump(data, fh, indent=1, sort_keys=True)
        fh.write("\n")

    lines = [f"| kernel | work-groups | dispatches | fetched MiB / dispatch | written MiB / dispatch |", "|---|---|---|---|---|"]
    for name, groups, n, f_avg, w_avg in rows:
        ours = name.startswith(("w4a8_", "splitk_", "hadamard_", "permute_rows", "remap_mask", "prepack_"))
        if not ours and not ("copyBuffer" in name and f_avg > 1e5):
            continue                                      # the framework's own set-up kernels
        lines.append(f"| `{name}` | {groups} | {n} | {f_avg / 1024.0:.1f} | {w_avg / 1024.0:.1f} |")
    table = "\n".join(lines)
    summary = (f"configs[{args.config}], build {args.build_id}: scale factors FETCH_SIZE x {ff:.3f}, WRITE_SIZE x {wf:.3f} "
               f"(from the 1 GiB copy); GEMM (with split-K reduce) {per_step / 2 ** 20:.1f} MiB per step, "
               f"{per_launch / 1e6:.1f} MB per GEMM launch over {gemm_launches} launches.")
    print(summary)
    print(table)
    if args.md:
        with open(args.md, "a") as fh:
            fh.write("\n" + summary + "\n\n" + table + "\n")


if __name__ == "__main__":
    main()
