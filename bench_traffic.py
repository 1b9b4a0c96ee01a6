"""Turns two rocprofv3 counter runs of bench.py into HBM bytes per launch of its kernels.

    rocprofv3 --pmc FETCH_SIZE -d <dir_f> -o run --output-format csv -- python3 bench.py --steps 1 --warmup 0 \\
              --cpu-budget 0 --no-torch-ops --calibration-copy [--workload c2|c3|c5]
    rocprofv3 --pmc WRITE_SIZE -d <dir_w> -o run --output-format csv -- python3 bench.py ... (same)
    python bench_traffic.py --fetch <dir_f>/run_counter_collection.csv --write <dir_w>/run_counter_collection.csv \\
           --workload c3_gpt2_xl

Both counters are reported in KiB per dispatch.  Each is scaled by what the same counter reads for the
plain copy kernel of known size that `--calibration-copy` adds to the run (1 GiB read, 1 GiB written).
The dominant kernel (the multi-tensor fold of whole layers) is reduced to bytes per launch; decay and
update dispatches are reduced to bytes per element of the step's whole state.  The result goes to
profiles/traffic_<workload>.json together with the build id of the library that ran, and bench.py quotes
it as roofline.traffic for as long as that build id is the loaded library's.
"""
from __future__ import annotations

import argparse
import csv
import json
import os
import re
import sys

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)
COPY_BYTES = 1 << 30


def _per_kernel(path: str, counter: str):
    rows = {}
    with open(path) as fh:
        for r in csv.DictReader(fh):
            if r["Counter_Name"] == counter:
                rows.setdefault(r["Kernel_Name"], []).append((int(r["Grid_Size"]), float(r["Counter_Value"])))
    return rows


def _scale(rows: dict, path: str) -> float:
    copy = [v for k, vals in rows.items() if "synth_copy_kernel" in k for _, v in vals]
    if len(copy) != 1:
        raise SystemExit(f"{path}: expected exactly one synth_copy_kernel dispatch, found {len(copy)}")
    if copy[0] <= 0:
        raise SystemExit(f"{path}: the calibration copy read {copy[0]} KiB")
    return COPY_BYTES / (copy[0] * 1024.0), copy[0]


def summarise(fetch_csv: str, write_csv: str, kernel_regex: str, workload: str, grid_min: int = 0) -> dict:
    """Bytes per launch of the kernels matching `kernel_regex` (dispatches of at least grid_min work-items),
    from one FETCH_SIZE and one WRITE_SIZE run, each scaled by the same counter's reading for the one
    calibration copy in that run."""
    out = {"workload": workload, "unit": "bytes"}
    per_launch = {}
    for name, path, counter in (("fetch", fetch_csv, "FETCH_SIZE"), ("write", write_csv, "WRITE_SIZE")):
        rows = _per_kernel(path, counter)
        scale, copy_kib = _scale(rows, path)
        dom = [v for k, vals in rows.items() if re.search(kernel_regex, k) for g, v in vals if g >= grid_min]
        if not dom:
            raise SystemExit(f"{path}: no dispatch matches {kernel_regex!r}")
        per_launch[name] = sum(dom) / len(dom) * 1024.0 * scale
        out[f"{name}_scale"] = round(scale, 4)
        out[f"{name}_copy_kib"] = copy_kib
        out[f"{name}_bytes_per_launch"] = round(per_launch[name])
        out["launches"] = len(dom)
    out["bytes_per_launch"] = round(per_launch["fetch"] + per_launch["write"])
    return out


def total_bytes(fetch_csv: str, write_csv: str, kernel_regex: str) -> tuple:
    """Scaled fetch + write bytes summed over every dispatch matching `kernel_regex`, and their number."""
    total, n = 0.0, 0
    for path, counter in ((fetch_csv, "FETCH_SIZE"), (write_csv, "WRITE_SIZE")):
        rows = _per_kernel(path, counter)
        scale, _ = _scale(rows, path)
        vals = [v for k, vs in rows.items() if re.search(kernel_regex, k) for _, v in vs]
        total += sum(vals) * 1024.0 * scale
        n = len(vals)
    return total, n


def main() -> None:
    ap = argparse.ArgumentParser()
    ap.add_argument("--fetch", required=True)
    ap.add_argument("--write", required=True)
    ap.add_argument("--workload", required=True, help="workload name as bench.py prints it, e.g. c3_gpt2_xl")
    ap.add_argument("--optimizer", default="adama", choices=["adama", "sgdm"])
    ap.add_argument("--steps", type=int, default=2, help="mini-batches of the separate-call path in the profiled run "
                    "(bench.py --steps 1 --warmup 0 runs one timed and one instrumented step)")
    args = ap.parse_args()
    from paper_2305_19982_amd import binding
    from synth import configs

    w = next(f() for f in configs.FULL.values() if f().name == args.workload)
    fold_op, decay_op, apply_op = (7, 6, 8) if args.optimizer == "sgdm" else (1, 0, 2)
    big = max(w.layer_elems(li) for li in range(len(w.layers)) if len(w.layers[li]) > 1)
    t = binding.adama_tuning(fold_op, big)
    gt = {"f32": 0, "bf16": 1, "f16": 2}[w.gdtype]
    kernel = rf"multi_tensor_kernel<{fold_op}, {gt}, {t['block']}, {t['groups_per_thread']}, \d+, false>"
    # the dominant kernel as bench.py defines it: every multi-tensor fold launch of at least big_launch_elems elements
    out = summarise(args.fetch, args.write, kernel, args.workload)
    out["kernel"] = kernel
    state = 8 if args.optimizer == "sgdm" else 16
    timed = [w.layer_elems(li) for li in range(len(w.layers)) if len(w.layers[li]) > 1 and w.layer_elems(li) >= t["big_launch_elems"]]
    out["algorithmic_bytes_per_launch"] = round(sum(timed) / len(timed) * (state + w.grad_bytes))
    out["ratio"] = round(out["bytes_per_launch"] / out["algorithmic_bytes_per_launch"], 5)
    for name, op, bytes_per_param in (("decay", decay_op, state), ("update", apply_op, 8 + state // 2)):
        tot, n = total_bytes(args.fetch, args.write, rf"multi_tensor_kernel<{op}, 0, ")
        out[name] = {"dispatches": n, "bytes_per_param": round(tot / (args.steps * w.P), 4), "algorithmic": bytes_per_param}
    out["build_id"] = binding.adama_build_id()
    os.makedirs(os.path.join(ROOT, "profiles"), exist_ok=True)
    suffix = "" if args.optimizer == "adama" else f"_{args.optimizer}"
    dst = os.path.join(ROOT, "profiles", f"traffic_{args.workload}{suffix}.json")
    with open(dst, "w") as fh:
        json.dump(out, fh, indent=1)
        fh.write("\n")
    print(json.dumps(out))


if __name__ == "__main__":
    main()
