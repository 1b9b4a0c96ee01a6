"""Turns two rocprofv3 counter runs of bench.py into HBM bytes per launch of the dominant kernel.

    rocprofv3 --pmc FETCH_SIZE -d <dir_f> -o run --output-format csv -- python3 bench.py --steps 1 --warmup 0 \\
              --cpu-budget 0 --calibration-copy
    rocprofv3 --pmc WRITE_SIZE -d <dir_w> -o run --output-format csv -- python3 bench.py ... (same)
    python -m paper_2305_19982_amd.traffic --fetch <dir_f>/run_counter_collection.csv \\
           --write <dir_w>/run_counter_collection.csv --workload c3_gpt2_xl

Both counters are reported in KiB per dispatch.  Each is scaled by what the same counter reads for the
plain copy kernel of known size that `--calibration-copy` adds to the run (1 GiB read, 1 GiB written).
The result goes to profiles/traffic_<workload>.json, which bench.py quotes as roofline.traffic, and a
short text summary next to it.
"""
from __future__ import annotations

import argparse
import csv
import json
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
COPY_BYTES = 1 << 30


def _per_kernel(path: str, counter: str):
    rows = {}
    with open(path) as fh:
        for r in csv.DictReader(fh):
            if r["Counter_Name"] == counter:
                rows.setdefault(r["Kernel_Name"], []).append((int(r["Grid_Size"]), float(r["Counter_Value"])))
    return rows


def summarise(fetch_csv: str, write_csv: str, kernel_regex: str, workload: str) -> dict:
    """Bytes per launch of the kernels matching `kernel_regex`, from one FETCH_SIZE and one WRITE_SIZE
    run, each scaled by the same counter's reading for the one calibration copy in that run."""
    out = {"workload": workload, "unit": "bytes"}
    per_launch = {}
    for name, path, counter in (("fetch", fetch_csv, "FETCH_SIZE"), ("write", write_csv, "WRITE_SIZE")):
        rows = _per_kernel(path, counter)
        copy = [v for k, vals in rows.items() if "synth_copy_kernel" in k for _, v in vals]
        if len(copy) != 1:
            raise SystemExit(f"{path}: expected exactly one synth_copy_kernel dispatch, found {len(copy)}")
        if copy[0] <= 0:
            raise SystemExit(f"{path}: the calibration copy read {copy[0]} KiB")
        scale = COPY_BYTES / (copy[0] * 1024.0)
        dom = [v for k, vals in rows.items() if re.search(kernel_regex, k) for _, v in vals]
        if not dom:
            raise SystemExit(f"{path}: no dispatch matches {kernel_regex!r}")
        per_launch[name] = sum(dom) / len(dom) * 1024.0 * scale
        out[f"{name}_scale"] = round(scale, 4)
        out[f"{name}_copy_kib"] = copy[0]
        out[f"{name}_bytes_per_launch"] = round(per_launch[name])
        out["launches"] = len(dom)
    out["bytes_per_launch"] = round(per_launch["fetch"] + per_launch["write"])
    return out


def main() -> None:
    ap = argparse.ArgumentParser()
    ap.add_argument("--fetch", required=True)
    ap.add_argument("--write", required=True)
    ap.add_argument("--workload", required=True)
    ap.add_argument("--kernel", default=None,
                    help="regex of the dominant kernel's name (default: the multi-tensor fold with the chunk size the "
                         "built library uses for --launch-elems)")
    ap.add_argument("--launch-elems", type=int, default=30_740_800, help="elements per launch of the dominant kernel")
    args = ap.parse_args()
    if args.kernel is None:
        from . import binding

        t = binding.adama_tuning("fold", args.launch_elems)
        args.kernel = rf"multi_tensor_kernel<1, \d, {t['block']}, {t['groups_per_thread']}, \d+, false>"
    out = summarise(args.fetch, args.write, args.kernel, args.workload)
    os.makedirs(os.path.join(ROOT, "profiles"), exist_ok=True)
    dst = os.path.join(ROOT, "profiles", f"traffic_{args.workload}.json")
    with open(dst, "w") as fh:
        json.dump(out, fh, indent=1)
        fh.write("\n")
    print(json.dumps(out))


if __name__ == "__main__":
    main()
