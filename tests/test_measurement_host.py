"""Host logic of the measurement tools: the counter-CSV reduction behind roofline.traffic and the
byte accounting of bench.py (no GPU)."""
import csv
import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

FOLD = "void adama::multi_tensor_kernel<1, 1, 128, 1, 7, false>(adama::Table<80>, adama::Scalars)"
OTHER = "void adama::multi_tensor_kernel<2, 0, 256, 1, 7, false>(adama::Table<80>, adama::Scalars)"
COPY = "synth_copy_kernel(float __vector(4)*, float __vector(4) const*, unsigned long)"


def _write(path, counter, rows):
    with open(path, "w", newline="") as fh:
        w = csv.writer(fh, quoting=csv.QUOTE_NONNUMERIC)
        w.writerow(["Dispatch_Id", "Grid_Size", "Kernel_Name", "Counter_Name", "Counter_Value"])
        for i, (kernel, value) in enumerate(rows):
            w.writerow([i, 256, kernel, counter, value])
            w.writerow([i, 256, kernel, "SOMETHING_ELSE", 1.0])


def test_traffic_summary_scales_by_the_calibration_copy(tmp_path):
    import bench_traffic as traffic

    f, w = str(tmp_path / "f.csv"), str(tmp_path / "w.csv")
    # the fetch counter reads half of the real KiB (as on MI355X), the write counter the real KiB
    _write(f, "FETCH_SIZE", [(COPY, 524288.0), (FOLD, 1000.0), (OTHER, 77.0), (FOLD, 3000.0)])
    _write(w, "WRITE_SIZE", [(COPY, 1048576.0), (FOLD, 1600.0), (FOLD, 4800.0), (OTHER, 5.0)])
    out = traffic.summarise(f, w, r"multi_tensor_kernel<1, \d, 128, 1, \d+, false>", "unit_test")
    assert out["fetch_scale"] == 2.0 and out["write_scale"] == 1.0 and out["launches"] == 2
    assert out["fetch_bytes_per_launch"] == 2000 * 1024 * 2
    assert out["write_bytes_per_launch"] == 3200 * 1024
    assert out["bytes_per_launch"] == 2000 * 1024 * 2 + 3200 * 1024


def test_traffic_summary_refuses_ambiguous_input(tmp_path):
    import bench_traffic as traffic

    f, w = str(tmp_path / "f.csv"), str(tmp_path / "w.csv")
    _write(f, "FETCH_SIZE", [(COPY, 1.0), (COPY, 1.0), (FOLD, 1.0)])
    _write(w, "WRITE_SIZE", [(COPY, 1.0), (FOLD, 1.0)])
    with pytest.raises(SystemExit, match="exactly one synth_copy_kernel"):
        traffic.summarise(f, w, "multi_tensor_kernel<1", "x")
    _write(f, "FETCH_SIZE", [(COPY, 1.0), (OTHER, 1.0)])
    with pytest.raises(SystemExit, match="no dispatch matches"):
        traffic.summarise(f, w, "multi_tensor_kernel<1", "x")


def test_bench_byte_accounting():
    import bench
    from synth import configs

    w = configs.FULL["c3"]()
    assert bench.per_param_bytes(w, "adama") == 16 + 16 * 18 + 16 == 320
    assert bench.per_param_bytes(w, "adamw") == 320
    assert bench.per_param_bytes(w, "adama", fused=True) == 16 * 18 + 8 == 296
    assert bench.per_param_bytes(w, "sgdm") == 8 + 16 * 10 + 12 == 180
    assert bench.per_param_bytes(w, "sgdm", fused=True) == 16 * 10 + 8 == 168
    assert bench.algorithmic_bytes_per_step(w) == 320 * 1557611200
    w2 = configs.FULL["c2"]()
    assert bench.per_param_bytes(w2, "adama") == 16 + 8 * 20 + 16 == 192


def test_bench_refuses_more_than_one_gpu():
    import subprocess

    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0 and "one GPU" in r.stderr and r.stdout.strip() == ""
