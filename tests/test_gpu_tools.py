"""The measurement tools run end to end on the GPU and print what their readers expect (each in a process of
its own, as a user would start them)."""
import json
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
pytestmark = pytest.mark.gpu


def _last_json(cmd, timeout):
    res = subprocess.run([sys.executable, "-u", *cmd], cwd=ROOT, capture_output=True, text=True, timeout=timeout)
    assert res.returncode == 0, res.stdout[-2000:] + res.stderr[-2000:]
    lines = [l for l in res.stdout.splitlines() if l.startswith("{")]
    assert lines, res.stdout[-2000:]
    return json.loads(lines[-1])


def test_bench_line_of_a_small_workload_has_every_field():
    """bench.py on the launch-bound 2000-tensor workload: one JSON line with the contract's fields, the roofline and
    cpu_baseline objects, and the placement search's record (2 allocations x 2 distances here)."""
    d = _last_json(["bench.py", "--workload", "c4", "--steps", "3", "--warmup", "1", "--cpu-budget", "1", "--no-torch-ops",
                    "--placement-tries", "2", "--pitch-tries", "2"], 300)
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline", "library_build", "arena_placement"):
        assert key in d, key
    assert d["n_gpus"] == 1 and d["steps"] == 3 and d["warmup"] == 1 and d["unit"] == "GB/s" and d["value"] > 0
    assert d["config"]["workload"] == "c4_ragged_small" and d["vs_baseline"] is None and d["data"] == "synthetic"
    rl = d["roofline"]
    assert rl["bound"] == "hbm" and rl["peak"] == 8000.0 and rl["unit"] == "GB/s"
    assert abs(rl["frac"] - rl["achieved"] / rl["peak"]) < 1e-3
    assert d["cpu_baseline"]["kind"] == "oracle" and d["cpu_baseline"]["extrapolated"] is True and d["cpu_baseline"]["cores"] == 1
    pl = d["arena_placement"]
    assert pl["layout"] == "slab" and pl["tries"] == 2 and [len(r) for r in pl["step_ms"]] == [2, 2]
    est = pl["estimated_GB/s"]
    assert est["slowest_candidate"] <= est["first_candidate"] <= est["kept"]
    assert len(d["library_build"]) == 16


def test_in_process_ab_tool_runs():
    """bench_ab.py with the package's own library: one figure per (op, library, bound), all plausible."""
    d = _last_json(["bench_ab.py", "--ops", "fold,decay,fold@8388608", "--residency=-1,0", "--rounds", "1"], 300)
    table = d["bench_ab"]
    assert d["unit"] == "GB/s" and d["contents"] == "realistic" and len(table) == 6
    assert all(2000.0 < v < 8000.0 for v in table.values()), table
