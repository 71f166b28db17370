"""bench.py end to end on the small configuration: the JSON line carries what its contract names (needs an MI355X)."""
import json
import os
import subprocess
import sys

import pytest

pytestmark = pytest.mark.gpu
ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _run(*args):
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py")] + list(args), stdout=subprocess.PIPE,
                       stderr=subprocess.PIPE, timeout=300)
    assert r.returncode == 0, r.stderr.decode()[-1500:]
    lines = [l for l in r.stdout.decode().splitlines() if l.startswith("{")]
    assert len(lines) == 1                                  # ONE JSON line
    return json.loads(lines[0])


def test_bench_line_of_the_small_configuration():
    d = _run("--workload", "cfg1", "--steps", "3", "--warmup", "1", "--prefill", "1", "--profile-steps", "2",
             "--cpu-budget", "2", "--others", "cfg1")
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert key in d, key
    assert d["n_gpus"] == 1 and d["steps"] == 3 and d["unit"] == "IDs/s" and d["data"] == "synthetic"
    assert d["vs_baseline"] is None and d["dtype"] == "f32" and "workload" in d["config"] and "model" not in d["config"]
    roof = d["roofline"]
    for key in ("bound", "achieved", "peak", "unit", "frac", "traffic"):
        assert key in roof and key in roof["dominant_kernel"], key
    assert roof["bound"] == "hbm" and roof["peak"] == 8000.0 and roof["unit"] == "GB/s"
    assert abs(roof["frac"] - roof["achieved"] / roof["peak"]) < 1e-3
    assert roof["traffic"] is None                           # no profile was taken of this workload: no figure is claimed
    cpu = d["cpu_baseline"]
    assert cpu["kind"] == "oracle" and cpu["cores"] == 1 and cpu["value"] > 0 and cpu["sample"]
    assert d["value"] > 0
    other = d["other_workloads"]["cfg1"]
    assert "error" not in other and other["ms_per_step"] > 0 and other["roofline_frac"] is not None


def test_bench_refuses_more_than_one_gpu():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], stdout=subprocess.PIPE,
                       stderr=subprocess.PIPE, timeout=120)
    assert r.returncode != 0 and b"ONE GPU" in r.stderr
