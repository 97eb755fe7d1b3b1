"""bench.py's command line and output contract: one JSON line with the agreed keys, the
roofline and cpu_baseline objects, and a refusal of more than one GPU."""
import json
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
BENCH = os.path.join(ROOT, "bench.py")


def test_more_than_one_gpu_is_refused():
    r = subprocess.run([sys.executable, BENCH, "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0
    assert "single-GPU" in r.stderr and r.stdout.strip() == ""


@pytest.mark.gpu
def test_one_json_line_with_the_agreed_keys():
    r = subprocess.run([sys.executable, BENCH, "--workload", "tiny", "--steps", "20", "--warmup", "3"],
                       capture_output=True, text=True, timeout=600)
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [l for l in r.stdout.splitlines() if l.strip()]
    assert len(lines) == 1
    d = json.loads(lines[0])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step",
                "higher_is_better", "scaling", "vs_baseline", "dtype", "data", "config",
                "roofline", "cpu_baseline"):
        assert key in d, key
    assert d["n_gpus"] == 1 and d["steps"] == 20 and d["warmup"] == 3
    assert d["unit"] == "params/s" and d["higher_is_better"] is True and d["vs_baseline"] is None
    assert d["dtype"] == "f32" and d["data"] == "synthetic"
    assert d["config"]["workload"] == "tiny" and "model" not in d["config"]
    assert d["value"] > 0 and abs(d["value"] - d["config"]["params"] / (d["ms_per_step"] * 1e-3)) \
        <= 1e-6 * d["value"]
    roof = d["roofline"]
    assert roof["bound"] == "hbm" and roof["unit"] == "GB/s" and roof["peak"] == 8000.0
    assert abs(roof["frac"] - roof["achieved"] / roof["peak"]) < 1e-12 and "traffic" in roof
    cpu = d["cpu_baseline"]
    assert cpu["kind"] == "oracle" and cpu["unit"] == "params/s" and cpu["value"] > 0
    assert cpu["cores"] >= 1 and isinstance(cpu["sample"], str)
    assert cpu["max_abs_err_vs_oracle"] is not None and cpu["max_err_over_bound"] < 1.0
    # parity is total: every element of the workload went through the oracle
    assert cpu["elements_compared"] == d["config"]["params"] and cpu["parity_ok"] is True
    assert cpu["fragments_covered"] == [0]
    assert roof["traffic"] is None or isinstance(roof["traffic"], int)
    assert isinstance(roof["traffic_source"], str)
    assert d["config"]["library_build"]
