"""bench.py: the command-line contract (one GPU only) and the shape of its JSON line."""
import json
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    p = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True, timeout=120)
    assert p.returncode != 0
    assert "ONE GPU" in p.stderr
    assert p.stdout.strip() == ""


@pytest.mark.gpu
def test_json_line_on_the_small_config():
    """config 1 (the case the oracle finishes at once), few steps: one JSON line with the fields
    of the contract, the output checked against the oracle inside the run"""
    p = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--config", "1", "--steps", "40",
                        "--warmup", "8", "--buffers", "4", "--no-prefetch"],
                       capture_output=True, text=True, timeout=600)
    assert p.returncode == 0, p.stderr[-2000:]
    lines = [ln for ln in p.stdout.splitlines() if ln.strip()]
    assert len(lines) == 1
    d = json.loads(lines[0])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step",
                "higher_is_better", "scaling", "vs_baseline", "dtype", "data", "config",
                "roofline", "cpu_baseline"):
        assert key in d, key
    assert d["n_gpus"] == 1 and d["steps"] == 40 and d["warmup"] == 8
    assert d["unit"] == "modMAC/s" and d["vs_baseline"] is None and d["data"] == "synthetic"
    assert d["config"]["workload"].startswith("config 1")
    r = d["roofline"]
    assert r["bound"] in ("hbm", "mfma") and r["peak"] > 0
    assert abs(r["frac"] - r["achieved"] / r["peak"]) < 1e-3
    c = d["cpu_baseline"]
    assert c["kind"] == "oracle" and c["cores"] >= 1 and c["value"] > 0
    assert d["output_matches_oracle"] is True
    assert d["two_streams"]["outputs_equal_one_stream"] is True
    # value = modular MACs per step / time per step
    assert abs(d["value"] - d["config"]["mod_macs_per_step"] / (d["ms_per_step"] * 1e-3)) <= 1e-3 * d["value"]
