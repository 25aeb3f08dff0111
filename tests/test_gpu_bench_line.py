"""The benchmark command exactly as the harness runs it at the end of a round: it must exit 0 and print
one JSON line with the contract's keys (this is the command that an index error once stopped)."""
import json
import os
import subprocess
import sys

import pytest

pytestmark = pytest.mark.gpu

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_driver_command_prints_the_contract_line():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "1", "--steps", "20", "--warmup", "5"],
                       cwd=ROOT, capture_output=True, text=True, timeout=400)
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [ln for ln in r.stdout.splitlines() if ln.strip()]
    assert len(lines) == 1, lines[:3]
    d = json.loads(lines[0])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert key in d, key
    assert d["steps"] == 20 and d["warmup"] == 5 and d["n_gpus"] == 1 and d["p99_samples"] == 20
    assert d["unit"] == "ms" and d["higher_is_better"] is False and d["vs_baseline"] is None and d["dtype"] == "bf16"
    assert d["config"]["workload"].startswith("cfg2") and "model" not in d["config"]
    assert 0.05 < d["value"] < 50.0 and d["value"] == d["hp_p99_ms"]
    assert 0.5 * 20 * 5.0 < d["ms_per_step"] * d["steps"] < 2.0 * 20 * 5.0 + 50      # 20 arrivals at 200/s: about 100 ms
    roof = d["roofline"]
    assert roof["bound"] == "mfma" and roof["unit"] == "TFLOP/s" and roof["peak"] == 2500.0
    assert abs(roof["frac"] - roof["achieved"] / roof["peak"]) < 1e-9 and 0.2 < roof["frac"] < 1.0
    assert roof["traffic"] > 0 and roof["traffic_over_algorithmic"] > 1.0
    cpu = d["cpu_baseline"]
    assert cpu["kind"] == "oracle" and cpu["cores"] >= 1 and cpu["value"] > 0 and cpu["sample"]
    tail = d["tail_study"]
    assert tail["full_scheduler"]["requests"] == 5000 and tail["static_masks"]["requests"] == 5000
    assert d["scheduler"]["context_totals"]["revocations"] >= d["scheduler"]["be_revocations"]
    # more than one GPU is refused with a message
    r2 = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], cwd=ROOT, capture_output=True, text=True, timeout=60)
    assert r2.returncode != 0 and "one GPU" in r2.stderr
