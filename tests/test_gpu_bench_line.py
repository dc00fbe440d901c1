"""The bench's one JSON line: the keys the harness reads, and the relations between its numbers."""
import json
import os
import subprocess
import sys

import pytest

pytestmark = pytest.mark.gpu
ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _run(*args):
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *args], capture_output=True, text=True, cwd=ROOT,
                       timeout=600)
    return r


def test_bench_line_contract():
    r = _run("--config", "480p", "--steps", "3", "--warmup", "1")
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [l for l in r.stdout.splitlines() if l.strip()]
    assert len(lines) == 1, "exactly one line on stdout"
    d = json.loads(lines[0])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert key in d, key
    assert d["n_gpus"] == 1 and d["steps"] == 3 and d["warmup"] == 1
    assert d["dtype"] == "bf16" and d["data"] == "synthetic" and d["higher_is_better"] is True
    assert d["vs_baseline"] is None
    cfg = d["config"]
    assert cfg["workload"] == "480p" and "model" not in cfg
    eff = 4.0 * cfg["N"] ** 2 * cfg["d"] * cfg["B"] * cfg["H"] * cfg["k"] / cfg["g"]
    assert abs(d["value"] - eff / (d["ms_per_step"] * 1e-3) / 1e12) <= 1e-6 * d["value"]
    roof = d["roofline"]
    for key in ("bound", "achieved", "peak", "unit", "frac", "traffic", "launch_ms", "executed", "no_drop"):
        assert key in roof, key
    assert roof["bound"] == "mfma" and roof["peak"] == 2500.0 and roof["unit"] == "TFLOP/s"
    assert abs(roof["frac"] - roof["achieved"] / roof["peak"]) < 1e-9
    assert abs(roof["achieved"] - eff / (roof["launch_ms"] * 1e-3) / 1e12) <= 1e-6 * roof["achieved"]
    assert 0.0 < roof["executed"]["frac"] < 1.0 and 0.0 < roof["no_drop"]["frac"] < roof["frac"] * 1.05
    assert roof["executed"]["tiles_carried_out"] <= roof["executed"]["tiles"] == roof["no_drop"]["tiles"]
    assert roof["no_drop"]["tiles_carried_out"] == roof["no_drop"]["tiles"]   # nothing dropped means nothing dropped
    assert roof["launch_ms"] < d["ms_per_step"]
    cpu = d["cpu_baseline"]
    for key in ("value", "unit", "cores", "kind", "sample"):
        assert key in cpu, key
    assert cpu["kind"] == "oracle" and cpu["cores"] >= 1


def test_bench_refuses_more_than_one_gpu():
    r = _run("--gpus", "2")
    assert r.returncode != 0
    assert "one GPU" in r.stderr
