"""bench.py prints one JSON line with the fields the harness reads; checked here on cut-down workloads."""
import json
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
pytestmark = pytest.mark.gpu


def bench_line(*args):
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *args], cwd=ROOT, capture_output=True, text=True,
                       timeout=600)
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [l for l in r.stdout.splitlines() if l.startswith("{")]
    assert len(lines) == 1, r.stdout[-2000:]
    return json.loads(lines[0])


@pytest.mark.parametrize("config,extra,bound,dtype", [
    (3, ["--chains", "256", "--iters", "20"], "mfma", "f64"),
    (2, ["--chains", "64", "--iters", "20"], "alu", "f64"),
    (4, ["--chains", "32", "--iters", "3"], "mfma", "f32"),
    (5, ["--chains", "256", "--iters", "3"], "hbm", "f32"),
])
def test_bench_line_has_the_contract_fields(config, extra, bound, dtype):
    d = bench_line("--config", str(config), "--steps", "2", "--warmup", "1", "--no-cpu-baseline", *extra)
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config", "roofline"):
        assert key in d, key
    assert d["n_gpus"] == 1 and d["steps"] == 2 and d["warmup"] == 1 and d["higher_is_better"] is True
    assert d["unit"] == "grad-evals/s" and d["value"] > 0 and d["ms_per_step"] > 0
    assert d["dtype"] == dtype and d["data"] == "synthetic" and d["vs_baseline"] is None
    assert "workload" in d["config"] and "model" not in d["config"]
    r = d["roofline"]
    assert r["bound"] == bound and r["peak"] > 0 and r["achieved"] > 0 and r["kernel_ms"] > 0
    assert r["frac"] is None or 0.0 < r["frac"] <= 1.0      # never a fraction above the roof
    assert 0.0 < d["occupancy"] <= 1.0
    if config == 3:
        g = r["gradient_phase"]
        assert 0.0 < g["share_of_kernel_time"] < 1.0 and r["frac"] < g["frac"] <= 1.0
