"""bench.py end to end on a cut-down run: the JSON line carries what its contract asks for (the headline fields,
the roofline of the dominant kernel measured with events, the rooflines of the other passes, the oracle baseline)."""
import json
import os
import subprocess
import sys

import pytest

pytestmark = pytest.mark.gpu
ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_bench_line_has_the_contract_fields():
    cmd = [sys.executable, os.path.join(ROOT, "bench.py"), "--workload", "deepseek-moe-16b", "--layers", "2", "--steps", "2",
           "--warmup", "1", "--no-probes", "--no-decode", "--no-forward", "--no-apply"]
    res = subprocess.run(cmd, capture_output=True, text=True, timeout=280)
    assert res.returncode == 0, res.stderr[-2000:]
    lines = [l for l in res.stdout.splitlines() if l.startswith("{")]
    assert len(lines) == 1, res.stdout[-500:]
    d = json.loads(lines[0])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config", "roofline", "rooflines", "cpu_baseline"):
        assert key in d, key
    assert d["n_gpus"] == 1 and d["steps"] == 2 and d["warmup"] == 1 and d["higher_is_better"] is True
    assert d["vs_baseline"] is None and d["data"] == "synthetic" and d["dtype"] == "bf16"
    assert d["config"]["workload"].startswith("deepseek-moe-16b") and "model" not in d["config"]
    assert d["value"] > 0 and abs(d["value"] - 8192 * 2 * 1e3 / d["ms_per_step"]) < 0.02 * d["value"]
    r = d["roofline"]
    assert r["bound"] == "mfma" and r["unit"] == "TFLOP/s" and r["peak"] == 2500.0
    assert abs(r["frac"] - r["achieved"] / r["peak"]) < 1e-3 and 0.05 < r["frac"] < 1.0
    assert abs(r["achieved"] - r["flops_per_launch"] / (r["avg_launch_ms"] * 1e-3) / 1e12) < 0.01 * r["achieved"]
    assert 0.0 < r["per_expert_bound"]["frac"] <= 1.0
    for name in ("down_norm", "route", "bucket", "finalize", "rank"):
        p = d["rooflines"][name]
        assert p["bound"] == "hbm" and p["peak"] == 8000.0 and p["us_per_call"] > 0 and 0 < p["frac"] < 1.0
    c = d["cpu_baseline"]
    assert c["kind"] == "oracle" and c["cores"] >= 1 and c["value"] > 0 and "sample" in c
