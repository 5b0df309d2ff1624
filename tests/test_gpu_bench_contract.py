"""bench.py prints exactly one JSON line with the fields its callers rely on (a short run)."""
import json
import os
import subprocess
import sys

import pytest

pytestmark = pytest.mark.gpu
ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.parametrize("extra", [[], ["--config", "5", "--no-cpu-baseline"]], ids=["default_workload", "bf16_workload"])
def test_bench_line(extra):
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "1", "--steps", "6", "--warmup", "2"] + extra,
                       capture_output=True, text=True, timeout=300, cwd=ROOT)
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [l for l in r.stdout.splitlines() if l.strip()]
    assert len(lines) == 1
    d = json.loads(lines[0])
    for key, typ in (("metric", str), ("value", float), ("unit", str), ("n_gpus", int), ("steps", int), ("warmup", int),
                     ("ms_per_step", float), ("higher_is_better", bool), ("scaling", str), ("dtype", str), ("data", str),
                     ("config", dict), ("roofline", dict)):
        assert isinstance(d[key], typ), key
    assert d["n_gpus"] == 1 and d["steps"] == 6 and d["warmup"] == 2 and d["vs_baseline"] is None
    assert d["unit"] == "TFLOP/s" and d["higher_is_better"] is True and d["data"] == "synthetic"
    assert "workload" in d["config"] and "model" not in d["config"]
    assert d["dtype"] == ("bf16" if extra else "f32")
    # value and ms_per_step describe the same measurement
    flop = d["config"]["conv_gflop_per_step"] * 1e9
    assert abs(flop / (d["ms_per_step"] * 1e-3) / 1e12 - d["value"]) <= 0.02 * d["value"]
    rf = d["roofline"]
    assert (rf["bound"], rf["unit"], rf["peak"]) in (("mfma", "TFLOP/s", 157.3), ("mfma", "TFLOP/s", 2500.0), ("hbm", "GB/s", 8000.0))
    assert rf["bound"] == ("hbm" if extra else "mfma")     # the bf16 stem pass sits below its ridge, conv1 above
    assert rf["algorithmic_bytes"] > 0
    assert abs(rf["achieved"] / rf["peak"] - rf["frac"]) <= 1e-3 and 0.0 < rf["frac"] < 1.0
    assert rf["traffic"] is None or rf["traffic"] > 0
    if not extra:
        cb = d["cpu_baseline"]
        assert cb["kind"] == "oracle" and cb["unit"] == "TFLOP/s" and cb["value"] > 0 and cb["cores"] >= 1 and cb["sample"]
