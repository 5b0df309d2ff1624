"""bench.py prints exactly one JSON line with the fields its callers rely on (a short run)."""
import json
import os
import subprocess
import sys

import pytest

pytestmark = pytest.mark.gpu
ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.parametrize("extra", [[], ["--config", "5", "--no-cpu-baseline", "--no-per-config"]], ids=["default_workload", "bf16_workload"])
def test_bench_line(extra):
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "1", "--steps", "6", "--warmup", "2"] + extra,
                       capture_output=True, text=True, timeout=600, cwd=ROOT)
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
    if not extra:
        assert rf["bound"] == "mfma"       # every pass of the fp32 stack sits above the fp32 ridge
    assert rf["algorithmic_bytes"] > 0
    assert abs(rf["achieved"] / rf["peak"] - rf["frac"]) <= 1e-3 and 0.0 < rf["frac"] < 1.0
    assert rf["traffic"] is None or rf["traffic"] > 0
    if not extra:
        # the headline is the largest fp32 workload; the other three ride along in the same line
        assert d["config"]["workload"] == "cfg4_alexnet_conv_stack_f32_n128"
        per = d["per_config"]
        assert sorted(per) == ["cfg2_nin_mlpconv_f32_n64", "cfg3_inception_f32_n128", "cfg5_googlenet_stem_bf16_n256"]
        for name, e in per.items():
            assert e["dtype"] == ("bf16" if "bf16" in name else "f32")
            assert e["ms_per_step"] > 0 and e["value"] > 0 and 0.0 < e["frac_of_mfma_peak"] < 1.0
            assert abs(e["conv_gflop_per_step"] * 1e9 / (e["ms_per_step"] * 1e-3) / 1e12 - e["value"]) <= 0.02 * e["value"]
            r2 = e["roofline"]
            assert r2["bound"] in ("mfma", "hbm") and 0.0 < r2["frac"] < 1.0 and r2["algorithmic_bytes"] > 0
        cb = d["cpu_baseline"]
        assert cb["kind"] == "oracle" and cb["unit"] == "TFLOP/s" and cb["value"] > 0 and cb["cores"] >= 1 and cb["sample"]
