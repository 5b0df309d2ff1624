"""bench.py takes `roofline.traffic` from the counter summary kept under profiles/: the table must
parse, and must hold the operators that come out dominant on each workload."""
import importlib.util
import os

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_traffic_table_parses_and_covers_the_dominant_operators():
    spec = importlib.util.spec_from_file_location("_bench", os.path.join(ROOT, "bench.py"))
    bench = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(bench)
    t = bench.measured_traffic()
    for key in ((4, "conv_bwd_data[conv2.dx]"), (4, "conv_fwd_bias_relu[conv2.a]"), (4, "conv_bwd_weight_bias[conv2.dw]"),
                (2, "conv_bwd_data[conv1.dx]"), (2, "conv_fwd_bias_relu[conv1.a]"), (3, "conv_bwd_data_relu[b2_3x3.dx]"),
                (5, "conv_bwd_data[stem7x7.dx]")):
        assert key in t, key
        assert 1e7 < t[key] < 2e9            # bytes per launch: tens of MB to under 2 GB
    # the bf16 stem's backward-data reads dy once and writes dx once: 411 + 77 MB within a few per cent
    assert abs(t[(5, "conv_bwd_data[stem7x7.dx]")] / 488130944 - 1.0) < 0.05
