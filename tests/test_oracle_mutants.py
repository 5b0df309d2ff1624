"""Do the pins pin? Each case plants ONE plausible mistake in a copy of the oracle's C source (a
wrong sign, a flipped kernel, a dropped term, an off-by-one extent, a wrong tie rule ...), builds
it, and runs the pin suite against that build in a child process: the suite has to fail. The
mistakes are planted in the oracle, on the CPU; every mutant stays inside its arrays."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "conv_oracle.c")

# name, text to replace, replacement, which occurrence (0-based) of the text
MUTANTS = [
    ("fwd_pad_sign", "const int64_t h = p * g->sh - g->ph + r;", "const int64_t h = p * g->sh + g->ph + r;", 0),
    ("fwd_kernel_flipped", "acc += (double)x[XI(n, c, h, w_)] * (double)w[WI(k, c, r, s)];",
     "acc += (double)x[XI(n, c, h, w_)] * (double)w[WI(k, c, g->R - 1 - r, g->S - 1 - s)];", 0),
    ("fwd_stride_of_the_other_axis", "const int64_t w_ = q * g->sw - g->pw + s;", "const int64_t w_ = q * g->sh - g->pw + s;", 0),
    ("fwd_drops_last_channel", "for (int64_t c = 0; c < g->C; ++c)", "for (int64_t c = 0; c + 1 < g->C || c == 0; ++c)", 0),
    ("bwd_data_sign", "dx[XI(n, c, h, w_)] += gy * (double)w[WI(k, c, r, s)];", "dx[XI(n, c, h, w_)] -= gy * (double)w[WI(k, c, r, s)];", 0),
    ("bwd_data_kernel_flipped", "dx[XI(n, c, h, w_)] += gy * (double)w[WI(k, c, r, s)];",
     "dx[XI(n, c, h, w_)] += gy * (double)w[WI(k, c, g->R - 1 - r, g->S - 1 - s)];", 0),
    ("bwd_data_pad_sign", "const int64_t w_ = q * g->sw - g->pw + s;", "const int64_t w_ = q * g->sw + g->pw + s;", 1),
    ("bwd_weight_tap_sign", "const int64_t h = p * g->sh - g->ph + r;", "const int64_t h = p * g->sh - g->ph - r;", 2),
    ("bwd_weight_drops_first_image", "for (int64_t n = 0; n < g->N; ++n)\n        for (int64_t p = 0; p < P; ++p) {",
     "for (int64_t n = (g->N > 1); n < g->N; ++n)\n        for (int64_t p = 0; p < P; ++p) {", 0),
    ("bias_fwd_wrong_channel", "row[i] += (double)b[k];", "row[i] += (double)b[0];", 0),
    ("bias_bwd_drops_last_pixel", "for (int64_t i = 0; i < PQ; ++i) acc += (double)row[i];",
     "for (int64_t i = 0; i + 1 < PQ || i == 0; ++i) acc += (double)row[i];", 0),
    ("extent_off_by_one", "return (in + 2 * pad - k) / stride + 1;", "return (in + 2 * pad - k + stride - 1) / stride + 1;", 0),
    ("pool_last_maximum_wins_ties", "if (best < 0 || v > bv) { best = (int32_t)(h * W + w_); bv = v; }",
     "if (best < 0 || v >= bv) { best = (int32_t)(h * W + w_); bv = v; }", 0),
    ("pool_gradient_overwrites", "if (a >= 0) plane[a] += (double)dy[nc * PQ + i];", "if (a >= 0) plane[a] = (double)dy[nc * PQ + i];", 0),
    ("pool_gradient_lands_one_position_off", "if (a >= 0) plane[a] += (double)dy[nc * PQ + i];",
     "if (a >= 0) plane[(a + 1) % HW] += (double)dy[nc * PQ + i];", 0),
    ("pool_gradient_reads_another_planes_dy", "if (a >= 0) plane[a] += (double)dy[nc * PQ + i];",
     "if (a >= 0) plane[a] += (double)dy[((nc + 1) % NC) * PQ + i];", 0),
    ("relu_passes_zero_gradient", "dx[i] = x[i] > 0.0f ? dy[i] : 0.0f;", "dx[i] = x[i] >= 0.0f ? dy[i] : 0.0f;", 0),
]


def nth_replace(text, old, new, n):
    pos = -1
    for _ in range(n + 1):
        pos = text.index(old, pos + 1)
    return text[:pos] + new + text[pos + len(old):]


def run_pins(lib):
    env = dict(os.environ)
    if lib:
        env["ORACLE_LIB_OVERRIDE"] = lib
    else:
        env.pop("ORACLE_LIB_OVERRIDE", None)
    return subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", "test_oracle_pins.py"), "-x", "-q",
                           "-p", "no:cacheprovider"], cwd=ROOT, env=env, capture_output=True, text=True, timeout=300)


def build(src_text, tmp_path, name):
    c = tmp_path / (name + ".c")
    so = tmp_path / (name + ".so")
    c.write_text(src_text)
    subprocess.run(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-o", str(so), str(c)], check=True,
                   capture_output=True)
    return str(so)


def test_an_unaltered_copy_passes(tmp_path):
    """The harness itself: the same source built elsewhere passes the pins through the override."""
    r = run_pins(build(open(SRC).read(), tmp_path, "copy"))
    assert r.returncode == 0, r.stdout[-2000:]


@pytest.mark.parametrize("name,old,new,nth", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_pins_notice_a_planted_mistake(tmp_path, name, old, new, nth):
    text = open(SRC).read()
    mutant = nth_replace(text, old, new, nth)
    assert mutant != text
    r = run_pins(build(mutant, tmp_path, name))
    assert r.returncode != 0, "the pin suite passed on the mutant " + name
    assert "failed" in r.stdout or "error" in r.stdout.lower(), r.stdout[-500:]
