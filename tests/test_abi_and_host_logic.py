"""CPU-only checks of the C-ABI library: it loads, exports every declared symbol, and its host-side
integer logic (shapes, workspace plans, reciprocal division, argument validation) is right.
No compute call is made here."""
import ctypes
import os
import re

import numpy as np
import pytest

import oracle
import paper_1412_6249_amd as pa
from paper_1412_6249_amd import binding
from synth.configs import CONV_LAYERS

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "purine.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(purine_[a-z_0-9]+)\s*\(", text)))


def test_every_declared_symbol_is_exported_and_bound():
    names = declared_symbols()
    assert len(names) == 55
    lib = ctypes.CDLL(binding.LIB_PATH)
    for n in names:
        assert hasattr(lib, n), n
    assert set(names) == set(binding.EXPORTED)
    for n in names:
        assert callable(getattr(pa, n)), n


def test_out_shape_matches_oracle_and_workload_table():
    for layers in CONV_LAYERS.values():
        for l in layers:
            d = pa.conv_desc(l.stride, l.pad)
            assert pa.purine_conv_out_shape(d, l.x_shape, l.w_shape) == l.y_shape
            assert oracle.out_shape(l.x_shape, l.w_shape, l.stride, l.pad) == l.y_shape
    rng = np.random.default_rng(0)
    for _ in range(300):
        H, W = rng.integers(1, 40, 2)
        R, S = rng.integers(1, 8, 2)
        sh, sw = rng.integers(1, 5, 2)
        ph, pw = rng.integers(0, 4, 2)
        xs, ws = (2, 3, int(H), int(W)), (5, 3, int(R), int(S))
        d = pa.conv_desc((int(sh), int(sw)), (int(ph), int(pw)))
        P, Q = oracle.out_extent(H, R, sh, ph), oracle.out_extent(W, S, sw, pw)
        if P <= 0 or Q <= 0:
            with pytest.raises(pa.PurineError) as e:
                pa.purine_conv_out_shape(d, xs, ws)
            assert e.value.status == -2
        else:
            assert pa.purine_conv_out_shape(d, xs, ws) == (2, 5, P, Q)


def test_out_shape_rejects_bad_arguments():
    with pytest.raises(pa.PurineError) as e:
        pa.purine_conv_out_shape(pa.conv_desc(1, 0), (1, 3, 8, 8), (4, 2, 3, 3))   # channel mismatch
    assert e.value.status == -2
    with pytest.raises(pa.PurineError) as e:
        pa.purine_conv_out_shape(pa.conv_desc(0, 0), (1, 3, 8, 8), (4, 3, 3, 3))   # stride 0
    assert e.value.status == -8
    with pytest.raises(pa.PurineError) as e:
        pa.purine_conv_out_shape(pa.conv_desc(1, -1), (1, 3, 8, 8), (4, 3, 3, 3))  # negative pad
    assert e.value.status == -8
    with pytest.raises(pa.PurineError) as e:
        pa.purine_conv_out_shape(pa.conv_desc(1, 0), (0, 3, 8, 8), (4, 3, 3, 3))   # empty batch
    assert e.value.status == -2


def test_fastdiv_exact():
    rng = np.random.default_rng(1)
    divisors = list(range(1, 70)) + [96, 121, 169, 363, 729, 3025, 12544, 50176, 65535, 65536,
                                     65537, 2 ** 20 + 1, 2 ** 30, 2 ** 31 - 1]
    for d in divisors:
        ns = [0, 1, d - 1, d, d + 1, 2 * d - 1, 2 * d, 2 ** 31 - 1, 2 ** 31 - d, 2 ** 30]
        ns += [int(v) for v in rng.integers(0, 2 ** 31, 200)]
        ns += [k * d + o for k in (3, 1000, (2 ** 31 - 1) // d) for o in (-1, 0, 1)]
        for n in ns:
            if 0 <= n < 2 ** 31:
                assert pa.purine_debug_fastdiv(n, d) == n // d, (n, d)


def test_workspace_queries():
    for layers in CONV_LAYERS.values():
        for l in layers:
            d = pa.conv_desc(l.stride, l.pad)
            dt = pa.PURINE_F32 if l.dtype == "f32" else pa.PURINE_BF16
            esz = 4 if l.dtype == "f32" else 2
            fwd = pa.purine_conv_workspace_bytes(pa.PURINE_CONV_FWD, d, l.x_shape, l.w_shape, dt)
            bwd = pa.purine_conv_workspace_bytes(pa.PURINE_CONV_BWD_DATA, d, l.x_shape, l.w_shape, dt)
            w_bytes = esz * int(np.prod(l.w_shape))

            def bound(rows, red, taps, gathered_elems):
                """A zero-padded filter copy (rows up to the widest row tile, reduction up to a
                whole slab more), plus, for bf16 layers with more than one tap, a channels-blocked
                copy of the gathered tensor."""
                pad_rows = max(192, (rows + 191) // 192 * 192)
                filt = esz * taps * (red + 32) * pad_rows
                blocked = 2 * gathered_elems if (l.dtype == "bf16" and taps > 1 and red >= 16) else 0
                return filt + blocked + 256

            taps = l.R * l.S
            c_pad = (l.C + 31) // 32 * 32
            k_pad = (l.K + 31) // 32 * 32
            if l.C < 16 and l.dtype == "f32":
                assert fwd == 0                                   # the flattened fp32 kernel reads KCRS
            else:
                assert w_bytes <= fwd <= bound(l.K, l.C * taps if l.C < 16 else l.C, 1 if l.C < 16 else taps,
                                               l.N * c_pad * l.H * l.W)
            s2 = l.stride * l.stride
            taps_b = taps if l.stride == 1 else ((l.R + l.stride - 1) // l.stride) * ((l.S + l.stride - 1) // l.stride)
            assert w_bytes <= bwd <= bound(l.C * s2, l.K, taps_b, l.N * k_pad * l.P * l.Q)
            nbytes = pa.purine_conv_workspace_bytes(pa.PURINE_CONV_BWD_WEIGHT, d, l.x_shape, l.w_shape, dt)
            dw_bytes = 4 * int(np.prod(l.w_shape))
            assert nbytes >= dw_bytes and nbytes % dw_bytes == 0      # whole partial copies of dw
            assert nbytes <= 1 << 30
            both = pa.purine_conv_workspace_bytes(pa.PURINE_CONV_BWD_WEIGHT_BIAS, d, l.x_shape, l.w_shape, dt)
            splits = nbytes // dw_bytes
            assert nbytes + 4 * splits * l.K <= both <= nbytes + 4 * splits * l.K + 256   # + bias partials
            assert 0 < pa.purine_bias_bwd_workspace_bytes(l.y_shape, dt) <= 4 * l.K * l.N
    # illegal shapes give 0 (the operator call reports the error)
    assert pa.purine_conv_workspace_bytes(2, pa.conv_desc(1, 0), (1, 3, 2, 2), (4, 3, 3, 3), 0) == 0


def test_operator_argument_validation_without_launch():
    """All of these must be rejected on the host before any HIP call (there is no GPU here)."""
    F32, BF16 = pa.PURINE_F32, pa.PURINE_BF16
    fake = 0x10000   # never dereferenced: validation fails first
    d = pa.conv_desc(1, 1)
    x = binding.raw_desc(fake, F32, (2, 3, 8, 8))
    w = binding.raw_desc(fake + 0x100000, F32, (4, 3, 3, 3))
    y = binding.raw_desc(fake + 0x200000, F32, (2, 4, 8, 8))

    def status(fn, *a, **k):
        with pytest.raises(pa.PurineError) as e:
            fn(*a, **k)
        return e.value.status

    class _S:   # stand-in stream handle so that torch is not consulted
        cuda_stream = 0
    s = _S()
    assert status(pa.purine_conv_fwd, d, x, w, binding.raw_desc(fake + 0x200000, F32, (2, 4, 7, 8)), stream=s) == -2
    assert status(pa.purine_conv_fwd, d, x, binding.raw_desc(fake + 0x100000, BF16, (4, 3, 3, 3)), y, stream=s) == -3
    assert status(pa.purine_conv_fwd, d, binding.raw_desc(0, F32, (2, 3, 8, 8)), w, y, stream=s) == -1
    assert status(pa.purine_conv_fwd, d, binding.raw_desc(fake + 4, F32, (2, 3, 8, 8)), w, y, stream=s) == -4
    assert status(pa.purine_conv_fwd, d, x, w, binding.raw_desc(fake, F32, (2, 4, 8, 8)), stream=s) == -4  # y aliases x
    assert status(pa.purine_conv_fwd, pa.conv_desc(0, 1), x, w, y, stream=s) == -8
    assert status(pa.purine_conv_bwd_data, d, y, w, x, beta=0.5, stream=s) == -8
    assert status(pa.purine_conv_bwd_data, d, y, w, x, stream=s) == -5                # no workspace
    dw = binding.raw_desc(fake + 0x300000, F32, (4, 3, 3, 3))
    assert status(pa.purine_conv_bwd_weight, d, x, y, dw, stream=s) == -5            # no workspace
    assert status(pa.purine_conv_bwd_weight, d, x, y, binding.raw_desc(fake + 0x300000, BF16, (4, 3, 3, 3)), stream=s) == -3
    db4 = binding.raw_desc(fake + 0x400000, F32, (4,))
    assert status(pa.purine_conv_bwd_weight_bias, d, x, y, dw, db4, stream=s) == -5     # no workspace
    assert status(pa.purine_conv_bwd_weight_bias, d, x, y, dw, binding.raw_desc(fake + 0x400000, F32, (5,)), stream=s) == -2
    assert status(pa.purine_conv_bwd_weight_bias, d, x, y, dw, binding.raw_desc(fake + 0x300000, F32, (4,)), stream=s) == -4  # db aliases dw
    b = binding.raw_desc(fake + 0x400000, F32, (5,))
    assert status(pa.purine_bias_fwd, b, y, stream=s) == -2                          # K mismatch
    db = binding.raw_desc(fake + 0x400000, F32, (4,))
    assert status(pa.purine_bias_bwd, y, db, stream=s) == -5
    wd = binding.raw_desc(fake + 0x600000, F32, (4, 3, 3, 3))
    nw = binding.raw_desc(fake + 0x700000, F32, (4, 3, 3, 3))
    assert status(pa.purine_sgd_update, w, wd, binding.raw_desc(fake + 0x700000, BF16, (4, 3, 3, 3)), 0.1, stream=s) == -3
    assert status(pa.purine_sgd_update, w, binding.raw_desc(fake + 0x600000, BF16, (4, 3, 3, 3)), nw, 0.1, stream=s) == -3
    assert status(pa.purine_sgd_update, w, wd, binding.raw_desc(fake + 0x700000, F32, (4, 3, 3, 2)), 0.1, stream=s) == -2
    assert status(pa.purine_sgd_update, w, wd, nw, float("nan"), stream=s) == -8
    assert status(pa.purine_sgd_update, w, wd, nw, float("inf"), stream=s) == -8
    assert status(pa.purine_sgd_update, w, wd, binding.raw_desc(fake + 0x100000 + 16, F32, (4, 3, 3, 3)), 0.1, stream=s) == -4  # partial overlap with w
    assert status(pa.purine_sgd_update, w, wd, wd, 0.1, stream=s) == -4                # new_w is dw
    # size limits: no tensor with 2^31 or more elements; the bf16 multi-tap kernels' blocked copy of
    # the gathered tensor must stay below 2^31 bytes (forward: x, backward-data: dy)
    big = 1 << 40   # made-up, well separated addresses
    x_big = binding.raw_desc(big, F32, (2, 64, 4096, 4096))                   # 2^31 elements
    assert status(pa.purine_conv_fwd, d, x_big, binding.raw_desc(fake, F32, (4, 64, 3, 3)),
                  binding.raw_desc(3 * big, F32, (2, 4, 4096, 4096)), stream=s) == -2
    xb = binding.raw_desc(big, BF16, (2, 32, 4096, 4096))                     # 2^30 elements: copy of 2^31 bytes
    wb = binding.raw_desc(fake, BF16, (8, 32, 3, 3))
    yb = binding.raw_desc(3 * big, BF16, (2, 8, 4096, 4096))
    assert status(pa.purine_conv_fwd, d, xb, wb, yb, stream=s) == -2
    wb2 = binding.raw_desc(fake, BF16, (32, 8, 3, 3))                         # backward-data gathers dy = xb
    assert status(pa.purine_conv_bwd_data, d, xb, wb2, yb, stream=s) == -2
    xh = binding.raw_desc(big, BF16, (1, 32, 4096, 4096))                     # half of that passes this check
    yh = binding.raw_desc(3 * big, BF16, (1, 8, 4096, 4096))
    assert status(pa.purine_conv_fwd, d, xh, wb, yh, stream=s) == -5          # (stops at the missing workspace)
    # channel-slice views: x is channels 4..6 of a [2, 12, 8, 8] buffer
    xv = binding.raw_desc(fake + 4 * 64 * 4, F32, (2, 3, 8, 8), nstride=12 * 64)
    assert status(pa.purine_conv_bwd_data, d, y, w, xv, stream=s) == -5                # accepted up to the workspace
    assert status(pa.purine_conv_fwd, d, binding.raw_desc(fake, F32, (2, 3, 8, 8), nstride=3 * 64 - 4), w, y, stream=s) == -2
    assert status(pa.purine_conv_fwd, d, binding.raw_desc(fake, F32, (2, 3, 8, 8), nstride=12 * 64 + 2), w, y, stream=s) == -4
    wb3 = binding.raw_desc(fake + 0x100000, BF16, (4, 3, 3, 3))
    yb3 = binding.raw_desc(fake + 0x200000, BF16, (2, 4, 8, 8))
    # bf16 views: the distance between images is a whole number of 8-element packets
    assert status(pa.purine_conv_fwd, d, binding.raw_desc(fake, BF16, (2, 3, 8, 8), nstride=12 * 64 + 4), wb3, yb3, stream=s) == -4
    assert status(pa.purine_conv_fwd, d, binding.raw_desc(fake, BF16, (2, 3, 8, 8), nstride=12 * 64), wb3, yb3, stream=s) == -5
    yv = binding.raw_desc(fake + 0x200000, F32, (2, 4, 8, 8), nstride=16 * 64)
    assert status(pa.purine_bias_fwd, binding.raw_desc(fake + 0x400000, F32, (4,)), yv, stream=s) == -4   # dense only
    assert status(pa.purine_bias_bwd, yv, db, stream=s) == -4
    assert status(pa.purine_conv_bwd_data_relu, d, y, w, x, xv, stream=s) == -4        # mask and dx differ in nstride
    # two slices of one buffer: disjoint channel ranges do not alias, overlapping ones do
    lo = binding.raw_desc(fake, F32, (2, 4, 8, 8), nstride=16 * 64)
    hi = binding.raw_desc(fake + 4 * 64 * 4, F32, (2, 4, 8, 8), nstride=16 * 64)
    mid = binding.raw_desc(fake + 2 * 64 * 4, F32, (2, 4, 8, 8), nstride=16 * 64)
    assert status(pa.purine_relu_fwd, lo, mid, stream=s) == -4
    assert status(pa.purine_relu_bwd, lo, hi, mid, stream=s) == -4
    assert status(pa.purine_relu_fwd, lo, binding.raw_desc(fake, F32, (2, 4, 8, 8)), stream=s) == -4   # same start, other stride
    # grouped convolution and fully-connected compositions: rejected before any launch
    xg = binding.raw_desc(fake, F32, (2, 8, 6, 6))
    wg = binding.raw_desc(fake + 0x100000, F32, (8, 4, 3, 3))
    yg = binding.raw_desc(fake + 0x200000, F32, (2, 8, 6, 6))
    assert status(pa.purine_grouped_conv_bwd_data, d, 2, yg, wg, xg, stream=s) == -5            # needs scratch
    assert status(pa.purine_grouped_conv_fwd, d, 3, xg, wg, None, yg, stream=s) == -2           # 8 % 3
    assert status(pa.purine_grouped_conv_fwd, d, 0, xg, wg, None, yg, stream=s) == -8
    assert status(pa.purine_grouped_conv_fwd, d, 4, xg, wg, None, yg, stream=s) == -2           # w has C/2 channels
    assert status(pa.purine_grouped_conv_fwd, d, 2, binding.raw_desc(fake, F32, (2, 6, 5, 5)),
                  binding.raw_desc(fake + 0x100000, F32, (8, 3, 3, 3)), None,
                  binding.raw_desc(fake + 0x200000, F32, (2, 8, 5, 5)), stream=s) == -4         # 3*25 elements per slice
    assert status(pa.purine_grouped_conv_fwd, d, 2, binding.raw_desc(fake, BF16, (2, 8, 6, 6)),
                  binding.raw_desc(fake + 0x100000, BF16, (8, 4, 3, 3)), None,
                  binding.raw_desc(fake + 0x200000, BF16, (2, 8, 6, 6)), stream=s) == -4         # K/G = 4 bf16 bias values
    assert status(pa.purine_grouped_conv_fwd, d, 2, binding.raw_desc(fake, BF16, (2, 16, 6, 6)),
                  binding.raw_desc(fake + 0x100000, BF16, (16, 8, 3, 3)), None,
                  binding.raw_desc(fake + 0x200000, BF16, (2, 16, 6, 6)), stream=s) == -5        # accepted up to the workspace
    assert pa.purine_grouped_conv_workspace_bytes(0, d, 2, (2, 8, 6, 6), (8, 4, 3, 3), F32) == \
        pa.purine_conv_workspace_bytes(0, d, (2, 4, 6, 6), (4, 4, 3, 3), F32)
    fx = binding.raw_desc(fake, F32, (4, 20))
    fw = binding.raw_desc(fake + 0x100000, F32, (6, 20))
    fy = binding.raw_desc(fake + 0x200000, F32, (4, 6))
    assert status(pa.purine_fc_fwd, fx, fw, None, fy, stream=s) == -5
    assert status(pa.purine_fc_fwd, fx, binding.raw_desc(fake + 0x100000, F32, (6, 21)), None, fy, stream=s) == -2
    assert status(pa.purine_fc_fwd, fx, fw, None, binding.raw_desc(fake + 0x200000, BF16, (4, 6)), stream=s) == -3
    assert status(pa.purine_fc_bwd_data, fy, fw, binding.raw_desc(fake, F32, (4, 21)), stream=s) == -2
    assert status(pa.purine_fc_bwd_weight, fx, fy, binding.raw_desc(fake + 0x300000, F32, (6, 20)), None, beta=0.5, stream=s) == -8
    assert status(pa.purine_fc_fwd, binding.raw_desc(fake, BF16, (4, 20)), binding.raw_desc(fake + 0x100000, BF16, (6, 20)),
                  None, binding.raw_desc(fake + 0x200000, BF16, (4, 6)), stream=s) == -5         # bf16: accepted up to the workspace
    assert status(pa.purine_fc_bwd_weight, binding.raw_desc(fake, BF16, (4, 20)), binding.raw_desc(fake + 0x200000, BF16, (4, 6)),
                  binding.raw_desc(fake + 0x300000, BF16, (6, 20)), None, stream=s) == -3        # dw is fp32
    assert pa.purine_fc_workspace_bytes(0, 4, 20, 6) > 0 and pa.purine_fc_workspace_bytes(7, 4, 20, 6) == 0
    assert pa.purine_fc_workspace_bytes(0, 4, 20, 6, BF16) >= 4 * 6 * 4 and pa.purine_fc_workspace_bytes(2, 4, 20, 6, BF16) >= 2 * (4 * 20 + 4 * 6)
    assert pa.purine_fc_workspace_bytes(0, 4, 20, 6, pa.PURINE_I32) == 0
    # bf16 backward-data with rows of whole 16-byte packets: fp32 tiles of the slices of the reduction
    # (whole multiples of N*C*4 bytes, none when one slice covers it); other shapes size the forward kernel's scratch
    n_, c_, k_ = 128, 9216, 4096
    sliced = pa.purine_fc_workspace_bytes(1, n_, c_, k_, BF16)
    assert sliced % (n_ * c_ * 4) == 0 and 2 <= sliced // (n_ * c_ * 4) <= 64
    assert pa.purine_fc_workspace_bytes(1, 8, 4096, 64, BF16) == 0                 # 32 column tiles, too short a reduction to slice
    assert pa.purine_fc_workspace_bytes(1, n_, c_, k_ + 4, BF16) == \
        pa.purine_conv_workspace_bytes(0, pa.conv_desc((1, 1), (0, 0)), (1, k_ + 4, 1, c_), (n_, k_ + 4, 1, 1), BF16)
    bdy = binding.raw_desc(fake, BF16, (n_, k_))
    bw = binding.raw_desc(fake + 0x10000000, BF16, (k_, c_))
    bdx = binding.raw_desc(fake + 0x20000000, BF16, (n_, c_))
    assert status(pa.purine_fc_bwd_data, bdy, bw, bdx, stream=s) == -5             # needs the slices' scratch
    assert status(pa.purine_fc_bwd_data, bdy, bw, bdy, stream=s) == -2             # dx of the wrong extent
    big = binding.raw_desc(fake, F32, (1 << 12, 1 << 12, 1 << 4, 1 << 4))           # 2^32 elements
    assert status(pa.purine_relu_fwd, big, big, stream=s) == -2
    assert status(pa.purine_maxpool_fwd, pa.pool_desc(3, 2, 3), x, y, binding.raw_desc(fake + 0x500000, pa.PURINE_I32, (2, 4, 8, 8)), stream=s) == -8


def test_static_scratch_entry_point_refuses_what_does_not_fit():
    """purine_conv_bwd_weight_static validates like purine_conv_bwd_weight and refuses, before
    any launch, a layer whose partial sums need more than the library's static device array."""
    fake = 0x7f0000000000   # never dereferenced: the call is refused on the host
    F32 = pa.PURINE_F32

    class _S:   # stand-in stream handle so that torch is not consulted
        cuda_stream = 0
    s = _S()
    cap = pa.purine_static_scratch_bytes()
    assert cap == 64 << 20
    d = pa.conv_desc(1, 1)
    # a layer with a large filter and many pixels: its split-reduction partials exceed the array
    xs, ws_, ys = (8, 512, 64, 64), (512, 512, 3, 3), (8, 512, 64, 64)
    need = pa.purine_conv_workspace_bytes(pa.PURINE_CONV_BWD_WEIGHT, d, xs, ws_, F32)
    assert need > cap
    x = binding.raw_desc(fake, F32, xs)
    dy = binding.raw_desc(fake + 0x40000000, F32, ys)
    dw = binding.raw_desc(fake + 0x80000000, F32, ws_)
    with pytest.raises(pa.PurineError) as e:
        pa.purine_conv_bwd_weight_static(d, x, dy, dw, stream=s)
    assert e.value.status == -9 and "static" in str(e.value)
    # argument errors come first, exactly as in the workspace form
    with pytest.raises(pa.PurineError) as e:
        pa.purine_conv_bwd_weight_static(d, x, dy, dw, beta=0.5, stream=s)
    assert e.value.status == -8
    bad = binding.raw_desc(fake + 0x80000000, F32, (512, 511, 3, 3))
    with pytest.raises(pa.PurineError) as e:
        pa.purine_conv_bwd_weight_static(d, x, dy, bad, stream=s)
    assert e.value.status == -2


def test_bench_refuses_more_than_one_gpu():
    """The path has no collectives: bench.py --gpus N with N above 1 must stop with a message that
    says so, before anything touches a device."""
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True, timeout=60)
    assert r.returncode != 0
    assert "one GPU" in r.stderr and r.stdout.strip() == ""


def test_header_is_plain_c_and_links_against_the_library(tmp_path):
    """include/purine.h must be usable from C: it compiles as C99 with warnings as errors, and a C
    program that calls host-only entry points links against the library and runs."""
    import os
    import subprocess
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    inc = os.path.join(root, "include")
    src = tmp_path / "use_purine.c"
    src.write_text(r'''
#include <stdio.h>
#include "purine.h"
int main(void) {
    purine_conv_desc d = {4, 4, 0, 0};
    int64_t x[4] = {64, 3, 224, 224}, w[4] = {96, 3, 11, 11}, y[4];
    if (purine_conv_out_shape(&d, x, w, y) != PURINE_OK) return 1;
    if (y[0] != 64 || y[1] != 96 || y[2] != 54 || y[3] != 54) return 2;
    purine_graph* g = purine_graph_create();
    if (!g) return 3;
    purine_tensor t = {0};
    t.dtype = PURINE_F32; t.ndim = 1; t.dim[0] = 4;
    int a = purine_graph_add_tensor(g, &t, "a"), b = purine_graph_add_tensor(g, &t, "b");
    int op = purine_graph_add_op(g, PURINE_OP_HOST_NOP, NULL, &a, 1, &b, 1, 0);
    if (a != 0 || b != 1 || op != 0) return 4;
    if (purine_graph_run(g) != PURINE_OK) return 5;
    int order[1];
    if (purine_graph_fire_log(g, order, 1) != 1 || order[0] != 0) return 6;
    purine_graph_destroy(g);
    printf("%s\n", purine_status_string(PURINE_E_SHAPE));
    return 0;
}
''')
    exe = tmp_path / "use_purine"
    lib_dir = os.path.dirname(binding.LIB_PATH)
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-Werror", "-pedantic", "-I", inc, str(src), "-o", str(exe),
                    "-L", lib_dir, "-l:libpurine_conv.so", "-Wl,-rpath," + lib_dir], check=True, capture_output=True)
    r = subprocess.run([str(exe)], capture_output=True, text=True, timeout=60)
    assert r.returncode == 0, (r.returncode, r.stderr)
    assert "shape" in r.stdout
