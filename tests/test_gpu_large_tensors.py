"""Tensors near the size limits of the boundary (fewer than 2^31 elements each; for the bf16
multi-tap kernels a gathered tensor below 2^30 elements): layers whose activations and gradients
are 2 to 5.8 GB, so that element offsets pass 2^30, byte offsets pass 2^32 (fp32), and the fp32
gathered tensors are too large for the range-checked raw buffer loads (the kernels take their
ordinary-load path at its real size), while the bf16 blocked copy sits just under its limit.
  - a 3x3 layer with 24 channels (tap-major forward / backward-data, per-tap weight gradient),
  - a strided 5x5 first layer with 3 channels (flattened forward and weight gradient, phase-folded
    backward-data with the depth-to-space epilogue),
  - the 3x3 layer in bf16.
Checked against the oracle on windows it can compute one by one, at the lowest addresses, in the
middle and in the last rows of the last image (the highest addresses), plain and fused operators;
the weight gradient on sampled elements summed over the whole batch; the bias gradient in full.
Tolerance: relative L2 <= 1e-5 (fp32), <= 1e-2 (bf16) per sample."""
import sys

import numpy as np
import pytest

import oracle

pytestmark = pytest.mark.gpu

WIN = 20
# name, dtype, N, C, H, W, K, R, stride, pad
CASES = [
    ("c24_3x3_f32", "f32", 3, 24, 3900, 3900, 32, 3, 1, 1),        # x 1.10e9 elements, y 1.46e9
    ("c3_5x5_s2_f32", "f32", 40, 3, 3000, 3000, 16, 5, 2, 2),      # x 1.08e9 elements, y 1.44e9
    ("c32_3x3_bf16", "bf16", 2, 32, 4000, 4000, 32, 3, 1, 1),      # x, y 1.02e9 elements: blocked copy 2.05e9 bytes
]


def say(*a):
    print(*a, file=sys.stderr, flush=True)


def window(t, n, a0, a1, b0, b1):
    """rows a0..a1-1, columns b0..b1-1 of image n as a [1, C, rows, cols] host array, zeros outside"""
    import torch
    from gpu_util import to_host
    Ht, Wt = t.shape[2], t.shape[3]
    out = torch.zeros((1, t.shape[1], a1 - a0, b1 - b0), dtype=t.dtype, device=t.device)
    hs, he, ws, we = max(a0, 0), min(a1, Ht), max(b0, 0), min(b1, Wt)
    if hs < he and ws < we:
        out[0, :, hs - a0:he - a0, ws - b0:we - b0] = t[n, :, hs:he, ws:we]
    return to_host(out)


@pytest.mark.parametrize("case", CASES, ids=[c[0] for c in CASES])
def test_layer_near_the_size_limits(case):
    import torch
    import paper_1412_6249_amd as pa
    from gpu_util import rel_l2, workspace, to_host, tdtype, pcode, TOL, DEV

    name, dtype, N, C, H, W, K, R, s, pad = case
    P, Q = (H + 2 * pad - R) // s + 1, (W + 2 * pad - R) // s + 1
    assert N * C * H * W < 2 ** 31 and N * K * P * Q < 2 ** 31 and N * C * H * W > 2 ** 30 - 2 ** 26
    free, _ = torch.cuda.mem_get_info()
    if free < 48 * 2 ** 30:
        pytest.skip("needs 48 GiB of free device memory")
    td, tol = tdtype(dtype), TOL[dtype]
    g = torch.Generator(device="cuda")
    g.manual_seed(14126249 + len(name))
    x = torch.rand((N, C, H, W), generator=g, device=DEV).to(td)
    w = (torch.randn((K, C, R, R), generator=g, device=DEV) * 0.05).to(td)
    b = (torch.randn((K,), generator=g, device=DEV) * 0.05).to(td)
    dy = (torch.rand((N, K, P, Q), generator=g, device=DEV) * 2 - 1).to(td)
    act = (torch.rand((N, C, H, W), generator=g, device=DEV) - 0.5).to(td)     # stands for a ReLU output
    y, y2 = torch.empty((N, K, P, Q), dtype=td, device=DEV), torch.empty((N, K, P, Q), dtype=td, device=DEV)
    dx, dx2 = torch.empty((N, C, H, W), dtype=td, device=DEV), torch.empty((N, C, H, W), dtype=td, device=DEV)
    dw = torch.empty((K, C, R, R), device=DEV)
    db, db2 = torch.empty((K,), device=DEV), torch.empty((K,), device=DEV)
    desc = pa.conv_desc(s, pad)
    code = pcode(dtype)
    q = lambda which: workspace(pa.purine_conv_workspace_bytes(which, desc, x.shape, w.shape, code))
    say(name, "forward, plain and fused")
    pa.purine_conv_fwd(desc, x, w, y, ws=q(pa.PURINE_CONV_FWD))
    pa.purine_bias_fwd(b, y)
    pa.purine_conv_fwd_bias_relu(desc, x, w, b, y2, relu=True, ws=q(pa.PURINE_CONV_FWD))
    torch.cuda.synchronize()
    say(name, "backward-data, plain and through a ReLU mask")
    pa.purine_conv_bwd_data(desc, dy, w, dx, ws=q(pa.PURINE_CONV_BWD_DATA))
    pa.purine_conv_bwd_data_relu(desc, dy, w, act, dx2, ws=q(pa.PURINE_CONV_BWD_DATA))
    torch.cuda.synchronize()
    say(name, "backward-weight with bias gradient, bias gradient alone")
    pa.purine_conv_bwd_weight_bias(desc, x, dy, dw, db, ws=q(pa.PURINE_CONV_BWD_WEIGHT_BIAS))
    pa.purine_bias_bwd(dy, db2, ws=workspace(pa.purine_bias_bwd_workspace_bytes(dy.shape, code)))
    torch.cuda.synchronize()

    hw, hb = to_host(w), to_host(b)
    # forward windows, in output coordinates
    for n, p0, q0 in [(0, 0, 0), (N // 2, P // 2 - 7, Q // 2 + 3), (N - 1, 0, Q - WIN), (N - 1, P - WIN, Q - WIN)]:
        say(name, "forward window", n, p0, q0)
        xp = window(x, n, p0 * s - pad, (p0 + WIN - 1) * s - pad + R, q0 * s - pad, (q0 + WIN - 1) * s - pad + R)
        ref = oracle.bias_fwd(oracle.conv_fwd(xp, hw, (s, s), (0, 0)), hb)[0]
        got = to_host(y[n, :, p0:p0 + WIN, q0:q0 + WIN])
        assert rel_l2(got, ref) <= tol, ("fwd", n, p0, q0, rel_l2(got, ref))
        got = to_host(y2[n, :, p0:p0 + WIN, q0:q0 + WIN])
        assert rel_l2(got, np.maximum(ref, 0.0)) <= tol, ("fused fwd", n, p0, q0)
    # backward-data windows, in input coordinates: every output row that reaches the window
    for n, h0, w0 in [(0, 0, 0), (N // 2, H // 2 - 7, W // 2 + 3), (N - 1, H - WIN, 0), (N - 1, H - WIN, W - WIN)]:
        say(name, "backward-data window", n, h0, w0)
        lo = lambda a: max(0, -((-(a + pad - (R - 1))) // s))          # ceil((a + pad - R + 1) / s), clamped
        hi = lambda a, lim: min(lim - 1, (a + WIN - 1 + pad) // s)
        pa_, pb_, qa_, qb_ = lo(h0), hi(h0, P), lo(w0), hi(w0, Q)
        dyp = window(dy, n, pa_, pb_ + 1, qa_, qb_ + 1)
        hv, wv = pa_ * s - pad, qa_ * s - pad                              # origin of the patch's own input image
        Hv, Wv = (pb_ - pa_) * s + R, (qb_ - qa_) * s + R
        full = oracle.conv_bwd_data(dyp, hw, (1, C, Hv, Wv), (s, s), (0, 0))[0]
        assert hv <= h0 and wv <= w0 and h0 + WIN <= hv + Hv and w0 + WIN <= wv + Wv
        ref = full[:, h0 - hv:h0 - hv + WIN, w0 - wv:w0 - wv + WIN]
        got = to_host(dx[n, :, h0:h0 + WIN, w0:w0 + WIN])
        assert rel_l2(got, ref) <= tol, ("bwd_data", n, h0, w0, rel_l2(got, ref))
        mask = to_host(act[n, :, h0:h0 + WIN, w0:w0 + WIN]) > 0
        got = to_host(dx2[n, :, h0:h0 + WIN, w0:w0 + WIN])
        assert rel_l2(got, np.where(mask, ref, 0.0)) <= tol, ("fused bwd_data", n, h0, w0)
        assert np.all(got[~mask] == 0)

    say(name, "weight and bias gradients")
    del y, y2, dx, dx2, act
    hx, hdy = to_host(x), to_host(dy)
    n_w = K * C * R * R
    rs = np.random.default_rng(6249)
    flat = np.unique(np.concatenate([rs.integers(0, n_w, size=10), [0, n_w - 1]]))
    ref_dw = oracle.conv_bwd_weight_at(hx, hdy, (K, C, R, R), flat, (s, s), (pad, pad))
    got_dw = dw.cpu().numpy().ravel()[flat]
    assert rel_l2(got_dw, ref_dw) <= tol, ("bwd_weight", rel_l2(got_dw, ref_dw))
    ref_db = oracle.bias_bwd(hdy)
    assert rel_l2(db.cpu().numpy(), ref_db) <= tol, ("fused bias_bwd", rel_l2(db.cpu().numpy(), ref_db))
    assert rel_l2(db2.cpu().numpy(), ref_db) <= tol, ("bias_bwd", rel_l2(db2.cpu().numpy(), ref_db))


def test_pointwise_operators_near_the_size_limits():
    """ReLU, fan-in sum, channel concatenation and both max-pooling forms of the workloads on a
    1.10e9-element (4.4 GB) tensor: exact operators, compared whole and bit for bit with the oracle
    (the pooling gradient with small-integer dy, so that its sums are exact in any order)."""
    import torch
    import paper_1412_6249_amd as pa
    from gpu_util import DEV

    N, C, H, W = 3, 24, 3900, 3900
    free, _ = torch.cuda.mem_get_info()
    if free < 48 * 2 ** 30:
        pytest.skip("needs 48 GiB of free device memory")
    g = torch.Generator(device="cuda")
    g.manual_seed(6249)
    x = torch.rand((N, C, H, W), generator=g, device=DEV) - 0.5
    gr = torch.rand((N, C, H, W), generator=g, device=DEV) * 2 - 1
    hx, hg = x.cpu().numpy(), gr.cpu().numpy()
    out = torch.empty_like(x)

    say("large pointwise: relu")
    pa.purine_relu_fwd(x, out)
    torch.cuda.synchronize()
    assert np.array_equal(out.cpu().numpy(), oracle.relu_fwd(hx))
    pa.purine_relu_bwd(x, gr, out)
    torch.cuda.synchronize()
    assert np.array_equal(out.cpu().numpy(), oracle.relu_bwd(hx, hg))

    say("large pointwise: sum")
    pa.purine_sum([x, gr], out)
    torch.cuda.synchronize()
    assert np.array_equal(out.cpu().numpy(), oracle.fan_in_sum([hx, hg]).astype(np.float32))

    say("large pointwise: concat")
    extra = torch.rand((N, 2, H, W), generator=g, device=DEV)
    cat = torch.empty((N, C + 2, H, W), device=DEV)
    pa.purine_concat_fwd([x, extra], cat)
    torch.cuda.synchronize()
    assert np.array_equal(cat.cpu().numpy(), oracle.concat_channels([hx, extra.cpu().numpy()]))
    del cat, extra, hg

    for window_, stride, pad in ((3, 1, 1), (3, 2, 0)):
        say("large pointwise: max-pool", window_, stride, pad)
        P = (H + 2 * pad - window_) // stride + 1
        desc = pa.pool_desc(window_, stride, pad)
        y = torch.empty((N, C, P, P), device=DEV)
        arg = torch.empty((N, C, P, P), dtype=torch.int32, device=DEV)
        pa.purine_maxpool_fwd(desc, x, y, arg)
        torch.cuda.synchronize()
        ref_y, ref_arg = oracle.maxpool_fwd(hx, window_, stride, pad)
        assert np.array_equal(y.cpu().numpy(), ref_y)
        assert np.array_equal(arg.cpu().numpy(), ref_arg)
        dy = torch.randint(-2, 3, (N, C, P, P), generator=g, device=DEV).float()
        pa.purine_maxpool_bwd(desc, dy, arg, out)
        torch.cuda.synchronize()
        ref_dx = oracle.maxpool_bwd(dy.cpu().numpy(), ref_arg, (N, C, H, W))
        assert np.array_equal(out.cpu().numpy(), ref_dx.astype(np.float32))
        del y, arg, dy, ref_y, ref_arg, ref_dx
