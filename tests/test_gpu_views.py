"""Channel-slice views (a tensor that is channels c0..c0+C-1 of a larger NCHW buffer) through every
fp32 convolution kernel family and through ReLU, against the oracle on the corresponding dense
slices. The rest of each buffer is filled with a sentinel and must come back untouched."""
import zlib

import numpy as np
import pytest

import oracle

pytestmark = pytest.mark.gpu

SENTINEL = 777.0

# name, N, C, H, W, K, R, S, stride, pad  (kernel family it exercises)
VIEW_CASES = [
    ("tap3x3_k130_c33", 2, 33, 15, 15, 130, 3, 3, (1, 1), (1, 1)),        # tap-major fwd/bwd, flattened wgrad
    ("tap_c70_k70_5x5", 2, 70, 12, 12, 70, 5, 5, (1, 1), (2, 2)),         # per-tap wgrad (96x96 tile)
    ("flat_stride4_11x11", 3, 3, 51, 47, 96, 11, 11, (4, 4), (0, 0)),     # flat fwd, phase-folded 48-row bwd
    ("stem_like_s2", 2, 3, 40, 40, 64, 7, 7, (2, 2), (3, 3)),             # flat fwd with padding, 12-row bwd
    ("stride3_pad2", 2, 7, 20, 18, 20, 5, 4, (3, 2), (2, 1)),
    ("pw_c48_k100", 3, 48, 10, 14, 100, 1, 1, (1, 1), (0, 0)),            # streaming 1x1 kernel (HW % 4 == 0)
    ("pw_c192_k96", 2, 192, 6, 10, 96, 1, 1, (1, 1), (0, 0)),
    ("pw_c64_k64_hw42", 2, 64, 7, 6, 64, 1, 1, (1, 1), (0, 0)),           # HW % 4 == 2
    ("inception_1x1_like", 2, 192, 28, 28, 176, 1, 1, (1, 1), (0, 0)),
]


def view_of(torch, arr, c_before, c_after, dev):
    """A device buffer [N, c_before + C + c_after, H, W] full of the sentinel whose middle channels
    hold `arr`; returns (buffer, view). c_before is a multiple of 4 (16-byte aligned first element)
    and the total channel count is rounded up to one (distance between images)."""
    n, c, h, w = arr.shape
    total = c_before + c + c_after
    total += -total % 4                                   # distance between images: a multiple of 4 elements
    big = torch.full((n, total, h, w), SENTINEL, dtype=torch.float32, device=dev)
    v = big[:, c_before:c_before + c]
    v.copy_(torch.from_numpy(arr).to(dev))
    assert v.data_ptr() % 16 == 0 and v.stride(0) % 4 == 0 and not v.is_contiguous()
    return big, v


def untouched(big, c_before, c):
    b = big.cpu().numpy()
    return np.all(b[:, :c_before] == SENTINEL) and np.all(b[:, c_before + c:] == SENTINEL)


@pytest.mark.parametrize("case", VIEW_CASES, ids=[c[0] for c in VIEW_CASES])
def test_conv_operators_on_views(case):
    import torch
    import paper_1412_6249_amd as pa
    from gpu_util import rel_l2, workspace, DEV
    name, N, C, H, W, K, R, S, stride, pad = case
    rs = np.random.default_rng(zlib.crc32(name.encode()))
    P, Q = oracle.out_shape((N, C, H, W), (K, C, R, S), stride, pad)[2:]
    u = lambda *s: rs.uniform(-1, 1, size=s).astype(np.float32)
    x, w, b, dy, act = u(N, C, H, W), u(K, C, R, S), u(K), u(N, K, P, Q), u(N, C, H, W)
    # channel paddings: multiples of 4 keep every alignment rule whatever H*W is
    xb, xv = view_of(torch, x, 4, 8, DEV)
    dyb, dyv = view_of(torch, dy, 8, 4, DEV)
    ab, av = view_of(torch, act, 4, 8, DEV)                       # same distance between images as dx below
    yb, yv = view_of(torch, np.zeros((N, K, P, Q), np.float32), 12, 4, DEV)
    dxb, dxv = view_of(torch, np.zeros((N, C, H, W), np.float32), 4, 8, DEV)
    dx2b, dx2v = view_of(torch, np.zeros((N, C, H, W), np.float32), 4, 8, DEV)
    tw, tb = torch.from_numpy(w).to(DEV), torch.from_numpy(b).to(DEV)
    dw = torch.empty((K, C, R, S), dtype=torch.float32, device=DEV)
    db = torch.empty((K,), dtype=torch.float32, device=DEV)
    desc = pa.conv_desc(stride, pad)
    q = lambda which: workspace(pa.purine_conv_workspace_bytes(which, desc, x.shape, w.shape, pa.PURINE_F32))
    pa.purine_conv_fwd_bias_relu(desc, xv, tw, tb, yv, relu=True, ws=q(pa.PURINE_CONV_FWD))
    pa.purine_conv_bwd_data(desc, dyv, tw, dxv, ws=q(pa.PURINE_CONV_BWD_DATA))
    pa.purine_conv_bwd_data_relu(desc, dyv, tw, av, dx2v, ws=q(pa.PURINE_CONV_BWD_DATA))
    pa.purine_conv_bwd_weight_bias(desc, xv, dyv, dw, db, ws=q(pa.PURINE_CONV_BWD_WEIGHT_BIAS))
    torch.cuda.synchronize()
    tol = 1e-5
    ref_y = np.maximum(oracle.bias_fwd(oracle.conv_fwd(x, w, stride, pad), b), 0.0)
    assert rel_l2(yv.cpu().numpy(), ref_y) <= tol, "fwd"
    ref_dx = oracle.conv_bwd_data(dy, w, x.shape, stride, pad)
    assert rel_l2(dxv.cpu().numpy(), ref_dx) <= tol, "bwd_data"
    assert rel_l2(dx2v.cpu().numpy(), np.where(act > 0, ref_dx, 0.0)) <= tol, "bwd_data through the mask"
    assert rel_l2(dw.cpu().numpy(), oracle.conv_bwd_weight(x, dy, w.shape, stride, pad)) <= tol, "bwd_weight"
    assert rel_l2(db.cpu().numpy(), oracle.bias_bwd(dy)) <= tol, "bias_bwd"
    assert untouched(yb, 12, K) and untouched(dxb, 4, C) and untouched(dx2b, 4, C)
    assert untouched(xb, 4, C) and untouched(dyb, 8, K) and untouched(ab, 4, C)

    # the same operators with dense tensors give the same bits (views change addresses only), and the
    # general kernels (raw buffer loads off, no streaming 1x1 kernel) agree with the oracle on views too
    dense = lambda a: torch.from_numpy(a).to(DEV)
    y_d = torch.empty((N, K, P, Q), dtype=torch.float32, device=DEV)
    dx_d = torch.empty((N, C, H, W), dtype=torch.float32, device=DEV)
    dw_d, db_d = torch.empty_like(dw), torch.empty_like(db)
    pa.purine_conv_fwd_bias_relu(desc, dense(x), tw, tb, y_d, relu=True, ws=q(pa.PURINE_CONV_FWD))
    pa.purine_conv_bwd_data(desc, dense(dy), tw, dx_d, ws=q(pa.PURINE_CONV_BWD_DATA))
    pa.purine_conv_bwd_weight_bias(desc, dense(x), dense(dy), dw_d, db_d, ws=q(pa.PURINE_CONV_BWD_WEIGHT_BIAS))
    torch.cuda.synchronize()
    assert torch.equal(y_d, yv) and torch.equal(dx_d, dxv) and torch.equal(dw_d, dw) and torch.equal(db_d, db)
    pa.purine_debug_force_tile(-1, -1)
    try:
        yv.fill_(SENTINEL)
        dxv.fill_(SENTINEL)
        pa.purine_conv_fwd_bias_relu(desc, xv, tw, tb, yv, relu=True, ws=q(pa.PURINE_CONV_FWD))
        pa.purine_conv_bwd_data(desc, dyv, tw, dxv, ws=q(pa.PURINE_CONV_BWD_DATA))
        pa.purine_conv_bwd_weight(desc, xv, dyv, dw_d, ws=q(pa.PURINE_CONV_BWD_WEIGHT))
        torch.cuda.synchronize()
    finally:
        pa.purine_debug_force_tile(0, 0)
    assert rel_l2(yv.cpu().numpy(), ref_y) <= tol and rel_l2(dxv.cpu().numpy(), ref_dx) <= tol
    assert rel_l2(dw_d.cpu().numpy(), oracle.conv_bwd_weight(x, dy, w.shape, stride, pad)) <= tol
    assert untouched(yb, 12, K) and untouched(dxb, 4, C)


@pytest.mark.parametrize("shape", [(3, 5, 7, 9), (2, 64, 28, 28), (5, 6, 3, 3)])
def test_relu_on_views(shape):
    import torch
    import paper_1412_6249_amd as pa
    from gpu_util import DEV
    rs = np.random.default_rng(shape[1])
    x = rs.uniform(-1, 1, shape).astype(np.float32)
    g = rs.uniform(-1, 1, shape).astype(np.float32)
    xb, xv = view_of(torch, x, 4, 4, DEV)
    gb, gv = view_of(torch, g, 8, 4, DEV)
    yb, yv = view_of(torch, np.zeros(shape, np.float32), 4, 12, DEV)
    pa.purine_relu_fwd(xv, yv)
    torch.cuda.synchronize()
    assert np.array_equal(yv.cpu().numpy(), oracle.relu_fwd(x)) and untouched(yb, 4, shape[1])
    pa.purine_relu_bwd(xv, gv, yv)
    torch.cuda.synchronize()
    assert np.array_equal(yv.cpu().numpy(), oracle.relu_bwd(x, g)) and untouched(yb, 4, shape[1])
    pa.purine_relu_bwd(xv, gv, gv)                                   # in place on the gradient view
    torch.cuda.synchronize()
    assert np.array_equal(gv.cpu().numpy(), oracle.relu_bwd(x, g)) and untouched(gb, 8, shape[1])
    dense = torch.empty(shape, dtype=torch.float32, device=DEV)      # view in, dense out
    pa.purine_relu_fwd(xv, dense)
    torch.cuda.synchronize()
    assert np.array_equal(dense.cpu().numpy(), oracle.relu_fwd(x)) and untouched(xb, 4, shape[1])
