"""Pins for the CPU oracle: things the mathematics fixes, none of which re-types the oracle's loops.

The paper gives no worked example (section 2 / Figure 1 define the conv layer by reference), so the
pins are closed forms, brute force on tiny inputs, special cases that reduce to a library matmul,
a second formulation (explicit lowering + matmul, the prior-art formulation the paper's math
routines used, section 1), adjoint identities and exact finite differences.
"""
import itertools
import os

import numpy as np
import pytest

import oracle
from synth import gen
from synth.configs import CONV_LAYERS

RNG = np.random.default_rng(1412_6249)
GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "ones_3x3_tap_counts.txt")


def rnd(*shape):
    return RNG.uniform(-1, 1, size=shape).astype(np.float32)


def rel(a, b):
    a, b = np.asarray(a, np.float64), np.asarray(b, np.float64)
    d = np.linalg.norm((a - b).ravel())
    n = np.linalg.norm(b.ravel())
    return d if n == 0 else d / n


SHAPES = [
    # N, C, H, W, K, R, S, (sh, sw), (ph, pw)
    (2, 3, 7, 6, 4, 3, 3, (1, 1), (1, 1)),
    (1, 2, 9, 11, 3, 3, 2, (2, 1), (0, 1)),
    (2, 1, 12, 10, 2, 5, 3, (3, 2), (2, 0)),
    (1, 4, 13, 13, 5, 4, 4, (4, 4), (3, 3)),
    (3, 2, 5, 8, 2, 1, 1, (1, 1), (0, 0)),
    (1, 3, 6, 6, 2, 2, 5, (1, 3), (1, 2)),
]


def lower(x, R, S, stride, pad):
    """Patch matrix [N*P*Q, C*R*S] built with explicit zero padding and strided slicing."""
    N, C, H, W = x.shape
    (sh, sw), (ph, pw) = stride, pad
    xp = np.zeros((N, C, H + 2 * ph, W + 2 * pw), dtype=np.float64)
    xp[:, :, ph:ph + H, pw:pw + W] = x
    P = (H + 2 * ph - R) // sh + 1
    Q = (W + 2 * pw - S) // sw + 1
    cols = np.empty((N, P, Q, C, R, S), dtype=np.float64)
    for r in range(R):
        for s in range(S):
            cols[:, :, :, :, r, s] = xp[:, :, r:r + sh * (P - 1) + 1:sh,
                                        s:s + sw * (Q - 1) + 1:sw].transpose(0, 2, 3, 1)
    return cols.reshape(N * P * Q, C * R * S), P, Q


def load_golden():
    rows = [l.split() for l in open(GOLDEN) if l.strip() and not l.startswith("#")]
    m = np.array([[float(v) for v in r] for r in rows[:3]])
    corners = np.array([[float(v) for v in r] for r in rows[3:5]])
    cover = np.array([[float(v) for v in r] for r in rows[5:8]])
    return m, corners, cover


# ---------------------------------------------------------------- P1 closed forms, hand-derived
def test_ones_tap_counts_golden():
    m, corners, cover = load_golden()
    one = np.ones((1, 1, 3, 3), np.float32)
    assert np.array_equal(oracle.conv_fwd(one, one, 1, 1)[0, 0], m)
    assert np.array_equal(oracle.conv_fwd(one, one, 2, 1)[0, 0], corners)
    assert np.array_equal(oracle.conv_bwd_data(one, one, (1, 1, 3, 3), 1, 1)[0, 0], m)
    assert np.array_equal(oracle.conv_bwd_weight(one, one, (1, 1, 3, 3), 1, 1)[0, 0], m)
    dy2 = np.ones((1, 1, 2, 2), np.float32)
    assert np.array_equal(oracle.conv_bwd_data(dy2, one, (1, 1, 3, 3), 2, 1)[0, 0], cover)
    assert np.array_equal(oracle.conv_bwd_weight(one, dy2, (1, 1, 3, 3), 2, 1)[0, 0], cover)
    assert np.array_equal(oracle.bias_bwd(one), [9.0])


def test_brute_force_tiny_python_loops():
    """Every product enumerated in pure Python with an independent index convention:
    iterate over INPUT positions and kernel taps and ask which output they feed."""
    N, C, H, W, K, R, S = 2, 2, 5, 4, 3, 3, 2
    (sh, sw), (ph, pw) = (2, 1), (1, 1)
    x, w = rnd(N, C, H, W), rnd(K, C, R, S)
    P = (H + 2 * ph - R) // sh + 1
    Q = (W + 2 * pw - S) // sw + 1
    dy = rnd(N, K, P, Q)
    y = np.zeros((N, K, P, Q))
    dx = np.zeros((N, C, H, W))
    dw = np.zeros((K, C, R, S))
    for n, c, h, ww, k, r, s in itertools.product(range(N), range(C), range(H), range(W),
                                                  range(K), range(R), range(S)):
        tp, tq = h + ph - r, ww + pw - s
        if tp % sh or tq % sw:
            continue
        p, q = tp // sh, tq // sw
        if not (0 <= p < P and 0 <= q < Q):
            continue
        y[n, k, p, q] += float(x[n, c, h, ww]) * float(w[k, c, r, s])
        dx[n, c, h, ww] += float(dy[n, k, p, q]) * float(w[k, c, r, s])
        dw[k, c, r, s] += float(dy[n, k, p, q]) * float(x[n, c, h, ww])
    assert rel(oracle.conv_fwd(x, w, (sh, sw), (ph, pw)), y) < 1e-14
    assert rel(oracle.conv_bwd_data(dy, w, x.shape, (sh, sw), (ph, pw)), dx) < 1e-14
    assert rel(oracle.conv_bwd_weight(x, dy, w.shape, (sh, sw), (ph, pw)), dw) < 1e-14


# ---------------------------------------------------------------- P2 second formulation
@pytest.mark.parametrize("shape", SHAPES)
def test_lowering_plus_matmul_agrees(shape):
    N, C, H, W, K, R, S, stride, pad = shape
    x, w = rnd(N, C, H, W), rnd(K, C, R, S)
    cols, P, Q = lower(x, R, S, stride, pad)
    wm = w.reshape(K, -1).astype(np.float64)
    y = (cols @ wm.T).reshape(N, P, Q, K).transpose(0, 3, 1, 2)
    assert oracle.out_shape(x.shape, w.shape, stride, pad) == (N, K, P, Q)
    assert rel(oracle.conv_fwd(x, w, stride, pad), y) < 1e-13
    dy = rnd(N, K, P, Q)
    dym = dy.transpose(0, 2, 3, 1).reshape(N * P * Q, K).astype(np.float64)
    dw = (dym.T @ cols).reshape(K, C, R, S)
    assert rel(oracle.conv_bwd_weight(x, dy, w.shape, stride, pad), dw) < 1e-13
    # bwd-data through the lowering: fold d(cols) = dy @ w back with the transpose of `lower`
    dcols = (dym @ wm).reshape(N, P, Q, C, R, S)
    (sh, sw), (ph, pw) = stride, pad
    dxp = np.zeros((N, C, H + 2 * ph, W + 2 * pw))
    for r in range(R):
        for s in range(S):
            dxp[:, :, r:r + sh * (P - 1) + 1:sh, s:s + sw * (Q - 1) + 1:sw] += \
                dcols[:, :, :, :, r, s].transpose(0, 3, 1, 2)
    dx = dxp[:, :, ph:ph + H, pw:pw + W]
    assert rel(oracle.conv_bwd_data(dy, w, x.shape, stride, pad), dx) < 1e-13


# ---------------------------------------------------------------- P3 1x1 = matmul
def test_1x1_is_matmul():
    N, C, H, W, K = 3, 5, 4, 6, 7
    x, w, dy = rnd(N, C, H, W), rnd(K, C, 1, 1), rnd(N, K, H, W)
    W2 = w[:, :, 0, 0].astype(np.float64)
    y = np.einsum("kc,nchw->nkhw", W2, x.astype(np.float64))
    assert rel(oracle.conv_fwd(x, w), y) < 1e-14
    dx = np.einsum("kc,nkhw->nchw", W2, dy.astype(np.float64))
    assert rel(oracle.conv_bwd_data(dy, w, x.shape), dx) < 1e-14
    dw = np.einsum("nkhw,nchw->kc", dy.astype(np.float64), x.astype(np.float64))
    assert rel(oracle.conv_bwd_weight(x, dy, w.shape)[:, :, 0, 0], dw) < 1e-14


# ---------------------------------------------------------------- P4 delta kernel = shift (no flip)
@pytest.mark.parametrize("r0,s0", [(0, 0), (1, 1), (2, 0), (0, 2), (1, 2)])
def test_delta_kernel_is_shift_cross_correlation(r0, s0):
    N, C, H, W = 2, 3, 6, 7
    x = rnd(N, C, H, W)
    w = np.zeros((C, C, 3, 3), np.float32)
    for c in range(C):
        w[c, c, r0, s0] = 1.0
    y = oracle.conv_fwd(x, w, 1, 1)
    expect = np.zeros_like(y)
    for p in range(H):
        for q in range(W):
            h, ww = p - 1 + r0, q - 1 + s0     # cross-correlation: tap (r0,s0) reads x[p-pad+r0]
            if 0 <= h < H and 0 <= ww < W:
                expect[:, :, p, q] = x[:, :, h, ww]
    assert np.array_equal(y, expect)
    if (r0, s0) == (1, 1):
        assert np.array_equal(y, x.astype(np.float64))


def test_delta_kernel_strided():
    x = rnd(1, 1, 9, 9)
    w = np.zeros((1, 1, 3, 3), np.float32)
    w[0, 0, 2, 1] = 1.0
    y = oracle.conv_fwd(x, w, 2, 0)
    assert y.shape == (1, 1, 4, 4)
    assert np.array_equal(y[0, 0], x[0, 0, 2:9:2, 1:8:2].astype(np.float64))


# ---------------------------------------------------------------- P5 adjoint identities
@pytest.mark.parametrize("shape", SHAPES)
def test_adjoint_identities(shape):
    N, C, H, W, K, R, S, stride, pad = shape
    x, w = rnd(N, C, H, W), rnd(K, C, R, S)
    y = oracle.conv_fwd(x, w, stride, pad)
    dy = rnd(*y.shape)
    b = rnd(K)
    lhs = np.vdot(y, dy.astype(np.float64))
    a1 = np.vdot(x.astype(np.float64), oracle.conv_bwd_data(dy, w, x.shape, stride, pad))
    a2 = np.vdot(w.astype(np.float64), oracle.conv_bwd_weight(x, dy, w.shape, stride, pad))
    scale = np.linalg.norm(y) * np.linalg.norm(dy)
    assert abs(lhs - a1) < 1e-12 * scale
    assert abs(lhs - a2) < 1e-12 * scale
    yb = oracle.bias_fwd(np.zeros_like(y), b)
    assert abs(np.vdot(yb, dy.astype(np.float64)) - np.vdot(b.astype(np.float64), oracle.bias_bwd(dy))) \
        < 1e-12 * np.linalg.norm(yb) * np.linalg.norm(dy)


# ---------------------------------------------------------------- P6 finite differences (exact: L is linear)
@pytest.mark.parametrize("shape", SHAPES[:4])
@pytest.mark.parametrize("step", [1.0, 2.0 ** -10])
def test_finite_differences(shape, step):
    N, C, H, W, K, R, S, stride, pad = shape
    # values on a 2^-12 grid so that x +- step is exact in fp32 for both steps
    x, w, b = (np.round(t * 4096) / 4096 for t in (rnd(N, C, H, W), rnd(K, C, R, S), rnd(K)))
    x, w, b = x.astype(np.float32), w.astype(np.float32), b.astype(np.float32)
    dy = rnd(*oracle.out_shape(x.shape, w.shape, stride, pad))
    dy64 = dy.astype(np.float64)

    def L(x_, w_, b_):
        return np.vdot(oracle.bias_fwd(oracle.conv_fwd(x_, w_, stride, pad), b_), dy64)

    dx = oracle.conv_bwd_data(dy, w, x.shape, stride, pad)
    dw = oracle.conv_bwd_weight(x, dy, w.shape, stride, pad)
    db = oracle.bias_bwd(dy)
    pick = np.random.default_rng(7)
    corners = [(0,) * 4, tuple(np.array(x.shape) - 1)]
    for idx in corners + [tuple(pick.integers(0, d) for d in x.shape) for _ in range(12)]:
        e = np.zeros_like(x)
        e[idx] = step
        fd = (L(x + e, w, b) - L(x - e, w, b)) / (2 * step)
        assert abs(fd - dx[idx]) <= 1e-10 * max(1.0, abs(dx[idx])), (idx, fd, dx[idx])
    for idx in [(0,) * 4, tuple(np.array(w.shape) - 1)] + \
               [tuple(pick.integers(0, d) for d in w.shape) for _ in range(12)]:
        e = np.zeros_like(w)
        e[idx] = step
        fd = (L(x, w + e, b) - L(x, w - e, b)) / (2 * step)
        assert abs(fd - dw[idx]) <= 1e-10 * max(1.0, abs(dw[idx])), (idx, fd, dw[idx])
    for k in range(K):
        e = np.zeros_like(b)
        e[k] = step
        fd = (L(x, w, b + e) - L(x, w, b - e)) / (2 * step)
        assert abs(fd - db[k]) <= 1e-10 * max(1.0, abs(db[k]))


# ---------------------------------------------------------------- P7 batch additivity (data-parallel invariant)
def test_batch_additivity():
    N, C, H, W, K, R, S, stride, pad = 5, 3, 8, 7, 4, 3, 3, (2, 1), (1, 1)
    x, w = rnd(N, C, H, W), rnd(K, C, R, S)
    y = oracle.conv_fwd(x, w, stride, pad)
    dy = rnd(*y.shape)
    dx = oracle.conv_bwd_data(dy, w, x.shape, stride, pad)
    dw = oracle.conv_bwd_weight(x, dy, w.shape, stride, pad)
    db = oracle.bias_bwd(dy)
    shards = [slice(0, 2), slice(2, 3), slice(3, 5)]
    dw_sum, db_sum = np.zeros_like(dw), np.zeros_like(db)
    for s in shards:
        assert np.array_equal(oracle.conv_fwd(x[s], w, stride, pad), y[s])
        assert np.array_equal(oracle.conv_bwd_data(dy[s], w, x[s].shape, stride, pad), dx[s])
        dw_sum += oracle.conv_bwd_weight(x[s], dy[s], w.shape, stride, pad)
        db_sum += oracle.bias_bwd(dy[s])
    assert rel(dw_sum, dw) < 1e-14 and rel(db_sum, db) < 1e-14


# ---------------------------------------------------------------- P8 stride / pad reductions
def test_stride_is_subsampling_and_pad_is_explicit_zeros():
    x, w = rnd(2, 3, 11, 10), rnd(4, 3, 3, 3)
    full = oracle.conv_fwd(x, w, 1, 1)
    assert np.array_equal(oracle.conv_fwd(x, w, (3, 2), 1), full[:, :, ::3, ::2])
    xp = np.zeros((2, 3, 11 + 4, 10 + 2), np.float32)
    xp[:, :, 2:13, 1:11] = x
    assert rel(oracle.conv_fwd(x, w, 1, (2, 1)), oracle.conv_fwd(xp, w, 1, 0)) < 1e-15


# ---------------------------------------------------------------- P9 constants
def test_zero_weights_and_unit_gradients():
    x, b = rnd(2, 3, 9, 8), rnd(5)
    w0 = np.zeros((5, 3, 3, 3), np.float32)
    y = oracle.bias_fwd(oracle.conv_fwd(x, w0, 1, 1), b)
    assert np.array_equal(y, np.broadcast_to(b.astype(np.float64)[None, :, None, None], y.shape))
    ones = np.ones((2, 5, 4, 3), np.float32)      # stride 2, pad 0 on 9x8 with 3x3: P=4, Q=3
    assert oracle.out_shape(x.shape, w0.shape, 2, 0) == (2, 5, 4, 3)
    assert np.array_equal(oracle.bias_bwd(ones), np.full(5, 2 * 4 * 3.0))
    dw = oracle.conv_bwd_weight(x, ones, w0.shape, 2, 0)
    # dy = 1  =>  dw[k,c,r,s] = sum of x over the strided lattice starting at (r,s)
    x64 = x.astype(np.float64)
    for r in range(3):
        for s in range(3):
            lattice = x64[:, :, r:r + 7:2, s:s + 5:2].sum(axis=(0, 2, 3))
            for k in range(5):
                assert np.allclose(dw[k, :, r, s], lattice, rtol=1e-14, atol=1e-14)


def test_unit_gradient_dw_matches_summed_area_table():
    """stride 1, pad 1: dw[k,c,r,s] is a window sum of x; take it from an integral image."""
    N, C, H, W = 2, 2, 6, 7
    x = gen.integers((N, C, H, W), 11, 4)
    ones = np.ones((N, 1, H, W), np.float32)
    dw = oracle.conv_bwd_weight(x, ones, (1, C, 3, 3), 1, 1)
    sat = np.zeros((N, C, H + 1, W + 1))
    sat[:, :, 1:, 1:] = x.astype(np.float64).cumsum(2).cumsum(3)
    for r in range(3):
        for s in range(3):
            h0, h1 = max(0, r - 1), min(H, H - 1 + r)     # rows p-1+r for p in [0,H) clipped
            w0, w1 = max(0, s - 1), min(W, W - 1 + s)
            box = sat[:, :, h1, w1] - sat[:, :, h0, w1] - sat[:, :, h1, w0] + sat[:, :, h0, w0]
            assert np.array_equal(dw[0, :, r, s], box.sum(0))


# ---------------------------------------------------------------- P10 shape table
def test_shape_table_of_the_workloads():
    expect = {("2", "conv1"): 54, ("2", "cccp1"): 54, ("3", "b2_3x3"): 28, ("3", "b3_5x5"): 28,
              ("4", "conv1"): 55, ("4", "conv2"): 27, ("4", "conv3"): 13, ("4", "conv5"): 13,
              ("5", "stem7x7"): 112, ("5", "c1x1"): 56, ("5", "c3x3"): 56, ("1", "conv"): 16}
    seen = 0
    for cfg, layers in CONV_LAYERS.items():
        for l in layers:
            shp = oracle.out_shape(l.x_shape, l.w_shape, l.stride, l.pad)
            assert shp == l.y_shape
            if (str(cfg), l.name) in expect:
                assert shp[2] == shp[3] == expect[(str(cfg), l.name)]
                seen += 1
    assert seen == len(expect)
    assert oracle.out_extent(224, 11, 4, 0) == 54      # floor, not ceil: 213/4 = 53.25
    assert oracle.out_extent(2, 3, 1, 0) == -1         # padded input smaller than the kernel
    assert oracle.out_extent(3, 3, 1, 0) == 1
    assert oracle.out_extent(5, 3, 0, 0) == -1 and oracle.out_extent(5, 0, 1, 0) == -1
    with pytest.raises(ValueError):
        oracle.out_shape((1, 3, 8, 8), (4, 2, 3, 3), 1, 1)


# ---------------------------------------------------------------- sampled dw equals full dw
def test_bwd_weight_at_matches_full():
    x, dy = rnd(3, 4, 9, 9), rnd(3, 5, 4, 4)
    dw = oracle.conv_bwd_weight(x, dy, (5, 4, 3, 3), 2, 0)
    idx = np.array([0, 7, 44, 179, 5 * 4 * 9 - 1])
    assert np.array_equal(oracle.conv_bwd_weight_at(x, dy, (5, 4, 3, 3), idx, 2, 0), dw.ravel()[idx])


# ---------------------------------------------------------------- integer inputs: exact in any order
def test_integer_inputs_are_exact():
    l = CONV_LAYERS[1][0]
    x, w, b, dy = gen.layer_tensors(l, 1, integer=True)
    y = oracle.conv_fwd(x, w, l.stride, l.pad)
    assert np.array_equal(y, np.round(y)) and np.abs(y).max() < 2 ** 24
    cols, P, Q = lower(x, l.R, l.S, (l.stride,) * 2, (l.pad,) * 2)
    y2 = (cols @ w.reshape(l.K, -1).astype(np.float64).T).reshape(l.N, P, Q, l.K).transpose(0, 3, 1, 2)
    assert np.array_equal(y, y2)


# ---------------------------------------------------------------- support operators
def test_relu_and_pool_and_concat():
    x = rnd(2, 3, 7, 7)
    x[0, 0, 0, 0] = 0.0
    dy = rnd(2, 3, 7, 7)
    assert np.array_equal(oracle.relu_fwd(x), np.maximum(x, 0))
    assert np.array_equal(oracle.relu_bwd(x, dy), np.where(x > 0, dy, 0))
    y, arg = oracle.maxpool_fwd(x, 3, 2, 0)
    assert y.shape == (2, 3, 3, 3)
    for p in range(3):
        for q in range(3):
            win = x[:, :, 2 * p:2 * p + 3, 2 * q:2 * q + 3].reshape(2, 3, 9)
            assert np.array_equal(y[:, :, p, q], win.max(-1))
            a = win.argmax(-1)                                   # numpy: first maximum
            assert np.array_equal(arg[:, :, p, q], (2 * p + a // 3) * 7 + 2 * q + a % 3)
    g = rnd(2, 3, 3, 3)
    dx = oracle.maxpool_bwd(g, arg, x.shape)
    assert abs(dx.sum() - g.astype(np.float64).sum()) < 1e-12
    assert np.count_nonzero(dx) <= g.size
    # ties: all-equal window -> first position wins; padding never wins
    z = np.zeros((1, 1, 4, 4), np.float32)
    y0, a0 = oracle.maxpool_fwd(z, 3, 1, 1)
    assert y0.shape == (1, 1, 4, 4) and a0[0, 0, 0, 0] == 0 and a0[0, 0, 3, 3] == 2 * 4 + 2
    neg = -np.ones((1, 1, 4, 4), np.float32)
    assert np.array_equal(oracle.maxpool_fwd(neg, 3, 1, 1)[0], neg)
    a, b = rnd(2, 2, 3, 3), rnd(2, 5, 3, 3)
    cat = oracle.concat_channels([a, b])
    assert cat.shape == (2, 7, 3, 3) and np.array_equal(cat[:, 2:], b)
    assert np.array_equal(oracle.fan_in_sum([a, a]), 2 * a.astype(np.float64))


def pool_winners_by_hand(x, k, stride, pad):
    """Winner of every pooling window found without the oracle: the window is cut out of a copy of
    the plane padded with -inf and numpy's argmax (first maximum in row-major order) picks it."""
    N, C, H, W = x.shape
    P, Q = (H + 2 * pad - k) // stride + 1, (W + 2 * pad - k) // stride + 1
    xp = np.full((N, C, H + 2 * pad, W + 2 * pad), -np.inf)
    xp[:, :, pad:pad + H, pad:pad + W] = x
    hh = np.empty((N, C, P, Q), np.int64)
    ww = np.empty((N, C, P, Q), np.int64)
    for p in range(P):
        for q in range(Q):
            a = xp[:, :, p * stride:p * stride + k, q * stride:q * stride + k].reshape(N, C, k * k).argmax(-1)
            hh[:, :, p, q] = p * stride - pad + a // k
            ww[:, :, p, q] = q * stride - pad + a % k
    return hh, ww


@pytest.mark.parametrize("k,stride,pad,H,W", [(3, 1, 1, 6, 7), (3, 2, 0, 9, 7), (3, 2, 1, 8, 8), (2, 2, 0, 6, 4),
                                               (5, 3, 2, 11, 9)])
def test_pool_gradient_lands_on_the_winner_of_its_own_window(k, stride, pad, H, W):
    """Brute force: every window adds its dy to dx[n, c, h*, w*] of ITS plane, (h*, w*) its winner;
    overlapping windows add up. The winners are found by hand (not by the oracle), the planes hold
    distinct values and different planes hold different data, so a gradient landing one position
    off, or read from another plane's dy, changes the result."""
    N, C = 2, 3
    x = RNG.permutation(N * C * H * W).reshape(N, C, H, W).astype(np.float32)   # all distinct
    hh, ww = pool_winners_by_hand(x, k, stride, pad)
    y, arg = oracle.maxpool_fwd(x, k, stride, pad)
    assert np.array_equal(arg, hh * W + ww)
    dy = rnd(*y.shape)
    want = np.zeros(x.shape, np.float64)
    for n, c, p, q in itertools.product(range(N), range(C), range(y.shape[2]), range(y.shape[3])):
        want[n, c, hh[n, c, p, q], ww[n, c, p, q]] += float(dy[n, c, p, q])
    got = oracle.maxpool_bwd(dy, arg, x.shape)
    assert np.abs(got - want).max() <= 1e-15
    if stride < k:      # overlapping windows: some position must have collected several gradients
        counts = np.zeros(x.shape, np.int64)
        np.add.at(counts, (np.arange(N)[:, None, None, None], np.arange(C)[None, :, None, None], hh, ww), 1)
        assert counts.max() >= 2


def test_pool_gradient_is_the_derivative_of_the_pooled_loss():
    """L(x) = <maxpool(x), dy> is piecewise linear; with distinct integer inputs a step of 0.25 at
    one position never changes a winner, so the one-sided difference quotient is exact and equals
    maxpool_bwd's element there (through the forward routine only, which has its own pins)."""
    x = RNG.permutation(2 * 2 * 7 * 7).reshape(2, 2, 7, 7).astype(np.float32)
    k, stride, pad = 3, 2, 1
    y, arg = oracle.maxpool_fwd(x, k, stride, pad)
    dy = np.round(rnd(*y.shape) * 64) / 64          # on a 2^-6 grid: every product below is exact
    dx = oracle.maxpool_bwd(dy, arg, x.shape)
    loss = lambda t: float((oracle.maxpool_fwd(t, k, stride, pad)[0].astype(np.float64) * dy).sum())
    base = loss(x)
    for idx in itertools.product(range(2), range(2), range(7), range(7)):
        t = x.copy()
        t[idx] += 0.25
        assert (loss(t) - base) / 0.25 == dx[idx], idx


# ---------------------------------------------------------------- SGD step (section 2.2)
def test_sgd_update_descends_a_linear_and_a_quadratic_loss():
    """Pins sign and scale of the update with functions other than itself. (1) L(w) = <conv(x, w), g>
    is linear in w with gradient dw = conv_bwd_weight(x, g), so a step changes it by exactly
    -lr * |dw|^2. (2) For L(w) = |w - t|^2 / 2 the gradient is w - t: a step with lr = 1 lands on
    t, lr = 0 stays, and lr = 1/2 halves the distance."""
    x, w, g = rnd(2, 3, 6, 5), rnd(4, 3, 3, 2), rnd(2, 4, 4, 4)
    stride, pad = (1, 1), (0, 0)
    loss = lambda ww: float((oracle.conv_fwd(x, ww.astype(np.float32), stride, pad) * g).sum())
    dw = oracle.conv_bwd_weight(x, g, w.shape, stride, pad)
    lr = 2.0 ** -6                                       # exact in fp32, keeps w_new close to fp32 grid
    w_new = oracle.sgd_update(w, dw, lr)
    # linearity: evaluate the loss change through the oracle's own forward pass on the DIFFERENCE
    step = (w_new - w.astype(np.float64)).astype(np.float32)
    change = float((oracle.conv_fwd(x, step, stride, pad) * g).sum())
    assert abs(change + lr * float((dw ** 2).sum())) <= 1e-5 * lr * float((dw ** 2).sum())
    assert loss(w_new) < loss(w.astype(np.float64))
    t = rnd(5, 7)
    v = rnd(5, 7)
    assert np.allclose(oracle.sgd_update(v, v.astype(np.float64) - t, 1.0), t, rtol=0, atol=1e-15)
    assert np.array_equal(oracle.sgd_update(v, v - t, 0.0), v.astype(np.float64))
    half = oracle.sgd_update(v, v.astype(np.float64) - t, 0.5)
    assert np.allclose(half - t, 0.5 * (v.astype(np.float64) - t), rtol=0, atol=1e-15)


# ---------------------------------------------------------------- fully connected, grouped convolution
def test_fc_against_loops_adjoints_and_the_conv_oracle():
    x, w, b, dy = rnd(3, 5), rnd(4, 5), rnd(4), rnd(3, 4)
    y = oracle.fc_fwd(x, w, b)
    for n in range(3):
        for k in range(4):
            assert abs(y[n, k] - (sum(float(x[n, c]) * float(w[k, c]) for c in range(5)) + float(b[k]))) < 1e-12
    dx = oracle.fc_bwd_data(dy, w)
    dw, db = oracle.fc_bwd_weight(x, dy)
    # adjoint identities: <fc(x), dy> = <x, dx> = <w, dw>, and the bias term gives <b, db>
    lin = float((oracle.fc_fwd(x, w) * dy).sum())
    assert abs(lin - float((x * dx).sum())) < 1e-12 and abs(lin - float((w * dw).sum())) < 1e-12
    assert abs(float((b.astype(np.float64)[None, :] * dy).sum()) - float((b * db).sum())) < 1e-12
    # a fully-connected layer is a convolution whose filter covers the whole input (C-routine route)
    xi, wi = rnd(2, 3, 4, 5), rnd(6, 3, 4, 5)
    yc = oracle.conv_fwd(xi, wi, 1, 0)
    assert yc.shape == (2, 6, 1, 1)
    assert rel(yc[:, :, 0, 0], oracle.fc_fwd(xi.reshape(2, -1), wi.reshape(6, -1))) < 1e-12


def test_grouped_conv_is_a_block_diagonal_plain_conv():
    """A grouped convolution equals the plain one whose filter is zero outside the diagonal blocks;
    so do its gradients (the weight gradient restricted to the blocks)."""
    G, N, C, K, H, W, R, S = 2, 2, 6, 4, 7, 6, 3, 2
    stride, pad = (2, 1), (1, 0)
    x, w = rnd(N, C, H, W), rnd(K, C // G, R, S)
    full = np.zeros((K, C, R, S), np.float32)
    for g in range(G):
        full[g * K // G:(g + 1) * K // G, g * C // G:(g + 1) * C // G] = w[g * K // G:(g + 1) * K // G]
    y = oracle.grouped_conv_fwd(x, w, G, stride, pad)
    assert rel(y, oracle.conv_fwd(x, full, stride, pad)) < 1e-12
    dy = rnd(*y.shape)
    assert rel(oracle.grouped_conv_bwd_data(dy, w, x.shape, G, stride, pad),
               oracle.conv_bwd_data(dy, full, x.shape, stride, pad)) < 1e-12
    dfull = oracle.conv_bwd_weight(x, dy, full.shape, stride, pad)
    dw = oracle.grouped_conv_bwd_weight(x, dy, w.shape, G, stride, pad)
    for g in range(G):
        ks, cs = slice(g * K // G, (g + 1) * K // G), slice(g * C // G, (g + 1) * C // G)
        assert rel(dw[ks], dfull[ks, cs]) < 1e-12
    assert rel(oracle.grouped_conv_fwd(x, full, 1, stride, pad), oracle.conv_fwd(x, full, stride, pad)) == 0
