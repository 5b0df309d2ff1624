"""GPU parity, element by element against the CPU oracle, at sizes the oracle finishes in seconds
that still span several tiles and ragged tails. Every call goes through the C ABI.

Tolerance: relative L2 <= 1e-5 (fp32), <= 1e-2 (bf16 inputs, fp32 accumulation); delta kernels and
integer-valued inputs must match bit for bit (index and shape bookkeeping)."""
import zlib

import numpy as np
import pytest

import oracle
from synth import gen
from synth.configs import CONV_LAYERS, ConvLayer

pytestmark = pytest.mark.gpu

# name, N, C, H, W, K, R, S, (sh,sw), (ph,pw): ragged against the 32/64/96/128-row tiles, the
# 128/256-pixel tiles and the 16-deep slabs; strides 1..4; non-square everything
CASES = [
    ("tiny", 1, 1, 3, 3, 1, 3, 3, (1, 1), (1, 1)),
    ("ragged_k37", 3, 5, 19, 23, 37, 3, 2, (2, 1), (1, 0)),
    ("one_by_one", 2, 40, 13, 11, 100, 1, 1, (1, 1), (0, 0)),
    ("k130_c33", 2, 33, 15, 15, 130, 3, 3, (1, 1), (1, 1)),
    ("stride4_11x11", 3, 3, 51, 47, 96, 11, 11, (4, 4), (0, 0)),
    ("stride3_pad2", 2, 7, 20, 18, 20, 5, 4, (3, 2), (2, 1)),
    ("k5x5_pad2", 2, 16, 14, 14, 32, 5, 5, (1, 1), (2, 2)),
    ("stem_like", 2, 3, 40, 40, 64, 7, 7, (2, 2), (3, 3)),
    ("pad_bigger_than_needed", 1, 2, 5, 6, 3, 3, 3, (1, 1), (2, 2)),
    ("many_pixels", 5, 4, 37, 41, 8, 3, 3, (1, 1), (1, 1)),
    ("c200", 1, 200, 9, 9, 48, 3, 3, (1, 1), (1, 1)),
    ("smallc_s3x2", 2, 2, 13, 17, 9, 4, 5, (3, 2), (1, 2)),
    ("smallc_tiny_h", 1, 3, 2, 9, 4, 3, 3, (4, 2), (1, 1)),
    ("smallc_s4_pad5", 2, 4, 21, 19, 6, 7, 6, (4, 4), (5, 4)),
    ("pq_multiple_of_32", 3, 8, 16, 16, 40, 3, 3, (1, 1), (1, 1)),
    ("c70_k70_5x5", 2, 70, 12, 12, 70, 5, 5, (1, 1), (2, 2)),
    # fewer than 16 channels but C*R*S beyond the flattened kernel's row table: tap-major kernel
    ("c15_12x12_long_reduction", 2, 15, 15, 14, 8, 12, 12, (1, 1), (1, 0)),
    # 1x1 / stride 1 / no padding with channel counts that are multiples of 16 and an even pixel
    # count: the streaming GEMM kernel (forward when C qualifies, backward-data when K does)
    ("pw_c48_k100", 3, 48, 10, 14, 100, 1, 1, (1, 1), (0, 0)),
    ("pw_c192_k96", 2, 192, 6, 10, 96, 1, 1, (1, 1), (0, 0)),
    ("pw_c16_k32", 5, 16, 9, 8, 32, 1, 1, (1, 1), (0, 0)),
    ("pw_c64_k64_hw42", 2, 64, 7, 6, 64, 1, 1, (1, 1), (0, 0)),
    ("pw_c160_k16_m_tail", 7, 160, 5, 14, 16, 1, 1, (1, 1), (0, 0)),
    # ... with so few tiles and so long a reduction (at least four 128-channel stages) that the channels
    # are split over workgroups and a second kernel adds the partial tiles: forward (C = 512, whole
    # stages) and backward-data (K = 640: five stages in splits of two, the last split shorter)
    ("pw_split_c512_k32", 2, 512, 6, 8, 32, 1, 1, (1, 1), (0, 0)),
    ("pw_split_c64_k640", 2, 64, 4, 10, 640, 1, 1, (1, 1), (0, 0)),
    # strided layers whose filter fits inside one stride step: backward-data folds onto a single tap
    # and still needs the depth-to-space epilogue
    ("pw_stride2", 2, 32, 9, 10, 24, 1, 1, (2, 2), (0, 0)),
    ("filter_inside_stride", 2, 64, 20, 21, 33, 1, 2, (1, 4), (0, 1)),
    # K % 4 != 0 with K*C*R*S % 4 == 0 and 64 splits of the pixel reduction: dw's partials are added
    # by the same kernel with and without the fused bias gradient (whose rows are not 16-byte aligned)
    ("k6_many_splits", 4, 2, 64, 64, 6, 3, 3, (1, 1), (1, 1)),
    # bf16: gathered rows of whole 16-byte packets and a unit-stride gather take the kernel that stages
    # the input patch in LDS (forward when W % 8 == 0 and C % 8 == 0, backward-data when Q and K are):
    # every row-tile shape (12, 40, 90, 100, 192 output rows), one and two fill rounds, tiles that end
    # inside an image row, images smaller than a tile, pads 0..2, channel counts that are not multiples of 32
    ("patch_c24_k40", 2, 24, 16, 24, 40, 3, 3, (1, 1), (1, 1)),
    ("patch_c64_k192_5x3", 3, 64, 9, 32, 192, 5, 3, (1, 1), (2, 1)),
    ("patch_c40_k104_wide", 1, 40, 7, 112, 104, 3, 3, (1, 1), (1, 1)),
    ("patch_c16_k90_nopad", 2, 16, 20, 24, 90, 3, 3, (1, 1), (0, 0)),
    ("patch_bwd_folded_s2", 2, 3, 32, 32, 32, 7, 7, (2, 2), (3, 3)),
    ("patch_bwd_folded_s2_k72", 3, 12, 31, 32, 72, 3, 4, (2, 2), (1, 1)),
    ("patch_c96_k96_56", 2, 96, 56, 56, 96, 3, 3, (1, 1), (1, 1)),
    # bf16 forward with fewer than 16 input channels and rows of whole 16-byte packets: input rows
    # staged in LDS, reduction over (c, r, block of 8 filter columns): strides 1..4, even and odd
    # pads, filter rows of one and two blocks, two row tiles, several tiles per image
    ("rows_s4_11x11_k96", 2, 3, 43, 48, 96, 11, 11, (4, 4), (0, 0)),
    ("rows_s1_5x5", 2, 5, 12, 24, 20, 5, 5, (1, 1), (2, 2)),
    ("rows_s3_3x5", 1, 4, 20, 32, 33, 3, 5, (3, 3), (1, 2)),
    ("rows_9x9_pad4", 1, 2, 10, 16, 8, 9, 9, (1, 1), (4, 4)),
    ("rows_s2_7x7_many_tiles", 3, 3, 64, 64, 64, 7, 7, (2, 2), (3, 3)),
    # bf16 3x3 / stride 1 / pad 1 with at least 32 channels on both sides and rows of whole packets: the
    # weight gradient that stages rows in LDS (ranges of rows that cross image boundaries, ragged
    # channel groups on both sides, a last 16-pixel step that is half empty, one-step rows)
    ("wgrows_c64_k192_w24", 3, 64, 9, 24, 192, 3, 3, (1, 1), (1, 1)),
    ("wgrows_c40_k72_w16_h5", 5, 40, 5, 16, 72, 3, 3, (1, 1), (1, 1)),
    ("wgrows_c130_k33_w40", 2, 130, 7, 40, 33, 3, 3, (1, 1), (1, 1)),
    ("wgrows_c32_k32_w8_h3", 7, 32, 3, 8, 32, 3, 3, (1, 1), (1, 1)),
    # ... many short images: every worker's range of rows crosses several image boundaries, the
    # widest rows the kernel takes (7 packets), requests in flight across the boundaries
    ("wgrows_c64_k96_w56_many_images", 37, 64, 4, 56, 96, 3, 3, (1, 1), (1, 1)),
    # bf16 layers with at most 160 filter elements per output channel and a column stride of 1 or 2:
    # the weight gradient whose wavefronts each hold the whole filter tile (input rows de-interleaved
    # by column parity in LDS; an odd number of output rows per image, so that a pair of rows
    # straddles two images; output channels past a multiple of 64; one to five column tiles)
    ("wgcols_7x7_s2_c3_k64", 3, 3, 36, 64, 64, 7, 7, (2, 2), (3, 3)),
    ("wgcols_7x7_s2_odd_rows", 5, 3, 18, 32, 64, 7, 7, (2, 2), (3, 3)),
    ("wgcols_5x5_s1_c3_k40", 2, 3, 12, 32, 40, 5, 5, (1, 1), (2, 2)),
    ("wgcols_3x3_s2_c8_k96", 2, 8, 10, 64, 96, 3, 3, (2, 2), (1, 1)),
    ("wgcols_3x5_s21_c4_k33", 3, 4, 9, 16, 33, 3, 5, (2, 1), (1, 2)),
    ("wgcols_1x1_s2_c16_k32", 2, 16, 6, 32, 32, 1, 1, (2, 2), (0, 0)),
    # ... and shapes only the general form of that kernel takes (a window per lane): more than 32
    # (channel, filter row) pairs, an even filter width
    ("wgcols_3x3_c12_k64", 2, 12, 9, 32, 64, 3, 3, (1, 1), (1, 1)),
    ("wgcols_4x4_s2_c5_k72", 3, 5, 10, 64, 72, 4, 4, (2, 2), (1, 1)),
]
PW = [c for c in CASES if c[0].startswith("pw_")]


def make(case, dtype, seed=0, integer=False):
    name, N, C, H, W, K, R, S, stride, pad = case
    rs = np.random.default_rng(zlib.crc32(name.encode()) + seed)
    P, Q = oracle.out_shape((N, C, H, W), (K, C, R, S), stride, pad)[2:]
    if integer:
        d = lambda *s: rs.integers(-2, 3, size=s).astype(np.float32)
    else:
        d = lambda *s: rs.uniform(-1, 1, size=s).astype(np.float32)
    x, w, b, dy = d(N, C, H, W), d(K, C, R, S), d(K), d(N, K, P, Q)
    if dtype == "bf16":
        x, w, b, dy = (gen.quantize_bf16(t) for t in (x, w, b, dy))
    return x, w, b, dy, stride, pad


def oracle_layer(x, w, b, dy, stride, pad):
    return (oracle.bias_fwd(oracle.conv_fwd(x, w, stride, pad), b),
            oracle.conv_bwd_data(dy, w, x.shape, stride, pad),
            oracle.conv_bwd_weight(x, dy, w.shape, stride, pad),
            oracle.bias_bwd(dy))


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("case", CASES, ids=[c[0] for c in CASES])
def test_layer_parity(case, dtype):
    from gpu_util import run_layer, rel_l2, TOL
    x, w, b, dy, stride, pad = make(case, dtype)
    got = run_layer(x, w, b, dy, stride, pad, dtype)
    ref = oracle_layer(x, w, b, dy, stride, pad)
    for name, g, r in zip(("y", "dx", "dw", "db"), got, ref):
        assert g.shape == r.shape
        assert np.isfinite(g).all(), name
        assert rel_l2(g, r) <= TOL[dtype], (case[0], name, rel_l2(g, r))


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("case", CASES, ids=[c[0] for c in CASES])
def test_fused_weight_and_bias_gradient(case, dtype):
    """ConvBwdWeight+BiasBwd as one operator: db against the oracle, on random and on
    small-integer inputs (exact), and dw bit-identical to the separate operator's (the bias sums
    ride along the same kernel). Also with beta = 1."""
    from gpu_util import run_layer, rel_l2, TOL
    x, w, b, dy, stride, pad = make(case, dtype)
    _, _, dw0, _ = run_layer(x, w, b, dy, stride, pad, dtype)
    _, _, dw, db = run_layer(x, w, b, dy, stride, pad, dtype, fused_wb=True)
    assert np.array_equal(dw, dw0)
    assert np.isfinite(db).all()
    assert rel_l2(db, oracle.bias_bwd(dy)) <= TOL[dtype], rel_l2(db, oracle.bias_bwd(dy))
    xi, wi, bi, dyi, _, _ = make(case, dtype, integer=True)
    _, _, dwi, dbi = run_layer(xi, wi, bi, dyi, stride, pad, dtype, fused_wb=True)
    assert np.array_equal(dbi, oracle.bias_bwd(dyi).astype(np.float32))
    assert np.array_equal(dwi, oracle.conv_bwd_weight(xi, dyi, wi.shape, stride, pad).astype(np.float32))
    rs = np.random.default_rng(11)
    prev = [rs.uniform(-1, 1, s).astype(np.float32) for s in (x.shape, w.shape, b.shape)]
    if dtype == "bf16":
        prev[0] = gen.quantize_bf16(prev[0])
    _, _, dw1, db1 = run_layer(x, w, b, dy, stride, pad, dtype, beta=1.0, prev=prev, fused_wb=True)
    assert rel_l2(db1, oracle.bias_bwd(dy) + prev[2]) <= TOL[dtype]
    assert rel_l2(dw1, oracle.conv_bwd_weight(x, dy, w.shape, stride, pad) + prev[1]) <= TOL[dtype]


def test_config1_all_operators():
    from gpu_util import run_layer, rel_l2
    l = CONV_LAYERS[1][0]
    x, w, b, dy = gen.layer_tensors(l, 1)
    got = run_layer(x, w, b, dy, l.stride, l.pad)
    ref = oracle_layer(x, w, b, dy, l.stride, l.pad)
    for name, g, r in zip(("y", "dx", "dw", "db"), got, ref):
        assert rel_l2(g, r) <= 1e-5, (name, rel_l2(g, r))


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("case", [CASES[1], CASES[4], CASES[5], CASES[3]] + PW[:3], ids=lambda c: c[0])
def test_integer_inputs_bit_exact(case, dtype):
    """Small-integer tensors: every partial sum is an exact integer below 2^24, so any summation
    order gives the same bits. fp32 outputs must equal the oracle exactly; bf16-stored outputs are
    compared after the oracle's value is rounded the same way (RNE)."""
    from gpu_util import run_layer
    x, w, b, dy, stride, pad = make(case, dtype, integer=True)
    got = run_layer(x, w, b, dy, stride, pad, dtype)
    ref = oracle_layer(x, w, b, dy, stride, pad)
    assert max(np.abs(r).max() for r in ref) < 2 ** 24
    for i, (g, r) in enumerate(zip(got, ref)):
        r32 = r.astype(np.float32)
        if dtype == "bf16" and i < 2:
            r32 = gen.quantize_bf16(r32)
        assert np.array_equal(g, r32), ("y", "dx", "dw", "db")[i]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("r0,s0,stride,pad", [(1, 1, 1, 1), (0, 2, 1, 1), (2, 0, 2, 1), (4, 3, 3, 2)])
def test_delta_kernel_is_an_exact_shift(r0, s0, stride, pad, dtype):
    """w = delta at tap (r0,s0) on the channel diagonal: y is x shifted (cross-correlation, zero
    fill), bit for bit; dx of a delta is dy scattered back, bit for bit."""
    from gpu_util import run_layer
    N, C, H, W, R = 2, 5, 17, 21, 5 if r0 > 2 else 3
    rs = np.random.default_rng(3)
    x = rs.uniform(-1, 1, (N, C, H, W)).astype(np.float32)
    w = np.zeros((C, C, R, R), np.float32)
    for c in range(C):
        w[c, c, r0, s0] = 1.0
    b = np.zeros(C, np.float32)
    P, Q = oracle.out_shape(x.shape, w.shape, stride, pad)[2:]
    dy = rs.uniform(-1, 1, (N, C, P, Q)).astype(np.float32)
    if dtype == "bf16":
        x, dy = gen.quantize_bf16(x), gen.quantize_bf16(dy)
    y, dx, dw, db = run_layer(x, w, b, dy, stride, pad, dtype)
    ey = np.zeros((N, C, P, Q), np.float32)
    edx = np.zeros_like(x)
    for p in range(P):
        for q in range(Q):
            h, ww = p * stride - pad + r0, q * stride - pad + s0
            if 0 <= h < H and 0 <= ww < W:
                ey[:, :, p, q] = x[:, :, h, ww]
                edx[:, :, h, ww] = dy[:, :, p, q]
    assert np.array_equal(y, ey)
    assert np.array_equal(dx, edx)
    assert np.array_equal(y.astype(np.float64), oracle.conv_fwd(x, w, stride, pad))


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("case", [CASES[5], PW[1], PW[-2]], ids=lambda c: c[0])
def test_beta_one_accumulates(case, dtype):
    from gpu_util import run_layer, rel_l2, TOL
    x, w, b, dy, stride, pad = make(case, dtype)
    rs = np.random.default_rng(9)
    prev = [rs.uniform(-1, 1, s).astype(np.float32) for s in (x.shape, w.shape, b.shape)]
    if dtype == "bf16":
        prev[0] = gen.quantize_bf16(prev[0])
    _, dx, dw, db = run_layer(x, w, b, dy, stride, pad, dtype, beta=1.0, prev=prev)
    _, rdx, rdw, rdb = oracle_layer(x, w, b, dy, stride, pad)
    assert rel_l2(dx, rdx + prev[0]) <= TOL[dtype]
    assert rel_l2(dw, rdw + prev[1]) <= TOL[dtype]
    assert rel_l2(db, rdb + prev[2]) <= TOL[dtype]


@pytest.mark.parametrize("shape", [(32, 2), (64, 2), (96, 2), (32, 4), (64, 4), (64, 1), (96, 1), (-1, 0)])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_pointwise_kernel_shapes_agree(shape, dtype):
    """Every (rows per workgroup, pixels per lane) variant of the streaming 1x1 kernel, and the
    general kernel on the same layer, against the oracle. HW = 60 is a multiple of 4."""
    import paper_1412_6249_amd as pa
    from gpu_util import run_layer, rel_l2, TOL
    x, w, b, dy, stride, pad = make(PW[1], dtype)
    ref = oracle_layer(x, w, b, dy, stride, pad)
    pa.purine_debug_force_tile(*shape)
    try:
        got = run_layer(x, w, b, dy, stride, pad, dtype)
    finally:
        pa.purine_debug_force_tile(0, 0)
    for name, g, r in zip(("y", "dx"), got, ref):
        assert rel_l2(g, r) <= TOL[dtype], (shape, name, rel_l2(g, r))


@pytest.mark.parametrize("C", [36, 100, 66, 3])
def test_pointwise_backward_with_rows_past_the_last_channel(C):
    """1x1 backward-data on the streaming kernel where the last 32-row tile is mostly empty (C % 32 in
    1..4): plain, accumulating and through the ReLU mask. dx and the mask are the LAST bytes of their
    buffers (anything the epilogue touched past the last channel would lie outside them) and the
    words in front of them must come back untouched."""
    import torch
    import paper_1412_6249_amd as pa
    from gpu_util import rel_l2, workspace, DEV
    N, K, H, W = 2, 32, 6, 6
    rs = np.random.default_rng(C)
    u = lambda *s: rs.uniform(-1, 1, size=s).astype(np.float32)
    w, dy, act, prev = u(K, C, 1, 1), u(N, K, H, W), u(N, C, H, W), u(N, C, H, W)
    desc = pa.conv_desc(1, 0)
    guard, n = 64, N * C * H * W

    def at_the_end(values):
        buf = torch.full((guard + n,), 777.0, dtype=torch.float32, device=DEV)
        t = buf[guard:].view(N, C, H, W)
        t.copy_(torch.from_numpy(values).to(DEV))
        return buf, t

    tw, tdy = torch.from_numpy(w).to(DEV), torch.from_numpy(dy).to(DEV)
    ws = workspace(pa.purine_conv_workspace_bytes(pa.PURINE_CONV_BWD_DATA, desc, act.shape, w.shape, pa.PURINE_F32))
    ref = oracle.conv_bwd_data(dy, w, act.shape, 1, 0)
    mb, tmask = at_the_end(act)
    for beta, masked in ((0.0, False), (1.0, False), (0.0, True), (1.0, True)):
        db_, tdx = at_the_end(prev)
        if masked:
            pa.purine_conv_bwd_data_relu(desc, tdy, tw, tmask, tdx, beta=beta, ws=ws)
        else:
            pa.purine_conv_bwd_data(desc, tdy, tw, tdx, beta=beta, ws=ws)
        torch.cuda.synchronize()
        want = (np.where(act > 0, ref, 0.0) if masked else ref) + (prev if beta else 0.0)
        assert rel_l2(tdx.cpu().numpy(), want) <= 1e-5, (beta, masked)
        assert bool((db_[:guard] == 777.0).all()) and bool((mb[:guard] == 777.0).all())


@pytest.mark.parametrize("case", [c for c in CASES if c[0].startswith("patch_")], ids=lambda c: c[0])
def test_patch_kernel_with_fill_and_multiply_wavefronts(case):
    """The bf16 patch kernel whose workgroups split into wavefronts that fill LDS and wavefronts that
    multiply (persistent over tiles; picked by itself only for layers of a thousand tiles or more) on
    the small patch shapes: against the oracle, and bit for bit against the one-role kernel (same
    MFMAs in the same order). Forward with bias, backward-data plain, accumulating and masked."""
    import torch
    import paper_1412_6249_amd as pa
    from gpu_util import rel_l2, to_dev, to_host, workspace, TOL, DEV
    x, w, b, dy, stride, pad = make(case, "bf16")
    act = gen.quantize_bf16(np.random.default_rng(3).uniform(-1, 1, x.shape).astype(np.float32))
    desc = pa.conv_desc(stride, pad)
    q = lambda which: workspace(pa.purine_conv_workspace_bytes(which, desc, x.shape, w.shape, pa.PURINE_BF16))
    tx, tw, tb, tdy, tact = (to_dev(a, "bf16") for a in (x, w, b, dy, act))

    def run():
        y = torch.full(dy.shape, float("nan"), dtype=torch.bfloat16, device=DEV)
        dx, dxm = (torch.full(x.shape, float("nan"), dtype=torch.bfloat16, device=DEV) for _ in range(2))
        dxa = to_dev(act, "bf16")
        pa.purine_conv_fwd_bias_relu(desc, tx, tw, tb, y, relu=True, ws=q(pa.PURINE_CONV_FWD))
        pa.purine_conv_bwd_data(desc, tdy, tw, dx, ws=q(pa.PURINE_CONV_BWD_DATA))
        pa.purine_conv_bwd_data(desc, tdy, tw, dxa, beta=1.0, ws=q(pa.PURINE_CONV_BWD_DATA))
        pa.purine_conv_bwd_data_relu(desc, tdy, tw, tact, dxm, ws=q(pa.PURINE_CONV_BWD_DATA))
        torch.cuda.synchronize()
        return [to_host(t) for t in (y, dx, dxa, dxm)]

    base = run()
    pa.purine_debug_force_tile(-5, 0)
    try:
        got = run()
    finally:
        pa.purine_debug_force_tile(0, 0)
    ref_dx = oracle.conv_bwd_data(dy, w, x.shape, stride, pad)
    refs = (np.maximum(oracle.bias_fwd(oracle.conv_fwd(x, w, stride, pad), b), 0), ref_dx, ref_dx + act,
            np.where(act > 0, ref_dx, 0.0))
    for name, g, b0, r in zip(("y", "dx", "dx accumulated", "dx masked"), got, base, refs):
        assert np.isfinite(g).all() and rel_l2(g, r) <= TOL["bf16"], (name, rel_l2(g, r))
        assert np.array_equal(g, b0), name


def test_results_are_bit_identical_run_to_run():
    from gpu_util import run_layer
    x, w, b, dy, stride, pad = make(CASES[3], "f32")
    a = run_layer(x, w, b, dy, stride, pad)
    c = run_layer(x, w, b, dy, stride, pad)
    for u, v in zip(a, c):
        assert np.array_equal(u, v)


def test_batch_shards_add_up():
    """Data-parallel invariant (paper section 3.4): y and dx of a batch are the concatenation of
    the shards' results, dw and db are the sums over shards."""
    from gpu_util import run_layer, rel_l2
    x, w, b, dy, stride, pad = make(CASES[9], "f32")
    y, dx, dw, db = run_layer(x, w, b, dy, stride, pad)
    parts = [slice(0, 2), slice(2, 5)]
    sdw, sdb = np.zeros_like(dw, dtype=np.float64), np.zeros_like(db, dtype=np.float64)
    for s in parts:
        ys, dxs, dws, dbs = run_layer(x[s], w, b, dy[s], stride, pad)
        assert np.array_equal(ys, y[s]) and np.array_equal(dxs, dx[s])
        sdw += dws
        sdb += dbs
    assert rel_l2(dw, sdw) <= 1e-5 and rel_l2(db, sdb) <= 1e-5


def _random_cases(n, seed):
    """Seeded random layer shapes: every kernel family and ragged edge gets hit without anyone
    choosing the shapes (channel counts on both sides of the 16 / 64 thresholds, 1x1 layers with
    and without the streaming kernel's alignment, strides up to 4, pads up to the filter size)."""
    rs = np.random.default_rng(seed)
    out = []
    while len(out) < n:
        C = int(rs.choice([1, 2, 3, 5, 8, 15, 16, 17, 32, 48, 63, 64, 70, 96]))
        K = int(rs.choice([1, 3, 8, 16, 31, 32, 33, 48, 64, 96, 100, 130]))
        R, S = (1, 1) if rs.random() < 0.3 else (int(rs.integers(1, 8)), int(rs.integers(1, 8)))
        sh, sw = int(rs.integers(1, 5)), int(rs.integers(1, 5))
        if R == 1 and S == 1 and rs.random() < 0.7:
            sh = sw = 1
        ph, pw = int(rs.integers(0, R)), int(rs.integers(0, S))
        H, W = int(rs.integers(max(1, R - 2 * ph), 26)), int(rs.integers(max(1, S - 2 * pw), 26))
        N = int(rs.integers(1, 5))
        if H + 2 * ph < R or W + 2 * pw < S:
            continue
        if N * C * H * W > 60000 or C * R * S * K > 120000:
            continue
        out.append(("rnd%d_%d_n%d_c%d_%dx%d_k%d_%dx%d_s%d%d_p%d%d" % (seed % 97, len(out), N, C, H, W, K, R, S, sh, sw, ph, pw),
                    N, C, H, W, K, R, S, (sh, sw), (ph, pw)))
    return out


RANDOM_CASES = _random_cases(48, 1412_6249) + _random_cases(48, 6249_1412)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("case", RANDOM_CASES, ids=[c[0] for c in RANDOM_CASES])
def test_random_shapes(case, dtype):
    from gpu_util import run_layer, rel_l2, TOL
    x, w, b, dy, stride, pad = make(case, dtype)
    got = run_layer(x, w, b, dy, stride, pad, dtype, fused_wb=(zlib.crc32(case[0].encode()) & 1) == 1)
    ref = oracle_layer(x, w, b, dy, stride, pad)
    for name, g, r in zip(("y", "dx", "dw", "db"), got, ref):
        assert g.shape == r.shape and np.isfinite(g).all(), name
        assert rel_l2(g, r) <= TOL[dtype], (case[0], name, rel_l2(g, r))
