"""The memory-bound operators of the layer graphs (max pooling and its gradient, ReLU, bias, concat,
fan-in sum) through the C ABI against the oracle, on small planes, planes larger than a workgroup's
chunk, ragged plane counts, every templated window shape and the generic one. Pool winners and the
ReLU / concat outputs are index or copy work: bit for bit."""
import numpy as np
import pytest
import torch

import oracle
from synth import gen

pytestmark = pytest.mark.gpu

# name, N, C, H, W, window, stride, pad
POOLS = [
    ("k3s1p1_28", 3, 5, 28, 28, 3, 1, 1),          # inception pool branch
    ("k3s2_55", 2, 3, 55, 55, 3, 2, 0),            # overlapping AlexNet pooling
    ("k3s2_13", 4, 7, 13, 13, 3, 2, 0),
    ("k2s2_even", 2, 6, 12, 16, 2, 2, 0),
    ("k2s2_odd", 1, 3, 9, 7, 2, 2, 0),
    ("k3s1p1_tiny", 5, 3, 3, 3, 3, 1, 1),          # many planes per workgroup
    ("k3s2p1_rect", 2, 2, 17, 33, 3, 2, 1),
    ("k5s3p2_generic", 2, 3, 20, 23, 5, 3, 2),     # runtime window / stride path
    ("k4s1p2_generic", 1, 2, 11, 10, 4, 1, 2),
    ("k3s1p1_big_plane", 1, 2, 70, 90, 3, 1, 1),   # one plane spans several chunks
    ("k3s2_big_plane", 1, 3, 101, 97, 3, 2, 0),
    ("k1s1_identity", 2, 2, 6, 5, 1, 1, 0),
    # 3x3 / stride 1 / pad 1 with rows of whole 16-byte packets: the packet kernels (fp32)
    ("k3s1p1_w8", 3, 5, 5, 8, 3, 1, 1),
    ("k3s1p1_w4_h1", 2, 3, 1, 4, 3, 1, 1),
    ("k3s1p1_w4_h2", 1, 1, 2, 4, 3, 1, 1),
    ("k3s1p1_56x12", 2, 3, 56, 12, 3, 1, 1),
]


def _random_pools(n, seed):
    rs = np.random.default_rng(seed)
    out = []
    while len(out) < n:
        k = int(rs.integers(1, 6))
        s = int(rs.integers(1, 5))
        p = int(rs.integers(0, k))
        H, W = int(rs.integers(1, 40)), int(rs.integers(1, 40))
        if H + 2 * p < k or W + 2 * p < k:
            continue
        N, C = int(rs.integers(1, 4)), int(rs.integers(1, 9))
        out.append(("rnd%d_k%ds%dp%d_%dx%dx%dx%d" % (len(out), k, s, p, N, C, H, W), N, C, H, W, k, s, p))
    return out


POOLS += _random_pools(24, 1412)


def pool_inputs(case, dtype, ties):
    name, N, C, H, W, k, s, p = case
    rs = np.random.default_rng([N, C, H, W, k, s, p])
    if ties:
        x = rs.integers(-2, 3, size=(N, C, H, W)).astype(np.float32)     # many equal maxima
    else:
        x = rs.uniform(-1, 1, size=(N, C, H, W)).astype(np.float32)
    if dtype == "bf16":
        x = gen.quantize_bf16(x)
    P = (H + 2 * p - k) // s + 1
    Q = (W + 2 * p - k) // s + 1
    dy = rs.uniform(-1, 1, size=(N, C, P, Q)).astype(np.float32)
    if dtype == "bf16":
        dy = gen.quantize_bf16(dy)
    return x, dy


@pytest.mark.parametrize("ties", [False, True], ids=["distinct", "ties"])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("case", POOLS, ids=[c[0] for c in POOLS])
def test_maxpool_forward_and_backward(case, dtype, ties):
    import paper_1412_6249_amd as pa
    from gpu_util import to_dev, to_host, tdtype, rel_l2, pool_bwd_in_order, DEV
    name, N, C, H, W, k, s, p = case
    x, dy = pool_inputs(case, dtype, ties)
    ey, earg = oracle.maxpool_fwd(x, k, s, p)
    desc = pa.pool_desc(k, s, p)
    tx, tdy = to_dev(x, dtype), to_dev(dy, dtype)
    ty = torch.full(ey.shape, float("nan"), dtype=tdtype(dtype), device=DEV)
    targ = torch.full(ey.shape, -7, dtype=torch.int32, device=DEV)
    pa.purine_maxpool_fwd(desc, tx, ty, targ)
    torch.cuda.synchronize()
    assert np.array_equal(to_host(ty), ey.astype(np.float32))
    assert np.array_equal(targ.cpu().numpy(), earg)

    edx = oracle.maxpool_bwd(dy, earg, x.shape)
    tdx = torch.full(x.shape, float("nan"), dtype=tdtype(dtype), device=DEV)
    pa.purine_maxpool_bwd(desc, tdy, targ, tdx)
    torch.cuda.synchronize()
    tol = 1e-2 if dtype == "bf16" else 1e-6
    assert rel_l2(to_host(tdx), edx) <= tol
    # positions no window chose get exactly zero
    assert np.all(to_host(tdx)[edx == 0] == 0)
    # and bit for bit the fp32 sum over the windows in (p, q) order
    assert np.array_equal(to_host(tdx), pool_bwd_in_order(dy, earg, x.shape, dtype))

    # accumulate into an existing gradient
    prev = np.random.default_rng(5).uniform(-1, 1, size=x.shape).astype(np.float32)
    if dtype == "bf16":
        prev = gen.quantize_bf16(prev)
    tdx2 = to_dev(prev, dtype)
    pa.purine_maxpool_bwd(desc, tdy, targ, tdx2, beta=1.0)
    torch.cuda.synchronize()
    assert rel_l2(to_host(tdx2), edx + prev) <= tol
    assert np.array_equal(to_host(tdx2), pool_bwd_in_order(dy, earg, x.shape, dtype, prev=prev))


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("case", POOLS, ids=[c[0] for c in POOLS])
def test_maxpool_backward_with_relu_mask(case, dtype):
    """MaxPoolBwd and the ReLU gradient of the pooled tensor as one operator, the mask read off the
    pooling output y (a position that won a window holds that window's y). With the forward pass's
    own y of a ReLU output: the oracle's two functions composed, and where the pooled tensor is
    positive the bits of purine_maxpool_bwd, elsewhere no pooling gradient; also accumulating.
    With a y unrelated to the winners (about half of the windows masked): the pooling gradient of
    dy with those windows' entries dropped, which is what the operator is defined to compute."""
    import paper_1412_6249_amd as pa
    from gpu_util import to_dev, to_host, tdtype, rel_l2, pool_bwd_in_order, DEV
    name, N, C, H, W, k, s, p = case
    x, dy = pool_inputs(case, dtype, False)
    act = np.maximum(x, 0.0)                                   # a ReLU output: zeros and positives
    ey, earg = oracle.maxpool_fwd(act, k, s, p)
    desc = pa.pool_desc(k, s, p)
    tdy = to_dev(dy, dtype)
    targ = torch.from_numpy(earg.astype(np.int32)).to(DEV)
    rs = np.random.default_rng(11)
    other = rs.uniform(-1, 1, size=dy.shape).astype(np.float32)  # a "y" unrelated to the winners
    prev = rs.uniform(-1, 1, size=x.shape).astype(np.float32)
    if dtype == "bf16":
        other, prev = gen.quantize_bf16(other), gen.quantize_bf16(prev)
    for y in (np.asarray(ey, dtype=np.float32), other):
        tdx = torch.full(x.shape, float("nan"), dtype=tdtype(dtype), device=DEV)
        pa.purine_maxpool_bwd_relu(desc, tdy, targ, to_dev(y, dtype), tdx)
        tdx2 = to_dev(prev, dtype)
        pa.purine_maxpool_bwd_relu(desc, tdy, targ, to_dev(y, dtype), tdx2, beta=1.0)
        torch.cuda.synchronize()
        kept = np.where(y > 0, dy, np.float32(0))               # windows whose winner was positive
        ref = oracle.maxpool_bwd(kept, earg, x.shape)
        assert rel_l2(to_host(tdx), ref) <= (1e-2 if dtype == "bf16" else 1e-6)
        assert np.array_equal(to_host(tdx), pool_bwd_in_order(kept, earg, x.shape, dtype))
        assert np.array_equal(to_host(tdx2), pool_bwd_in_order(kept, earg, x.shape, dtype, prev=prev))
        if y is not other:
            # the forward pass's own y: MaxPoolBwd followed by ReLUBwd on the pooled tensor
            composed = oracle.relu_bwd(act, oracle.maxpool_bwd(dy, earg, x.shape))
            assert rel_l2(to_host(tdx), composed) <= (1e-2 if dtype == "bf16" else 1e-6)
            exact = pool_bwd_in_order(dy, earg, x.shape, dtype)
            assert np.array_equal(to_host(tdx), np.where(act > 0, exact, np.float32(0)))
            exact2 = pool_bwd_in_order(dy, earg, x.shape, dtype, prev=prev)
            assert np.array_equal(to_host(tdx2), np.where(act > 0, exact2, prev))


def test_maxpool_backward_is_deterministic():
    import paper_1412_6249_amd as pa
    from gpu_util import to_dev, DEV
    case = POOLS[0]
    x, dy = pool_inputs(case, "f32", True)
    desc = pa.pool_desc(*case[5:])
    tx, tdy = to_dev(x), to_dev(dy)
    P, Q = dy.shape[2:]
    ty = torch.empty(dy.shape, device=DEV)
    targ = torch.empty(dy.shape, dtype=torch.int32, device=DEV)
    pa.purine_maxpool_fwd(desc, tx, ty, targ)
    outs = []
    for _ in range(3):
        tdx = torch.empty(x.shape, device=DEV)
        pa.purine_maxpool_bwd(desc, tdy, targ, tdx)
        torch.cuda.synchronize()
        outs.append(tdx.clone())
    assert torch.equal(outs[0], outs[1]) and torch.equal(outs[0], outs[2])


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("shape", [(2, 3, 5, 7), (1, 1, 1, 1), (3, 8, 16, 16), (2, 5, 33, 31)])
def test_relu_bias_and_sum(shape, dtype):
    import paper_1412_6249_amd as pa
    from gpu_util import to_dev, to_host, tdtype, rel_l2, DEV, workspace, pcode
    rs = np.random.default_rng(sum(shape))
    q = (lambda a: gen.quantize_bf16(a)) if dtype == "bf16" else (lambda a: a)
    x = q(rs.uniform(-1, 1, size=shape).astype(np.float32))
    dy = q(rs.uniform(-1, 1, size=shape).astype(np.float32))
    b = q(rs.uniform(-1, 1, size=shape[1]).astype(np.float32))
    tx, tdy, tb = to_dev(x, dtype), to_dev(dy, dtype), to_dev(b, dtype)
    ty = torch.empty(shape, dtype=tdtype(dtype), device=DEV)
    pa.purine_relu_fwd(tx, ty)
    tdx = torch.empty(shape, dtype=tdtype(dtype), device=DEV)
    pa.purine_relu_bwd(ty, tdy, tdx)
    torch.cuda.synchronize()
    assert np.array_equal(to_host(ty), oracle.relu_fwd(x).astype(np.float32))
    assert np.array_equal(to_host(tdx), oracle.relu_bwd(oracle.relu_fwd(x), dy).astype(np.float32))

    tyb = to_dev(x, dtype)
    pa.purine_bias_fwd(tb, tyb)
    tdb = torch.empty(shape[1], dtype=torch.float32, device=DEV)
    ws = workspace(pa.purine_bias_bwd_workspace_bytes(shape, pcode(dtype)))
    pa.purine_bias_bwd(tdy, tdb, ws=ws)
    torch.cuda.synchronize()
    tol = 1e-2 if dtype == "bf16" else 1e-6
    assert rel_l2(to_host(tyb), oracle.bias_fwd(x, b)) <= tol
    assert rel_l2(to_host(tdb), oracle.bias_bwd(dy)) <= 1e-5

    terms = [q(rs.uniform(-1, 1, size=shape).astype(np.float32)) for _ in range(4)]
    tout = torch.empty(shape, dtype=tdtype(dtype), device=DEV)
    pa.purine_sum([to_dev(t, dtype) for t in terms], tout)
    torch.cuda.synchronize()
    assert rel_l2(to_host(tout), oracle.fan_in_sum(terms)) <= tol


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_concat_and_split_are_copies(dtype):
    import paper_1412_6249_amd as pa
    from gpu_util import to_dev, to_host, tdtype, DEV
    rs = np.random.default_rng(11)
    q = (lambda a: gen.quantize_bf16(a)) if dtype == "bf16" else (lambda a: a)
    parts = [q(rs.uniform(-1, 1, size=(3, c, 7, 9)).astype(np.float32)) for c in (4, 1, 6, 3)]
    tparts = [to_dev(t, dtype) for t in parts]
    tcat = torch.empty((3, 14, 7, 9), dtype=tdtype(dtype), device=DEV)
    pa.purine_concat_fwd(tparts, tcat)
    torch.cuda.synchronize()
    assert np.array_equal(to_host(tcat), oracle.concat_channels(parts).astype(np.float32))
    back = [torch.empty_like(t) for t in tparts]
    pa.purine_concat_bwd(tcat, back)
    torch.cuda.synchronize()
    for t, r in zip(back, parts):
        assert np.array_equal(to_host(t), r)
