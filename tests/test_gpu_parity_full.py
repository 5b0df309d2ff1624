"""GPU parity at the FULL workload shapes (configs 2-5, every conv layer), in the launch
configuration bench.py times, on outputs the oracle can compute one by one:
  - forward (+bias) and backward-data: every image of configs 2 and 3; for configs 4 and 5 whole
    images sampled by seed (these passes are independent per image, so an image of the batch is an
    exact sub-problem);
  - backward-weight: EVERY element of dw, summed by the oracle over the whole batch;
  - bias gradient: all of it.
The fused operators bench.py's graphs use (Conv+Bias+ReLU, ConvBwdData through a ReLU mask,
ConvBwdWeight+BiasBwd) are
checked on the same samples. A second test feeds small-integer tensors at full shape, where every
partial sum is an exact integer below 2^24, so the outputs (sampled images, all of dw and db) must
match bit for bit whatever the summation order (index and shape bookkeeping at the real sizes).
Tolerance: relative L2 <= 1e-5 (fp32), <= 1e-2 (bf16 in, fp32 accumulate), over each sample."""
import sys

import numpy as np
import pytest

import oracle
from synth.configs import CONV_LAYERS

pytestmark = pytest.mark.gpu

CASES = [(cfg, i) for cfg in (2, 3, 4, 5) for i in range(len(CONV_LAYERS[cfg]))]


@pytest.mark.parametrize("cfg,idx", CASES, ids=["cfg%d_%s" % (c, CONV_LAYERS[c][i].name) for c, i in CASES])
def test_full_shape_layer(cfg, idx):
    import torch
    import paper_1412_6249_amd as pa
    from gpu_util import rel_l2, TOL, to_host, pcode, tdtype, workspace, DEV

    L = CONV_LAYERS[cfg][idx]
    print("full-shape parity", cfg, L, file=sys.stderr, flush=True)
    td = tdtype(L.dtype)
    g = torch.Generator(device="cuda")
    g.manual_seed(14126249 * 1000 + 100 * cfg + idx)
    x = torch.rand(L.x_shape, generator=g, device=DEV).to(td)
    w = (torch.randn(L.w_shape, generator=g, device=DEV) * 0.01).to(td)
    b = (torch.randn((L.K,), generator=g, device=DEV) * 0.01).to(td)
    dy = (torch.rand(L.y_shape, generator=g, device=DEV) * 2 - 1).to(td)
    y = torch.empty(L.y_shape, dtype=td, device=DEV)
    dx = torch.empty(L.x_shape, dtype=td, device=DEV)
    dw = torch.empty(L.w_shape, dtype=torch.float32, device=DEV)
    db = torch.empty((L.K,), dtype=torch.float32, device=DEV)
    desc = pa.conv_desc(L.stride, L.pad)
    code = pcode(L.dtype)
    q = lambda which: workspace(pa.purine_conv_workspace_bytes(which, desc, L.x_shape, L.w_shape, code))
    pa.purine_conv_fwd(desc, x, w, y, ws=q(pa.PURINE_CONV_FWD))
    pa.purine_bias_fwd(b, y)
    pa.purine_conv_bwd_data(desc, dy, w, dx, ws=q(pa.PURINE_CONV_BWD_DATA))
    pa.purine_conv_bwd_weight(desc, x, dy, dw, ws=q(pa.PURINE_CONV_BWD_WEIGHT))
    pa.purine_bias_bwd(dy, db, ws=workspace(pa.purine_bias_bwd_workspace_bytes(L.y_shape, code)))
    torch.cuda.synchronize()

    tol = TOL[L.dtype]
    rs = np.random.default_rng(1000 * cfg + idx)
    imgs = list(range(L.N)) if cfg in (2, 3) else sorted(rs.choice(L.N - 1, size=2, replace=False).tolist() + [L.N - 1])
    hw, hb = to_host(w), to_host(b)
    hx_s, hdy_s = to_host(x[imgs]), to_host(dy[imgs])
    ref_y = oracle.bias_fwd(oracle.conv_fwd(hx_s, hw, L.stride, L.pad), hb)
    assert rel_l2(to_host(y[imgs]), ref_y) <= tol, ("fwd", rel_l2(to_host(y[imgs]), ref_y))
    ref_dx = oracle.conv_bwd_data(hdy_s, hw, hx_s.shape, L.stride, L.pad)
    assert rel_l2(to_host(dx[imgs]), ref_dx) <= tol, ("bwd_data", rel_l2(to_host(dx[imgs]), ref_dx))

    # fused vertices of the benchmark graphs, on the same samples
    y2 = torch.empty_like(y)
    pa.purine_conv_fwd_bias_relu(desc, x, w, b, y2, relu=True, ws=q(pa.PURINE_CONV_FWD))
    act = (torch.rand(L.x_shape, generator=g, device=DEV) - 0.5).to(td)     # stands for the ReLU output below
    dx2 = torch.empty_like(dx)
    pa.purine_conv_bwd_data_relu(desc, dy, w, act, dx2, ws=q(pa.PURINE_CONV_BWD_DATA))
    torch.cuda.synchronize()
    assert rel_l2(to_host(y2[imgs]), np.maximum(ref_y, 0.0)) <= tol, "fused fwd"
    mask = to_host(act[imgs]) > 0
    got_dx2 = to_host(dx2[imgs])
    assert rel_l2(got_dx2, np.where(mask, ref_dx, 0.0)) <= tol, "fused bwd_data"
    assert np.all(got_dx2[~mask] == 0)
    del hx_s, hdy_s, y2, dx2, act
    hx, hdy = to_host(x), to_host(dy)
    ref_dw = oracle.conv_bwd_weight(hx, hdy, L.w_shape, L.stride, L.pad)
    got_dw = dw.cpu().numpy()
    assert rel_l2(got_dw, ref_dw) <= tol, ("bwd_weight", rel_l2(got_dw, ref_dw))
    # no single filter (one k: a row of the weight-gradient GEMM) may hide behind the others
    per_k = [rel_l2(got_dw[k], ref_dw[k]) for k in range(L.K)]
    assert max(per_k) <= 4 * tol, ("bwd_weight, worst filter", int(np.argmax(per_k)), max(per_k))
    ref_db = oracle.bias_bwd(hdy)
    assert rel_l2(db.cpu().numpy(), ref_db) <= tol, ("bias_bwd", rel_l2(db.cpu().numpy(), ref_db))
    # the two parameter gradients from the single fused operator
    dw2, db2 = torch.empty_like(dw), torch.empty_like(db)
    pa.purine_conv_bwd_weight_bias(desc, x, dy, dw2, db2, ws=q(pa.PURINE_CONV_BWD_WEIGHT_BIAS))
    torch.cuda.synchronize()
    assert torch.equal(dw2, dw), "fused bwd_weight"
    assert rel_l2(db2.cpu().numpy(), ref_db) <= tol, ("fused bias_bwd", rel_l2(db2.cpu().numpy(), ref_db))


INT_CASES = [(2, 0), (2, 1), (3, 4), (4, 2), (5, 0), (5, 2)]


@pytest.mark.parametrize("cfg,idx", INT_CASES, ids=["cfg%d_%s" % (c, CONV_LAYERS[c][i].name) for c, i in INT_CASES])
def test_full_shape_integer_inputs_bit_exact(cfg, idx):
    """One layer per kernel family (flattened forward + phase-folded backward, 1x1 streaming,
    small-channel 5x5, tap-major 3x3 with per-tap weight gradient, bf16 flattened, bf16 tap-major)
    at full shape with values in {-2..2}: sampled images of y and dx, every element of dw and all
    of db must equal the oracle exactly (bf16-stored outputs after the same RNE rounding)."""
    import torch
    import paper_1412_6249_amd as pa
    from gpu_util import to_host, pcode, tdtype, workspace, DEV
    from synth import gen

    L = CONV_LAYERS[cfg][idx]
    print("full-shape integer parity", cfg, L, file=sys.stderr, flush=True)
    td = tdtype(L.dtype)
    g = torch.Generator(device="cuda")
    g.manual_seed(77 + 100 * cfg + idx)
    ri = lambda shape: torch.randint(-2, 3, shape, generator=g, device=DEV).to(td)
    x, w, b, dy = ri(L.x_shape), ri(L.w_shape), ri((L.K,)), ri(L.y_shape)
    y = torch.empty(L.y_shape, dtype=td, device=DEV)
    dx = torch.empty(L.x_shape, dtype=td, device=DEV)
    dw = torch.empty(L.w_shape, dtype=torch.float32, device=DEV)
    db = torch.empty((L.K,), dtype=torch.float32, device=DEV)
    desc = pa.conv_desc(L.stride, L.pad)
    code = pcode(L.dtype)
    q = lambda which: workspace(pa.purine_conv_workspace_bytes(which, desc, L.x_shape, L.w_shape, code))
    pa.purine_conv_fwd_bias_relu(desc, x, w, b, y, relu=False, ws=q(pa.PURINE_CONV_FWD))
    pa.purine_conv_bwd_data(desc, dy, w, dx, ws=q(pa.PURINE_CONV_BWD_DATA))
    pa.purine_conv_bwd_weight(desc, x, dy, dw, ws=q(pa.PURINE_CONV_BWD_WEIGHT))
    pa.purine_bias_bwd(dy, db, ws=workspace(pa.purine_bias_bwd_workspace_bytes(L.y_shape, code)))
    torch.cuda.synchronize()

    stored = (lambda a: gen.quantize_bf16(a.astype(np.float32))) if L.dtype == "bf16" else (lambda a: a.astype(np.float32))
    rs = np.random.default_rng(2000 * cfg + idx)
    imgs = sorted(rs.choice(L.N - 1, size=1, replace=False).tolist() + [L.N - 1])
    hw, hb = to_host(w), to_host(b)
    hx_s, hdy_s = to_host(x[imgs]), to_host(dy[imgs])
    ref_y = oracle.bias_fwd(oracle.conv_fwd(hx_s, hw, L.stride, L.pad), hb)
    assert np.abs(ref_y).max() < 2 ** 24
    assert np.array_equal(to_host(y[imgs]), stored(ref_y)), "fwd"
    ref_dx = oracle.conv_bwd_data(hdy_s, hw, hx_s.shape, L.stride, L.pad)
    assert np.array_equal(to_host(dx[imgs]), stored(ref_dx)), "bwd_data"
    del hx_s, hdy_s
    hx, hdy = to_host(x), to_host(dy)
    ref_dw = oracle.conv_bwd_weight(hx, hdy, L.w_shape, L.stride, L.pad)
    assert np.abs(ref_dw).max() < 2 ** 24
    assert np.array_equal(dw.cpu().numpy(), ref_dw.astype(np.float32)), "bwd_weight"
    assert np.array_equal(db.cpu().numpy(), oracle.bias_bwd(hdy).astype(np.float32)), "bias_bwd"
    dw2, db2 = torch.empty_like(dw), torch.empty_like(db)
    pa.purine_conv_bwd_weight_bias(desc, x, dy, dw2, db2, ws=q(pa.PURINE_CONV_BWD_WEIGHT_BIAS))
    torch.cuda.synchronize()
    assert torch.equal(dw2, dw) and torch.equal(db2, db), "fused bwd_weight + bias_bwd"
