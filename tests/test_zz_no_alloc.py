"""The entry point that allocates nothing (purine_conv_bwd_weight_static: the split-reduction
partial sums go to a fixed array inside the library's device image) against the workspace form of
the same operator, through the C ABI: bit-identical dw on two calls in a row, the second with a
smaller layer (the array keeps the first call's contents), plus an accumulating call and a bf16
layer; and against the oracle within the operator's tolerance."""
import numpy as np
import pytest

import oracle

pytestmark = pytest.mark.gpu

# name, N, C, H, W, K, R, S, stride, pad
FIRST = ("larger", 4, 70, 24, 24, 70, 3, 3, 1, 1)
SECOND = ("smaller", 2, 5, 19, 23, 37, 3, 2, 2, 1)


def _run(case, dtype, beta=0.0):
    import torch
    import paper_1412_6249_amd as pa
    from gpu_util import to_dev, workspace, pcode, rel_l2, TOL
    from synth import gen
    name, N, C, H, W, K, R, S, stride, pad = case
    rs = np.random.default_rng(len(name) + N)
    P, Q = oracle.out_shape((N, C, H, W), (K, C, R, S), stride, pad)[2:]
    x = rs.uniform(-1, 1, (N, C, H, W)).astype(np.float32)
    dy = rs.uniform(-1, 1, (N, K, P, Q)).astype(np.float32)
    prev = rs.uniform(-1, 1, (K, C, R, S)).astype(np.float32)
    if dtype == "bf16":
        x, dy = gen.quantize_bf16(x), gen.quantize_bf16(dy)
    desc = pa.conv_desc(stride, pad)
    tx, tdy = to_dev(x, dtype), to_dev(dy, dtype)
    need = pa.purine_conv_workspace_bytes(pa.PURINE_CONV_BWD_WEIGHT, desc, x.shape, prev.shape, pcode(dtype))
    assert 0 < need <= pa.purine_static_scratch_bytes()
    want = to_dev(prev)
    pa.purine_conv_bwd_weight(desc, tx, tdy, want, beta=beta, ws=workspace(need))
    got = to_dev(prev)
    pa.purine_conv_bwd_weight_static(desc, tx, tdy, got, beta=beta)
    torch.cuda.synchronize()
    assert torch.equal(got, want), (name, dtype, beta)
    ref = oracle.conv_bwd_weight(x, dy, prev.shape, stride, pad) + (prev if beta else 0.0)
    assert rel_l2(got.cpu().numpy(), ref) <= TOL[dtype], (name, dtype, beta)


def test_static_scratch_weight_gradient_two_calls_in_a_row():
    _run(FIRST, "f32")
    _run(SECOND, "f32")          # smaller layer: most of the array still holds the first call's partials
    _run(SECOND, "f32", beta=1.0)
    _run(FIRST, "bf16")
    _run(SECOND, "bf16")
