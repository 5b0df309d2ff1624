"""Helpers for the GPU parity tests: upload seeded host tensors, call the operators through the
C-ABI binding, bring results back as numpy. The only arithmetic here is `pool_bwd_in_order`, the
fp32 restatement of the pooling gradient's summation order that lets it be compared bit for bit."""
import numpy as np
import torch

import paper_1412_6249_amd as pa
from synth import gen

DEV = "cuda:0"
TOL = {"f32": 1e-5, "bf16": 1e-2}     # relative L2 error allowed against the fp64 oracle


def rel_l2(got, ref):
    got = np.asarray(got, dtype=np.float64).ravel()
    ref = np.asarray(ref, dtype=np.float64).ravel()
    n = np.linalg.norm(ref)
    d = np.linalg.norm(got - ref)
    if n == 0.0:
        return 0.0 if np.linalg.norm(got) == 0.0 else np.inf
    return d / n


def to_dev(a, dtype="f32"):
    """numpy fp32 array -> device tensor; bf16 goes through the exact 16-bit patterns."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    if dtype == "bf16":
        bits = gen.to_bf16_bits(a).reshape(a.shape)
        return torch.from_numpy(bits.view(np.int16)).to(DEV).view(torch.bfloat16)
    return torch.from_numpy(a).to(DEV)


def to_host(t):
    """device tensor -> numpy fp32 (bf16 widened exactly)."""
    if t.dtype == torch.bfloat16:
        return t.float().cpu().numpy()
    return t.cpu().numpy()


def pool_bwd_in_order(dy, arg, x_shape, dtype="f32", prev=None):
    """Pooling gradient summed the way the operator is specified to sum it: per input position an
    fp32 accumulator that starts from the previous gradient (accumulating call) or zero and takes
    the windows that chose the position in ascending (p, q) order; a bf16 result is that fp32 sum
    rounded to nearest even once. The fp64 oracle fixes WHERE each gradient lands and the value up
    to rounding; this fixes the rounding, so the GPU result can be compared exactly."""
    N, C, H, W = (int(v) for v in x_shape)
    P, Q = dy.shape[2:]
    dx = np.zeros((N * C, H * W), np.float32) if prev is None else np.array(prev, np.float32).reshape(N * C, H * W)
    g = np.ascontiguousarray(dy, np.float32).reshape(N * C, P, Q)
    a = np.asarray(arg).reshape(N * C, P, Q)
    planes = np.arange(N * C)
    for p in range(P):
        for q in range(Q):
            ok = a[:, p, q] >= 0
            dx[planes[ok], a[ok, p, q]] += g[ok, p, q]      # one target per plane: no repeated index
    dx = dx.reshape(N, C, H, W)
    return gen.quantize_bf16(dx) if dtype == "bf16" else dx


def tdtype(dtype):
    return torch.bfloat16 if dtype == "bf16" else torch.float32


def pcode(dtype):
    return pa.PURINE_BF16 if dtype == "bf16" else pa.PURINE_F32


def workspace(nbytes):
    return torch.empty(max(256, int(nbytes)), dtype=torch.uint8, device=DEV)


def run_layer(x, w, b, dy, stride, pad, dtype="f32", beta=0.0, prev=None, fused_wb=False):
    """One conv layer through the five operators. Inputs are numpy fp32 (bf16-valued if dtype is
    bf16). Returns y (with bias), dx, dw, db as numpy arrays. fused_wb: dw and db come from the
    single ConvBwdWeight+BiasBwd operator instead of the two separate ones."""
    desc = pa.conv_desc(stride, pad)
    tx, tw, tb, tdy = to_dev(x, dtype), to_dev(w, dtype), to_dev(b, dtype), to_dev(dy, dtype)
    ys = pa.purine_conv_out_shape(desc, x.shape, w.shape)
    assert tuple(dy.shape) == ys
    ty = torch.empty(ys, dtype=tdtype(dtype), device=DEV)
    if prev is None:
        tdx = torch.full(x.shape, float("nan"), dtype=tdtype(dtype), device=DEV)
        tdw = torch.full(w.shape, float("nan"), dtype=torch.float32, device=DEV)
        tdb = torch.full(b.shape, float("nan"), dtype=torch.float32, device=DEV)
    else:
        tdx, tdw, tdb = to_dev(prev[0], dtype), to_dev(prev[1]), to_dev(prev[2])
    ws = workspace(pa.purine_conv_workspace_bytes(pa.PURINE_CONV_BWD_WEIGHT, desc, x.shape, w.shape,
                                                  pcode(dtype)))
    ws2 = workspace(pa.purine_bias_bwd_workspace_bytes(dy.shape, pcode(dtype)))
    wsf = workspace(pa.purine_conv_workspace_bytes(pa.PURINE_CONV_FWD, desc, x.shape, w.shape, pcode(dtype)))
    wsd = workspace(pa.purine_conv_workspace_bytes(pa.PURINE_CONV_BWD_DATA, desc, x.shape, w.shape,
                                                   pcode(dtype)))
    pa.purine_conv_fwd(desc, tx, tw, ty, ws=wsf)
    pa.purine_bias_fwd(tb, ty)
    pa.purine_conv_bwd_data(desc, tdy, tw, tdx, beta=beta, ws=wsd)
    if fused_wb:
        wsb = workspace(pa.purine_conv_workspace_bytes(pa.PURINE_CONV_BWD_WEIGHT_BIAS, desc, x.shape, w.shape,
                                                       pcode(dtype)))
        pa.purine_conv_bwd_weight_bias(desc, tx, tdy, tdw, tdb, beta=beta, ws=wsb)
    else:
        pa.purine_conv_bwd_weight(desc, tx, tdy, tdw, beta=beta, ws=ws)
        pa.purine_bias_bwd(tdy, tdb, beta=beta, ws=ws2)
    torch.cuda.synchronize()
    return to_host(ty), to_host(tdx), to_host(tdw), to_host(tdb)
