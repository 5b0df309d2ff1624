"""Per-layer, per-operator timing of the conv-layer operators at the workload shapes.

    python -m paper_1412_6249_amd.layer_bench --config 4 [--layer conv2] [--op fwd] [--iters 20]

Each operator is launched alone on the current stream and bracketed with HIP events through the
library's kernel probe, so the figure is the main kernel's duration (no concurrency, no launch gaps).
Useful on its own and as the command to put after `rocprofv3 ... --` for counters of one kernel.
"""
import argparse
import sys

import torch

from . import binding as B
from synth.configs import CONV_LAYERS

PEAK = {"f32": 157.3, "bf16": 2500.0}
HBM_TBS = 8.0   # TB/s


def time_op(fn, iters, warmup=10):
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    starts = [torch.cuda.Event(enable_timing=True) for _ in range(iters)]
    stops = [torch.cuda.Event(enable_timing=True) for _ in range(iters)]
    for i in range(iters):
        starts[i].record()
        stops[i].record()     # create the underlying hipEvent handles
    torch.cuda.synchronize()
    for i in range(iters):
        B.purine_set_kernel_probe(starts[i].cuda_event, stops[i].cuda_event)
        fn()
    B.purine_set_kernel_probe(None, None)
    torch.cuda.synchronize()
    ms = sorted(s.elapsed_time(e) for s, e in zip(starts, stops))
    return ms[len(ms) // 2], ms[0]


def bench_layer(L, ops, iters, out=sys.stdout):
    td = torch.bfloat16 if L.dtype == "bf16" else torch.float32
    code = B.PURINE_BF16 if L.dtype == "bf16" else B.PURINE_F32
    dev = "cuda:0"
    g = torch.Generator(device="cuda")
    g.manual_seed(1412)
    x = torch.rand(L.x_shape, generator=g, device=dev).to(td)
    w = (torch.randn(L.w_shape, generator=g, device=dev) * 0.01).to(td)
    b = (torch.randn((L.K,), generator=g, device=dev) * 0.01).to(td)
    dy = (torch.rand(L.y_shape, generator=g, device=dev) * 2 - 1).to(td)
    y = torch.empty(L.y_shape, dtype=td, device=dev)
    dx = torch.empty(L.x_shape, dtype=td, device=dev)
    dw = torch.empty(L.w_shape, dtype=torch.float32, device=dev)
    db = torch.empty((L.K,), dtype=torch.float32, device=dev)
    desc = B.conv_desc(L.stride, L.pad)
    ws = torch.empty(max(256, B.purine_conv_workspace_bytes(B.PURINE_CONV_BWD_WEIGHT_BIAS, desc, L.x_shape,
                                                            L.w_shape, code)),
                     dtype=torch.uint8, device=dev)
    ws2 = torch.empty(max(256, B.purine_bias_bwd_workspace_bytes(L.y_shape, code)), dtype=torch.uint8,
                      device=dev)
    wsf = torch.empty(max(256, B.purine_conv_workspace_bytes(B.PURINE_CONV_FWD, desc, L.x_shape, L.w_shape,
                                                             code)), dtype=torch.uint8, device=dev)
    wsd = torch.empty(max(256, B.purine_conv_workspace_bytes(B.PURINE_CONV_BWD_DATA, desc, L.x_shape,
                                                             L.w_shape, code)), dtype=torch.uint8, device=dev)
    table = {
        "fwd": (lambda: B.purine_conv_fwd(desc, x, w, y, ws=wsf), L.flop_per_pass),
        "fwd_fused": (lambda: B.purine_conv_fwd_bias_relu(desc, x, w, b, y, relu=True, ws=wsf), L.flop_per_pass),
        "bwd_data": (lambda: B.purine_conv_bwd_data(desc, dy, w, dx, ws=wsd), L.flop_per_pass),
        "bwd_weight": (lambda: B.purine_conv_bwd_weight(desc, x, dy, dw, ws=ws), L.flop_per_pass),
        "bwd_weight_bias": (lambda: B.purine_conv_bwd_weight_bias(desc, x, dy, dw, db, ws=ws), L.flop_per_pass),
        "bias_fwd": (lambda: B.purine_bias_fwd(b, y), 0),
        "bias_bwd": (lambda: B.purine_bias_bwd(dy, db, ws=ws2), 0),
    }
    results = {}
    for name in ops:
        fn, flop = table[name]
        med, best = time_op(fn, iters)
        tf = flop / (med * 1e-3) / 1e12 if flop else 0.0
        results[name] = (med, tf)
        if flop:
            # algorithmic bytes of the pass: each operand tensor once; attainable = min(MFMA peak,
            # arithmetic intensity x 8 TB/s)
            es = x.element_size()
            nb = {"fwd": (x.numel() + w.numel() + y.numel()) * es, "fwd_fused": (x.numel() + w.numel() + y.numel()) * es,
                  "bwd_data": (dy.numel() + w.numel() + dx.numel()) * es,
                  "bwd_weight": (x.numel() + dy.numel()) * es + dw.numel() * 4,
                  "bwd_weight_bias": (x.numel() + dy.numel()) * es + dw.numel() * 4}[name]
            attainable = min(PEAK[L.dtype], flop / nb * HBM_TBS)
            out.write("%-10s %-10s %9.4f ms (best %9.4f)  %8.2f TFLOP/s  %5.1f%% of %s MFMA peak  "
                      "%5.1f%% of attainable (%s-bound)  %7.1f GB/s algorithmic\n"
                      % (L.name, name, med, best, tf, 100 * tf / PEAK[L.dtype], L.dtype,
                         100 * tf / attainable, "MFMA" if attainable >= PEAK[L.dtype] else "HBM",
                         nb / (med * 1e-3) / 1e9))
        else:
            nbytes = y.numel() * y.element_size() * (2 if name == "bias_fwd" else 1)
            out.write("%-10s %-10s %9.4f ms (best %9.4f)  %8.1f GB/s\n"
                      % (L.name, name, med, best, nbytes / (med * 1e-3) / 1e9))
        out.flush()
    return results


def copy_calibration(mib, iters=5):
    """A plain device copy of known size (the one-term Sum operator): reads mib MiB, writes mib MiB.
    Run it under `rocprofv3 --pmc FETCH_SIZE` / `WRITE_SIZE` to get the counter-to-bytes factor."""
    n = mib * (1 << 20) // 4
    src = torch.rand(n, device="cuda:0")
    dst = torch.empty_like(src)
    for _ in range(iters):
        B.purine_sum([src], dst)
    torch.cuda.synchronize()
    assert torch.equal(src, dst)
    print("copy calibration: sum_kernel<float> moved %d bytes in and %d bytes out per launch, %d launches"
          % (n * 4, n * 4, iters))


def time_whole(fn, iters, warmup=5):
    """Whole-operator time (every kernel of a composed operator), events on the current stream."""
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    ms = []
    for _ in range(iters):
        s, e = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        s.record()
        fn()
        e.record()
        torch.cuda.synchronize()
        ms.append(s.elapsed_time(e))
    ms.sort()
    return ms[len(ms) // 2], ms[0]


def bench_fc(N, C, K, iters, dtype="f32", out=sys.stdout):
    """The three passes of a fully-connected layer [N, C] x [K, C]."""
    dev = "cuda:0"
    td = torch.bfloat16 if dtype == "bf16" else torch.float32
    x, w, b = torch.rand(N, C, device=dev).to(td), (torch.randn(K, C, device=dev) * 0.01).to(td), torch.zeros(K, device=dev, dtype=td)
    dy = (torch.rand(N, K, device=dev) * 2 - 1).to(td)
    y, dx = torch.empty(N, K, device=dev, dtype=td), torch.empty(N, C, device=dev, dtype=td)
    dw, db = torch.empty(K, C, device=dev), torch.empty(K, device=dev)
    code = B.PURINE_BF16 if dtype == "bf16" else B.PURINE_F32
    ws = [torch.empty(max(256, B.purine_fc_workspace_bytes(p, N, C, K, code)), dtype=torch.uint8, device=dev) for p in (0, 1, 2)]
    flop = 2.0 * N * C * K
    w_bytes = (2.0 if dtype == "bf16" else 4.0) * K * C
    passes = (("fc_fwd", lambda: B.purine_fc_fwd(x, w, b, y, ws=ws[0])),
              ("fc_bwd_data", lambda: B.purine_fc_bwd_data(dy, w, dx, ws=ws[1])),
              ("fc_bwd_weight", lambda: B.purine_fc_bwd_weight(x, dy, dw, db, ws=ws[2])))
    for name, fn in passes:
        med, best = time_whole(fn, iters)
        out.write("fc %dx%d->%d %s %-14s %8.4f ms (best %8.4f)  %7.2f TFLOP/s  %5.1f%% of %s MFMA peak  weights at %6.0f GB/s\n"
                  % (N, C, K, dtype, name, med, best, flop / med / 1e9, 100 * flop / med / 1e9 / PEAK[dtype], dtype, w_bytes / med / 1e6))


def bench_grouped(L, groups, iters, out=sys.stdout):
    """Grouped variant of a conv layer (fp32): the filter keeps C/groups input channels."""
    dev = "cuda:0"
    ws_shape = (L.K, L.C // groups, L.R, L.S)
    x, w, b = torch.rand(L.x_shape, device=dev), torch.randn(ws_shape, device=dev) * 0.01, torch.zeros(L.K, device=dev)
    dy = torch.rand(L.y_shape, device=dev) * 2 - 1
    y, dx = torch.empty(L.y_shape, device=dev), torch.empty(L.x_shape, device=dev)
    dw, db = torch.empty(ws_shape, device=dev), torch.empty(L.K, device=dev)
    desc = B.conv_desc(L.stride, L.pad)
    q = lambda which: torch.empty(max(256, B.purine_grouped_conv_workspace_bytes(which, desc, groups, L.x_shape, ws_shape,
                                                                                 B.PURINE_F32)), dtype=torch.uint8, device=dev)
    wsf, wsd, wsw = q(0), q(1), q(3)
    flop = L.flop_per_pass / groups
    passes = (("fwd+bias+relu", lambda: B.purine_grouped_conv_fwd(desc, groups, x, w, b, y, relu=True, ws=wsf)),
              ("bwd_data", lambda: B.purine_grouped_conv_bwd_data(desc, groups, dy, w, dx, ws=wsd)),
              ("bwd_weight+bias", lambda: B.purine_grouped_conv_bwd_weight(desc, groups, x, dy, dw, db, ws=wsw)))
    for name, fn in passes:
        med, best = time_whole(fn, iters)
        out.write("%-8s groups=%d  %-16s %8.4f ms (best %8.4f)  %7.2f TFLOP/s  %5.1f%% of f32 MFMA peak\n"
                  % (L.name, groups, name, med, best, flop / med / 1e9, 100 * flop / med / 1e9 / PEAK["f32"]))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--config", type=int, default=4)
    ap.add_argument("--layer", default=None)
    ap.add_argument("--op", default="all")
    ap.add_argument("--iters", type=int, default=20)
    ap.add_argument("--batch", type=int, default=None)
    ap.add_argument("--tile", default=None, metavar="BM,BN",
                    help="force the forward / backward-data tile shape (tuning)")
    ap.add_argument("--copy-cal", type=int, default=0, metavar="MiB",
                    help="run only a plain device copy of this many MiB (counter calibration)")
    ap.add_argument("--fc", default=None, metavar="N,C,K", help="time a fully-connected layer instead")
    ap.add_argument("--dtype", default="f32", choices=["f32", "bf16"], help="dtype of the --fc layer")
    ap.add_argument("--groups", type=int, default=0, help="time the grouped variant of the selected layers")
    a = ap.parse_args()
    if a.copy_cal:
        copy_calibration(a.copy_cal)
        return
    if a.fc:
        bench_fc(*[int(v) for v in a.fc.split(",")], a.iters, a.dtype)
        return
    if a.tile:
        B.purine_debug_force_tile(*[int(v) for v in a.tile.split(",")])
    ops = ["fwd", "bwd_data", "bwd_weight", "bias_fwd", "bias_bwd"] if a.op == "all" else a.op.split(",")
    for L in CONV_LAYERS[a.config]:
        if a.layer and L.name != a.layer:
            continue
        if a.batch:
            L = L.with_batch(a.batch)
        if a.groups:
            bench_grouped(L, a.groups, a.iters)
            continue
        bench_layer(L, ops, a.iters)


if __name__ == "__main__":
    main()
