#!/usr/bin/env python3
"""Throughput of the conv-layer hot path on one MI355X.

One step = one forward + backward pass of the whole workload bi-graph (every Conv, Bias,
ConvBwdData, ConvBwdWeight and BiasBwd operator, plus the ReLU/pool/concat glue), driven by the
C-ABI executor with inputs already resident in HBM. value = conv FLOPs of the step (dense
convention, 3 passes x 2*N*K*C*R*S*P*Q per layer) / wall time, in TFLOP/s.

The default run times the AlexNet-shaped five-layer stack at batch 128 (the largest fp32 workload,
driven end to end by the bi-graph executor) and prints ONE JSON line for it. `roofline` describes
the single kernel that takes the most time in the step (its FLOPs, or below the ridge of its dtype
its algorithmic bytes, / its average duration measured with HIP events on its own stream inside
the timed region); `cpu_baseline` is the CPU oracle timed on a bounded sample of the same layers;
`per_config` repeats the measurement (same steps, same warm-up, each with its own dominant-kernel
roofline) for the NIN block, the inception module and the bf16 GoogLeNet stem.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_TFLOPS = {"f32": 157.3, "bf16": 2500.0}     # MI355X dense MFMA peaks
HBM_PEAK_GBS = 8000.0

TRAFFIC_TABLE = os.path.join(ROOT, "profiles", "hbm_traffic_dominant_kernels.md")


def measured_traffic():
    """(config, operator) -> HBM bytes per launch, read from the counter summary kept under
    profiles/ (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this same command, scaled by what the
    counters read for a plain copy of known size). Rows: | cfgN | operator | kernel | fetch_MB | write_MB |.
    An operator that is not in the table (a kernel changed, another one came out dominant) gets null."""
    out = {}
    try:
        with open(TRAFFIC_TABLE) as f:
            for line in f:
                cells = [c.strip() for c in line.strip().strip("|").split("|")]
                if len(cells) >= 5 and cells[0].startswith("cfg") and cells[0][3:].isdigit():
                    try:
                        out[(int(cells[0][3:]), cells[1])] = (float(cells[3]) + float(cells[4])) * 1e6
                    except ValueError:
                        pass
    except OSError:
        pass
    return out


KIND_NAMES = {0: "conv_fwd", 1: "bias_fwd", 2: "conv_bwd_data", 3: "conv_bwd_weight", 4: "bias_bwd",
              5: "relu_fwd", 6: "relu_bwd", 7: "maxpool_fwd", 8: "maxpool_bwd", 9: "concat_fwd",
              10: "concat_bwd", 11: "sum", 13: "conv_fwd_bias_relu", 14: "conv_bwd_data_relu",
              15: "conv_bwd_weight_bias", 16: "sgd_update", 17: "alias", 24: "maxpool_bwd_relu"}


def cpu_baseline(cfg, budget_s=15.0):
    """The oracle as it stands, on a batch-subset of every conv layer of the workload (standalone
    layers with synthetic inputs of the same recipe): fwd + bias, bwd-data, bwd-weight, bias-bwd."""
    import oracle
    from synth import gen
    from synth.configs import CONV_LAYERS
    layers = CONV_LAYERS[cfg]

    def run(n_img):
        flop = 0
        for i, L in enumerate(layers):
            Ls = L.with_batch(n_img)
            x, w, b, dy = gen.layer_tensors_fast(Ls, cfg, i)
            ts = time.perf_counter()
            oracle.bias_fwd(oracle.conv_fwd(x, w, L.stride, L.pad), b)
            oracle.conv_bwd_data(dy, w, x.shape, L.stride, L.pad)
            oracle.conv_bwd_weight(x, dy, w.shape, L.stride, L.pad)
            oracle.bias_bwd(dy)
            run.compute += time.perf_counter() - ts
            flop += 3 * Ls.flop_per_pass
        return flop
    run.compute = 0.0
    run(1)
    t1 = run.compute
    n_img = int(max(1, min(layers[0].N, budget_s / max(t1, 1e-3))))
    run.compute = 0.0
    flop = run(n_img)
    secs = run.compute
    if secs < 0.6 * budget_s and n_img < layers[0].N:      # one image under-uses the cores: rescale once
        n_img = int(max(1, min(layers[0].N, n_img * budget_s / secs)))
        run.compute = 0.0
        flop = run(n_img)
        secs = run.compute
    return {"value": flop / secs / 1e12, "unit": "TFLOP/s", "cores": oracle.num_threads(),
            "kind": "oracle", "seconds": round(secs, 2),
            "sample": "%d of %d images of every conv layer of the workload, all five operators, "
                      "standalone layers with the same input recipe" % (n_img, layers[0].N)}


def bracket_overhead_ms(reps=30):
    """Median bracketed duration of a 64-element ReLU (a kernel of about 2 us)."""
    import torch
    import paper_1412_6249_amd as pa
    a = torch.zeros(64, device="cuda:0")
    b = torch.empty_like(a)
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
    for s, e in evs:            # create the underlying handles
        s.record(); e.record()
    torch.cuda.synchronize()
    for s, e in evs:
        pa.purine_set_kernel_probe(s.cuda_event, e.cuda_event)
        pa.purine_relu_fwd(a, b)
    pa.purine_set_kernel_probe(None, None)
    torch.cuda.synchronize()
    ms = sorted(s.elapsed_time(e) for s, e in evs)
    return max(ms[len(ms) // 2] - 0.002, 0.0)


def run_config(cfg, args, secondary_figures):
    """Times one workload: warm-up, one serial step per operator (per-operator table, dominant
    kernel), then exactly args.steps timed steps between two device synchronisations."""
    import torch
    import paper_1412_6249_amd as pa
    from paper_1412_6249_amd.layers import build_workload
    from synth.configs import CONV_LAYERS, WORKLOAD_NAMES, total_flop

    merge = cfg == 3 and not args.no_merge_1x1 and not args.unfused
    gb = build_workload(cfg, multi_stream=not args.single_stream, fuse=not args.unfused, merge_1x1=merge, fan_in_add=merge)
    n_streams = len(gb.threads)      # `thread` ids of the timed graph: one HIP stream each
    # Warm-up and one step per operator with that operator's main kernel bracketed (twice, keeping
    # the shorter): the per-operator table, and which kernel dominates. These steps run serially
    # (every operator alone on the device), so that each bracket measures its kernel and so that a
    # profiler's per-kernel averages over the whole run are of kernels that ran alone.
    pa.purine_graph_set_serial(gb.g, True)
    pa.purine_graph_enable_timing(gb.g, False)
    for _ in range(max(1, args.warmup)):
        gb.run()
    warm_ms = {}
    for op in gb.ops:
        if op[1] in (12, 17):          # host and alias operators launch nothing
            warm_ms[op[0]] = 0.0
            continue
        best = float("inf")
        for _ in range(2):
            pa.purine_graph_time_only(gb.g, op[0])
            gb.run()
            best = min(best, pa.purine_graph_op_elapsed_ms(gb.g, op[0]))
        warm_ms[op[0]] = best
    # What an event bracket adds around a kernel (the gaps between the event time stamps and the
    # kernel's first and last cycle): measured on a kernel that does next to nothing, and taken off
    # the bracketed durations below, so that they are kernel durations as a profiler reports them.
    bracket_ms = bracket_overhead_ms()
    warm_ms = {k: max(v - bracket_ms, 1e-4) for k, v in warm_ms.items()}
    conv_kinds = (0, 2, 3, 13, 14, 15)
    dominant = max((op for op in gb.ops if op[1] in conv_kinds), key=lambda op: warm_ms[op[0]])[0]
    # Timed region: the graph runs on its streams with operators overlapping as their thread ids
    # allow. On every n-th step (default 4) the dominant kernel is bracketed (one event pair) and
    # keeps the device to itself, so the bracket measures the kernel's own duration. Such a step
    # loses the overlap this one operator would otherwise have had (about 6 % of the step when
    # done every step, 1.5 % at every fourth); that cost is part of the reported value.
    pa.purine_graph_set_serial(gb.g, False)
    if args.replay:
        pa.purine_graph_set_replay(gb.g, True)
        pa.purine_graph_enable_timing(gb.g, False)
        gb.run()                      # records the pass (outside the timed region)
    # The serial per-operator steps above leave the device between host waits most of the time; a run
    # of untimed steps issued exactly like the timed ones brings it back to its steady state (the
    # first steps after such a phase measure up to a fifth slower than the twentieth).
    pa.purine_graph_enable_timing(gb.g, False)
    gb.iterate(max(1, args.warmup))
    dom_ms, dom_n = 0.0, 0
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    # The steps between two sampled ones go through the library's graph iteration: the barrier
    # between consecutive steps is kept by the device (every stream waits for all the others) and
    # the host waits once per group instead of once per step.
    i = 0
    while i < args.steps:
        if i % args.sample_every == 0:
            pa.purine_graph_time_only(gb.g, dominant)
            gb.run()                  # returns after every sink's device work has completed
            dom_ms += pa.purine_graph_op_elapsed_ms(gb.g, dominant)
            dom_n += 1
            i += 1
        else:
            n = min(args.steps - i, args.sample_every - i % args.sample_every)
            pa.purine_graph_enable_timing(gb.g, False)
            gb.iterate(n)
            i += n
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    flop = total_flop(cfg)
    dtype = CONV_LAYERS[cfg][0].dtype

    # per-operator table (warm-up steps) and the dominant kernel (timed steps)
    by_out = {rec[k]: (rec["layer"], k) for rec in gb.conv_records for k in ("y", "out", "dx", "dw")
              if rec[k] is not None}
    rows = []
    for oid, kind, ins, outs, _ in gb.ops:
        avg = warm_ms[oid]
        L = by_out.get(outs[0], (None, None))[0] if kind in conv_kinds else None
        rows.append((avg, oid, kind, outs[0], L))
    rows.sort(reverse=True)
    if args.ops:
        sys.stderr.write("---- %s\n" % WORKLOAD_NAMES[cfg])
        for avg, oid, kind, out, L in rows:
            extra = "  %.1f TFLOP/s" % (L.flop_per_pass / avg / 1e9) if L is not None and avg > 0 else ""
            sys.stderr.write("%9.3f ms  %-16s %s%s\n" % (avg, KIND_NAMES[kind], out, extra))
        sys.stderr.write("sum of kernels (each timed alone) %.3f ms, timed step %.3f ms\n"
                         % (sum(r[0] for r in rows), ms_per_step))
    _, _, kind, out_name, L = next(r for r in rows if r[1] == dominant)
    avg_ms = dom_ms / dom_n - bracket_ms
    kname = "%s[%s]" % (KIND_NAMES[kind], out_name)
    # Which roof bounds this pass: its algorithmic bytes are the three tensors it touches, each once
    # (the ReLU mask of the fused backward-data counts as a fourth); below the ridge
    # peak flop/s / peak bytes/s the pass is priced against HBM, else against the MFMA peak.
    elem = 2 if dtype == "bf16" else 4
    sizes = {"x": elem, "w": elem, "y": elem}
    for nm, shp in (("x", L.x_shape), ("w", L.w_shape), ("y", L.y_shape)):
        for s in shp:
            sizes[nm] *= s
    if kind in (3, 15):
        sizes["w"] = sizes["w"] // elem * 4          # the weight gradient is fp32
    algo_bytes = sizes["x"] + sizes["w"] + sizes["y"] + (sizes["x"] if kind == 14 else 0)
    ridge = PEAK_TFLOPS[dtype] * 1e12 / (HBM_PEAK_GBS * 1e9)
    if L.flop_per_pass / algo_bytes >= ridge:
        achieved = L.flop_per_pass / (avg_ms * 1e-3) / 1e12
        bound, peak, unit = "mfma", PEAK_TFLOPS[dtype], "TFLOP/s"
    else:
        achieved = algo_bytes / (avg_ms * 1e-3) / 1e9
        bound, peak, unit = "hbm", HBM_PEAK_GBS, "GB/s"
    roofline = {"bound": bound, "kernel": kname, "achieved": round(achieved, 3),
                "peak": peak, "unit": unit,
                "frac": round(achieved / peak, 4),
                "avg_kernel_ms": round(avg_ms, 4),
                "bracket_overhead_ms": round(bracket_ms, 4),
                "algorithmic_bytes": algo_bytes,
                "traffic": measured_traffic().get((cfg, kname))}

    secondary = None
    if secondary_figures:
        # secondary figure: the same step without the first layer's backward-data (the gradient with
        # respect to the images, which training does not need); its flops leave the numerator too
        if cfg in (2, 4):
            gb.close()
            gb2 = build_workload(cfg, multi_stream=not args.single_stream, fuse=not args.unfused, first_layer_dx=False)
            if args.replay:
                pa.purine_graph_set_replay(gb2.g, True)
            for _ in range(max(1, args.warmup)):
                gb2.run()
            torch.cuda.synchronize()
            s0 = time.perf_counter()
            n2 = max(5, args.steps // 2)
            gb2.iterate(n2)
            torch.cuda.synchronize()
            ms2 = (time.perf_counter() - s0) * 1e3 / n2
            flop2 = flop - CONV_LAYERS[cfg][0].flop_per_pass
            secondary = {"without_first_layer_dx": {"ms_per_step": round(ms2, 4),
                                                    "value": round(flop2 / (ms2 * 1e-3) / 1e12, 3)}}
            gb = gb2
        # third figure: whole training iterations (paper section 2.2): the step above plus one SGD update
        # operator per parameter tensor and the swap of old and new parameters, iterated natively
        gb.close()
        gb = build_workload(cfg, multi_stream=not args.single_stream, fuse=not args.unfused,
                            first_layer_dx=cfg not in (2, 4), sgd_lr=1e-6, merge_1x1=merge, fan_in_add=merge)
        if args.replay:
            pa.purine_graph_set_replay(gb.g, True)
        gb.iterate(max(2, args.warmup))
        torch.cuda.synchronize()
        s0 = time.perf_counter()
        n3 = max(6, args.steps // 2) // 2 * 2
        gb.iterate(n3)
        torch.cuda.synchronize()
        ms3 = (time.perf_counter() - s0) * 1e3 / n3
        flop3 = flop - (CONV_LAYERS[cfg][0].flop_per_pass if cfg in (2, 4) else 0)
        secondary = dict(secondary or {})
        secondary["sgd_iterations"] = {"ms_per_iteration": round(ms3, 4), "value": round(flop3 / (ms3 * 1e-3) / 1e12, 3),
                                       "first_layer_dx": cfg not in (2, 4)}
    gb.close()
    del gb
    torch.cuda.empty_cache()
    value = flop / (ms_per_step * 1e-3) / 1e12
    return {"workload": WORKLOAD_NAMES[cfg], "ms_per_step": round(ms_per_step, 4), "value": round(value, 3),
            "dtype": dtype, "conv_gflop_per_step": round(flop / 1e9, 2),
            "frac_of_mfma_peak": round(value / PEAK_TFLOPS[dtype], 4),
            "roofline": roofline, "secondary": secondary, "merge": merge, "streams": n_streams}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=40)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", type=int, default=4,
                    help="workload 1..5 of the headline line (default 4: AlexNet-shaped conv stack, batch 128)")
    ap.add_argument("--no-per-config", action="store_true",
                    help="leave out the per_config block (workloads 2, 3 and 5 measured the same way)")
    ap.add_argument("--single-stream", action="store_true", help="all operators on one thread id")
    ap.add_argument("--unfused", action="store_true",
                    help="separate Bias / ReLU / ReLU-gradient operators instead of the fused conv vertices")
    ap.add_argument("--no-merge-1x1", action="store_true",
                    help="config 3: keep the three 1x1 convolutions on the module input as separate operators "
                         "and the Concat copies (default: one merged operator, concatenation by address "
                         "through channel-slice views)")
    ap.add_argument("--replay", action="store_true",
                    help="executor replay mode: the unbracketed steps launch a recorded HIP graph of the pass")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--sample-every", type=int, default=8,
                    help="bracket the dominant kernel (which then runs alone) on every n-th timed step")
    ap.add_argument("--ops", action="store_true", help="print the per-operator tables to stderr")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.stderr.write("bench.py: this build runs on exactly one GPU (the path has no collectives); "
                         "--gpus %d is not supported\n" % args.gpus)
        sys.exit(2)

    import torch
    torch.cuda.set_device(0)
    cfg = args.config
    main_res = run_config(cfg, args, secondary_figures=True)
    result = {
        "metric": "conv fwd+bwd TFLOP/s on one MI355X",
        "value": main_res["value"],
        "unit": "TFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": main_res["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": main_res["dtype"], "data": "synthetic",
        "config": {"workload": main_res["workload"], "conv_gflop_per_step": main_res["conv_gflop_per_step"],
                   "executor": "bi-graph, %s%s, %s" % ("%d stream%s" % (main_res["streams"], "" if main_res["streams"] == 1 else "s"),
                                                        ", recorded pass replayed" if args.replay else "",
                                                      "separate bias/relu ops" if args.unfused
                                                      else "bias+relu fused into conv vertices"
                                                      + (", merged 1x1 + concat by address" if main_res["merge"] else "")),
                   "frac_of_mfma_peak": main_res["frac_of_mfma_peak"]},
        "roofline": main_res["roofline"],
    }
    if main_res["secondary"]:
        result["secondary"] = main_res["secondary"]
    if not args.no_per_config:
        # the other large workloads, measured the same way (same steps and warm-up): the NIN block and
        # the inception module in fp32, the GoogLeNet stem in bf16
        per = {}
        for c in (2, 3, 4, 5):
            if c == cfg:
                continue
            r = run_config(c, args, secondary_figures=False)
            per[r["workload"]] = {k: r[k] for k in ("ms_per_step", "value", "dtype", "conv_gflop_per_step",
                                                    "frac_of_mfma_peak", "roofline", "streams")}
        result["per_config"] = per
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(cfg)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
