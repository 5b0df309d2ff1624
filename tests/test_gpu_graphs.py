"""The five workloads as bi-graphs run by the executor on the GPU, at full layer shapes and a small
batch, checked operator by operator against the oracle with GPU-side teacher forcing: each
operator's ACTUAL device inputs are downloaded and fed to the oracle, and that operator's device
output is compared (conv/bias/sum within tolerance; ReLU, pooling, concat bit for bit). An
end-to-end comparison against an independent fp64 chain would flip ReLU signs and pool winners of
near-zero activations and measure nothing."""
import numpy as np
import pytest

import oracle

pytestmark = pytest.mark.gpu


def host(gb, name):
    from gpu_util import to_host
    return to_host(gb.t[name])


def check_conv_record(gb, rec, tol):
    from gpu_util import rel_l2
    L = rec["layer"]
    x, w, b = host(gb, rec["x"]), host(gb, rec["w"]), host(gb, rec["b"])
    if rec["fused_fwd"]:
        # fused Conv+Bias(+ReLU) vertex: ReLU is continuous, so the composition is compared as one
        ref = oracle.bias_fwd(oracle.conv_fwd(x, w, L.stride, L.pad), b)
        if rec["relu"]:
            ref = np.maximum(ref, 0.0)
        assert rel_l2(host(gb, rec["out"]), ref) <= tol, (L.name, "fused fwd")
    else:
        y = host(gb, rec["y"])
        assert rel_l2(y, oracle.conv_fwd(x, w, L.stride, L.pad)) <= tol, (L.name, "fwd")
        yb = host(gb, rec["yb"])
        # Bias works in place on an exact copy of the Conv output, so y is what it read
        assert rel_l2(yb, oracle.bias_fwd(y, b)) <= tol, (L.name, "bias")
        if rec["relu"]:
            assert np.array_equal(host(gb, rec["out"]), oracle.relu_fwd(yb)), (L.name, "relu")
    dy = host(gb, rec["dy"])
    if rec["relu_bwd_op"]:
        dout_name = gb.ops_by_out[rec["dy"]][2][1]
        assert np.array_equal(dy, oracle.relu_bwd(host(gb, rec["out"]), host(gb, dout_name))), (L.name, "relu_bwd")
    ref_dx = oracle.conv_bwd_data(dy, w, x.shape, L.stride, L.pad)
    if rec.get("fused_bwd"):
        ref_dx = np.where(x > 0, ref_dx, 0.0)        # mask of the ReLU below, taken from its actual output
        assert np.array_equal(host(gb, rec["dx"]) != 0, (x > 0) & (host(gb, rec["dx"]) != 0))
    assert rel_l2(host(gb, rec["dx"]), ref_dx) <= tol, (L.name, "dx")
    assert rel_l2(host(gb, rec["dw"]), oracle.conv_bwd_weight(x, dy, w.shape, L.stride, L.pad)) <= tol, (L.name, "dw")
    assert rel_l2(host(gb, rec["db"]), oracle.bias_bwd(dy)) <= tol, (L.name, "db")


def check_pool_record(gb, rec, check_dx=True):
    from gpu_util import rel_l2, pool_bwd_in_order
    x = host(gb, rec["x"])
    d = rec["desc"]
    ey, earg = oracle.maxpool_fwd(x, d.window, d.stride, d.pad)
    assert np.array_equal(host(gb, rec["y"]), ey)
    assert np.array_equal(gb.t[rec["arg"]].cpu().numpy(), earg)
    if not check_dx:            # a later operator accumulated onto the pooling gradient's storage
        return
    dy = host(gb, rec["dy"])
    dx = host(gb, rec["dx"])
    edx = oracle.maxpool_bwd(dy, earg, x.shape)
    exact = pool_bwd_in_order(dy, earg, x.shape)
    if rec.get("fused_relu"):
        # MaxPoolBwd + the ReLU gradient of the pooled tensor as one operator
        edx, exact = oracle.relu_bwd(x, edx), np.where(x > 0, exact, np.float32(0))
    assert rel_l2(dx, edx) <= 1e-6
    # exact operator: the fp32 sum over the windows in (p, q) order, bit for bit
    assert np.array_equal(dx, exact)


def index_ops(gb):
    gb.ops_by_out = {}
    for op in gb.ops:
        for o in op[3]:
            gb.ops_by_out[o] = op


def legal_order(gb):
    order = gb.fire_log()
    pos = {o: i for i, o in enumerate(order)}
    assert sorted(order) == sorted(op[0] for op in gb.ops)
    writers = {}
    for oid, _, ins, outs, _ in gb.ops:
        for t in outs:
            writers.setdefault(t, []).append(oid)
    for oid, _, ins, outs, _ in gb.ops:
        for t in ins:
            for wtr in writers.get(t, []):
                assert pos[wtr] < pos[oid]


@pytest.mark.parametrize("fuse", [False, True], ids=["plain", "fused"])
@pytest.mark.parametrize("cfg,batch", [(1, None), (2, 2), (3, 2), (4, 2), (5, 1)])
def test_workload_graph_teacher_forced(cfg, batch, fuse):
    from paper_1412_6249_amd.layers import build_workload
    gb = build_workload(cfg, batch=batch, inplace=False, fuse=fuse)
    try:
        index_ops(gb)
        gb.run()
        legal_order(gb)
        tol = 1e-2 if cfg == 5 else 1e-5
        for rec in gb.conv_records:
            check_conv_record(gb, rec, tol)
        for rec in getattr(gb, "pool_records", []):
            check_pool_record(gb, rec)
            assert rec["fused_relu"] == (fuse and cfg == 4)   # every pooled tensor of config 4 is a ReLU output
        if cfg == 4 and fuse:
            assert sum(op[1] == 6 for op in gb.ops) == 0      # no ReLUBwd pass left: three ride on the pooling gradients,
            assert sum(op[1] == 14 for op in gb.ops) == 2     # two (conv3, conv4) on the backward-data of the layer above
        if cfg == 3:
            from gpu_util import rel_l2
            cat = host(gb, "cat")
            parts = [host(gb, r["out"]) for r in gb.conv_records if r["prefix"] in ("b1_1x1", "b2_3x3", "b3_5x5", "b4_proj")]
            assert np.array_equal(cat, oracle.concat_channels(parts))
            terms = [host(gb, n) for n in ("b1_1x1.dx", "b2_reduce.dx", "b3_reduce.dx", "pool.dx")]
            assert rel_l2(host(gb, "dx"), oracle.fan_in_sum(terms)) <= 1e-6
    finally:
        gb.close()


def test_benchmark_graph_of_the_five_layer_stack_at_full_batch():
    """The graph bench.py times by default (config 4 at batch 128: fused vertices, in-place buffers,
    three streams), teacher-forced per conv layer on the device values each operator actually read:
    two sampled images of the fused forward and of backward-data, ALL of dw (summed by the oracle
    over the whole batch) and all of db."""
    import torch
    from gpu_util import rel_l2, to_host
    from paper_1412_6249_amd.layers import build_workload
    gb = build_workload(4, multi_stream=True, fuse=True)
    tol = 1e-5
    try:
        gb.run()
        legal_order(gb)
        rs = np.random.default_rng(404)
        for rec in gb.conv_records:
            L = rec["layer"]
            assert L.N == 128 and rec["fused_fwd"]
            imgs = sorted(rs.choice(L.N - 1, size=1, replace=False).tolist() + [L.N - 1])
            w, b = host(gb, rec["w"]), host(gb, rec["b"])
            x, dy = host(gb, rec["x"]), host(gb, rec["dy"])
            ref = oracle.bias_fwd(oracle.conv_fwd(x[imgs], w, L.stride, L.pad), b)
            if rec["relu"]:
                ref = np.maximum(ref, 0.0)
            assert rel_l2(to_host(gb.t[rec["out"]][imgs]), ref) <= tol, (L.name, "fused fwd")
            if rec["dx"] is not None:
                ref_dx = oracle.conv_bwd_data(dy[imgs], w, x[imgs].shape, L.stride, L.pad)
                if rec.get("fused_bwd"):
                    ref_dx = np.where(x[imgs] > 0, ref_dx, 0.0)
                assert rel_l2(to_host(gb.t[rec["dx"]][imgs]), ref_dx) <= tol, (L.name, "dx")
            assert rel_l2(host(gb, rec["dw"]), oracle.conv_bwd_weight(x, dy, w.shape, L.stride, L.pad)) <= tol, (L.name, "dw")
            assert rel_l2(host(gb, rec["db"]), oracle.bias_bwd(dy)) <= tol, (L.name, "db")
        # the pooling operators of that graph, whole batch, bit for bit (the gradient goes through the
        # fused MaxPoolBwd + ReLU-gradient operator: every pooled tensor here is a ReLU output)
        assert len(gb.pool_records) == 3
        for rec in gb.pool_records:
            assert rec["fused_relu"]
            check_pool_record(gb, rec)
    finally:
        gb.close()


@pytest.mark.parametrize("cfg,batch", [(2, 2), (3, 2), (4, 2)])
def test_inplace_and_multistream_graphs_give_identical_bits(cfg, batch):
    """Buffer-version aliasing (in-place Bias/ReLU) and the thread-to-stream mapping are scheduling
    choices: gradients must be bit-identical to the out-of-place, single-stream run, twice in a row."""
    import torch
    from paper_1412_6249_amd.layers import build_workload
    ref = build_workload(cfg, batch=batch, inplace=False, multi_stream=False, fuse=True)
    fast = build_workload(cfg, batch=batch, inplace=True, multi_stream=True, fuse=True)
    try:
        ref.run()
        for _ in range(2):
            fast.run()
            for r, f in zip(ref.conv_records, fast.conv_records):
                for key in ("dw", "db"):
                    assert torch.equal(ref.t[r[key]], fast.t[f[key]]), (r["prefix"], key)
            # intermediate dx buffers are reused in place by the next ReLUBwd; the gradient at
            # the workload input is the one that survives
            final = "dx" if cfg == 3 else ref.conv_records[0]["dx"]
            assert torch.equal(ref.t[final], fast.t[final])
    finally:
        ref.close()
        fast.close()


@pytest.mark.parametrize("fan_in_add", [False, True], ids=["fan_in_sum", "fan_in_add"])
def test_inception_with_merged_1x1_and_concat_by_address(fan_in_add):
    """Config 3 with the three 1x1 convolutions on the module input merged into one operator and the
    concatenation done through channel-slice views: every operator against the oracle on the device
    values it actually read (the output gradient is saved before the in-place ReLU gradients
    overwrite their slices), and the whole step against the plain graph on the same parameters.
    fan_in_add: the merged operator's backward-data adds to the pooling branch's gradient (no Sum)."""
    from gpu_util import rel_l2, to_host
    from paper_1412_6249_amd.layers import build_workload
    plain = build_workload(3, batch=2, inplace=True, fuse=True)
    gb = build_workload(3, batch=2, inplace=True, fuse=True, merge_1x1=True, fan_in_add=fan_in_add)
    tol = 1e-5
    try:
        assert not any(op[1] in (9, 10) for op in gb.ops)             # no Concat operator either way
        dout0 = to_host(gb.t["dout"]).copy()
        assert np.array_equal(dout0, to_host(plain.t["dout"]))
        plain.run()
        gb.run()
        legal_order(gb)
        H = lambda name: to_host(gb.t[name])
        recs = {r["prefix"]: r for r in gb.conv_records}
        sl = gb.slices
        x = H("x")
        # merged forward and its three slices
        rF = recs["merged_1x1"]
        w_m, b_m = H(rF["w"]), H(rF["b"])
        F = H(rF["out"])
        assert rel_l2(F, np.maximum(oracle.bias_fwd(oracle.conv_fwd(x, w_m, 1, 0), b_m), 0)) <= tol
        assert np.array_equal(H("b2_reduce.a"), F[:, 0:96]) and np.array_equal(H("b3_reduce.a"), F[:, 96:112])
        assert np.array_equal(H("b1_1x1.a"), F[:, 112:176])
        for k, name in enumerate(gb.merged_order):                    # stacked filters = the branches' own
            lo = sum(plain.t[n + ".w"].shape[0] for n in gb.merged_order[:k])
            assert np.array_equal(w_m[lo:lo + plain.t[name + ".w"].shape[0]], to_host(plain.t[name + ".w"]))
        # branch convolutions read slices and write slices
        for p in ("b2_3x3", "b3_5x5", "b4_proj"):
            r = recs[p]
            L = r["layer"]
            ref = np.maximum(oracle.bias_fwd(oracle.conv_fwd(H(r["x"]), H(r["w"]), L.stride, L.pad), H(r["b"])), 0)
            assert rel_l2(H(r["out"]), ref) <= tol, p
        cat = H("cat")
        assert np.array_equal(cat, oracle.concat_channels([H("b1_1x1.a"), H("b2_3x3.a"), H("b3_5x5.a"), H("b4_proj.a")]))
        assert rel_l2(cat, to_host(plain.t["cat"])) <= tol
        # backward of the branches: in-place ReLU gradient on the slice, then the two conv gradients
        first = {"b1_1x1": 0, "b2_3x3": 64, "b3_5x5": 192, "b4_proj": 224}
        for p in ("b2_3x3", "b3_5x5", "b4_proj"):
            r = recs[p]
            L = r["layer"]
            dy = H(r["dy"])
            assert np.array_equal(dy, oracle.relu_bwd(H(r["out"]), dout0[:, first[p]:first[p] + L.K])), p
            xin = H(r["x"])
            ref_dx = oracle.conv_bwd_data(dy, H(r["w"]), xin.shape, L.stride, L.pad)
            if r["fused_bwd"]:
                ref_dx = np.where(xin > 0, ref_dx, 0.0)
            assert rel_l2(H(r["dx"]), ref_dx) <= tol, p
            assert rel_l2(H(r["dw"]), oracle.conv_bwd_weight(xin, dy, H(r["w"]).shape, L.stride, L.pad)) <= tol, p
            assert rel_l2(H(r["db"]), oracle.bias_bwd(dy)) <= tol, p
        assert recs["b2_3x3"]["fused_bwd"] and recs["b3_5x5"]["fused_bwd"] and not recs["b4_proj"]["fused_bwd"]
        assert np.array_equal(H("b1_1x1.dyb"), oracle.relu_bwd(H("b1_1x1.a"), dout0[:, 0:64]))
        # merged backward on the 176-channel gradient slice
        dF = H("merged_1x1.dout")
        assert np.array_equal(dF[:, 0:96], H("b2_3x3.dx")) and np.array_equal(dF[:, 112:176], H("b1_1x1.dyb"))
        assert rel_l2(H(rF["dw"]), oracle.conv_bwd_weight(x, dF, w_m.shape, 1, 0)) <= tol
        assert rel_l2(H(rF["db"]), oracle.bias_bwd(dF)) <= tol
        if fan_in_add:
            assert not any(op[1] == 11 for op in gb.ops)              # no Sum operator
            rp = gb.pool_records[0]
            pool_dx = oracle.maxpool_bwd(H(rp["dy"]), gb.t[rp["arg"]].cpu().numpy(), x.shape)
            assert rel_l2(H("dx"), oracle.conv_bwd_data(dF, w_m, x.shape, 1, 0) + pool_dx) <= tol
            assert gb.t["dx"].data_ptr() == gb.t["pool.dx"].data_ptr()
            check_pool_record(gb, rp, check_dx=False)
        else:
            assert rel_l2(H(rF["dx"]), oracle.conv_bwd_data(dF, w_m, x.shape, 1, 0)) <= tol
            assert rel_l2(H("dx"), oracle.fan_in_sum([H(rF["dx"]), H("pool.dx")])) <= 1e-6
            check_pool_record(gb, gb.pool_records[0])
        # against the plain graph (same parameters, same inputs): the whole step agrees
        assert rel_l2(H("dx"), to_host(plain.t["dx"])) <= tol
        lo = 0
        for name in gb.merged_order:
            k = plain.t[name + ".w"].shape[0]
            assert rel_l2(H(rF["dw"])[lo:lo + k], to_host(plain.t[name + ".dw"])) <= tol, name
            assert rel_l2(H(rF["db"])[lo:lo + k], to_host(plain.t[name + ".db"])) <= tol, name
            lo += k
        for p in ("b2_3x3", "b3_5x5", "b4_proj"):
            assert rel_l2(H(recs[p]["dw"]), to_host(plain.t[p + ".dw"])) <= tol, p
        # a second run gives the same bits (the gradient slices are rewritten from the saved source)
        snap = {n: H(n).copy() for n in ("dx", rF["dw"], rF["db"], "b2_3x3.dw")}
        gb.t["dout"].copy_(__import__("torch").from_numpy(dout0).to(gb.t["dout"].device))
        gb.run()
        for n, v in snap.items():
            assert np.array_equal(H(n), v), n
    finally:
        gb.close()
        plain.close()


@pytest.mark.parametrize("seed", range(6))
def test_random_multi_stream_graphs_equal_their_single_stream_run(seed):
    """Random bi-graphs of Sum and ReLU operators spread over up to five streams, with tensors large
    enough (8 MB) for operators on different streams to overlap in time: every tensor must hold the
    same bits as when the same graph runs on one stream, run after run. A completion event that is
    missing where a consumer on another stream needs it shows up here as a mismatch."""
    import random
    import torch
    import paper_1412_6249_amd as pa
    from paper_1412_6249_amd import binding as B
    rng = random.Random(4200 + seed)
    shape = (2, 16, 256, 256)
    n_ops = rng.randint(20, 45)
    plan = []                                  # (kind, input indices, thread)
    n_src = 3
    for i in range(n_ops):
        avail = n_src + i
        if rng.random() < 0.25:
            plan.append((B.OP_RELU_FWD, [rng.randrange(avail)], rng.randrange(5)))
        else:
            plan.append((B.OP_SUM, rng.sample(range(avail), rng.randint(1, min(3, avail))), rng.randrange(5)))
    gen = torch.Generator(device="cuda")
    gen.manual_seed(seed)
    src = [torch.rand(shape, generator=gen, device="cuda") - 0.5 for _ in range(n_src)]

    def build(single):
        g = pa.purine_graph_create()
        ts = [s.clone() for s in src] + [torch.full(shape, float("nan"), device="cuda") for _ in plan]
        ids = [pa.purine_graph_add_tensor(g, t, "t%d" % i) for i, t in enumerate(ts)]
        for i, (kind, ins, thread) in enumerate(plan):
            pa.purine_graph_add_op(g, kind, [ids[j] for j in ins], [ids[n_src + i]], 0 if single else thread)
        return g, ts

    g1, t1 = build(True)
    gm, tm = build(False)
    try:
        pa.purine_graph_run(g1)
        for rep in range(3):
            for t in tm[n_src:]:
                t.fill_(float("nan"))
            torch.cuda.synchronize()
            pa.purine_graph_run(gm) if rep != 1 else pa.purine_graph_iterate(gm, 2)
            for i, (a, b) in enumerate(zip(t1, tm)):
                assert torch.equal(a, b), (rep, i)
        waits = sum(len(pa.purine_graph_op_waits(gm, o)) for o in range(n_ops))
        assert waits <= n_ops * 4
    finally:
        pa.purine_graph_destroy(g1)
        pa.purine_graph_destroy(gm)
