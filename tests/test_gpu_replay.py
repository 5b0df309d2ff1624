"""Replay mode of the executor: one pass recorded into a HIP graph and launched again, against the
same graph issued operator by operator. Every replay is checked, with eager work (fills of every
output by the framework that owns the storage) and synchronisations between the replays, and the
SGD iteration with its two alternating storage bindings is replayed across several calls."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


def snapshot(gb):
    from gpu_util import to_host
    return {name: to_host(t) for name, t in gb.t.items()}


def same(a, b):
    assert set(a) == set(b)
    for name in a:
        assert np.array_equal(a[name], b[name], equal_nan=True), name


@pytest.mark.parametrize("cfg,batch,merge", [(2, 4, False), (3, 4, True), (4, 2, False), (5, 1, False)])
def test_every_replay_matches_direct_issue(cfg, batch, merge):
    import torch
    import paper_1412_6249_amd as pa
    from paper_1412_6249_amd.layers import build_workload
    a = build_workload(cfg, batch=batch, fuse=True, merge_1x1=merge, fan_in_add=merge)
    b = build_workload(cfg, batch=batch, fuse=True, merge_1x1=merge, fan_in_add=merge)
    try:
        a.run()
        ref = snapshot(a)
        order = pa.purine_graph_fire_log(a.g)
        # what device operators write, leaving out storage shared with a source tensor (slices of a
        # union buffer can be inputs; alias operators only name storage)
        written = {name for op in b.ops if op[1] not in (12, 17) for name in op[3]}
        sources = set(b.t) - {name for op in b.ops for name in op[3]}
        span = lambda t: (t.data_ptr(), t.data_ptr() + (t.untyped_storage().nbytes() - t.storage_offset() * t.element_size()))
        src_spans = [span(b.t[s]) for s in sources]
        touches = lambda u, v: u[0] < v[1] and v[0] < u[1]
        produced = sorted(n for n in written if not any(touches(span(b.t[n]), s) for s in src_spans))
        assert produced
        pa.purine_graph_set_replay(b.g, True)
        for rep in range(5):
            for name in produced:                       # eager work between the replays
                b.t[name].fill_(float(rep) + 0.5) if b.t[name].dtype != torch.int32 else b.t[name].fill_(-7)
            torch.cuda.synchronize()
            b.run()
            same(snapshot(b), ref)
            assert pa.purine_graph_fire_log(b.g) == order
        # timing mode issues directly again, and replay resumes afterwards
        some_op = next(op[0] for op in b.ops if op[1] not in (12, 17))
        pa.purine_graph_time_only(b.g, some_op)
        b.run()
        assert pa.purine_graph_op_elapsed_ms(b.g, some_op) > 0.0
        same(snapshot(b), ref)
        pa.purine_graph_enable_timing(b.g, False)
        b.run()
        same(snapshot(b), ref)
        pa.purine_graph_set_replay(b.g, False)
        b.run()
        same(snapshot(b), ref)
    finally:
        a.close()
        b.close()


@pytest.mark.parametrize("cfg,batch,merge", [(2, 8, False), (3, 4, True)])
def test_replayed_sgd_iterations_match_direct_ones(cfg, batch, merge):
    import paper_1412_6249_amd as pa
    from paper_1412_6249_amd.layers import build_workload
    a = build_workload(cfg, batch=batch, fuse=True, sgd_lr=1e-3, merge_1x1=merge, fan_in_add=merge)
    b = build_workload(cfg, batch=batch, fuse=True, sgd_lr=1e-3, merge_1x1=merge, fan_in_add=merge)
    try:
        pa.purine_graph_set_replay(b.g, True)
        a.iterate(5)
        b.iterate(3)          # records both bindings, replays the first again
        b.iterate(2)          # starts from the second binding
        same(snapshot(a), snapshot(b))
        a.run()
        b.run()
        same(snapshot(a), snapshot(b))
    finally:
        a.close()
        b.close()
