"""Bi-graph executor bookkeeping on the CPU (host-only operators, no device work).

Dispatcher rules under test (paper section 2.1 and the `thread` property of section 3): every
operator fires exactly once; never before all its incoming tensors are ready; a tensor is ready
only when all its incoming operators have fired; operators of one thread keep FIFO order; the run
ends only when all sinks are reached; an illegal graph is an error, not a hang."""
import random

import pytest

import paper_1412_6249_amd as pa
from paper_1412_6249_amd import binding

F32 = pa.PURINE_F32


def host_tensor(g, name=None, ptr=0, dims=(1,)):
    return pa.purine_graph_add_tensor(g, binding.raw_desc(ptr, F32, dims), name)


def nop(g, ins, outs, thread=0):
    return pa.purine_graph_add_op(g, pa.OP_HOST_NOP, ins, outs, thread)


def check_legal(order, ops):
    """ops: id -> (ins, outs, thread). Legal = every producer of every input fired earlier."""
    pos = {o: i for i, o in enumerate(order)}
    assert sorted(order) == sorted(ops), "each operator fires exactly once"
    writers = {}
    for o, (ins, outs, _) in ops.items():
        for t in outs:
            writers.setdefault(t, []).append(o)
    for o, (ins, outs, _) in ops.items():
        for t in ins:
            for wtr in writers.get(t, []):
                assert pos[wtr] < pos[o], (wtr, o)


def test_chain_single_thread_is_insertion_topological_order():
    g = pa.purine_graph_create()
    t = [host_tensor(g, "t%d" % i) for i in range(6)]
    a = nop(g, [t[0]], [t[1]])
    b = nop(g, [t[1]], [t[2]])
    c = nop(g, [t[0]], [t[3]])
    d = nop(g, [t[2], t[3]], [t[4]])
    e = nop(g, [t[4]], [t[5]])
    pa.purine_graph_run(g)
    assert pa.purine_graph_fire_log(g) == [a, c, b, d, e]
    pa.purine_graph_run(g)                      # graphs can be iterated (section 2.2)
    assert pa.purine_graph_fire_log(g) == [a, c, b, d, e]
    assert pa.purine_graph_num_ops(g) == 5 and pa.purine_graph_num_tensors(g) == 6
    pa.purine_graph_destroy(g)


def test_tensor_with_two_incoming_operators_waits_for_both():
    g = pa.purine_graph_create()
    s0, s1, mid, out = (host_tensor(g) for _ in range(4))
    late = nop(g, [s1], [mid], thread=1)
    early = nop(g, [s0], [mid], thread=0)
    consumer = nop(g, [mid], [out], thread=2)
    pa.purine_graph_run(g)
    order = pa.purine_graph_fire_log(g)
    assert order.index(consumer) == 2 and set(order[:2]) == {late, early}
    pa.purine_graph_destroy(g)


def test_conv_layer_bigraph_shape():
    """Figure 1(b): the conv layer as five operators over eight tensors, backward ops on own threads."""
    g = pa.purine_graph_create()
    names = ["bottom", "weight", "bias", "top", "top_b", "top_grad", "bottom_grad", "weight_grad", "bias_grad"]
    t = {n: host_tensor(g, n) for n in names}
    ops = {}
    ops[nop(g, [t["bottom"], t["weight"]], [t["top"]], 0)] = ([t["bottom"], t["weight"]], [t["top"]], 0)
    ops[nop(g, [t["top"], t["bias"]], [t["top_b"]], 0)] = ([t["top"], t["bias"]], [t["top_b"]], 0)
    ops[nop(g, [t["top_grad"], t["weight"]], [t["bottom_grad"]], 0)] = ([t["top_grad"], t["weight"]], [t["bottom_grad"]], 0)
    ops[nop(g, [t["bottom"], t["top_grad"]], [t["weight_grad"]], 1)] = ([t["bottom"], t["top_grad"]], [t["weight_grad"]], 1)
    ops[nop(g, [t["top_grad"]], [t["bias_grad"]], 2)] = ([t["top_grad"]], [t["bias_grad"]], 2)
    pa.purine_graph_run(g)
    check_legal(pa.purine_graph_fire_log(g), ops)
    pa.purine_graph_destroy(g)


@pytest.mark.parametrize("seed", range(8))
def test_random_dags_fire_legally_with_fifo_threads(seed):
    rnd = random.Random(seed)
    g = pa.purine_graph_create()
    n_src, n_ops = 4, 60
    tensors = [host_tensor(g) for _ in range(n_src)]
    ops = {}
    for _ in range(n_ops):
        ins = rnd.sample(tensors, rnd.randint(1, min(3, len(tensors))))
        outs = [host_tensor(g) for _ in range(rnd.randint(1, 2))]
        if rnd.random() < 0.2 and len(tensors) > n_src:   # a second writer for an existing non-source tensor
            extra = rnd.choice(tensors[n_src:])
            if extra not in ins:
                outs.append(extra)
        th = rnd.randint(0, 3)
        try:
            o = nop(g, ins, outs, th)
        except pa.PurineError:
            continue
        ops[o] = (ins, outs, th)
        tensors.extend(t for t in outs if t not in tensors)
    try:
        pa.purine_graph_run(g)
    except pa.PurineError as e:
        assert e.status == -6          # the extra writer closed a cycle: must be reported, not hang
        pa.purine_graph_destroy(g)
        return
    order = pa.purine_graph_fire_log(g)
    check_legal(order, ops)
    # FIFO per thread: among operators of one thread, firing order = the order they became ready,
    # and "ready" is monotone in the firing order of their last producer
    pos = {o: i for i, o in enumerate(order)}
    writers = {}
    for o, (ins, outs, _) in ops.items():
        for t in outs:
            writers.setdefault(t, []).append(o)

    def ready_time(o):
        return max([pos[w] for t in ops[o][0] for w in writers.get(t, [])], default=-1)
    for th in range(4):
        mine = [o for o in order if ops[o][2] == th]
        times = [ready_time(o) for o in mine]
        assert times == sorted(times), (th, times)
    pa.purine_graph_destroy(g)


def test_cycle_is_an_error_not_a_hang():
    g = pa.purine_graph_create()
    a, b = host_tensor(g), host_tensor(g)
    nop(g, [a], [b])
    nop(g, [b], [a])
    with pytest.raises(pa.PurineError) as e:
        pa.purine_graph_run(g)
    assert e.value.status == -6
    with pytest.raises(pa.PurineError) as e:
        pa.purine_graph_validate(g)
    assert e.value.status == -6
    pa.purine_graph_destroy(g)


def test_bipartite_rules_and_bad_ids():
    g = pa.purine_graph_create()
    a, b = host_tensor(g), host_tensor(g)
    for bad in ([a], [99]), ([-1], [b]):
        with pytest.raises(pa.PurineError) as e:
            nop(g, bad[0], bad[1]) if bad[1] != [99] else nop(g, [a], [99])
        assert e.value.status == -8
    with pytest.raises(pa.PurineError) as e:
        nop(g, [a], [a])                       # operator reading and writing one vertex
    assert e.value.status == -6
    with pytest.raises(pa.PurineError) as e:
        nop(g, [a], [b, b])
    assert e.value.status == -6
    with pytest.raises(pa.PurineError) as e:
        pa.purine_graph_add_op(g, pa.OP_CONV_FWD, [a], [b])     # conv needs two inputs
    assert e.value.status == -8
    with pytest.raises(pa.PurineError) as e:
        nop(g, [a], [b], thread=-1)
    assert e.value.status == -8
    with pytest.raises(pa.PurineError) as e:
        pa.purine_graph_add_op(g, 77, [a], [b])
    assert e.value.status == -8
    pa.purine_graph_destroy(g)


def test_unordered_writers_of_shared_storage_are_rejected():
    """Two device operators that write overlapping bytes with no path between them: validate()
    refuses (pure host analysis, nothing is launched)."""
    g = pa.purine_graph_create()
    x = pa.purine_graph_add_tensor(g, binding.raw_desc(0x1000, F32, (1, 2, 4, 4)), "x")
    y1 = pa.purine_graph_add_tensor(g, binding.raw_desc(0x9000, F32, (1, 2, 4, 4)), "y1")
    y2 = pa.purine_graph_add_tensor(g, binding.raw_desc(0x9000 + 64, F32, (1, 2, 4, 4)), "y2")
    pa.purine_graph_add_op(g, pa.OP_RELU_FWD, [x], [y1], 0)
    pa.purine_graph_add_op(g, pa.OP_RELU_FWD, [x], [y2], 1)
    with pytest.raises(pa.PurineError) as e:
        pa.purine_graph_validate(g)
    assert e.value.status == -6
    pa.purine_graph_destroy(g)
    # the same two writers chained through a version edge are fine
    g = pa.purine_graph_create()
    x = pa.purine_graph_add_tensor(g, binding.raw_desc(0x1000, F32, (1, 2, 4, 4)), "x")
    v0 = pa.purine_graph_add_tensor(g, binding.raw_desc(0x9000, F32, (1, 2, 4, 4)), "v0")
    v1 = pa.purine_graph_add_tensor(g, binding.raw_desc(0x9000, F32, (1, 2, 4, 4)), "v1")
    pa.purine_graph_add_op(g, pa.OP_RELU_FWD, [x], [v0], 0)
    pa.purine_graph_add_op(g, pa.OP_RELU_FWD, [v0], [v1], 1)   # in place: version 0 -> version 1
    pa.purine_graph_validate(g)
    pa.purine_graph_destroy(g)
    # a reader racing an in-place writer is refused as well
    g = pa.purine_graph_create()
    x = pa.purine_graph_add_tensor(g, binding.raw_desc(0x1000, F32, (1, 2, 4, 4)), "x")
    v0 = pa.purine_graph_add_tensor(g, binding.raw_desc(0x9000, F32, (1, 2, 4, 4)), "v0")
    v1 = pa.purine_graph_add_tensor(g, binding.raw_desc(0x9000, F32, (1, 2, 4, 4)), "v1")
    z = pa.purine_graph_add_tensor(g, binding.raw_desc(0x5000, F32, (1, 2, 4, 4)), "z")
    pa.purine_graph_add_op(g, pa.OP_RELU_FWD, [x], [v0], 0)
    pa.purine_graph_add_op(g, pa.OP_RELU_FWD, [v0], [v1], 0)
    pa.purine_graph_add_op(g, pa.OP_RELU_FWD, [v0], [z], 1)
    with pytest.raises(pa.PurineError) as e:
        pa.purine_graph_validate(g)
    assert e.value.status == -6
    pa.purine_graph_destroy(g)


def test_empty_graph_runs():
    g = pa.purine_graph_create()
    pa.purine_graph_run(g)
    assert pa.purine_graph_fire_log(g) == []
    pa.purine_graph_destroy(g)


def test_swap_storage_and_iteration_bookkeeping():
    """The swap step of graph iteration (paper section 2.2, Figure 2(b)) as host bookkeeping: every
    vertex bound to either address moves with it, the graph stays valid, and what would change the
    set of conflicting operators is refused."""
    g = pa.purine_graph_create()
    dims = (1, 2, 4, 4)                                              # 128 bytes
    old = pa.purine_graph_add_tensor(g, binding.raw_desc(0x1000, F32, dims), "old")
    old_v = pa.purine_graph_add_tensor(g, binding.raw_desc(0x1000, F32, dims), "old.v1")   # second version
    new = pa.purine_graph_add_tensor(g, binding.raw_desc(0x9000, F32, dims), "new")
    other = pa.purine_graph_add_tensor(g, binding.raw_desc(0x5000, F32, dims), "other")
    half = pa.purine_graph_add_tensor(g, binding.raw_desc(0x5000, F32, (1, 1, 4, 4)), "other.half")
    small = pa.purine_graph_add_tensor(g, binding.raw_desc(0x7000, F32, (1, 1, 4, 4)), "small")
    near = pa.purine_graph_add_tensor(g, binding.raw_desc(0x1040, F32, dims), "straddles old")
    nop(g, [old], [old_v])
    nop(g, [old_v], [new])
    addr = lambda t: pa.purine_graph_tensor_data(g, t)

    def status(a, b):
        with pytest.raises(pa.PurineError) as e:
            pa.purine_graph_swap_storage(g, a, b)
        return e.value.status

    assert status(old, small) == -2          # extents differ
    assert status(old, old) == -8
    assert status(old, 99) == -8
    assert status(old, old_v) == -4          # same storage
    assert status(old, near) == -4           # overlapping ranges
    assert status(other, new) == -4          # `half` covers part of `other`
    assert status(old, new) == -4            # `near` straddles old's range
    pa.purine_graph_destroy(g)

    g = pa.purine_graph_create()
    old = pa.purine_graph_add_tensor(g, binding.raw_desc(0x1000, F32, dims), "old")
    old_v = pa.purine_graph_add_tensor(g, binding.raw_desc(0x1000, F32, dims), "old.v1")
    new = pa.purine_graph_add_tensor(g, binding.raw_desc(0x9000, F32, dims), "new")
    other = pa.purine_graph_add_tensor(g, binding.raw_desc(0x5000, F32, dims), "other")
    nop(g, [old], [old_v])
    nop(g, [old_v, other], [new])
    addr = lambda t: pa.purine_graph_tensor_data(g, t)
    pa.purine_graph_swap_storage(g, old, new)
    assert (addr(old), addr(old_v), addr(new), addr(other)) == (0x9000, 0x9000, 0x1000, 0x5000)
    pa.purine_graph_validate(g)
    pa.purine_graph_iterate(g, 3, [(old, new)])                      # three runs, three more swaps
    assert (addr(old), addr(old_v), addr(new)) == (0x1000, 0x1000, 0x9000)
    assert pa.purine_graph_fire_log(g) == [0, 1]
    pa.purine_graph_iterate(g, 2, [])                                # no swaps: plain repetition
    assert addr(old) == 0x1000
    assert pa.purine_graph_tensor_data(g, 77) == 0
    with pytest.raises(pa.PurineError):
        pa.purine_graph_iterate(g, -1, [])
    pa.purine_graph_destroy(g)


def test_channel_slice_views_in_the_hazard_analysis():
    """Two operators that write disjoint channel slices of one buffer (same distance between
    images) do not conflict; overlapping slices, or a slice against the whole buffer, do."""
    dims, ns = (2, 4, 4, 4), 16 * 16                       # 4 of 16 channels, 16 elements per channel
    base = 0x20000

    def build(off_a, off_b, whole_reader=False):
        g = pa.purine_graph_create()
        x = pa.purine_graph_add_tensor(g, binding.raw_desc(0x1000, F32, dims), "x")
        a = pa.purine_graph_add_tensor(g, binding.raw_desc(base + off_a * 64, F32, dims, nstride=ns), "a")
        b = pa.purine_graph_add_tensor(g, binding.raw_desc(base + off_b * 64, F32, dims, nstride=ns), "b")
        pa.purine_graph_add_op(g, pa.OP_RELU_FWD, [x], [a], 0)
        pa.purine_graph_add_op(g, pa.OP_RELU_FWD, [x], [b], 1)
        if whole_reader:
            whole = pa.purine_graph_add_tensor(g, binding.raw_desc(base, F32, (2, 16, 4, 4)), "whole")
            z = pa.purine_graph_add_tensor(g, binding.raw_desc(0x90000, F32, (2, 16, 4, 4)), "z")
            pa.purine_graph_add_op(g, pa.OP_RELU_FWD, [whole], [z], 2)
        return g

    g = build(0, 4)                                        # channels 0..3 and 4..7
    pa.purine_graph_validate(g)
    pa.purine_graph_destroy(g)
    g = build(0, 12)                                       # first and last slice
    pa.purine_graph_validate(g)
    pa.purine_graph_destroy(g)
    for offs in ((0, 2), (4, 4), (8, 5)):                  # overlapping channel ranges
        g = build(*offs)
        with pytest.raises(pa.PurineError) as e:
            pa.purine_graph_validate(g)
        assert e.value.status == -6
        pa.purine_graph_destroy(g)
    g = build(0, 4, whole_reader=True)                     # an unordered reader of the whole buffer
    with pytest.raises(pa.PurineError) as e:
        pa.purine_graph_validate(g)
    assert e.value.status == -6
    pa.purine_graph_destroy(g)
    g = pa.purine_graph_create()                           # a view's nstride below its image size
    with pytest.raises(pa.PurineError) as e:
        pa.purine_graph_add_tensor(g, binding.raw_desc(base, F32, dims, nstride=8))
    assert e.value.status == -2
    pa.purine_graph_destroy(g)


# ---------------------------------------------------------------------------------------------
# Planned waits: an event is recorded, and waited for, only where stream order does not already
# give the ordering. Checked against an independent model of what each operator can rely on.

def _random_device_graph(rng, n_ops, n_threads, host_share):
    """Random bi-graph of Sum operators (device kind, made-up addresses: nothing is launched) and
    host operators spread over threads. Returns (g, ops) with ops: id -> (ins, outs, thread, kind)."""
    g = pa.purine_graph_create()
    dims = (1, 2, 4, 4)
    nbytes = 1 * 2 * 4 * 4 * 4
    tensors = [pa.purine_graph_add_tensor(g, binding.raw_desc(0x10000 + i * 0x1000, F32, dims), "src%d" % i)
               for i in range(3)]
    next_ptr = 0x100000
    ops = {}
    for i in range(n_ops):
        ins = rng.sample(tensors, rng.randint(1, min(3, len(tensors))))
        out = pa.purine_graph_add_tensor(g, binding.raw_desc(next_ptr, F32, dims), "t%d" % i)
        next_ptr += max(0x1000, nbytes)
        thread = rng.randrange(n_threads)
        kind = pa.OP_HOST_NOP if rng.random() < host_share else pa.OP_SUM
        o = pa.purine_graph_add_op(g, kind, ins, [out], thread)
        ops[o] = (ins, [out], thread, kind)
        tensors.append(out)
    return g, ops


def _check_planned_waits(g, ops):
    pa.purine_graph_validate(g)
    plan = pa.purine_graph_issue_plan(g)
    check_legal(plan, {o: v[:3] for o, v in ops.items()})
    writers = {}
    for o, (ins, outs, _, _) in ops.items():
        for t in outs:
            writers.setdefault(t, []).append(o)
    known = {}            # device operator -> operators certain to have completed when it starts
    host_known = set()    # what the host has waited for so far
    last_on_stream = {}
    n_waits = 0
    for o in plan:
        ins, outs, thread, kind = ops[o]
        waits = pa.purine_graph_op_waits(g, o)
        producers = {w for t in ins for w in writers.get(t, []) if ops[w][3] != pa.OP_HOST_NOP}
        assert set(waits) <= producers
        assert len(set(waits)) == len(waits)
        if kind == pa.OP_HOST_NOP:
            for p in waits:
                host_known |= known[p] | {p}
            assert producers <= host_known, (o, producers - host_known)
            continue
        n_waits += len(waits)
        assert all(ops[p][2] != thread for p in waits), "same-stream producers need no event"
        assert len({ops[p][2] for p in waits}) == len(waits), "at most one wait per producer stream"
        k = set(host_known)
        prev = last_on_stream.get(thread)
        if prev is not None:
            k |= known[prev] | {prev}
        for p in waits:
            k |= known[p] | {p}
        known[o] = k
        last_on_stream[thread] = o
        assert producers <= k, (o, producers - k)
    return n_waits


@pytest.mark.parametrize("seed", range(40))
def test_planned_waits_cover_every_cross_stream_dependency(seed):
    rng = random.Random(1000 + seed)
    g, ops = _random_device_graph(rng, n_ops=rng.randint(5, 60), n_threads=rng.randint(1, 5),
                                  host_share=rng.choice([0.0, 0.0, 0.15, 0.4]))
    try:
        _check_planned_waits(g, ops)
    finally:
        pa.purine_graph_destroy(g)


def test_planned_waits_of_a_two_stream_layer_stack():
    """Data path on thread 0, gradient-like consumers on thread 1: a consumer waits for the LAST
    producer of the other stream only, and a later consumer does not wait again for what an earlier
    one on its stream already waited for."""
    g = pa.purine_graph_create()
    dims = (1, 2, 4, 4)
    def T(i, name):
        return pa.purine_graph_add_tensor(g, binding.raw_desc(0x10000 + i * 0x1000, F32, dims), name)
    x, a1, a2, a3, g1, g2, g3 = (T(i, n) for i, n in enumerate(["x", "a1", "a2", "a3", "g1", "g2", "g3"]))
    f1 = pa.purine_graph_add_op(g, pa.OP_SUM, [x], [a1], 0)
    f2 = pa.purine_graph_add_op(g, pa.OP_SUM, [a1], [a2], 0)
    f3 = pa.purine_graph_add_op(g, pa.OP_SUM, [a2], [a3], 0)
    c1 = pa.purine_graph_add_op(g, pa.OP_SUM, [a1, a3], [g1], 1)    # needs f1 and f3: waits for f3 only
    c2 = pa.purine_graph_add_op(g, pa.OP_SUM, [a2, g1], [g2], 1)    # fires after c1; f2 is older than f3
    c3 = pa.purine_graph_add_op(g, pa.OP_SUM, [g1, g2], [g3], 1)    # same stream: no event
    pa.purine_graph_validate(g)
    assert pa.purine_graph_op_waits(g, f1) == [] and pa.purine_graph_op_waits(g, f2) == []
    assert pa.purine_graph_op_waits(g, c1) == [f3]
    assert pa.purine_graph_op_waits(g, c2) == []
    assert pa.purine_graph_op_waits(g, c3) == []
    assert sorted(pa.purine_graph_issue_plan(g)) == [f1, f2, f3, c1, c2, c3]
    pa.purine_graph_destroy(g)


def test_plan_queries_need_a_validated_graph():
    g = pa.purine_graph_create()
    a, b = host_tensor(g), host_tensor(g)
    o = nop(g, [a], [b])
    with pytest.raises(pa.PurineError) as e:
        pa.purine_graph_issue_plan(g)
    assert e.value.status == -6
    with pytest.raises(pa.PurineError) as e:
        pa.purine_graph_op_waits(g, o)
    assert e.value.status == -6
    pa.purine_graph_validate(g)
    assert pa.purine_graph_issue_plan(g) == [o]
    with pytest.raises(pa.PurineError) as e:
        pa.purine_graph_op_waits(g, 5)
    assert e.value.status == -8
    pa.purine_graph_destroy(g)
