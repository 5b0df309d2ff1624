"""Bi-graphs of the five synthetic workloads, built on the C-ABI executor.

Each conv layer becomes the operator subgraph of the paper's Figure 1(b): Conv and Bias forward,
ConvBwdData, ConvBwdWeight and BiasBwd backward, with one tensor vertex per buffer VERSION (an
in-place operator reads version i and writes version i+1 of the same storage). Operators get
`thread` ids (paper section 3) so that the three backward operators of a layer, which share only
inputs, can overlap on separate HIP streams. Only graph wiring lives here: every computation is an
operator of libpurine_conv.so.
"""
import torch

from . import binding as B
from synth.configs import CONV_LAYERS

T_MAIN, T_WGRAD, T_BGRAD = 0, 1, 2     # default thread ids: data path, weight grads, bias grads


def _tdtype(dtype):
    return torch.bfloat16 if dtype == "bf16" else torch.float32


def _pcode(dtype):
    return B.PURINE_BF16 if dtype == "bf16" else B.PURINE_F32


class GraphBuilder:
    """Owns the device tensors (by name) and the purine_graph handle."""

    def __init__(self, device="cuda:0", inplace=True, fuse=False):
        self.device = torch.device(device)
        self.inplace = inplace
        self.fuse = fuse                 # fold Bias/ReLU and the ReLU gradient into the conv operators
        self.relu_outputs = set()        # tensors that are the output of a ReLU
        self.masked_grads = set()        # gradients that already carry their layer's ReLU mask
        self.g = B.purine_graph_create()
        self.t = {}          # name -> torch tensor (storage)
        self.ids = {}        # name -> tensor vertex id
        self.ops = []        # (op id, kind, in names, out names, attrs kept alive)
        self.threads = set() # `thread` ids in use: one HIP stream each
        self.conv_records = []   # one dict per conv layer, naming the vertices around each operator
        self.swaps = []          # (old, new) parameter vertices exchanged after every iteration
        self._keep = []

    def close(self):
        if self.g is not None:
            B.purine_graph_destroy(self.g)
            self.g = None

    # ---- vertices
    def new(self, name, shape, dtype="f32", fill=None):
        td = torch.int32 if dtype == "i32" else _tdtype(dtype)
        ten = torch.empty(tuple(int(s) for s in shape), dtype=td, device=self.device)
        if fill is not None:
            ten.fill_(fill)
        return self.bind(name, ten)

    def bind(self, name, tensor):
        assert name not in self.ids, name
        self.t[name] = tensor
        self.ids[name] = B.purine_graph_add_tensor(self.g, tensor, name)
        return name

    def version(self, name, of):
        """A new vertex for the next version of `of`: same storage when in-place, fresh otherwise."""
        if self.inplace:
            return self.bind(name, self.t[of])
        return self.bind(name, torch.empty_like(self.t[of]))

    def workspace(self, nbytes):
        ws = torch.empty(max(256, int(nbytes)), dtype=torch.uint8, device=self.device)
        self._keep.append(ws)
        return ws

    def op(self, kind, ins, outs, thread=T_MAIN, attrs=None):
        oid = B.purine_graph_add_op(self.g, kind, [self.ids[n] for n in ins],
                                    [self.ids[n] for n in outs], thread, attrs)
        self.ops.append((oid, kind, list(ins), list(outs), attrs))
        self.threads.add(int(thread))
        return oid

    # ---- layer-level wiring
    def conv_forward(self, L, x, w, b, prefix, relu, thread=T_MAIN, out=None):
        """x -> Conv -> Bias [-> ReLU]; returns the name of the layer output vertex. `out` (fused
        operators only): an already bound vertex, e.g. a channel slice of a larger buffer."""
        desc = B.conv_desc(L.stride, L.pad)
        ws = self.workspace(B.purine_conv_workspace_bytes(B.PURINE_CONV_FWD, desc, L.x_shape, L.w_shape,
                                                          _pcode(L.dtype)))
        if self.fuse:
            if out is None:
                out = self.new(prefix + (".a" if relu else ".yb"), L.y_shape, L.dtype)
            self.op(B.OP_CONV_FWD_BIAS_RELU, [x, w, b], [out], thread,
                    B.op_attrs(conv=desc, ws=ws, relu=relu))
            if relu:
                self.relu_outputs.add(out)
            rec = dict(layer=L, prefix=prefix, x=x, w=w, b=b, y=None, yb=None, out=out, relu=relu,
                       fused_fwd=True)
            self.conv_records.append(rec)
            return out, rec
        y0 = self.new(prefix + ".y", L.y_shape, L.dtype)
        self.op(B.OP_CONV_FWD, [x, w], [y0], thread, B.op_attrs(conv=desc, ws=ws))
        # Bias is in place by definition of the operator (y += b)
        if self.inplace:
            y1 = self.bind(prefix + ".yb", self.t[y0])
            self.op(B.OP_BIAS_FWD, [y0, b], [y1], thread)
        else:
            # out-of-place variant for the tests: copy version 0 with a one-term Sum, then add bias
            yc = self.new(prefix + ".yc", L.y_shape, L.dtype)
            self.op(B.OP_SUM, [y0], [yc], thread)
            y1 = self.bind(prefix + ".yb", self.t[yc])
            self.op(B.OP_BIAS_FWD, [yc, b], [y1], thread)
        out = y1
        if relu:
            out = self.version(prefix + ".a", y1)
            self.op(B.OP_RELU_FWD, [y1], [out], thread)
            self.relu_outputs.add(out)
        rec = dict(layer=L, prefix=prefix, x=x, w=w, b=b, y=y0, yb=y1, out=out, relu=relu,
                   fused_fwd=False)
        self.conv_records.append(rec)
        return out, rec

    def conv_backward(self, rec, dout, thread=T_MAIN, t_w=T_WGRAD, t_b=T_BGRAD, need_dx=True, dx=None,
                      grad_in_place=False, add_to=None):
        """dout is the gradient at the layer output (after ReLU if the layer has one). `dx`: an
        already bound vertex to receive the input gradient (e.g. a channel slice of a larger buffer);
        `grad_in_place`: the ReLU gradient overwrites dout whatever the builder's default.
        `add_to`: a vertex that already holds another branch's gradient of the same input; the
        backward-data operator then adds to it (beta = 1) and the returned vertex is the next
        version of that storage, so that no separate Sum operator runs for the fan-in."""
        L, p = rec["layer"], rec["prefix"]
        desc = B.conv_desc(L.stride, L.pad)
        dy = dout
        rec["relu_bwd_op"] = False
        if rec["relu"] and dout not in self.masked_grads:
            dy = self.bind(p + ".dyb", self.t[dout]) if grad_in_place else self.version(p + ".dyb", dout)
            self.op(B.OP_RELU_BWD, [rec["out"], dout], [dy], thread)
            rec["relu_bwd_op"] = True
        db = self.new(p + ".db", (L.K,), "f32")
        dw = self.new(p + ".dw", L.w_shape, "f32")
        if self.fuse:
            # both gradients of the layer's parameters from one pass over dy
            ws = self.workspace(B.purine_conv_workspace_bytes(B.PURINE_CONV_BWD_WEIGHT_BIAS, desc, L.x_shape,
                                                              L.w_shape, _pcode(L.dtype)))
            self.op(B.OP_CONV_BWD_WEIGHT_BIAS, [rec["x"], dy], [dw, db], t_w, B.op_attrs(conv=desc, ws=ws))
        else:
            self.op(B.OP_BIAS_BWD, [dy], [db], t_b,
                    B.op_attrs(ws=self.workspace(B.purine_bias_bwd_workspace_bytes(L.y_shape, _pcode(L.dtype)))))
            ws = self.workspace(B.purine_conv_workspace_bytes(B.PURINE_CONV_BWD_WEIGHT, desc, L.x_shape,
                                                              L.w_shape, _pcode(L.dtype)))
            self.op(B.OP_CONV_BWD_WEIGHT, [rec["x"], dy], [dw], t_w, B.op_attrs(conv=desc, ws=ws))
        if not need_dx:
            dx = None
        else:
            ws = self.workspace(B.purine_conv_workspace_bytes(B.PURINE_CONV_BWD_DATA, desc, L.x_shape,
                                                              L.w_shape, _pcode(L.dtype)))
            if add_to is not None:
                assert rec["x"] not in self.relu_outputs          # a mask would have to cover both terms
                dx = self.bind(p + ".dx+", self.t[add_to])
                self.op(B.OP_CONV_BWD_DATA, [dy, rec["w"], add_to], [dx], thread,
                        B.op_attrs(conv=desc, ws=ws, beta=1.0))
                rec["fused_bwd"] = False
                rec.update(dy=dy, db=db, dw=dw, dx=dx, t_w=t_w, t_b=t_w if self.fuse else t_b)
                return dx
            if dx is None:
                dx = self.new(p + ".dx", L.x_shape, L.dtype)
            if self.fuse and rec["x"] in self.relu_outputs:
                # the layer below ends in a ReLU whose output is our input: apply its gradient mask here
                self.op(B.OP_CONV_BWD_DATA_RELU, [dy, rec["w"], rec["x"]], [dx], thread,
                        B.op_attrs(conv=desc, ws=ws))
                self.masked_grads.add(dx)
                rec["fused_bwd"] = True
            else:
                self.op(B.OP_CONV_BWD_DATA, [dy, rec["w"]], [dx], thread, B.op_attrs(conv=desc, ws=ws))
                rec["fused_bwd"] = False
        rec.update(dy=dy, db=db, dw=dw, dx=dx, t_w=t_w, t_b=t_w if self.fuse else t_b)
        return dx

    def add_sgd(self, lr):
        """SGD by graph iteration (paper section 2.2, Figure 2): for every parameter tensor one
        operator leaves w - lr*dw in a separate "new" tensor (writing w itself would close a cycle);
        `swaps` lists the (old, new) vertex pairs whose storage addresses the swap step exchanges
        between two runs of the graph."""
        self.swaps = []
        for rec in self.conv_records:
            for par, grad, th in ((rec["w"], rec["dw"], rec["t_w"]), (rec["b"], rec["db"], rec["t_b"])):
                new = self.bind(par + ".new", torch.empty_like(self.t[par]))
                self.op(B.OP_SGD_UPDATE, [par, grad], [new], th, B.op_attrs(lr=lr))
                self.swaps.append((par, new))

    def iterate(self, n):
        """n times: run the graph, then swap old and new parameters. Afterwards the "old" vertices
        (and this object's tensors of the same names) hold the latest parameters."""
        B.purine_graph_iterate(self.g, n, [(self.ids[a], self.ids[b]) for a, b in self.swaps])
        if n % 2:
            for a, b in self.swaps:
                self.t[a], self.t[b] = self.t[b], self.t[a]

    def maxpool_forward(self, x, shape, dtype, window, stride, pad, prefix, thread=T_MAIN):
        N, C, H, W = shape
        P = (H + 2 * pad - window) // stride + 1
        Q = (W + 2 * pad - window) // stride + 1
        y = self.new(prefix + ".y", (N, C, P, Q), dtype)
        arg = self.new(prefix + ".arg", (N, C, P, Q), "i32")
        pd = B.pool_desc(window, stride, pad)
        self.op(B.OP_MAXPOOL_FWD, [x], [y, arg], thread, B.op_attrs(pool=pd))
        return y, dict(prefix=prefix, x=x, y=y, arg=arg, desc=pd, x_shape=shape, dtype=dtype)

    def maxpool_backward(self, rec, dy, thread=T_MAIN):
        dx = self.new(rec["prefix"] + ".dx", rec["x_shape"], rec["dtype"])
        if self.fuse and rec["x"] in self.relu_outputs:
            # the pooled tensor is a ReLU output: its gradient mask rides along, read off the pooling
            # output (no ReLUBwd pass over dx, and the pooled tensor is not read again)
            self.op(B.OP_MAXPOOL_BWD_RELU, [dy, rec["arg"], rec["y"]], [dx], thread, B.op_attrs(pool=rec["desc"]))
            self.masked_grads.add(dx)
            rec["fused_relu"] = True
        else:
            self.op(B.OP_MAXPOOL_BWD, [dy, rec["arg"]], [dx], thread, B.op_attrs(pool=rec["desc"]))
            rec["fused_relu"] = False
        rec.update(dy=dy, dx=dx)
        return dx

    def run(self):
        B.purine_graph_run(self.g)

    def fire_log(self):
        return B.purine_graph_fire_log(self.g)


# ------------------------------------------------------------------------------------------------
def _default_init(seed):
    """Device-side seeded initialiser: x ~ U[0,1), w, b ~ N(0, 0.01), dy ~ U[-1,1)."""
    gen = torch.Generator(device="cuda")
    gen.manual_seed(int(seed))

    def init(name, shape, dtype, kind):
        if kind == "x":
            t = torch.rand(shape, generator=gen, device="cuda", dtype=torch.float32)
        elif kind == "dy":
            t = torch.rand(shape, generator=gen, device="cuda", dtype=torch.float32) * 2 - 1
        else:
            t = torch.randn(shape, generator=gen, device="cuda", dtype=torch.float32) * 0.01
        return t.to(_tdtype(dtype)).contiguous()
    return init


def _build_inception_merged(gb, layers, src, params, multi_stream, fan_in_add=False):
    """The inception module with its three 1x1 convolutions on the module input merged into one
    operator (filters stacked along K: 96 + 16 + 64 = 176 output channels) and the concatenation done
    by address: every branch writes its channel slice of one activation buffer, and the gradients
    live in a buffer with the same channel map, so neither Concat nor its inverse runs.

    channel map of both buffers (368 channels):
      [0:96] b2_reduce out | [96:112] b3_reduce out | [112:176] b1 out | [176:304] b2_3x3 out |
      [304:336] b3_5x5 out | [336:368] b4_proj out
    merged operator output = [0:176]; module output (concat order b1, b2, b3, b4) = [112:368]."""
    from synth.configs import ConvLayer
    b1, b2r, b2, b3r, b3, b4 = layers
    N, HW = b1.N, (b1.H, b1.W)
    th = (lambda i: i) if multi_stream else (lambda i: 0)
    x = src("x", b1.x_shape, "f32", "x")
    P = {L.name: params(L, L.name) for L in layers}          # same draw order as the plain graph
    merged = ConvLayer("merged_1x1", N, b1.C, b1.H, b1.W, b2r.K + b3r.K + b1.K, 1, 1, 1, 0)
    order = (b2r, b3r, b1)
    w_m = gb.bind("merged_1x1.w", torch.cat([gb.t[P[L.name][0]] for L in order], 0).contiguous())
    b_m = gb.bind("merged_1x1.b", torch.cat([gb.t[P[L.name][1]] for L in order], 0).contiguous())
    act = torch.zeros((N, 368) + HW, dtype=torch.float32, device=gb.device)
    grad = torch.zeros((N, 368) + HW, dtype=torch.float32, device=gb.device)
    gb.t["act_buffer"], gb.t["grad_buffer"] = act, grad
    sl = dict(m2=(0, 96), m3=(96, 112), o1=(112, 176), o2=(176, 304), o3=(304, 336), o4=(336, 368),
              F=(0, 176), cat=(112, 368))
    A = lambda k, name: gb.bind(name, act[:, sl[k][0]:sl[k][1]])
    G = lambda k, name: gb.bind(name, grad[:, sl[k][0]:sl[k][1]])

    # forward
    F, rF = gb.conv_forward(merged, x, w_m, b_m, "merged_1x1", True, th(0), out=A("F", "merged_1x1.a"))
    m2, m3, o1 = A("m2", "b2_reduce.a"), A("m3", "b3_reduce.a"), A("o1", "b1_1x1.a")
    gb.op(B.OP_ALIAS, [F], [m2, m3, o1], th(0))               # the three slices of the merged output
    for v in (m2, m3, o1):
        gb.relu_outputs.add(v)
    o2, r2 = gb.conv_forward(b2, m2, *P[b2.name], b2.name, True, th(1), out=A("o2", "b2_3x3.a"))
    o3, r3 = gb.conv_forward(b3, m3, *P[b3.name], b3.name, True, th(2), out=A("o3", "b3_5x5.a"))
    p4, rp = gb.maxpool_forward(x, b1.x_shape, "f32", 3, 1, 1, "pool", th(3))
    o4, r4 = gb.conv_forward(b4, p4, *P[b4.name], b4.name, True, th(3), out=A("o4", "b4_proj.a"))
    cat = A("cat", "cat")
    gb.op(B.OP_ALIAS, [o1, o2, o3, o4], [cat], th(0))         # the concatenation: no copy

    # backward: the output gradient arrives in the slice [112:368] of the gradient buffer
    dcat = G("cat", "dout")
    gb.t[dcat].copy_(gb.init_value("dout", (N, 256) + HW, "f32", "dy"))
    d1, d2, d3, d4 = G("o1", "db1"), G("o2", "db2"), G("o3", "db3"), G("o4", "db4")
    gb.op(B.OP_ALIAS, [dcat], [d1, d2, d3, d4], th(0))
    tw3 = 4 if multi_stream else 0
    dm2 = gb.conv_backward(r2, d2, th(1), tw3, tw3, dx=G("m2", "b2_3x3.dx"), grad_in_place=True)
    dm3 = gb.conv_backward(r3, d3, th(2), tw3, tw3, dx=G("m3", "b3_5x5.dx"), grad_in_place=True)
    dp4 = gb.conv_backward(r4, d4, th(3), tw3, tw3, grad_in_place=True)
    dx4 = gb.maxpool_backward(rp, dp4, th(3))
    d1m = gb.bind("b1_1x1.dyb", gb.t[d1])                     # b1's ReLU gradient, in place on its slice
    gb.op(B.OP_RELU_BWD, [o1, d1], [d1m], th(0))
    dF = G("F", "merged_1x1.dout")
    gb.op(B.OP_ALIAS, [dm2, dm3, d1m], [dF], th(0))
    gb.masked_grads.add(dF)                                   # every slice already carries its ReLU mask
    if fan_in_add:
        # the module input has two consumers left (merged 1x1, pooling): the merged operator's
        # backward-data adds to the pooling gradient instead of a Sum over two full tensors
        dx = gb.conv_backward(rF, dF, th(0), tw3, tw3, add_to=dx4)
        gb.bind("dx", gb.t[dx])
        gb.op(B.OP_ALIAS, [dx], ["dx"], th(0))
    else:
        dxF = gb.conv_backward(rF, dF, th(0), tw3, tw3)
        dx = gb.new("dx", b1.x_shape, "f32")
        gb.op(B.OP_SUM, [dxF, dx4], [dx], th(0))              # gradient fan-in, fixed order
    gb.pool_records = [rp]
    gb.slices = sl
    gb.merged_order = [L.name for L in order]


def build_workload(cfg, batch=None, inplace=True, init=None, seed=14126249, multi_stream=True,
                   fuse=False, first_layer_dx=True, sgd_lr=None, merge_1x1=False, fan_in_add=False):
    """Builds the bi-graph of config `cfg` (1..5). `batch` overrides the batch size (tests).
    `init(name, shape, dtype, kind)` supplies source tensors (kind in x, w, b, dy); by default they
    are drawn on the device from the seed. `first_layer_dx=False` leaves out the backward-data
    operator of the layer that reads the images in the chained configs 2 and 4 (a training step
    does not need that gradient). `sgd_lr`: also add one SGD update operator per parameter tensor
    (gb.iterate(n) then runs n training iterations). `merge_1x1` (config 3 with fused operators):
    the module's three 1x1 convolutions on its input run as one operator and the concatenation is
    done by address (channel-slice views), see _build_inception_merged; `fan_in_add` (with merge_1x1):
    the gradient fan-in at the module input is an accumulating backward-data operator instead of a
    Sum. Returns the GraphBuilder; gb.run() performs one
    full forward + backward step."""
    init = init or _default_init(seed)
    layers = [l.with_batch(batch) if batch else l for l in CONV_LAYERS[cfg]]
    gb = GraphBuilder(inplace=inplace, fuse=fuse)
    tw = T_WGRAD if multi_stream else T_MAIN
    tb = T_BGRAD if multi_stream else T_MAIN

    def src(name, shape, dtype, kind):
        return gb.bind(name, init(name, tuple(shape), dtype, kind))

    def params(L, p):
        return src(p + ".w", L.w_shape, L.dtype, "w"), src(p + ".b", (L.K,), L.dtype, "b")

    if cfg in (1, 5):
        # independent layers, each with its own synthetic input and output gradient. Config 1 (one small
        # layer) spreads its operators over streams; config 5's kernels each fill the chip on their own
        # (measured: the same step takes 3-4 % longer spread over nine streams), so they share thread 0.
        spread = multi_stream and cfg == 1
        for i, L in enumerate(layers):
            p = L.name
            th = (3 * i) if spread else 0
            x = src(p + ".x", L.x_shape, L.dtype, "x")
            w, b = params(L, p)
            out, rec = gb.conv_forward(L, x, w, b, p, relu=False, thread=th)
            dy = src(p + ".dout", L.y_shape, L.dtype, "dy")
            gb.conv_backward(rec, dy, thread=th, t_w=th + 1 if spread else 0,
                             t_b=th + 2 if spread else 0)
    elif cfg == 2:
        L1, L2, L3 = layers
        x = src("x", L1.x_shape, L1.dtype, "x")
        recs = []
        cur = x
        for L, relu in ((L1, True), (L2, True), (L3, False)):
            w, b = params(L, L.name)
            cur, rec = gb.conv_forward(L, cur, w, b, L.name, relu)
            recs.append(rec)
        grad = src("dout", L3.y_shape, L3.dtype, "dy")
        for rec in reversed(recs):
            grad = gb.conv_backward(rec, grad, t_w=tw, t_b=tb, need_dx=first_layer_dx or rec is not recs[0])
    elif cfg == 3 and merge_1x1:
        if not (fuse and inplace):
            raise ValueError("merge_1x1 needs the fused operators and in-place buffer versions")
        gb.init_value = init
        _build_inception_merged(gb, layers, src, params, multi_stream, fan_in_add)
    elif cfg == 3:
        b1, b2r, b2, b3r, b3, b4 = layers
        N = b1.N
        x = src("x", b1.x_shape, "f32", "x")
        th = (lambda i: i) if multi_stream else (lambda i: 0)
        P = {}
        for L in layers:
            P[L.name] = params(L, L.name)
        o1, r1 = gb.conv_forward(b1, x, *P[b1.name], b1.name, True, th(0))
        m2, r2r = gb.conv_forward(b2r, x, *P[b2r.name], b2r.name, True, th(1))
        o2, r2 = gb.conv_forward(b2, m2, *P[b2.name], b2.name, True, th(1))
        m3, r3r = gb.conv_forward(b3r, x, *P[b3r.name], b3r.name, True, th(2))
        o3, r3 = gb.conv_forward(b3, m3, *P[b3.name], b3.name, True, th(2))
        p4, rp = gb.maxpool_forward(x, b1.x_shape, "f32", 3, 1, 1, "pool", th(3))
        o4, r4 = gb.conv_forward(b4, p4, *P[b4.name], b4.name, True, th(3))
        cat = gb.new("cat", (N, 256, 28, 28), "f32")
        gb.op(B.OP_CONCAT_FWD, [o1, o2, o3, o4], [cat], th(0))
        dcat = src("dout", (N, 256, 28, 28), "f32", "dy")
        d = [gb.new("d" + o, gb.t[o].shape, "f32") for o in (o1, o2, o3, o4)]
        gb.op(B.OP_CONCAT_BWD, [dcat], d, th(0))
        tw3 = 4 if multi_stream else 0
        tb3 = 5 if multi_stream else 0
        dx1 = gb.conv_backward(r1, d[0], th(0), tw3, tb3)
        dm2 = gb.conv_backward(r2, d[1], th(1), tw3, tb3)
        dx2 = gb.conv_backward(r2r, dm2, th(1), tw3, tb3)
        dm3 = gb.conv_backward(r3, d[2], th(2), tw3, tb3)
        dx3 = gb.conv_backward(r3r, dm3, th(2), tw3, tb3)
        dp4 = gb.conv_backward(r4, d[3], th(3), tw3, tb3)
        dx4 = gb.maxpool_backward(rp, dp4, th(3))
        dx = gb.new("dx", b1.x_shape, "f32")
        gb.op(B.OP_SUM, [dx1, dx2, dx3, dx4], [dx], th(0))     # gradient fan-in, fixed order
        gb.pool_records = [rp]
    elif cfg == 4:
        c1, c2, c3, c4, c5 = layers
        x = src("x", c1.x_shape, "f32", "x")
        recs, pools = [], []
        cur = x
        for L, pool in ((c1, True), (c2, True), (c3, False), (c4, False), (c5, True)):
            w, b = params(L, L.name)
            cur, rec = gb.conv_forward(L, cur, w, b, L.name, True)
            recs.append(rec)
            if pool:
                cur, prec = gb.maxpool_forward(cur, L.y_shape, "f32", 3, 2, 0, L.name + ".pool")
                pools.append(prec)
            else:
                pools.append(None)
        grad = src("dout", tuple(gb.t[cur].shape), "f32", "dy")
        for rec, prec in zip(reversed(recs), reversed(pools)):
            if prec is not None:
                grad = gb.maxpool_backward(prec, grad)
            grad = gb.conv_backward(rec, grad, t_w=tw, t_b=tb, need_dx=first_layer_dx or rec is not recs[0])
        gb.pool_records = [p for p in pools if p is not None]
    else:
        raise ValueError("config must be 1..5")
    if sgd_lr is not None:
        gb.add_sgd(sgd_lr)
    B.purine_graph_validate(gb.g)
    return gb
