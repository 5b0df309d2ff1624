"""Thin ctypes binding over libpurine_conv.so: argument marshalling only.

Every function has the name of the C entry point it calls (see include/purine.h). Tensors are
torch tensors that live on the GPU (PyTorch supplies device memory and streams, nothing else);
each call raises PurineError on a non-zero status. There is no fallback path: if the shared
library is missing, importing this module fails.
"""
import ctypes
import os

# PyTorch-ROCm ships its own HIP runtime; it must be in the process before our library is loaded
# so that both resolve to that one runtime instance (two instances do not share a device context).
import torch  # noqa: F401

PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(PKG, "libpurine_conv.so")

PURINE_F32, PURINE_BF16, PURINE_I32 = 0, 1, 2
PURINE_CONV_FWD, PURINE_CONV_BWD_DATA, PURINE_CONV_BWD_WEIGHT, PURINE_CONV_BWD_WEIGHT_BIAS = 0, 1, 2, 3

OP_CONV_FWD, OP_BIAS_FWD, OP_CONV_BWD_DATA, OP_CONV_BWD_WEIGHT, OP_BIAS_BWD = 0, 1, 2, 3, 4
OP_RELU_FWD, OP_RELU_BWD, OP_MAXPOOL_FWD, OP_MAXPOOL_BWD = 5, 6, 7, 8
OP_CONCAT_FWD, OP_CONCAT_BWD, OP_SUM, OP_HOST_NOP = 9, 10, 11, 12
OP_CONV_FWD_BIAS_RELU, OP_CONV_BWD_DATA_RELU, OP_CONV_BWD_WEIGHT_BIAS, OP_SGD_UPDATE, OP_ALIAS = 13, 14, 15, 16, 17
OP_FC_FWD, OP_FC_BWD_DATA, OP_FC_BWD_WEIGHT = 18, 19, 20
OP_GROUPED_CONV_FWD, OP_GROUPED_CONV_BWD_DATA, OP_GROUPED_CONV_BWD_WEIGHT = 21, 22, 23
OP_MAXPOOL_BWD_RELU = 24

STATUS = {0: "PURINE_OK", -1: "PURINE_E_NULL", -2: "PURINE_E_SHAPE", -3: "PURINE_E_DTYPE",
          -4: "PURINE_E_LAYOUT", -5: "PURINE_E_WORKSPACE", -6: "PURINE_E_GRAPH",
          -7: "PURINE_E_HIP", -8: "PURINE_E_ARG", -9: "PURINE_E_STATIC_SCRATCH"}


class PurineError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        msg = _lib.purine_status_string(status).decode()
        if status == -7:
            msg += ": " + _lib.purine_last_hip_error().decode()
        super().__init__("%s: %s (%s)" % (where, STATUS.get(status, status), msg))


class purine_tensor(ctypes.Structure):
    _fields_ = [("data", ctypes.c_void_p), ("dtype", ctypes.c_int32), ("ndim", ctypes.c_int32),
                ("dim", ctypes.c_int64 * 4), ("nstride", ctypes.c_int64)]


class purine_conv_desc(ctypes.Structure):
    _fields_ = [("stride_h", ctypes.c_int32), ("stride_w", ctypes.c_int32),
                ("pad_h", ctypes.c_int32), ("pad_w", ctypes.c_int32)]


class purine_pool_desc(ctypes.Structure):
    _fields_ = [("window", ctypes.c_int32), ("stride", ctypes.c_int32), ("pad", ctypes.c_int32)]


class purine_op_attrs(ctypes.Structure):
    _fields_ = [("conv", purine_conv_desc), ("pool", purine_pool_desc), ("beta", ctypes.c_float),
                ("relu", ctypes.c_int32), ("ws", ctypes.c_void_p), ("ws_bytes", ctypes.c_size_t),
                ("lr", ctypes.c_float), ("groups", ctypes.c_int32)]


if not os.path.exists(LIB_PATH):
    raise ImportError("libpurine_conv.so is not built: run `python -c 'import __graft_entry__ as g; "
                      "g.build()'` (or paper_1412_6249_amd/build.py) first")
_lib = ctypes.CDLL(LIB_PATH)

_P = ctypes.POINTER
_T, _D, _PD = _P(purine_tensor), _P(purine_conv_desc), _P(purine_pool_desc)
_i64p, _vp, _sz, _ip = _P(ctypes.c_int64), ctypes.c_void_p, ctypes.c_size_t, _P(ctypes.c_int)

_SIGS = {
    "purine_status_string": (ctypes.c_char_p, [ctypes.c_int]),
    "purine_last_hip_error": (ctypes.c_char_p, []),
    "purine_conv_out_shape": (ctypes.c_int, [_D, _i64p, _i64p, _i64p]),
    "purine_conv_workspace_bytes": (_sz, [ctypes.c_int, _D, _i64p, _i64p, ctypes.c_int32]),
    "purine_bias_bwd_workspace_bytes": (_sz, [_i64p, ctypes.c_int32]),
    "purine_conv_fwd": (ctypes.c_int, [_D, _T, _T, _T, _vp, _sz, _vp]),
    "purine_conv_bwd_data": (ctypes.c_int, [_D, _T, _T, _T, ctypes.c_float, _vp, _sz, _vp]),
    "purine_conv_bwd_weight": (ctypes.c_int, [_D, _T, _T, _T, ctypes.c_float, _vp, _sz, _vp]),
    "purine_conv_bwd_weight_bias": (ctypes.c_int, [_D, _T, _T, _T, _T, ctypes.c_float, _vp, _sz, _vp]),
    "purine_conv_bwd_weight_static": (ctypes.c_int, [_D, _T, _T, _T, ctypes.c_float, _vp]),
    "purine_static_scratch_bytes": (_sz, []),
    "purine_grouped_conv_workspace_bytes": (_sz, [ctypes.c_int, _D, ctypes.c_int, _i64p, _i64p, ctypes.c_int32]),
    "purine_grouped_conv_fwd": (ctypes.c_int, [_D, ctypes.c_int, _T, _T, _T, _T, ctypes.c_int, _vp, _sz, _vp]),
    "purine_grouped_conv_bwd_data": (ctypes.c_int, [_D, ctypes.c_int, _T, _T, _T, ctypes.c_float, _vp, _sz, _vp]),
    "purine_grouped_conv_bwd_weight": (ctypes.c_int, [_D, ctypes.c_int, _T, _T, _T, _T, ctypes.c_float, _vp, _sz, _vp]),
    "purine_fc_workspace_bytes": (_sz, [ctypes.c_int, ctypes.c_int64, ctypes.c_int64, ctypes.c_int64, ctypes.c_int32]),
    "purine_fc_fwd": (ctypes.c_int, [_T, _T, _T, _T, _vp, _sz, _vp]),
    "purine_fc_bwd_data": (ctypes.c_int, [_T, _T, _T, _vp, _sz, _vp]),
    "purine_fc_bwd_weight": (ctypes.c_int, [_T, _T, _T, _T, ctypes.c_float, _vp, _sz, _vp]),
    "purine_conv_fwd_bias_relu": (ctypes.c_int, [_D, _T, _T, _T, _T, ctypes.c_int, _vp, _sz, _vp]),
    "purine_conv_bwd_data_relu": (ctypes.c_int, [_D, _T, _T, _T, _T, ctypes.c_float, _vp, _sz, _vp]),
    "purine_bias_fwd": (ctypes.c_int, [_T, _T, _vp]),
    "purine_bias_bwd": (ctypes.c_int, [_T, _T, ctypes.c_float, _vp, _sz, _vp]),
    "purine_relu_fwd": (ctypes.c_int, [_T, _T, _vp]),
    "purine_relu_bwd": (ctypes.c_int, [_T, _T, _T, _vp]),
    "purine_maxpool_fwd": (ctypes.c_int, [_PD, _T, _T, _T, _vp]),
    "purine_maxpool_bwd": (ctypes.c_int, [_PD, _T, _T, _T, ctypes.c_float, _vp]),
    "purine_maxpool_bwd_relu": (ctypes.c_int, [_PD, _T, _T, _T, _T, ctypes.c_float, _vp]),
    "purine_concat_fwd": (ctypes.c_int, [_P(_T), ctypes.c_int, _T, _vp]),
    "purine_concat_bwd": (ctypes.c_int, [_T, _P(_T), ctypes.c_int, _vp]),
    "purine_sum": (ctypes.c_int, [_P(_T), ctypes.c_int, _T, _vp]),
    "purine_graph_create": (_vp, []),
    "purine_graph_destroy": (None, [_vp]),
    "purine_graph_add_tensor": (ctypes.c_int, [_vp, _T, ctypes.c_char_p]),
    "purine_graph_add_op": (ctypes.c_int, [_vp, ctypes.c_int, _P(purine_op_attrs), _ip, ctypes.c_int,
                                           _ip, ctypes.c_int, ctypes.c_int]),
    "purine_graph_set_stream": (ctypes.c_int, [_vp, ctypes.c_int, _vp]),
    "purine_graph_validate": (ctypes.c_int, [_vp]),
    "purine_graph_run": (ctypes.c_int, [_vp]),
    "purine_graph_swap_storage": (ctypes.c_int, [_vp, ctypes.c_int, ctypes.c_int]),
    "purine_graph_tensor_data": (_vp, [_vp, ctypes.c_int]),
    "purine_graph_iterate": (ctypes.c_int, [_vp, ctypes.c_int, _ip, _ip, ctypes.c_int]),
    "purine_sgd_update": (ctypes.c_int, [_T, _T, _T, ctypes.c_float, _vp]),
    "purine_graph_fire_log": (ctypes.c_int, [_vp, _ip, ctypes.c_int]),
    "purine_graph_set_replay": (ctypes.c_int, [_vp, ctypes.c_int]),
    "purine_graph_issue_plan": (ctypes.c_int, [_vp, _ip, ctypes.c_int]),
    "purine_graph_op_waits": (ctypes.c_int, [_vp, ctypes.c_int, _ip, ctypes.c_int]),
    "purine_graph_num_ops": (ctypes.c_int, [_vp]),
    "purine_graph_num_tensors": (ctypes.c_int, [_vp]),
    "purine_debug_fastdiv": (ctypes.c_uint32, [ctypes.c_uint32, ctypes.c_uint32]),
    "purine_debug_force_tile": (None, [ctypes.c_int, ctypes.c_int]),
    "purine_graph_enable_timing": (ctypes.c_int, [_vp, ctypes.c_int]),
    "purine_graph_time_only": (ctypes.c_int, [_vp, ctypes.c_int]),
    "purine_graph_set_serial": (ctypes.c_int, [_vp, ctypes.c_int]),
    "purine_graph_op_elapsed_ms": (ctypes.c_int, [_vp, ctypes.c_int, _P(ctypes.c_float)]),
    "purine_set_kernel_probe": (None, [_vp, _vp]),
}
for _name, (_res, _args) in _SIGS.items():
    _f = getattr(_lib, _name)
    _f.restype, _f.argtypes = _res, _args

EXPORTED = sorted(_SIGS)


# ------------------------------------------------------------------ marshalling helpers
def _dtype_code(t):
    import torch
    if t.dtype == torch.float32:
        return PURINE_F32
    if t.dtype == torch.bfloat16:
        return PURINE_BF16
    if t.dtype == torch.int32:
        return PURINE_I32
    raise TypeError("unsupported torch dtype %s" % t.dtype)


def tensor_desc(t):
    """purine_tensor for a CUDA torch tensor that is contiguous or a channel slice of a contiguous
    NCHW tensor (or passes a ready-made descriptor through)."""
    if isinstance(t, purine_tensor):
        return t
    if not t.is_cuda:
        raise ValueError("tensor must live on the GPU")
    if t.dim() < 1 or t.dim() > 4:
        raise ValueError("1 to 4 dimensions")
    nstride = 0
    if not t.is_contiguous():
        n, c, h, w = t.shape if t.dim() == 4 else (0, 0, 0, 0)
        if t.dim() != 4 or tuple(t.stride()[1:]) != (h * w, w, 1) or t.stride(0) < c * h * w:
            raise ValueError("tensor must be contiguous (dense NCHW / KCRS) or a channel slice of one")
        nstride = int(t.stride(0))
    d = purine_tensor()
    d.nstride = nstride
    d.data = t.data_ptr()
    d.dtype = _dtype_code(t)
    d.ndim = t.dim()
    for i, v in enumerate(t.shape):
        d.dim[i] = int(v)
    return d


def raw_desc(data_ptr, dtype, dims, nstride=0):
    """Descriptor from a raw pointer (tests of the error paths, host-only graphs)."""
    d = purine_tensor()
    d.nstride = int(nstride)
    d.data = data_ptr
    d.dtype = dtype
    d.ndim = len(dims)
    for i, v in enumerate(dims):
        d.dim[i] = int(v)
    return d


def conv_desc(stride=1, pad=0):
    sh, sw = (stride, stride) if isinstance(stride, int) else stride
    ph, pw = (pad, pad) if isinstance(pad, int) else pad
    return purine_conv_desc(int(sh), int(sw), int(ph), int(pw))


def pool_desc(window, stride, pad=0):
    return purine_pool_desc(int(window), int(stride), int(pad))


def _stream(stream):
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    return getattr(stream, "cuda_stream", stream)


def _ws(ws):
    if ws is None:
        return None, 0
    return ws.data_ptr(), ws.numel() * ws.element_size()


def _dims(shape):
    return (ctypes.c_int64 * 4)(*[int(v) for v in shape])


def _check(rc, where):
    if rc != 0:
        raise PurineError(rc, where)


def _ref(x):
    return ctypes.byref(x)


# ------------------------------------------------------------------ host-only entry points
def purine_status_string(status):
    return _lib.purine_status_string(int(status)).decode()


def purine_last_hip_error():
    return _lib.purine_last_hip_error().decode()


def purine_conv_out_shape(desc, x_shape, w_shape):
    out = (ctypes.c_int64 * 4)()
    _check(_lib.purine_conv_out_shape(_ref(desc), _dims(x_shape), _dims(w_shape), out),
           "purine_conv_out_shape")
    return tuple(int(v) for v in out)


def purine_conv_workspace_bytes(which, desc, x_shape, w_shape, dtype):
    return int(_lib.purine_conv_workspace_bytes(int(which), _ref(desc), _dims(x_shape),
                                                _dims(w_shape), int(dtype)))


def purine_bias_bwd_workspace_bytes(dy_shape, dtype):
    return int(_lib.purine_bias_bwd_workspace_bytes(_dims(dy_shape), int(dtype)))


def purine_debug_force_tile(bm=0, bn=0):
    _lib.purine_debug_force_tile(int(bm), int(bn))


def purine_debug_fastdiv(n, d):
    return int(_lib.purine_debug_fastdiv(int(n), int(d)))


# ------------------------------------------------------------------ operators
def purine_conv_fwd(desc, x, w, y, ws=None, stream=None):
    p, n = _ws(ws)
    _check(_lib.purine_conv_fwd(_ref(desc), _ref(tensor_desc(x)), _ref(tensor_desc(w)),
                                _ref(tensor_desc(y)), p, n, _stream(stream)), "purine_conv_fwd")


def purine_conv_bwd_data(desc, dy, w, dx, beta=0.0, ws=None, stream=None):
    p, n = _ws(ws)
    _check(_lib.purine_conv_bwd_data(_ref(desc), _ref(tensor_desc(dy)), _ref(tensor_desc(w)),
                                     _ref(tensor_desc(dx)), float(beta), p, n, _stream(stream)),
           "purine_conv_bwd_data")


def purine_conv_fwd_bias_relu(desc, x, w, b, y, relu=True, ws=None, stream=None):
    p, n = _ws(ws)
    bd = _ref(tensor_desc(b)) if b is not None else None
    _check(_lib.purine_conv_fwd_bias_relu(_ref(desc), _ref(tensor_desc(x)), _ref(tensor_desc(w)), bd,
                                          _ref(tensor_desc(y)), 1 if relu else 0, p, n, _stream(stream)),
           "purine_conv_fwd_bias_relu")


def purine_conv_bwd_data_relu(desc, dy, w, act, dx, beta=0.0, ws=None, stream=None):
    p, n = _ws(ws)
    _check(_lib.purine_conv_bwd_data_relu(_ref(desc), _ref(tensor_desc(dy)), _ref(tensor_desc(w)),
                                          _ref(tensor_desc(act)), _ref(tensor_desc(dx)), float(beta), p, n,
                                          _stream(stream)), "purine_conv_bwd_data_relu")


def purine_conv_bwd_weight(desc, x, dy, dw, beta=0.0, ws=None, stream=None):
    p, n = _ws(ws)
    _check(_lib.purine_conv_bwd_weight(_ref(desc), _ref(tensor_desc(x)), _ref(tensor_desc(dy)),
                                       _ref(tensor_desc(dw)), float(beta), p, n, _stream(stream)),
           "purine_conv_bwd_weight")


def purine_conv_bwd_weight_static(desc, x, dy, dw, beta=0.0, stream=None):
    _check(_lib.purine_conv_bwd_weight_static(_ref(desc), _ref(tensor_desc(x)), _ref(tensor_desc(dy)),
                                              _ref(tensor_desc(dw)), float(beta), _stream(stream)),
           "purine_conv_bwd_weight_static")


def purine_static_scratch_bytes():
    return int(_lib.purine_static_scratch_bytes())


def purine_conv_bwd_weight_bias(desc, x, dy, dw, db, beta=0.0, ws=None, stream=None):
    p, n = _ws(ws)
    _check(_lib.purine_conv_bwd_weight_bias(_ref(desc), _ref(tensor_desc(x)), _ref(tensor_desc(dy)),
                                            _ref(tensor_desc(dw)), _ref(tensor_desc(db)), float(beta), p, n,
                                            _stream(stream)), "purine_conv_bwd_weight_bias")


def _opt(t):
    return _ref(tensor_desc(t)) if t is not None else None


def purine_grouped_conv_workspace_bytes(which, desc, groups, x_shape, w_shape, dtype):
    return int(_lib.purine_grouped_conv_workspace_bytes(int(which), _ref(desc), int(groups), _dims(x_shape),
                                                        _dims(w_shape), int(dtype)))


def purine_grouped_conv_fwd(desc, groups, x, w, b, y, relu=False, ws=None, stream=None):
    p, n = _ws(ws)
    _check(_lib.purine_grouped_conv_fwd(_ref(desc), int(groups), _ref(tensor_desc(x)), _ref(tensor_desc(w)), _opt(b),
                                        _ref(tensor_desc(y)), 1 if relu else 0, p, n, _stream(stream)),
           "purine_grouped_conv_fwd")


def purine_grouped_conv_bwd_data(desc, groups, dy, w, dx, beta=0.0, ws=None, stream=None):
    p, n = _ws(ws)
    _check(_lib.purine_grouped_conv_bwd_data(_ref(desc), int(groups), _ref(tensor_desc(dy)), _ref(tensor_desc(w)),
                                             _ref(tensor_desc(dx)), float(beta), p, n, _stream(stream)),
           "purine_grouped_conv_bwd_data")


def purine_grouped_conv_bwd_weight(desc, groups, x, dy, dw, db=None, beta=0.0, ws=None, stream=None):
    p, n = _ws(ws)
    _check(_lib.purine_grouped_conv_bwd_weight(_ref(desc), int(groups), _ref(tensor_desc(x)), _ref(tensor_desc(dy)),
                                               _ref(tensor_desc(dw)), _opt(db), float(beta), p, n, _stream(stream)),
           "purine_grouped_conv_bwd_weight")


def purine_fc_workspace_bytes(which, N, C, K, dtype=PURINE_F32):
    return int(_lib.purine_fc_workspace_bytes(int(which), int(N), int(C), int(K), int(dtype)))


def purine_fc_fwd(x, w, b, y, ws=None, stream=None):
    p, n = _ws(ws)
    _check(_lib.purine_fc_fwd(_ref(tensor_desc(x)), _ref(tensor_desc(w)), _opt(b), _ref(tensor_desc(y)), p, n,
                              _stream(stream)), "purine_fc_fwd")


def purine_fc_bwd_data(dy, w, dx, ws=None, stream=None):
    p, n = _ws(ws)
    _check(_lib.purine_fc_bwd_data(_ref(tensor_desc(dy)), _ref(tensor_desc(w)), _ref(tensor_desc(dx)), p, n,
                                   _stream(stream)), "purine_fc_bwd_data")


def purine_fc_bwd_weight(x, dy, dw, db=None, beta=0.0, ws=None, stream=None):
    p, n = _ws(ws)
    _check(_lib.purine_fc_bwd_weight(_ref(tensor_desc(x)), _ref(tensor_desc(dy)), _ref(tensor_desc(dw)), _opt(db),
                                     float(beta), p, n, _stream(stream)), "purine_fc_bwd_weight")


def purine_sgd_update(w, dw, new_w, lr, stream=None):
    _check(_lib.purine_sgd_update(_ref(tensor_desc(w)), _ref(tensor_desc(dw)), _ref(tensor_desc(new_w)),
                                  float(lr), _stream(stream)), "purine_sgd_update")


def purine_bias_fwd(b, y, stream=None):
    _check(_lib.purine_bias_fwd(_ref(tensor_desc(b)), _ref(tensor_desc(y)), _stream(stream)),
           "purine_bias_fwd")


def purine_bias_bwd(dy, db, beta=0.0, ws=None, stream=None):
    p, n = _ws(ws)
    _check(_lib.purine_bias_bwd(_ref(tensor_desc(dy)), _ref(tensor_desc(db)), float(beta), p, n,
                                _stream(stream)), "purine_bias_bwd")


def purine_relu_fwd(x, y, stream=None):
    _check(_lib.purine_relu_fwd(_ref(tensor_desc(x)), _ref(tensor_desc(y)), _stream(stream)),
           "purine_relu_fwd")


def purine_relu_bwd(x, dy, dx, stream=None):
    _check(_lib.purine_relu_bwd(_ref(tensor_desc(x)), _ref(tensor_desc(dy)), _ref(tensor_desc(dx)),
                                _stream(stream)), "purine_relu_bwd")


def purine_maxpool_fwd(desc, x, y, arg, stream=None):
    _check(_lib.purine_maxpool_fwd(_ref(desc), _ref(tensor_desc(x)), _ref(tensor_desc(y)),
                                   _ref(tensor_desc(arg)), _stream(stream)), "purine_maxpool_fwd")


def purine_maxpool_bwd(desc, dy, arg, dx, beta=0.0, stream=None):
    _check(_lib.purine_maxpool_bwd(_ref(desc), _ref(tensor_desc(dy)), _ref(tensor_desc(arg)),
                                   _ref(tensor_desc(dx)), float(beta), _stream(stream)),
           "purine_maxpool_bwd")


def purine_maxpool_bwd_relu(desc, dy, arg, y, dx, beta=0.0, stream=None):
    _check(_lib.purine_maxpool_bwd_relu(_ref(desc), _ref(tensor_desc(dy)), _ref(tensor_desc(arg)),
                                        _ref(tensor_desc(y)), _ref(tensor_desc(dx)), float(beta), _stream(stream)),
           "purine_maxpool_bwd_relu")


def _tensor_ptr_array(tensors):
    descs = [tensor_desc(t) for t in tensors]
    arr = (_T * len(descs))(*[ctypes.pointer(d) for d in descs])
    return arr, descs


def purine_concat_fwd(parts, out, stream=None):
    arr, keep = _tensor_ptr_array(parts)
    _check(_lib.purine_concat_fwd(arr, len(keep), _ref(tensor_desc(out)), _stream(stream)),
           "purine_concat_fwd")


def purine_concat_bwd(dout, dparts, stream=None):
    arr, keep = _tensor_ptr_array(dparts)
    _check(_lib.purine_concat_bwd(_ref(tensor_desc(dout)), arr, len(keep), _stream(stream)),
           "purine_concat_bwd")


def purine_sum(terms, out, stream=None):
    arr, keep = _tensor_ptr_array(terms)
    _check(_lib.purine_sum(arr, len(keep), _ref(tensor_desc(out)), _stream(stream)), "purine_sum")


# ------------------------------------------------------------------ bi-graph executor
def purine_graph_create():
    g = _lib.purine_graph_create()
    if not g:
        raise MemoryError("purine_graph_create")
    return g


def purine_graph_destroy(g):
    _lib.purine_graph_destroy(g)


def purine_graph_add_tensor(g, t, name=None):
    rc = _lib.purine_graph_add_tensor(g, _ref(tensor_desc(t)), name.encode() if name else None)
    if rc < 0:
        raise PurineError(rc, "purine_graph_add_tensor")
    return rc


def purine_graph_add_op(g, kind, in_ids, out_ids, thread_id=0, attrs=None):
    ins = (ctypes.c_int * max(1, len(in_ids)))(*in_ids)
    outs = (ctypes.c_int * max(1, len(out_ids)))(*out_ids)
    rc = _lib.purine_graph_add_op(g, int(kind), _ref(attrs) if attrs is not None else None, ins,
                                  len(in_ids), outs, len(out_ids), int(thread_id))
    if rc < 0:
        raise PurineError(rc, "purine_graph_add_op")
    return rc


def op_attrs(conv=None, pool=None, beta=0.0, ws=None, relu=False, lr=0.0, groups=0):
    a = purine_op_attrs()
    a.groups = int(groups)
    a.relu = 1 if relu else 0
    a.lr = float(lr)
    if conv is not None:
        a.conv = conv
    if pool is not None:
        a.pool = pool
    a.beta = float(beta)
    p, n = _ws(ws)
    a.ws = p
    a.ws_bytes = n
    return a


def purine_graph_set_stream(g, thread_id, stream):
    _check(_lib.purine_graph_set_stream(g, int(thread_id), getattr(stream, "cuda_stream", stream)),
           "purine_graph_set_stream")


def purine_graph_validate(g):
    _check(_lib.purine_graph_validate(g), "purine_graph_validate")


def purine_graph_run(g):
    _check(_lib.purine_graph_run(g), "purine_graph_run")


def purine_graph_swap_storage(g, tensor_a, tensor_b):
    _check(_lib.purine_graph_swap_storage(g, int(tensor_a), int(tensor_b)), "purine_graph_swap_storage")


def purine_graph_tensor_data(g, tensor_id):
    return int(_lib.purine_graph_tensor_data(g, int(tensor_id)) or 0)


def purine_graph_iterate(g, n_iters, swaps=()):
    """swaps: pairs of tensor ids whose storage addresses are exchanged after every run."""
    n = len(swaps)
    a = (ctypes.c_int * max(1, n))(*[int(s[0]) for s in swaps])
    b = (ctypes.c_int * max(1, n))(*[int(s[1]) for s in swaps])
    _check(_lib.purine_graph_iterate(g, int(n_iters), a, b, n), "purine_graph_iterate")


def purine_graph_set_replay(g, on):
    _check(_lib.purine_graph_set_replay(g, 1 if on else 0), "purine_graph_set_replay")


def purine_graph_issue_plan(g):
    """Firing order planned by validation (the graph must have been validated)."""
    n = _lib.purine_graph_num_ops(g)
    buf = (ctypes.c_int * max(1, n))()
    got = _lib.purine_graph_issue_plan(g, buf, n)
    if got < 0:
        _check(got, "purine_graph_issue_plan")
    return [int(buf[i]) for i in range(min(n, got))]


def purine_graph_op_waits(g, op_id):
    """Producers whose completion operator op_id waits for before it is issued."""
    n = _lib.purine_graph_num_ops(g)
    buf = (ctypes.c_int * max(1, n))()
    got = _lib.purine_graph_op_waits(g, int(op_id), buf, n)
    if got < 0:
        _check(got, "purine_graph_op_waits")
    return [int(buf[i]) for i in range(min(n, got))]


def purine_graph_fire_log(g):
    n = _lib.purine_graph_num_ops(g)
    buf = (ctypes.c_int * max(1, n))()
    fired = _lib.purine_graph_fire_log(g, buf, n)
    return [int(buf[i]) for i in range(min(n, fired))]


def purine_graph_num_ops(g):
    return int(_lib.purine_graph_num_ops(g))


def purine_graph_num_tensors(g):
    return int(_lib.purine_graph_num_tensors(g))


def purine_graph_enable_timing(g, on=True):
    _check(_lib.purine_graph_enable_timing(g, 1 if on else 0), "purine_graph_enable_timing")


def purine_graph_time_only(g, op_id):
    _check(_lib.purine_graph_time_only(g, int(op_id)), "purine_graph_time_only")


def purine_graph_set_serial(g, on):
    _check(_lib.purine_graph_set_serial(g, 1 if on else 0), "purine_graph_set_serial")


def purine_graph_op_elapsed_ms(g, op_id):
    ms = ctypes.c_float()
    _check(_lib.purine_graph_op_elapsed_ms(g, int(op_id), ctypes.byref(ms)), "purine_graph_op_elapsed_ms")
    return float(ms.value)


def purine_set_kernel_probe(start_event, stop_event):
    """start/stop: raw hipEvent_t handles (ints) or None."""
    _lib.purine_set_kernel_probe(start_event, stop_event)
