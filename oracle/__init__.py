"""numpy front end of the CPU oracle (`conv_oracle.c`).

TEST INFRASTRUCTURE ONLY: imported by tests/, by `__graft_entry__.smoke()` and by the
`cpu_baseline` leg of bench.py. The product package never imports this module.

Every function takes fp32 numpy arrays (bfloat16 data is passed as the fp32 values it denotes)
and returns fp64 results. Parity pins: see the tests in tests/test_oracle_*.py (closed forms,
brute force, a second lowering+matmul formulation, adjoint identities, finite differences).
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "conv_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")
_lib = None


def build(force=False):
    """Compile conv_oracle.c with gcc (-O2, OpenMP, no fast-math)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11",
                               "-Wall", "-o", _LIB, _SRC])
    return _LIB


class _Shape(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int64) for n in
                ("N", "C", "H", "W", "K", "R", "S", "sh", "sw", "ph", "pw")]


def _load():
    global _lib
    if _lib is None:
        # ORACLE_LIB_OVERRIDE: a library built elsewhere from a (deliberately altered) copy of the
        # source; used only by the test that checks that the pins notice planted mistakes
        override = os.environ.get("ORACLE_LIB_OVERRIDE")
        if not override:
            build()
        _lib = ctypes.CDLL(override or _LIB)
        _lib.oracle_out_extent.restype = ctypes.c_int64
        _lib.oracle_out_extent.argtypes = [ctypes.c_int64] * 4
        _lib.oracle_num_threads.restype = ctypes.c_int
    return _lib


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


def _p(a):
    return a.ctypes.data_as(ctypes.c_void_p)


def _pair(v):
    return (int(v), int(v)) if np.isscalar(v) else (int(v[0]), int(v[1]))


def num_threads():
    return int(_load().oracle_num_threads())


def out_extent(size, k, stride, pad):
    return int(_load().oracle_out_extent(size, k, stride, pad))


def _shape(x_shape, w_shape, stride, pad):
    N, C, H, W = (int(v) for v in x_shape)
    K, C2, R, S = (int(v) for v in w_shape)
    if C != C2:
        raise ValueError("channel mismatch")
    sh, sw = _pair(stride)
    ph, pw = _pair(pad)
    P, Q = out_extent(H, R, sh, ph), out_extent(W, S, sw, pw)
    if P <= 0 or Q <= 0:
        raise ValueError("empty or illegal convolution")
    return _Shape(N, C, H, W, K, R, S, sh, sw, ph, pw), (N, K, P, Q)


def out_shape(x_shape, w_shape, stride, pad):
    return _shape(x_shape, w_shape, stride, pad)[1]


def conv_fwd(x, w, stride=1, pad=0):
    x, w = _f32(x), _f32(w)
    g, ys = _shape(x.shape, w.shape, stride, pad)
    y = np.empty(ys, dtype=np.float64)
    _load().oracle_conv_fwd(ctypes.byref(g), _p(x), _p(w), _p(y))
    return y


def bias_fwd(y, b):
    """Returns y + b[k] broadcast over (n, p, q); y is not modified."""
    out = np.array(y, dtype=np.float64, order="C", copy=True)
    b = _f32(b)
    N, K = out.shape[0], out.shape[1]
    assert b.shape == (K,)
    _load().oracle_bias_fwd(_p(out), _p(b), ctypes.c_int64(N), ctypes.c_int64(K),
                            ctypes.c_int64(out.size // max(N * K, 1)))
    return out


def conv_bwd_data(dy, w, x_shape, stride=1, pad=0):
    dy, w = _f32(dy), _f32(w)
    g, ys = _shape(x_shape, w.shape, stride, pad)
    assert tuple(dy.shape) == ys, (dy.shape, ys)
    dx = np.empty(tuple(int(v) for v in x_shape), dtype=np.float64)
    _load().oracle_conv_bwd_data(ctypes.byref(g), _p(dy), _p(w), _p(dx))
    return dx


def conv_bwd_weight(x, dy, w_shape, stride=1, pad=0):
    x, dy = _f32(x), _f32(dy)
    g, ys = _shape(x.shape, w_shape, stride, pad)
    assert tuple(dy.shape) == ys, (dy.shape, ys)
    dw = np.empty(tuple(int(v) for v in w_shape), dtype=np.float64)
    _load().oracle_conv_bwd_weight(ctypes.byref(g), _p(x), _p(dy), _p(dw))
    return dw


def conv_bwd_weight_at(x, dy, w_shape, flat_idx, stride=1, pad=0):
    """dw at the given flat indices only (sampled parity on full-size layers)."""
    x, dy = _f32(x), _f32(dy)
    g, ys = _shape(x.shape, w_shape, stride, pad)
    assert tuple(dy.shape) == ys, (dy.shape, ys)
    idx = np.ascontiguousarray(flat_idx, dtype=np.int64)
    assert idx.min(initial=0) >= 0 and idx.max(initial=0) < int(np.prod(w_shape))
    out = np.empty(idx.shape, dtype=np.float64)
    _load().oracle_conv_bwd_weight_at(ctypes.byref(g), _p(x), _p(dy), _p(idx),
                                      ctypes.c_int64(idx.size), _p(out))
    return out


def bias_bwd(dy):
    dy = _f32(dy)
    N, K = dy.shape[0], dy.shape[1]
    db = np.empty((K,), dtype=np.float64)
    _load().oracle_bias_bwd(_p(dy), _p(db), ctypes.c_int64(N), ctypes.c_int64(K),
                            ctypes.c_int64(dy.size // max(N * K, 1)))
    return db


def relu_fwd(x):
    x = _f32(x)
    y = np.empty_like(x)
    _load().oracle_relu_fwd(_p(x), _p(y), ctypes.c_int64(x.size))
    return y


def relu_bwd(x, dy):
    x, dy = _f32(x), _f32(dy)
    assert x.shape == dy.shape
    dx = np.empty_like(x)
    _load().oracle_relu_bwd(_p(x), _p(dy), _p(dx), ctypes.c_int64(x.size))
    return dx


def maxpool_fwd(x, k, stride, pad):
    x = _f32(x)
    N, C, H, W = x.shape
    P, Q = out_extent(H, k, stride, pad), out_extent(W, k, stride, pad)
    if P <= 0 or Q <= 0:
        raise ValueError("empty pooling output")
    y = np.empty((N, C, P, Q), dtype=np.float32)
    arg = np.empty((N, C, P, Q), dtype=np.int32)
    _load().oracle_maxpool_fwd(_p(x), _p(y), _p(arg), ctypes.c_int64(N * C), ctypes.c_int64(H),
                               ctypes.c_int64(W), ctypes.c_int64(k), ctypes.c_int64(stride),
                               ctypes.c_int64(pad))
    return y, arg


def maxpool_bwd(dy, arg, x_shape):
    dy = _f32(dy)
    arg = np.ascontiguousarray(arg, dtype=np.int32)
    N, C, H, W = (int(v) for v in x_shape)
    assert dy.shape == arg.shape and dy.shape[:2] == (N, C)
    dx = np.empty((N, C, H, W), dtype=np.float64)
    _load().oracle_maxpool_bwd(_p(dy), _p(arg), _p(dx), ctypes.c_int64(N * C),
                               ctypes.c_int64(H * W), ctypes.c_int64(dy.shape[2] * dy.shape[3]))
    return dx


def concat_channels(tensors):
    """Channel concatenation (exact copy)."""
    return np.concatenate([np.asarray(t) for t in tensors], axis=1)


def fan_in_sum(tensors):
    """Gradient fan-in: elementwise sum in fp64, operands taken in the given order."""
    acc = np.zeros(np.shape(tensors[0]), dtype=np.float64)
    for t in tensors:
        acc = acc + np.asarray(t, dtype=np.float64)
    return acc


def sgd_update(w, dw, lr):
    """One SGD step on a parameter tensor (paper section 2.2, Figure 2(a): every iteration computes
    a modification of the parameters and applies it before the next one). The paper fixes no
    formula beyond that; the reading taken is the plain rule new = w - lr * dw, in fp64."""
    return np.asarray(w, dtype=np.float64) - float(lr) * np.asarray(dw, dtype=np.float64)


# ---- fully-connected layer and grouped convolution (the other layer types of the networks that the
# paper's section 3 discusses): plain definitions in fp64
def fc_fwd(x, w, b=None):
    """y[n,k] = sum_c x[n,c] * w[k,c] (+ b[k])."""
    y = np.asarray(x, dtype=np.float64) @ np.asarray(w, dtype=np.float64).T
    return y if b is None else y + np.asarray(b, dtype=np.float64)[None, :]


def fc_bwd_data(dy, w):
    """dx[n,c] = sum_k dy[n,k] * w[k,c]."""
    return np.asarray(dy, dtype=np.float64) @ np.asarray(w, dtype=np.float64)


def fc_bwd_weight(x, dy):
    """dw[k,c] = sum_n dy[n,k] * x[n,c]; db[k] = sum_n dy[n,k]."""
    dy64 = np.asarray(dy, dtype=np.float64)
    return dy64.T @ np.asarray(x, dtype=np.float64), dy64.sum(axis=0)


def _group_slices(C, K, groups):
    cg, kg = C // groups, K // groups
    return [(slice(g * cg, (g + 1) * cg), slice(g * kg, (g + 1) * kg)) for g in range(groups)]


def grouped_conv_fwd(x, w, groups, stride=1, pad=0):
    """Output channels of group g see only the input channels of group g; w is [K, C/groups, R, S]."""
    x, w = _f32(x), _f32(w)
    parts = [conv_fwd(x[:, cs], w[ks], stride, pad) for cs, ks in _group_slices(x.shape[1], w.shape[0], groups)]
    return np.concatenate(parts, axis=1)


def grouped_conv_bwd_data(dy, w, x_shape, groups, stride=1, pad=0):
    dy, w = _f32(dy), _f32(w)
    N, C, H, W = x_shape
    parts = [conv_bwd_data(dy[:, ks], w[ks], (N, C // groups, H, W), stride, pad)
             for cs, ks in _group_slices(C, w.shape[0], groups)]
    return np.concatenate(parts, axis=1)


def grouped_conv_bwd_weight(x, dy, w_shape, groups, stride=1, pad=0):
    x, dy = _f32(x), _f32(dy)
    K, Cg, R, S = w_shape
    parts = [conv_bwd_weight(x[:, cs], dy[:, ks], (K // groups, Cg, R, S), stride, pad)
             for cs, ks in _group_slices(x.shape[1], K, groups)]
    return np.concatenate(parts, axis=0)
