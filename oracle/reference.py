"""ctypes front of the fp64 C oracle, plus the model interpreter.

Test infrastructure only (see ``oracle.c``).  Arrays are numpy float64,
activations (N, C, H, W), convolution weights (K, C, R, S), FC weights
(Out, In).  A model (a ``workloads.Model`` table) is evaluated node by node
with no rounding in between; the flatten before the first FC is PyTorch's
(channel-major).
"""

import ctypes
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "liboracle.so")
_lib = None

_DP = ctypes.POINTER(ctypes.c_double)
_I = ctypes.c_int


def _load():
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            from . import build as _build
            _build.build()
        lib = ctypes.CDLL(_LIB_PATH)
        lib.oracle_out_dim.argtypes = [_I] * 4
        lib.oracle_out_dim.restype = _I
        lib.oracle_conv2d.argtypes = [_DP, _DP, _DP, _DP, _DP] + [_I] * 10
        lib.oracle_conv2d.restype = None
        lib.oracle_depthwise_conv2d.argtypes = [_DP, _DP, _DP, _DP] + [_I] * 9
        lib.oracle_depthwise_conv2d.restype = None
        lib.oracle_maxpool.argtypes = [_DP, _DP] + [_I] * 7
        lib.oracle_maxpool.restype = None
        lib.oracle_avgpool.argtypes = [_DP, _DP] + [_I] * 7
        lib.oracle_avgpool.restype = None
        lib.oracle_global_avgpool.argtypes = [_DP, _DP] + [_I] * 4
        lib.oracle_global_avgpool.restype = None
        lib.oracle_fc.argtypes = [_DP, _DP, _DP, _DP] + [_I] * 4
        lib.oracle_fc.restype = None
        lib.oracle_num_threads.argtypes = []
        lib.oracle_num_threads.restype = _I
        _lib = lib
    return _lib


def _f64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


def _p(a):
    return a.ctypes.data_as(_DP) if a is not None else None


def num_threads():
    return int(_load().oracle_num_threads())


def out_dim(n, k, stride, pad):
    return int(_load().oracle_out_dim(n, k, stride, pad))


def conv2d(x, w, b=None, stride=1, pad=0, relu=False, residual=None):
    """Convolution layer (paper Sec. 5: the executor's forward pass; PyTorch
    conventions).  x (N,C,H,W), w (K,C,R,S), b (K,), residual like the output."""
    lib = _load()
    x, w = _f64(x), _f64(w)
    N, C, H, W = x.shape
    K, C2, R, S = w.shape
    if C2 != C:
        raise ValueError("channel mismatch: x has %d, w has %d" % (C, C2))
    P, Q = out_dim(H, R, stride, pad), out_dim(W, S, stride, pad)
    if P <= 0 or Q <= 0:
        raise ValueError("empty output")
    b = _f64(b) if b is not None else None
    if b is not None and b.shape != (K,):
        raise ValueError("bias shape")
    residual = _f64(residual) if residual is not None else None
    if residual is not None and residual.shape != (N, K, P, Q):
        raise ValueError("residual shape")
    y = np.empty((N, K, P, Q), dtype=np.float64)
    lib.oracle_conv2d(_p(x), _p(w), _p(b), _p(residual), _p(y), N, C, H, W, K, R, S, stride, pad,
                      int(bool(relu)))
    return y


def _pool(fn, x, k, stride, pad):
    x = _f64(x)
    N, C, H, W = x.shape
    if pad >= k:
        raise ValueError("pad must be smaller than the window")
    P, Q = out_dim(H, k, stride, pad), out_dim(W, k, stride, pad)
    if P <= 0 or Q <= 0:
        raise ValueError("empty output")
    y = np.empty((N, C, P, Q), dtype=np.float64)
    fn(_p(x), _p(y), N, C, H, W, k, stride, pad)
    return y


def maxpool(x, k, stride, pad=0):
    return _pool(_load().oracle_maxpool, x, k, stride, pad)


def avgpool(x, k, stride, pad=0):
    return _pool(_load().oracle_avgpool, x, k, stride, pad)


def global_avgpool(x):
    x = _f64(x)
    N, C, H, W = x.shape
    y = np.empty((N, C), dtype=np.float64)
    _load().oracle_global_avgpool(_p(x), _p(y), N, C, H, W)
    return y


def fc(x, w, b=None, relu=False):
    x, w = _f64(x), _f64(w)
    N, In = x.shape
    Out, In2 = w.shape
    if In2 != In:
        raise ValueError("feature mismatch: x has %d, w has %d" % (In, In2))
    b = _f64(b) if b is not None else None
    y = np.empty((N, Out), dtype=np.float64)
    _load().oracle_fc(_p(x), _p(w), _p(b), _p(y), N, In, Out, int(bool(relu)))
    return y


def depthwise_conv2d(x, w, b=None, stride=1, pad=0, relu=False):
    """Depthwise convolution layer (MobileNet blocks of the paper's SSD-MobileNet,
    Table 4).  x (N,C,H,W), w (C,1,R,S) as PyTorch stores a grouped filter, b (C,)."""
    lib = _load()
    x, w = _f64(x), _f64(w)
    N, C, H, W = x.shape
    if w.ndim != 4 or w.shape[0] != C or w.shape[1] != 1:
        raise ValueError("depthwise filter must be (C, 1, R, S)")
    R, S = w.shape[2], w.shape[3]
    P, Q = out_dim(H, R, stride, pad), out_dim(W, S, stride, pad)
    if P <= 0 or Q <= 0:
        raise ValueError("empty output")
    b = _f64(b) if b is not None else None
    if b is not None and b.shape != (C,):
        raise ValueError("bias shape")
    y = np.empty((N, C, P, Q), dtype=np.float64)
    lib.oracle_depthwise_conv2d(_p(x), _p(w), _p(b), _p(y), N, C, H, W, R, S, stride, pad, int(bool(relu)))
    return y


def run_model(model, params, x, keep=False, storage=None):
    """Forward pass of a ``workloads.Model`` on batch ``x`` (N,C,H,W) in fp64.

    Returns the output tensor, or with ``keep`` the dict of every named
    tensor (for per-layer comparisons).  ``storage``, if given, is applied to
    the output of every layer that computes (not to pooling by maximum or
    concatenation, which only move values): a test passes the rounding of an
    implementation's tensor format there to tell the error of the format from
    the error of the arithmetic.  The arithmetic of every layer stays fp64."""
    keep_as = storage if storage is not None else (lambda a: a)
    t = {"x": _f64(x)}
    for nd in model.nodes:
        a = nd.attr
        if nd.op == "conv":
            w, b = params[nd.name]
            res = t[a["residual"]] if a["residual"] else None
            t[nd.dst] = keep_as(conv2d(t[nd.src], w, b, a["stride"], a["pad"], a["relu"], res))
        elif nd.op == "dwconv":
            w, b = params[nd.name]
            t[nd.dst] = keep_as(depthwise_conv2d(t[nd.src], w, b, a["stride"], a["pad"], a["relu"]))
        elif nd.op == "maxpool":
            t[nd.dst] = maxpool(t[nd.src], a["k"], a["stride"], a["pad"])
        elif nd.op == "gavgpool":
            t[nd.dst] = keep_as(global_avgpool(t[nd.src]))
        elif nd.op == "fc":
            w, b = params[nd.name]
            src = t[nd.src]
            t[nd.dst] = keep_as(fc(src.reshape(src.shape[0], -1), w, b, a["relu"]))
        elif nd.op == "concat":
            t[nd.dst] = np.concatenate([t[s] for s in nd.src], axis=1)
        else:
            raise ValueError("unknown node kind %r" % (nd.op,))
    return t if keep else t[model.out]


def model_flops(model):
    """Multiply-add work of one image as 2*MAC, padding taps counted, split
    into (conv, fc).  Spatial sizes come from the oracle's own output-size
    rule."""
    shapes = {"x": tuple(model.in_shape)}
    conv = fcf = 0
    for nd in model.nodes:
        a = nd.attr
        if nd.op == "conv":
            C, H, W = shapes[nd.src]
            assert C == a["C"], (nd.name, C, a["C"])
            P, Q = out_dim(H, a["k"], a["stride"], a["pad"]), out_dim(W, a["k"], a["stride"], a["pad"])
            conv += 2 * P * Q * a["K"] * C * a["k"] * a["k"]
            shapes[nd.dst] = (a["K"], P, Q)
            if a["residual"]:
                assert shapes[a["residual"]] == shapes[nd.dst], nd.name
        elif nd.op == "dwconv":
            C, H, W = shapes[nd.src]
            assert C == a["C"], (nd.name, C, a["C"])
            P, Q = out_dim(H, a["k"], a["stride"], a["pad"]), out_dim(W, a["k"], a["stride"], a["pad"])
            conv += 2 * P * Q * C * a["k"] * a["k"]
            shapes[nd.dst] = (C, P, Q)
        elif nd.op == "maxpool":
            C, H, W = shapes[nd.src]
            shapes[nd.dst] = (C, out_dim(H, a["k"], a["stride"], a["pad"]),
                              out_dim(W, a["k"], a["stride"], a["pad"]))
        elif nd.op == "gavgpool":
            shapes[nd.dst] = (shapes[nd.src][0], 1, 1)
        elif nd.op == "fc":
            C, H, W = shapes[nd.src]
            assert C * H * W == a["In"], (nd.name, C * H * W, a["In"])
            fcf += 2 * a["In"] * a["Out"]
            shapes[nd.dst] = (a["Out"], 1, 1)
        elif nd.op == "concat":
            parts = [shapes[s] for s in nd.src]
            assert all(p[1:] == parts[0][1:] for p in parts), nd.name
            shapes[nd.dst] = (sum(p[0] for p in parts),) + parts[0][1:]
    return conv, fcf


def model_params(model):
    """Number of weights plus biases of a model."""
    n = 0
    for nd in model.nodes:
        if nd.op == "conv":
            a = nd.attr
            n += a["K"] * a["C"] * a["k"] * a["k"] + a["K"]
        elif nd.op == "dwconv":
            a = nd.attr
            n += a["C"] * a["k"] * a["k"] + a["C"]
        elif nd.op == "fc":
            n += nd.attr["Out"] * nd.attr["In"] + nd.attr["Out"]
    return n


def rel_err(got, ref):
    """Normwise relative error ||got - ref||_2 / ||ref||_2 over the whole
    tensor and the largest per-image value (axis 0 is the batch)."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    d = (got - ref).reshape(ref.shape[0], -1)
    r = ref.reshape(ref.shape[0], -1)
    whole = np.linalg.norm(d) / max(np.linalg.norm(r), 1e-300)
    per = np.linalg.norm(d, axis=1) / np.maximum(np.linalg.norm(r, axis=1), 1e-300)
    return float(whole), float(per.max())
