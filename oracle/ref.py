"""ctypes front end of the C oracle (test infrastructure; never on the product path).

Every function takes numpy arrays on the host and returns a new numpy array.  The
quantisation parameters are read from any object with the attributes
fl_x, fl_w, fl_y, clip_lo, clip_hi, x_type, y_type and, if a residual is given,
res_type and fl_res; the *_type attributes are the strings 'u8', 's8', 's32'.

The whole-network runner at the bottom walks a layer list (see the workload
generators) in execution order and calls the C oracle once per layer; it holds no
arithmetic of its own.
"""
import ctypes
import os
from concurrent.futures import ThreadPoolExecutor

import numpy as np

from . import build as _build

_TYPES = {"u8": 0, "s8": 1, "s32": 2}
_NP = {"u8": np.uint8, "s8": np.int8, "s32": np.int32}
ERRORS = {0: "OK", 1: "NULL", 2: "SHAPE", 3: "FL", 4: "CLIP", 5: "DTYPE", 6: "ACC_OVERFLOW"}


class OracleError(RuntimeError):
    def __init__(self, code):
        super().__init__("oracle error %d (%s)" % (code, ERRORS.get(code, "?")))
        self.code = code


class _Quant(ctypes.Structure):
    _fields_ = [("fl_x", ctypes.c_int32), ("fl_w", ctypes.c_int32), ("fl_y", ctypes.c_int32),
                ("clip_lo", ctypes.c_int32), ("clip_hi", ctypes.c_int32),
                ("x_type", ctypes.c_int32), ("y_type", ctypes.c_int32),
                ("res", ctypes.c_void_p), ("res_type", ctypes.c_int32),
                ("fl_res", ctypes.c_int32)]


_lib = None


def lib():
    global _lib
    if _lib is None:
        # F8REF_LIB selects another build of the same source (the sanitizer build of the tests)
        path = os.environ.get("F8REF_LIB") or _build.build(force=False)
        L = ctypes.CDLL(path)
        L.f8ref_shift_round.restype = ctypes.c_int64
        L.f8ref_shift_round.argtypes = [ctypes.c_int64, ctypes.c_int]
        vp, ip = ctypes.c_void_p, ctypes.c_int
        qp = ctypes.POINTER(_Quant)
        L.f8ref_gemm_fixed.argtypes = [vp, vp, vp, vp, ip, ip, ip, qp]
        L.f8ref_conv2d_fixed.argtypes = [vp, vp, vp, vp] + [ip] * 11 + [qp]
        L.f8ref_dwconv_fixed.argtypes = [vp, vp, vp, vp] + [ip] * 10 + [qp]
        L.f8ref_maxpool.argtypes = [vp, vp] + [ip] * 11
        L.f8ref_global_pool_fixed.argtypes = [vp, vp, ip, ip, ip, ip, qp]
        _lib = L
    return _lib


def shift_round(a: int, s: int) -> int:
    return int(lib().f8ref_shift_round(int(a), int(s)))


def _ptr(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _as(a, kind):
    a = np.ascontiguousarray(a)
    if a.dtype != _NP[kind]:
        raise TypeError("expected %s array, got %s" % (kind, a.dtype))
    return a


def _quant(q, res):
    c = _Quant()
    c.fl_x, c.fl_w, c.fl_y = int(q.fl_x), int(q.fl_w), int(q.fl_y)
    c.clip_lo, c.clip_hi = int(q.clip_lo), int(q.clip_hi)
    c.x_type, c.y_type = _TYPES[q.x_type], _TYPES[q.y_type]
    keep = None
    if res is not None:
        keep = _as(res, q.res_type)
        c.res = keep.ctypes.data
        c.res_type = _TYPES[q.res_type]
        c.fl_res = int(q.fl_res)
    return c, keep


def _check(rc):
    if rc != 0:
        raise OracleError(rc)


def out_hw(H, W, R, S, stride, pad):
    sh, sw = stride
    ph, pw = pad
    P = 0 if H + 2 * ph - R < 0 else (H + 2 * ph - R) // sh + 1
    Q = 0 if W + 2 * pw - S < 0 else (W + 2 * pw - S) // sw + 1
    return P, Q


def gemm_fixed(x, w, bias, q, res=None):
    x = _as(x, q.x_type)
    w = _as(w, "s8")
    bias = None if bias is None else _as(bias, "s32")
    M, K = x.shape
    N = w.shape[0]
    assert w.shape == (N, K)
    y = np.empty((M, N), _NP[q.y_type])
    c, keep = _quant(q, res)
    if keep is not None:
        assert keep.shape == y.shape
    _check(lib().f8ref_gemm_fixed(_ptr(x), _ptr(w), _ptr(bias), _ptr(y), M, K, N, ctypes.byref(c)))
    return y


def conv2d_fixed(x, w, bias, q, stride=(1, 1), pad=(0, 0), res=None):
    x = _as(x, q.x_type)
    w = _as(w, "s8")
    bias = None if bias is None else _as(bias, "s32")
    B, H, W, Cin = x.shape
    Cout, R, S, Cin2 = w.shape
    assert Cin == Cin2
    P, Q = out_hw(H, W, R, S, stride, pad)
    y = np.empty((B, P, Q, Cout), _NP[q.y_type])
    c, keep = _quant(q, res)
    if keep is not None:
        assert keep.shape == y.shape
    _check(lib().f8ref_conv2d_fixed(_ptr(x), _ptr(w), _ptr(bias), _ptr(y), B, H, W, Cin, Cout, R, S,
                                    stride[0], stride[1], pad[0], pad[1], ctypes.byref(c)))
    return y


def dwconv_fixed(x, w, bias, q, stride=(1, 1), pad=(0, 0), res=None):
    x = _as(x, q.x_type)
    w = _as(w, "s8")
    bias = None if bias is None else _as(bias, "s32")
    B, H, W, C = x.shape
    R, S, C2 = w.shape
    assert C == C2
    P, Q = out_hw(H, W, R, S, stride, pad)
    y = np.empty((B, P, Q, C), _NP[q.y_type])
    c, keep = _quant(q, res)
    if keep is not None:
        assert keep.shape == y.shape
    _check(lib().f8ref_dwconv_fixed(_ptr(x), _ptr(w), _ptr(bias), _ptr(y), B, H, W, C, R, S,
                                    stride[0], stride[1], pad[0], pad[1], ctypes.byref(c)))
    return y


def maxpool(x, kind, window=(3, 3), stride=(2, 2), pad=(1, 1)):
    x = _as(x, kind)
    B, H, W, C = x.shape
    P, Q = out_hw(H, W, window[0], window[1], stride, pad)
    y = np.empty((B, P, Q, C), _NP[kind])
    _check(lib().f8ref_maxpool(_ptr(x), _ptr(y), B, H, W, C, window[0], window[1],
                               stride[0], stride[1], pad[0], pad[1], _TYPES[kind]))
    return y


def global_pool_fixed(x, q):
    x = _as(x, q.x_type)
    B, H, W, C = x.shape
    y = np.empty((B, C), _NP[q.y_type])
    c, _ = _quant(q, None)
    _check(lib().f8ref_global_pool_fixed(_ptr(x), _ptr(y), B, H, W, C, ctypes.byref(c)))
    return y


# ---------------------------------------------------------------------------------
# whole-network runner: one oracle call per layer, in execution order
# ---------------------------------------------------------------------------------

class _SecondFormat:
    """The quantisation record of a layer with its output format replaced by the second one."""

    def __init__(self, L):
        self.fl_x, self.fl_w, self.x_type = L.fl_x, L.fl_w, L.x_type
        self.res_type, self.fl_res = L.res_type, L.fl_res
        self.fl_y, self.clip_lo, self.clip_hi, self.y_type = L.fl_y2, L.clip_lo2, L.clip_hi2, L.y2_type


def conv2d_fixed_dual(x, w, bias, q, stride=(1, 1), pad=(0, 0), res=None):
    """A layer with two output formats (paper Sec. 4.3, children with private fractional
    lengths): by definition each output is the layer evaluated with that format, so the oracle
    simply evaluates it twice."""
    return (conv2d_fixed(x, w, bias, q, stride, pad, res),
            conv2d_fixed(x, w, bias, _SecondFormat(q), stride, pad, res))


def run_layer(L, x, res=None):
    """Run one layer description on host arrays through the C oracle."""
    if L.op == "conv":
        return conv2d_fixed(x, L.w, L.bias, L, (L.stride, L.stride), (L.pad, L.pad), res)
    if L.op == "dwconv":
        return dwconv_fixed(x, L.w, L.bias, L, (L.stride, L.stride), (L.pad, L.pad), res)
    if L.op == "maxpool":
        return maxpool(x, L.x_type, (L.R, L.S), (L.stride, L.stride), (L.pad, L.pad))
    if L.op == "gpool":
        y = global_pool_fixed(x, L)
        return y.reshape(y.shape[0], 1, 1, y.shape[1])
    raise ValueError(L.op)


def _SecondFormat_layer(L):
    """Copy of a layer description whose output format is the second one."""
    import copy
    M = copy.copy(L)
    M.fl_y, M.clip_lo, M.clip_hi, M.y_type = L.fl_y2, L.clip_lo2, L.clip_hi2, L.y2_type
    M.dst2 = -1
    return M


def run_network(net, x, keep_all=False):
    """Evaluate the layer list `net.layers` on the batch x (NHWC numpy array).

    Tensor ids: 0 is the network input; layer i reads tensor L.src (and L.res, if >= 0)
    and writes tensor L.dst.  Returns the last tensor, or every tensor if keep_all.
    """
    t = {0: x}
    for L in net.layers:
        res = t[L.res] if L.res >= 0 else None
        t[L.dst] = run_layer(L, t[L.src], res)
        if getattr(L, "dst2", -1) > 0:
            t[L.dst2] = run_layer(_SecondFormat_layer(L), t[L.src], res)
    return t if keep_all else t[net.layers[-1].dst]


def run_network_parallel(net, x, workers, keep_all=False):
    """Same as run_network with the batch split image by image over `workers` host
    threads (images are independent; the C oracle itself stays single-threaded and
    releases the interpreter lock while it runs)."""
    B = x.shape[0]
    workers = max(1, min(workers, B))
    parts = [x[i::workers] for i in range(workers)]
    with ThreadPoolExecutor(workers) as ex:
        outs = list(ex.map(lambda xs: run_network(net, np.ascontiguousarray(xs), keep_all), parts))

    def merge(arrs):
        full = np.empty((B,) + arrs[0].shape[1:], arrs[0].dtype)
        for i, a in enumerate(arrs):
            full[i::workers] = a
        return full

    if keep_all:
        return {k: merge([o[k] for o in outs]) for k in outs[0]}
    return merge(outs)
