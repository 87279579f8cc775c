"""ctypes binding of libf8.so: the same names as the C ABI, argument marshalling only.

Tensors are torch tensors on the GPU (torch is used for device memory and streams); the
binding passes `tensor.data_ptr()` and the current torch stream to the library.  Every
step of the layer arithmetic runs inside the library's kernels.  If the library has not
been built, loading raises: there is no fallback path.
"""
import ctypes
import os

import torch

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libf8.so")

F8_U8, F8_S8, F8_S32 = 0, 1, 2
F8_OP_CONV, F8_OP_DWCONV, F8_OP_MAXPOOL, F8_OP_GPOOL = 0, 1, 2, 3
_TYPES = {"u8": F8_U8, "s8": F8_S8, "s32": F8_S32}
_OPS = {"conv": F8_OP_CONV, "dwconv": F8_OP_DWCONV, "maxpool": F8_OP_MAXPOOL, "gpool": F8_OP_GPOOL}
TORCH_DTYPE = {"u8": torch.uint8, "s8": torch.int8, "s32": torch.int32,
               F8_U8: torch.uint8, F8_S8: torch.int8, F8_S32: torch.int32}

EXPORTS = [
    "f8_gemm_fixed", "f8_conv2d_fixed", "f8_conv2d_fixed_noalloc", "f8_conv2d_fixed_ws", "f8_conv_workspace_bytes", "f8_conv2d_fixed_dual", "f8_dwconv_fixed", "f8_maxpool", "f8_global_pool_fixed",
    "f8_chain_create", "f8_chain_workspace_bytes", "f8_chain_prepare", "f8_chain_run",
    "f8_chain_tensor", "f8_chain_set_keep_all", "f8_chain_set_fusion", "f8_chain_set_streams", "f8_chain_destroy",
    "f8_chain_num_layers", "f8_chain_layer_info", "f8_chain_profile",
    "f8_clip_from_alpha", "f8_status_str", "f8_release_scratch", "f8_abi_version", "f8_copy_bytes",
    "f8_tuning_set", "f8_tuning_get", "f8_mfma_i8_yardstick", "f8_mfma_i8_yardstick_operands",
    "f8_fix_quant_f32", "f8_fix_quant_code", "f8_pact_f32", "f8_pact_fix_f32", "f8_eta_fix", "f8_opt_fl",
    "f8_tensor_stats_f32", "f8_quant_error_f32", "f8_fold_work_doubles", "f8_fold_conv_bn",
]
F8_STATS_WORK_DOUBLES = 4096


class F8Error(RuntimeError):
    def __init__(self, code, where):
        msg = lib().f8_status_str(code).decode()
        super().__init__("%s: f8 status %d (%s)" % (where, code, msg))
        self.code = code


class f8_quant(ctypes.Structure):
    _fields_ = [("fl_x", ctypes.c_int32), ("fl_w", ctypes.c_int32), ("fl_y", ctypes.c_int32),
                ("clip_lo", ctypes.c_int32), ("clip_hi", ctypes.c_int32),
                ("x_type", ctypes.c_int32), ("y_type", ctypes.c_int32),
                ("res", ctypes.c_void_p), ("res_type", ctypes.c_int32), ("fl_res", ctypes.c_int32)]


class f8_requant2(ctypes.Structure):
    _fields_ = [("fl_y", ctypes.c_int32), ("clip_lo", ctypes.c_int32), ("clip_hi", ctypes.c_int32),
                ("y_type", ctypes.c_int32)]


class f8_layer_desc(ctypes.Structure):
    _fields_ = [("op", ctypes.c_int32), ("src", ctypes.c_int32), ("dst", ctypes.c_int32),
                ("res", ctypes.c_int32), ("Cin", ctypes.c_int32), ("Cout", ctypes.c_int32),
                ("R", ctypes.c_int32), ("S", ctypes.c_int32),
                ("stride_h", ctypes.c_int32), ("stride_w", ctypes.c_int32),
                ("pad_h", ctypes.c_int32), ("pad_w", ctypes.c_int32),
                ("q", f8_quant), ("w", ctypes.c_void_p), ("bias", ctypes.c_void_p),
                ("dst2", ctypes.c_int32), ("q2", f8_requant2)]


class f8_stats(ctypes.Structure):
    _fields_ = [("mean", ctypes.c_double), ("std", ctypes.c_double),
                ("fl_signed", ctypes.c_int32), ("fl_unsigned", ctypes.c_int32)]


class f8_fold_desc(ctypes.Structure):
    _fields_ = [("cout", ctypes.c_int32), ("k", ctypes.c_int32),
                ("eta_in", ctypes.c_double), ("eta_out", ctypes.c_double),
                ("fl_x", ctypes.c_int32), ("fl_w", ctypes.c_int32)]


_lib = None


def lib():
    """Load libf8.so (raises if it was not built) and declare the signatures."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError("libf8.so is missing: build it with `python -m paper_2202_05239_amd.build` "
                           "(there is no fallback implementation)")
    L = ctypes.CDLL(LIB_PATH)
    vp, i32, qp = ctypes.c_void_p, ctypes.c_int, ctypes.POINTER(f8_quant)
    L.f8_gemm_fixed.argtypes = [vp, vp, vp, vp, i32, i32, i32, qp, vp]
    L.f8_conv2d_fixed.argtypes = [vp, vp, vp, vp] + [i32] * 11 + [qp, vp]
    L.f8_conv2d_fixed_noalloc.argtypes = [vp, vp, vp, vp] + [i32] * 11 + [qp, vp]
    L.f8_conv2d_fixed_ws.argtypes = [vp, vp, vp, vp] + [i32] * 11 + [qp, vp, ctypes.c_size_t, vp]
    L.f8_conv_workspace_bytes.argtypes = [i32]
    L.f8_conv_workspace_bytes.restype = ctypes.c_size_t
    L.f8_conv2d_fixed_dual.argtypes = [vp, vp, vp, vp, vp] + [i32] * 11 + [qp, ctypes.POINTER(f8_requant2), vp]
    L.f8_dwconv_fixed.argtypes = [vp, vp, vp, vp] + [i32] * 10 + [qp, vp]
    L.f8_maxpool.argtypes = [vp, vp] + [i32] * 11 + [vp]
    L.f8_global_pool_fixed.argtypes = [vp, vp, i32, i32, i32, i32, qp, vp]
    L.f8_chain_create.argtypes = [ctypes.POINTER(f8_layer_desc), i32, i32, i32, i32, i32,
                                  ctypes.POINTER(vp)]
    L.f8_chain_workspace_bytes.argtypes = [vp, i32, ctypes.POINTER(ctypes.c_size_t)]
    L.f8_chain_prepare.argtypes = [vp, vp, i32, vp]
    L.f8_chain_run.argtypes = [vp, vp, vp, vp, i32, vp]
    L.f8_chain_tensor.argtypes = [vp, i32, vp, i32, ctypes.POINTER(vp)] + [ctypes.POINTER(i32)] * 5
    L.f8_chain_set_keep_all.argtypes = [vp, i32]
    L.f8_chain_set_fusion.argtypes = [vp, i32]
    L.f8_chain_set_streams.argtypes = [vp, i32]
    L.f8_chain_destroy.argtypes = [vp]
    L.f8_chain_num_layers.argtypes = [vp]
    L.f8_chain_layer_info.argtypes = [vp, i32, i32, ctypes.c_char_p, i32, ctypes.POINTER(ctypes.c_double),
                                      ctypes.POINTER(ctypes.c_double)]
    L.f8_chain_profile.argtypes = [vp, vp, vp, vp, i32, vp, i32, ctypes.POINTER(ctypes.c_float)]
    L.f8_chain_destroy.restype = None
    L.f8_clip_from_alpha.argtypes = [ctypes.c_double, i32, i32]
    L.f8_clip_from_alpha.restype = ctypes.c_int32
    L.f8_status_str.argtypes = [i32]
    L.f8_status_str.restype = ctypes.c_char_p
    L.f8_copy_bytes.argtypes = [vp, vp, ctypes.c_size_t, vp]
    L.f8_release_scratch.restype = None
    sz, f32, f64 = ctypes.c_size_t, ctypes.c_float, ctypes.c_double
    L.f8_fix_quant_f32.argtypes = [vp, vp, sz, i32, i32, vp]
    L.f8_fix_quant_code.argtypes = [vp, vp, sz, i32, i32, vp]
    L.f8_pact_f32.argtypes = [vp, vp, sz, f32, vp]
    L.f8_pact_fix_f32.argtypes = [vp, vp, sz, f32, i32, vp]
    L.f8_eta_fix.argtypes = [f64, i32]
    L.f8_eta_fix.restype = f64
    L.f8_opt_fl.argtypes = [f64, i32]
    L.f8_tensor_stats_f32.argtypes = [vp, sz, vp, vp, vp]
    L.f8_quant_error_f32.argtypes = [vp, sz, i32, i32, vp, vp, vp]
    L.f8_fold_work_doubles.argtypes = [i32]
    L.f8_fold_work_doubles.restype = sz
    L.f8_fold_conv_bn.argtypes = [vp] * 5 + [ctypes.POINTER(f8_fold_desc)] + [vp] * 5
    L.f8_mfma_i8_yardstick.argtypes = [vp, i32, ctypes.POINTER(ctypes.c_double), vp]
    L.f8_mfma_i8_yardstick_operands.argtypes = [vp, i32, ctypes.c_uint32, ctypes.POINTER(ctypes.c_double), vp]
    L.f8_tuning_set.argtypes = [ctypes.c_char_p, i32]
    L.f8_tuning_get.argtypes = [ctypes.c_char_p]
    L.f8_abi_version.restype = ctypes.c_int
    if L.f8_abi_version() != 3:
        raise RuntimeError("libf8.so has ABI version %d, binding expects 3" % L.f8_abi_version())
    _lib = L
    return L


F8_YARDSTICK_SINK_INTS = 512 * 256


def f8_mfma_i8_yardstick(sink, iters):
    """One launch of the register-only int8 matrix-instruction loop; returns its operation count."""
    assert sink.numel() >= F8_YARDSTICK_SINK_INTS and sink.dtype == torch.int32
    ops = ctypes.c_double()
    _check(lib().f8_mfma_i8_yardstick(_ptr(sink), int(iters), ctypes.byref(ops), _stream()), "f8_mfma_i8_yardstick")
    return ops.value


def f8_mfma_i8_yardstick_operands(sink, iters, seed):
    """The same loop with pseudo-random operand bytes (seed != 0); returns its operation count."""
    assert sink.numel() >= F8_YARDSTICK_SINK_INTS and sink.dtype == torch.int32
    ops = ctypes.c_double()
    _check(lib().f8_mfma_i8_yardstick_operands(_ptr(sink), int(iters), int(seed), ctypes.byref(ops), _stream()),
           "f8_mfma_i8_yardstick_operands")
    return ops.value


def f8_tuning_set(name, value):
    """Set one of the library's tuning switches (kernel choice only, never results)."""
    if lib().f8_tuning_set(name.encode(), int(value)) != 0:
        raise ValueError("unknown tuning switch %r" % name)


def f8_tuning_get(name):
    return lib().f8_tuning_get(name.encode())


def _check(rc, where):
    if rc != 0:
        raise F8Error(rc, where)


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def make_quant(q, res=None):
    """f8_quant from any record with fl_x, fl_w, fl_y, clip_lo, clip_hi, x_type, y_type
    (and res_type, fl_res when a residual tensor is given)."""
    c = f8_quant()
    c.fl_x, c.fl_w, c.fl_y = int(q.fl_x), int(q.fl_w), int(q.fl_y)
    c.clip_lo, c.clip_hi = int(q.clip_lo), int(q.clip_hi)
    c.x_type, c.y_type = _TYPES[q.x_type], _TYPES[q.y_type]
    c.res = None
    if res is not None:
        c.res = res.data_ptr()
        c.res_type, c.fl_res = _TYPES[q.res_type], int(q.fl_res)
    return c


def f8_gemm_fixed(x, w, bias, y, q, res=None):
    """y[M][N] = layer(x[M][K], w[N][K], bias[N]); all tensors on the GPU, y preallocated."""
    M, K = x.shape
    N = w.shape[0]
    c = make_quant(q, res)
    _check(lib().f8_gemm_fixed(_ptr(x), _ptr(w), _ptr(bias), _ptr(y), M, K, N, ctypes.byref(c), _stream()),
           "f8_gemm_fixed")
    return y


def f8_conv2d_fixed(x, w, bias, y, q, stride=(1, 1), pad=(0, 0), res=None):
    """x NHWC, w [Cout][R][S][Cin], y NHWC preallocated."""
    B, H, W, Cin = x.shape
    Cout, R, S, _ = w.shape
    c = make_quant(q, res)
    _check(lib().f8_conv2d_fixed(_ptr(x), _ptr(w), _ptr(bias), _ptr(y), B, H, W, Cin, Cout, R, S,
                                 stride[0], stride[1], pad[0], pad[1], ctypes.byref(c), _stream()),
           "f8_conv2d_fixed")
    return y


def f8_conv2d_fixed_ws(x, w, bias, y, q, workspace, stride=(1, 1), pad=(0, 0), res=None, stream=None):
    """f8_conv2d_fixed with caller-supplied scratch (a uint8 tensor of f8_conv_workspace_bytes(Cout) bytes)."""
    B, H, W, Cin = x.shape
    Cout, R, S, _ = w.shape
    c = make_quant(q, res)
    st = _stream() if stream is None else ctypes.c_void_p(stream.cuda_stream)
    _check(lib().f8_conv2d_fixed_ws(_ptr(x), _ptr(w), _ptr(bias), _ptr(y), B, H, W, Cin, Cout, R, S, stride[0], stride[1],
                                    pad[0], pad[1], ctypes.byref(c), _ptr(workspace), workspace.numel(), st),
           "f8_conv2d_fixed_ws")
    return y


def f8_conv2d_fixed_noalloc(x, w, bias, y, q, stride=(1, 1), pad=(0, 0), res=None):
    """f8_conv2d_fixed through the entry point that allocates nothing (scratch inside the library)."""
    B, H, W, Cin = x.shape
    Cout, R, S, _ = w.shape
    c = make_quant(q, res)
    _check(lib().f8_conv2d_fixed_noalloc(_ptr(x), _ptr(w), _ptr(bias), _ptr(y), B, H, W, Cin, Cout, R, S,
                                         stride[0], stride[1], pad[0], pad[1], ctypes.byref(c), _stream()),
           "f8_conv2d_fixed_noalloc")
    return y


def make_requant2(q):
    """f8_requant2 from a record with fl_y2, clip_lo2, clip_hi2, y2_type."""
    c = f8_requant2()
    c.fl_y, c.clip_lo, c.clip_hi, c.y_type = int(q.fl_y2), int(q.clip_lo2), int(q.clip_hi2), _TYPES[q.y2_type]
    return c


def f8_conv2d_fixed_dual(x, w, bias, y, y2, q, stride=(1, 1), pad=(0, 0), res=None):
    """f8_conv2d_fixed with a second output y2 in the format q.fl_y2 / clip_lo2 / clip_hi2 / y2_type."""
    B, H, W, Cin = x.shape
    Cout, R, S, _ = w.shape
    c = make_quant(q, res)
    c2 = make_requant2(q)
    _check(lib().f8_conv2d_fixed_dual(_ptr(x), _ptr(w), _ptr(bias), _ptr(y), _ptr(y2), B, H, W, Cin, Cout, R, S,
                                      stride[0], stride[1], pad[0], pad[1], ctypes.byref(c), ctypes.byref(c2),
                                      _stream()), "f8_conv2d_fixed_dual")
    return y, y2


def f8_dwconv_fixed(x, w, bias, y, q, stride=(1, 1), pad=(0, 0), res=None):
    """x NHWC, w [R][S][C], y NHWC preallocated."""
    B, H, W, C = x.shape
    R, S, _ = w.shape
    c = make_quant(q, res)
    _check(lib().f8_dwconv_fixed(_ptr(x), _ptr(w), _ptr(bias), _ptr(y), B, H, W, C, R, S,
                                 stride[0], stride[1], pad[0], pad[1], ctypes.byref(c), _stream()),
           "f8_dwconv_fixed")
    return y


def f8_maxpool(x, y, kind, window=(3, 3), stride=(2, 2), pad=(1, 1)):
    B, H, W, C = x.shape
    _check(lib().f8_maxpool(_ptr(x), _ptr(y), B, H, W, C, window[0], window[1], stride[0], stride[1],
                            pad[0], pad[1], _TYPES[kind], _stream()), "f8_maxpool")
    return y


def f8_global_pool_fixed(x, y, q):
    B, H, W, C = x.shape
    c = make_quant(q)
    _check(lib().f8_global_pool_fixed(_ptr(x), _ptr(y), B, H, W, C, ctypes.byref(c), _stream()),
           "f8_global_pool_fixed")
    return y


def f8_clip_from_alpha(alpha, fl_y, is_signed=False):
    return int(lib().f8_clip_from_alpha(float(alpha), int(fl_y), int(bool(is_signed))))


def f8_copy_bytes(src, dst):
    """Plain streaming copy of src into dst (same byte size, a multiple of 16)."""
    n = src.numel() * src.element_size()
    _check(lib().f8_copy_bytes(_ptr(src), _ptr(dst), n, _stream()), "f8_copy_bytes")
    return dst


# ---- upstream of the integer layers (float32 tensors on the GPU) ------------------------------

def _f32(t):
    if t.dtype != torch.float32 or not t.is_contiguous():
        raise TypeError("expected a contiguous float32 tensor")
    return t


def f8_fix_quant_f32(x, fl, is_signed, out=None):
    out = torch.empty_like(x) if out is None else out
    _check(lib().f8_fix_quant_f32(_ptr(_f32(x)), _ptr(_f32(out)), x.numel(), int(fl), int(bool(is_signed)),
                                  _stream()), "f8_fix_quant_f32")
    return out


def f8_fix_quant_code(x, fl, is_signed, out=None):
    if out is None:
        out = torch.empty(x.shape, dtype=torch.int8 if is_signed else torch.uint8, device=x.device)
    _check(lib().f8_fix_quant_code(_ptr(_f32(x)), _ptr(out), x.numel(), int(fl), int(bool(is_signed)),
                                   _stream()), "f8_fix_quant_code")
    return out


def f8_pact_f32(x, alpha, out=None):
    out = torch.empty_like(x) if out is None else out
    _check(lib().f8_pact_f32(_ptr(_f32(x)), _ptr(_f32(out)), x.numel(), float(alpha), _stream()), "f8_pact_f32")
    return out


def f8_pact_fix_f32(x, alpha, fl, out=None):
    out = torch.empty_like(x) if out is None else out
    _check(lib().f8_pact_fix_f32(_ptr(_f32(x)), _ptr(_f32(out)), x.numel(), float(alpha), int(fl), _stream()),
           "f8_pact_fix_f32")
    return out


def f8_eta_fix(alpha, fl):
    return float(lib().f8_eta_fix(float(alpha), int(fl)))


def f8_opt_fl(sigma, is_signed):
    return int(lib().f8_opt_fl(float(sigma), int(bool(is_signed))))


def _read_stats(buf):
    """f8_stats out of a 24-byte device buffer (synchronises)."""
    raw = buf.cpu().numpy().tobytes()
    s = f8_stats.from_buffer_copy(raw)
    return {"mean": s.mean, "std": s.std, "fl_signed": s.fl_signed, "fl_unsigned": s.fl_unsigned}


def f8_tensor_stats_f32(x, work=None):
    """Mean, population standard deviation and the Eq. 1 fractional lengths of x, as a dict
    (reads the 24-byte result back, which synchronises)."""
    if work is None:
        work = torch.empty(F8_STATS_WORK_DOUBLES, dtype=torch.float64, device=x.device)
    buf = torch.empty(24, dtype=torch.uint8, device=x.device)
    _check(lib().f8_tensor_stats_f32(_ptr(_f32(x)), x.numel(), _ptr(buf), _ptr(work), _stream()),
           "f8_tensor_stats_f32")
    return _read_stats(buf)


def f8_quant_error_f32(x, fl, is_signed, out=None, work=None):
    """Device tensor of three doubles: sum |v - fix_quant(v)|, sum |v|, their ratio."""
    if work is None:
        work = torch.empty(F8_STATS_WORK_DOUBLES, dtype=torch.float64, device=x.device)
    if out is None:
        out = torch.empty(3, dtype=torch.float64, device=x.device)
    _check(lib().f8_quant_error_f32(_ptr(_f32(x)), x.numel(), int(fl), int(bool(is_signed)), _ptr(out), _ptr(work),
                                    _stream()), "f8_quant_error_f32")
    return out


def f8_fold_conv_bn(w, gamma, beta, mu, sigma, eta_in, eta_out, fl_x, fl_w=None, want_stats=True):
    """Integer parameters of a folded Conv-BN block: (wq int8 like w, bq int32 [cout], stats dict or
    None).  w is [cout][...]; fl_w=None lets the library choose it (Eq. 1), reported in
    stats['fl_signed']."""
    cout = w.shape[0]
    k = w.numel() // max(cout, 1)
    d = f8_fold_desc(cout, k, float(eta_in), float(eta_out), int(fl_x), -1 if fl_w is None else int(fl_w))
    wq = torch.empty(w.shape, dtype=torch.int8, device=w.device)
    bq = torch.empty(cout, dtype=torch.int32, device=w.device)
    work = torch.empty(lib().f8_fold_work_doubles(cout), dtype=torch.float64, device=w.device)
    buf = torch.empty(24, dtype=torch.uint8, device=w.device) if (want_stats or fl_w is None) else None
    _check(lib().f8_fold_conv_bn(_ptr(_f32(w)), _ptr(_f32(gamma)), _ptr(_f32(beta)), _ptr(_f32(mu)),
                                 _ptr(_f32(sigma)), ctypes.byref(d), _ptr(wq), _ptr(bq), _ptr(buf), _ptr(work),
                                 _stream()), "f8_fold_conv_bn")
    return wq, bq, (None if buf is None else _read_stats(buf))


def out_hw(H, W, R, S, stride, pad):
    P = 0 if H + 2 * pad[0] - R < 0 else (H + 2 * pad[0] - R) // stride[0] + 1
    Q = 0 if W + 2 * pad[1] - S < 0 else (W + 2 * pad[1] - S) // stride[1] + 1
    return P, Q


class Chain:
    """Handle on an f8_chain built from a layer list (see workloads.Net).

    Weights and biases are uploaded once and kept alive here; the workspace is a torch
    uint8 tensor allocated by prepare()."""

    def __init__(self, net, device="cuda", keep_all=False, fusion=False, streams=1):
        L = lib()
        self.net = net
        self.device = device
        self._keep = []
        descs = (f8_layer_desc * len(net.layers))()
        for d, S in zip(descs, net.layers):
            d.op = _OPS[S.op]
            d.src, d.dst, d.res = S.src, S.dst, S.res
            d.Cin, d.Cout, d.R, d.S = S.Cin, S.Cout, S.R, S.S
            d.stride_h = d.stride_w = S.stride
            d.pad_h = d.pad_w = S.pad
            d.q = make_quant(S)
            if S.res >= 0:
                d.q.res_type, d.q.fl_res = _TYPES[S.res_type], int(S.fl_res)
            d.w = d.bias = None
            d.dst2 = getattr(S, "dst2", -1)
            if d.dst2 > 0:
                d.q2 = make_requant2(S)
            if S.w is not None:
                wt = torch.from_numpy(S.w).contiguous().to(device)
                self._keep.append(wt)
                d.w = wt.data_ptr()
            if S.bias is not None:
                bt = torch.from_numpy(S.bias).contiguous().to(device)
                self._keep.append(bt)
                d.bias = bt.data_ptr()
        h = ctypes.c_void_p()
        _check(L.f8_chain_create(descs, len(net.layers), net.in_hw[0], net.in_hw[1], net.in_c,
                                 _TYPES[net.x_type], ctypes.byref(h)), "f8_chain_create")
        self.handle = h
        if keep_all:
            _check(L.f8_chain_set_keep_all(h, 1), "f8_chain_set_keep_all")
        if fusion:
            _check(L.f8_chain_set_fusion(h, 1), "f8_chain_set_fusion")
        if streams != 1:
            _check(L.f8_chain_set_streams(h, streams), "f8_chain_set_streams")
        self.workspace = None
        self.batch = None
        last = net.layers[-1]
        self.out_shape = (last.out_hw[0], last.out_hw[1], last.Cout)
        self.out_dtype = TORCH_DTYPE[last.y_type]

    def workspace_bytes(self, batch):
        n = ctypes.c_size_t()
        _check(lib().f8_chain_workspace_bytes(self.handle, batch, ctypes.byref(n)), "f8_chain_workspace_bytes")
        return n.value

    def prepare(self, batch):
        self.workspace = torch.empty(self.workspace_bytes(batch), dtype=torch.uint8, device=self.device)
        self.batch = batch
        _check(lib().f8_chain_prepare(self.handle, _ptr(self.workspace), batch, _stream()), "f8_chain_prepare")
        return self

    def run(self, x, out=None):
        B = x.shape[0]
        if out is None:
            out = torch.empty((B,) + self.out_shape, dtype=self.out_dtype, device=x.device)
        _check(lib().f8_chain_run(self.handle, _ptr(x), _ptr(out), _ptr(self.workspace), B, _stream()),
               "f8_chain_run")
        return out

    def capture(self, x, out):
        """Record one run of the chain on (x, out) into a HIP graph and return it (a
        torch.cuda.CUDAGraph; call .replay()).  The chain only launches kernels, so the capture
        holds nothing else; run the chain once before capturing so that one-time set-up calls
        (kernel attributes) are not part of the capture."""
        self.run(x, out)
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            self.run(x, out)
        return g

    def tensor(self, tid):
        """Copy of intermediate tensor `tid` after a run (None if its memory was reused)."""
        p = ctypes.c_void_p()
        h, w, c, dt, live = (ctypes.c_int() for _ in range(5))
        _check(lib().f8_chain_tensor(self.handle, tid, _ptr(self.workspace), self.batch, ctypes.byref(p),
                                     ctypes.byref(h), ctypes.byref(w), ctypes.byref(c), ctypes.byref(dt),
                                     ctypes.byref(live)), "f8_chain_tensor")
        if not p.value or not live.value:
            return None
        off = p.value - self.workspace.data_ptr()
        n = self.batch * h.value * w.value * c.value
        esz = 4 if dt.value == F8_S32 else 1
        flat = self.workspace[off:off + n * esz].view(TORCH_DTYPE[dt.value])
        return flat.view(self.batch, h.value, w.value, c.value).clone()

    def layer_info(self, i, batch):
        """(kernel name, algorithmic ops, algorithmic bytes) of layer i for `batch` images."""
        name = ctypes.create_string_buffer(64)
        ops, nbytes = ctypes.c_double(), ctypes.c_double()
        _check(lib().f8_chain_layer_info(self.handle, i, batch, name, 64, ctypes.byref(ops),
                                         ctypes.byref(nbytes)), "f8_chain_layer_info")
        return name.value.decode(), ops.value, nbytes.value

    def profile(self, x, out, repeats=1):
        """Per-layer device time in ms (HIP events on the current stream), mean of `repeats` runs."""
        n = lib().f8_chain_num_layers(self.handle)
        ms = (ctypes.c_float * n)()
        _check(lib().f8_chain_profile(self.handle, _ptr(x), _ptr(out), _ptr(self.workspace), x.shape[0],
                                      _stream(), repeats, ms), "f8_chain_profile")
        return list(ms)

    def close(self):
        if self.handle:
            lib().f8_chain_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
