"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every symbol
the header declares, rejects bad arguments before launching anything, and the chain
planner's book-keeping."""
import ctypes
import os
import re

import numpy as np
import pytest

from paper_2202_05239_amd import binding as f8
from paper_2202_05239_amd import workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE = ctypes.c_void_p(0x1000)        # never dereferenced: every call below fails validation first


def declared_functions():
    text = open(os.path.join(ROOT, "include", "f8.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(f8_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    L = f8.lib()
    names = declared_functions()
    assert len(names) >= 16
    for n in names:
        assert hasattr(L, n), n
    assert sorted(f8.EXPORTS) == names
    assert L.f8_abi_version() == 3


def quant(**kw):
    q = f8.f8_quant()
    q.fl_x, q.fl_w, q.fl_y, q.clip_lo, q.clip_hi = 4, 4, 4, 0, 255
    q.x_type, q.y_type, q.res, q.res_type, q.fl_res = f8.F8_U8, f8.F8_U8, None, 0, 0
    for k, v in kw.items():
        setattr(q, k, v)
    return q


def conv(q, x=FAKE, w=FAKE, bias=None, y=FAKE, B=1, H=8, W=8, Cin=16, Cout=16, R=3, S=3, sh=1, sw=1, ph=1, pw=1):
    return f8.lib().f8_conv2d_fixed(x, w, bias, y, B, H, W, Cin, Cout, R, S, sh, sw, ph, pw,
                                    ctypes.byref(q) if q is not None else None, None)


def test_conv_argument_validation():
    assert conv(quant(), x=None) == 1
    assert conv(quant(), w=None) == 1
    assert conv(quant(), y=None) == 1
    assert conv(None) == 1
    assert conv(quant(), H=0) == 2
    assert conv(quant(), sh=0) == 2
    assert conv(quant(), ph=-1) == 2
    assert conv(quant(), Cin=8192, R=3, S=3) == 2                 # K = 73728 > 65536
    assert conv(quant(fl_y=17)) == 3                               # shift -9
    assert conv(quant(fl_x=12, fl_w=13, fl_y=0)) == 3              # shift 25
    assert conv(quant(clip_lo=3, clip_hi=2)) == 4
    assert conv(quant(clip_hi=256)) == 4
    assert conv(quant(y_type=f8.F8_S8, clip_lo=-128, clip_hi=127)) == 4
    assert conv(quant(x_type=f8.F8_S32)) == 5
    assert conv(quant(y_type=7)) == 5
    assert conv(quant(res=0x2000, res_type=9)) == 5
    assert conv(quant(res=0x2000, res_type=f8.F8_U8, fl_res=40)) == 3
    assert conv(quant(), bias=ctypes.c_void_p(0x1002)) == 7
    assert conv(quant(y_type=f8.F8_S32), y=ctypes.c_void_p(0x1001)) == 7
    assert conv(quant(res=0x1000, res_type=f8.F8_U8, fl_res=4), y=ctypes.c_void_p(0x1000)) == 8
    assert conv(quant(), B=70000, H=256, W=256, Cin=16) == 8      # beyond 2^31-1 bytes
    # empty problems are fine and launch nothing
    assert conv(quant(), B=0) == 0
    assert conv(quant(), Cout=0) == 0
    assert conv(quant(), H=1, W=1, R=3, S=3, ph=0, pw=0) == 0     # window larger than image: P = Q = 0


def test_other_entry_points_validate():
    L = f8.lib()
    q = quant()
    assert L.f8_gemm_fixed(FAKE, FAKE, None, FAKE, -1, 8, 8, ctypes.byref(q), None) == 2
    assert L.f8_gemm_fixed(FAKE, FAKE, None, FAKE, 8, 0, 8, ctypes.byref(q), None) == 2
    assert L.f8_gemm_fixed(None, FAKE, None, FAKE, 8, 8, 8, ctypes.byref(q), None) == 1
    assert L.f8_gemm_fixed(FAKE, FAKE, None, FAKE, 0, 8, 8, ctypes.byref(q), None) == 0
    assert L.f8_dwconv_fixed(FAKE, FAKE, None, FAKE, 1, 8, 8, 0, 3, 3, 1, 1, 1, 1, ctypes.byref(q), None) == 2
    assert L.f8_dwconv_fixed(FAKE, None, None, FAKE, 1, 8, 8, 4, 3, 3, 1, 1, 1, 1, ctypes.byref(q), None) == 1
    assert L.f8_maxpool(FAKE, FAKE, 1, 8, 8, 4, 3, 3, 2, 2, 3, 1, f8.F8_U8, None) == 2   # pad >= window
    assert L.f8_maxpool(FAKE, FAKE, 1, 8, 8, 4, 3, 3, 2, 2, 1, 1, f8.F8_S32, None) == 5
    assert L.f8_global_pool_fixed(FAKE, FAKE, 1, 300, 300, 4, ctypes.byref(q), None) == 2
    qr = quant(res=0x3000)
    assert L.f8_global_pool_fixed(FAKE, FAKE, 1, 7, 7, 4, ctypes.byref(qr), None) == 8
    assert L.f8_status_str(3).decode().startswith("fractional")


def test_clip_from_alpha():
    assert f8.f8_clip_from_alpha(6.0, 5) == 192                    # 6.0 * 2^5
    assert f8.f8_clip_from_alpha(6.0, 6) == 255                    # saturates at the type's top
    assert f8.f8_clip_from_alpha(1.0, 7, True) == 127
    assert f8.f8_clip_from_alpha(0.7, 3) == 6                      # 5.6 -> 6
    assert f8.f8_clip_from_alpha(0.3125, 3) == 3                   # 2.5 -> 3 (half up)
    assert f8.f8_clip_from_alpha(-1.0, 3) == 0
    assert f8.f8_clip_from_alpha(3.0, 0) == 3


def make_descs(net):
    descs = (f8.f8_layer_desc * len(net.layers))()
    for d, S in zip(descs, net.layers):
        d.op = {"conv": 0, "dwconv": 1, "maxpool": 2, "gpool": 3}[S.op]
        d.src, d.dst, d.res = S.src, S.dst, S.res
        d.Cin, d.Cout, d.R, d.S = S.Cin, S.Cout, S.R, S.S
        d.stride_h = d.stride_w = S.stride
        d.pad_h = d.pad_w = S.pad
        d.q = f8.make_quant(S)
        if S.res >= 0:
            d.q.res_type, d.q.fl_res = {"u8": 0, "s8": 1, "s32": 2}[S.res_type], S.fl_res
        d.w = 0x10000 if S.w is not None else None
        d.bias = 0x20000 if S.bias is not None else None
        d.dst2 = S.dst2
        if S.dst2 > 0:
            d.q2 = f8.make_requant2(S)
    return descs


def test_chain_planner_host_side():
    L = f8.lib()
    _, net = wl.config4(batch=1, hw=64)
    descs = make_descs(net)
    h = ctypes.c_void_p()
    assert L.f8_chain_create(descs, len(net.layers), 64, 64, 3, f8.F8_S8, ctypes.byref(h)) == 0
    n1, n2, n8, nk = ctypes.c_size_t(), ctypes.c_size_t(), ctypes.c_size_t(), ctypes.c_size_t()
    assert L.f8_chain_workspace_bytes(h, 1, ctypes.byref(n1)) == 0
    assert L.f8_chain_workspace_bytes(h, 2, ctypes.byref(n2)) == 0
    assert L.f8_chain_workspace_bytes(h, 8, ctypes.byref(n8)) == 0
    total = sum(l.out_hw[0] * l.out_hw[1] * l.Cout for l in net.layers[:-1])
    biggest = max(l.out_hw[0] * l.out_hw[1] * l.Cout for l in net.layers[:-1])
    # reuse: the per-image arena is far smaller than the sum of all tensors, yet holds the
    # largest few; it scales linearly with the batch, the constants do not
    arena = n2.value - n1.value
    consts = n1.value - arena
    assert biggest <= arena < total / 4
    assert n8.value - n1.value == 7 * arena
    assert consts >= sum((l.Cout + 255) // 256 * 256 * 4 for l in net.layers if l.op == "conv")
    # run before prepare is refused; so is a wrong batch
    assert L.f8_chain_run(h, FAKE, FAKE, ctypes.c_void_p(0x100000), 1, None) == 10
    assert L.f8_chain_set_keep_all(h, 1) == 0
    assert L.f8_chain_workspace_bytes(h, 1, ctypes.byref(nk)) == 0
    assert nk.value - consts >= total
    L.f8_chain_destroy(h)
    # inconsistent chains are rejected
    bad = make_descs(net)
    bad[3].q.fl_x += 1
    assert L.f8_chain_create(bad, len(net.layers), 64, 64, 3, f8.F8_S8, ctypes.byref(h)) == 3
    bad = make_descs(net)
    bad[2].Cin += 1
    assert L.f8_chain_create(bad, len(net.layers), 64, 64, 3, f8.F8_S8, ctypes.byref(h)) == 2
    bad = make_descs(net)
    bad[5].src = 40
    assert L.f8_chain_create(bad, len(net.layers), 64, 64, 3, f8.F8_S8, ctypes.byref(h)) == 2
    assert L.f8_chain_create(make_descs(net), len(net.layers), 64, 64, 3, f8.F8_U8, ctypes.byref(h)) == 2


def test_chain_pairs_a_1x1_layer_with_the_layer_in_front_host_side():
    """The 1x1 64 -> 256 layers of the first ResNet stage and the 1x1 128 -> 512 layers of the second also
    compute the 1x1 layer that reads their output (the next block's first layer; at the boundary between
    the first two stages it sits behind the shortcut projection): which layers are paired, at which batch, and that the planner never lets the extra output share
    memory with anything the launch reads or with the launch's own output (no GPU needed: names and
    addresses only)."""
    L = f8.lib()
    _, net = wl.config4(batch=1)
    h = ctypes.c_void_p()
    assert L.f8_chain_create(make_descs(net), len(net.layers), 224, 224, 3, f8.F8_S8, ctypes.byref(h)) == 0

    def name(i, batch):
        buf = ctypes.create_string_buffer(64)
        assert L.f8_chain_layer_info(h, i, batch, buf, 64, None, None) == 0
        return buf.value.decode()

    names = [name(i, 256) for i in range(len(net.layers))]
    by_name = {S.name: i for i, S in enumerate(net.layers)}
    pairs = {"s1b1.conv_c": "s1b2.conv_a", "s1b2.conv_c": "s1b3.conv_a", "s1b3.conv_c": "s2b1.conv_a",
             "s2b1.conv_c": "s2b2.conv_a", "s2b2.conv_c": "s2b3.conv_a", "s2b3.conv_c": "s2b4.conv_a"}
    for front, behind in pairs.items():
        width = net.layers[by_name[behind]].Cout
        kernel = "pw1x1_ws<64x256>" if front.startswith("s1") else "pw1x1_mid<128x512>"
        assert names[by_name[front]] == "%s+1x1<%d>" % (kernel, width)
        assert names[by_name[behind]] == "(fused)"
    assert "+1x1" not in names[by_name["s2b4.conv_c"]]             # the third stage's first layer is 256 wide: on its own
    assert names[by_name["s2b1.ds"]] != "(fused)"                  # the layer between the last pair runs on its own
    assert names.count("(fused)") == len(pairs) + 1                # + the max pool inside the stem kernel
    assert not any("+1x1" in name(i, 8) for i in range(len(net.layers)))       # small batches: two launches

    base, batch = 1 << 32, 256
    def span(tid):
        p, dims = ctypes.c_void_p(), [ctypes.c_int() for _ in range(5)]
        assert L.f8_chain_tensor(h, tid, ctypes.c_void_p(base), batch, ctypes.byref(p), *[ctypes.byref(d) for d in dims]) == 0
        hh, ww, cc = (d.value for d in dims[:3])
        return p.value, p.value + batch * hh * ww * cc
    for front, behind in pairs.items():
        F, T = net.layers[by_name[front]], net.layers[by_name[behind]]
        spans = [span(t) for t in (F.src, F.res, F.dst, T.dst)]
        for a in range(4):
            for b in range(a + 1, 4):
                assert spans[a][1] <= spans[b][0] or spans[b][1] <= spans[a][0], (front, a, b)
    L.f8_chain_destroy(h)


def test_binding_refuses_to_run_without_library(monkeypatch):
    monkeypatch.setattr(f8, "_lib", None)
    monkeypatch.setattr(f8, "LIB_PATH", "/nonexistent/libf8.so")
    with pytest.raises(RuntimeError, match="no fallback"):
        f8.lib()


def test_quant_tools_host_side():
    """Eq. 1 and Eq. 5 on the host against the oracle, and argument validation of the device
    entry points (every call below fails before anything is launched)."""
    from oracle import quant_ref as qr
    L = f8.lib()
    rng = np.random.default_rng(5)
    sig = np.concatenate([10 ** rng.uniform(-4, 4, 2000), [40.0, 20.0, 70.0, 35.0, 0.3125, 0.0,
                                                            np.nextafter(20.0, 30.0), np.nextafter(20.0, 0.0), 1e-320, 1e308]])
    for s in sig:
        for is_signed in (True, False):
            assert f8.f8_opt_fl(s, is_signed) == qr.opt_fl(float(s), is_signed), (s, is_signed)
    assert f8.f8_opt_fl(float("nan"), True) == 7
    for alpha, fl in ((3.0, 4), (255.0, 0), (0.7, 8), (6.0, 1)):
        assert f8.f8_eta_fix(alpha, fl) == qr.eta_fix(alpha, fl)
    assert L.f8_fix_quant_f32(FAKE, FAKE, 16, 9, 0, None) == 3
    assert L.f8_fix_quant_f32(FAKE, FAKE, 16, 8, 1, None) == 3
    assert L.f8_fix_quant_f32(FAKE, FAKE, 16, -1, 0, None) == 3
    assert L.f8_fix_quant_f32(None, FAKE, 16, 4, 0, None) == 1
    assert L.f8_fix_quant_f32(None, None, 0, 4, 0, None) == 0           # empty: no-op
    assert L.f8_fix_quant_f32(ctypes.c_void_p(0x1002), FAKE, 16, 4, 0, None) == 7
    assert L.f8_fix_quant_code(FAKE, None, 16, 4, 0, None) == 1
    assert L.f8_pact_f32(FAKE, FAKE, 16, 0.0, None) == 4
    assert L.f8_pact_f32(FAKE, FAKE, 16, float("inf"), None) == 4
    assert L.f8_pact_fix_f32(FAKE, FAKE, 16, 2.0, 9, None) == 3
    assert L.f8_tensor_stats_f32(FAKE, 16, None, FAKE, None) == 1
    assert L.f8_tensor_stats_f32(FAKE, 16, FAKE, None, None) == 1
    assert L.f8_quant_error_f32(FAKE, 16, 8, 1, FAKE, FAKE, None) == 3
    assert L.f8_quant_error_f32(FAKE, 16, 3, 1, None, FAKE, None) == 1
    assert L.f8_fold_work_doubles(64) == 4096 + 128

    def fold(cout=8, k=16, eta_in=1.0, eta_out=1.0, fl_x=4, fl_w=-1, w=FAKE, stats=FAKE):
        d = f8.f8_fold_desc(cout, k, eta_in, eta_out, fl_x, fl_w)
        return L.f8_fold_conv_bn(w, FAKE, FAKE, FAKE, FAKE, ctypes.byref(d), FAKE, FAKE, stats, FAKE, None)
    assert fold(cout=-1) == 2
    assert fold(cout=65536, k=65536) == 2
    assert fold(cout=0) == 0
    assert fold(w=None) == 1
    assert fold(stats=None) == 1                      # Eq. 1 needs the statistics buffer
    assert fold(fl_w=8) == 3
    assert fold(fl_x=9) == 3
    assert fold(eta_out=0.0) == 4
    assert fold(eta_in=float("inf")) == 4
    assert L.f8_fold_conv_bn(FAKE, FAKE, FAKE, FAKE, FAKE, None, FAKE, FAKE, FAKE, FAKE, None) == 1


def test_second_output_format_host_side():
    """Validation of the two-format entry point, and a chain whose blocks write two formats."""
    L = f8.lib()

    def dual(q=None, q2=None, y=FAKE, y2=ctypes.c_void_p(0x2000), drop_q2=False):
        q = q or quant()
        r = q2 or f8.f8_requant2(4, 0, 255, f8.F8_U8)
        return L.f8_conv2d_fixed_dual(FAKE, FAKE, None, y, y2, 1, 8, 8, 16, 16, 3, 3, 1, 1, 1, 1, ctypes.byref(q),
                                      None if drop_q2 else ctypes.byref(r), None)
    assert dual(y2=None) == 1
    assert dual(drop_q2=True) == 1
    assert dual(q=quant(y_type=f8.F8_S32)) == 5
    assert dual(q2=f8.f8_requant2(4, 0, 255, f8.F8_S32)) == 5
    assert dual(q2=f8.f8_requant2(17, 0, 255, f8.F8_U8)) == 3          # second shift -9
    assert dual(q2=f8.f8_requant2(4, 0, 256, f8.F8_U8)) == 4
    assert dual(q2=f8.f8_requant2(4, -128, 127, f8.F8_S8)) == 4
    assert dual(q2=f8.f8_requant2(4, 9, 3, f8.F8_U8)) == 4
    assert dual(y2=FAKE) == 8                                          # y2 must not be y
    _, net = wl.resnet50_private_fl(batch=1, hw=64)
    _, plain = wl.config4(batch=1, hw=64)
    h = ctypes.c_void_p()
    assert L.f8_chain_create(make_descs(net), len(net.layers), 64, 64, 3, f8.F8_S8, ctypes.byref(h)) == 0
    n1, n2 = ctypes.c_size_t(), ctypes.c_size_t()
    assert L.f8_chain_workspace_bytes(h, 1, ctypes.byref(n1)) == 0
    assert L.f8_chain_set_keep_all(h, 1) == 0
    assert L.f8_chain_workspace_bytes(h, 1, ctypes.byref(n2)) == 0
    extra = sum(l.out_hw[0] * l.out_hw[1] * l.Cout for l in net.layers if l.dst2 > 0)
    total = sum(l.out_hw[0] * l.out_hw[1] * l.Cout for l in net.layers[:-1])
    assert n2.value - n1.value > 0 and n2.value >= total + extra
    L.f8_chain_destroy(h)
    bad = make_descs(net)
    i = next(k for k, l in enumerate(net.layers) if l.dst2 > 0)
    bad[i].dst2 = bad[i].dst                                           # both outputs in one tensor
    assert L.f8_chain_create(bad, len(net.layers), 64, 64, 3, f8.F8_S8, ctypes.byref(h)) == 2
    bad = make_descs(net)
    bad[i].q2.fl_y += 1                                                # the consumer expects another format
    assert L.f8_chain_create(bad, len(net.layers), 64, 64, 3, f8.F8_S8, ctypes.byref(h)) == 3
    bad = make_descs(net)
    bad[i].q2.y_type = f8.F8_S32
    assert L.f8_chain_create(bad, len(net.layers), 64, 64, 3, f8.F8_S8, ctypes.byref(h)) == 5


def test_bench_refuses_more_than_one_gpu():
    """The build runs on one GPU: bench.py with --gpus above 1 exits with a message and a non-zero
    status before it touches a device."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "ONE GPU" in r.stderr and r.stdout.strip() == ""
