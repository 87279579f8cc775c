"""The entry point that allocates nothing (f8_conv2d_fixed_noalloc, scratch inside the library)
against the ordinary one (f8_conv2d_fixed, per-stream hipMalloc'd scratch), through the C ABI.

Integer work: the bar is equality of every output byte.  The calls come in pairs, the second
smaller than the first, because all calls on a GPU share one scratch array that keeps the last
call's contents: whatever the second call needs must have been rewritten by the second call.
"""
import ctypes
import zlib

import numpy as np
import pytest
import torch

from paper_2202_05239_amd import binding as f8
from paper_2202_05239_amd import workloads as wl

pytestmark = pytest.mark.gpu

DEV = "cuda"


def raw_conv(entry, xt, wt, bt, yt, L, rt):
    """One call of `entry` (a ctypes function of the library) with plain pointers and sizes."""
    B, H, W, Cin = xt.shape
    Cout, R, S, _ = wt.shape
    q = f8.make_quant(L, rt)
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    rc = entry(ctypes.c_void_p(xt.data_ptr()), ctypes.c_void_p(wt.data_ptr()),
               ctypes.c_void_p(bt.data_ptr()) if bt is not None else None, ctypes.c_void_p(yt.data_ptr()),
               B, H, W, Cin, Cout, R, S, L.stride, L.stride, L.pad, L.pad, ctypes.byref(q), stream)
    return rc


def both_ways(case, rng, oracle=None):
    B, H, W, Cin, Cout, R, S, st, pd, xty, yty, rty = case
    x, L, res = wl.random_conv_case(rng, B, H, W, Cin, Cout, R, S, st, pd, xty, yty, rty)
    xt = torch.from_numpy(x).to(DEV)
    wt = torch.from_numpy(L.w).to(DEV)
    bt = torch.from_numpy(L.bias).to(DEV)
    rt = torch.from_numpy(res).to(DEV) if res is not None else None
    P, Q = L.out_hw
    lib = f8.lib()
    outs = []
    for entry in (lib.f8_conv2d_fixed_noalloc, lib.f8_conv2d_fixed):
        y = torch.full((B, P, Q, Cout), 77, dtype=f8.TORCH_DTYPE[yty], device=DEV)
        rc = raw_conv(entry, xt, wt, bt, y, L, rt)
        assert rc == 0, (case, rc)
        torch.cuda.synchronize()
        outs.append(y.cpu().numpy())
    got, want = outs
    assert got.dtype == want.dtype and got.shape == want.shape
    assert np.array_equal(got, want), "%s: %d of %d bytes differ" % (str(case), int((got != want).sum()), got.size)
    assert len(np.unique(want)) > 4, "degenerate draw"
    return got


# (first call, second and smaller call): the pair shares the library's scratch array
PAIRS = [
    # large then small, both through the LDS-direct dense kernel
    ((2, 28, 28, 128, 512, 1, 1, 1, 0, "u8", "u8", "u8"), (1, 14, 14, 64, 64, 3, 3, 1, 1, "u8", "u8", None)),
    # many channels (start values near the scratch limit), then few: the stale tail must not matter
    ((1, 7, 7, 256, 4096, 1, 1, 1, 0, "u8", "s8", None), (1, 9, 9, 7, 5, 3, 3, 1, 1, "u8", "s8", None)),
    # signed input (no sign correction in the start values) after unsigned, int32 logits after 8-bit
    ((2, 19, 23, 64, 192, 3, 3, 2, 1, "u8", "u8", None), (1, 1, 40, 512, 1000, 1, 1, 1, 0, "s8", "s32", None)),
]


@pytest.mark.parametrize("pair", PAIRS)
def test_noalloc_entry_point_matches_the_allocating_one(pair):
    rng = np.random.default_rng(zlib.crc32(repr(pair).encode()))
    for case in pair:          # two calls in a row, the second with the smaller input
        both_ways(case, rng)


def test_noalloc_matches_the_oracle_on_a_ragged_layer():
    # also pinned to the CPU oracle directly, not only to the other entry point
    from oracle import ref
    case = (3, 17, 17, 32, 160, 3, 3, 1, 1, "u8", "u8", "u8")
    rng = np.random.default_rng(7)
    B, H, W, Cin, Cout, R, S, st, pd, xty, yty, rty = case
    x, L, res = wl.random_conv_case(rng, B, H, W, Cin, Cout, R, S, st, pd, xty, yty, rty)
    want = ref.conv2d_fixed(x, L.w, L.bias, L, (st, st), (pd, pd), res)
    xt, wt, bt, rt = (torch.from_numpy(a).to(DEV) for a in (x, L.w, L.bias, res))
    y = torch.empty(want.shape, dtype=torch.uint8, device=DEV)
    assert raw_conv(f8.lib().f8_conv2d_fixed_noalloc, xt, wt, bt, y, L, rt) == 0
    torch.cuda.synchronize()
    assert np.array_equal(y.cpu().numpy(), want)


def test_noalloc_rejects_more_channels_than_its_scratch_holds():
    # validation only: nothing is launched, the pointers are never dereferenced
    lib = f8.lib()
    q = f8.f8_quant()
    q.fl_x, q.fl_w, q.fl_y, q.clip_lo, q.clip_hi = 4, 4, 4, 0, 255
    q.x_type, q.y_type, q.res = f8.F8_U8, f8.F8_U8, None
    fake = ctypes.c_void_p(0x1000)
    rc = lib.f8_conv2d_fixed_noalloc(fake, fake, None, fake, 1, 4, 4, 16, 4097, 1, 1, 1, 1, 0, 0, ctypes.byref(q), None)
    assert rc == 8 and b"unsupported" in lib.f8_status_str(rc)
