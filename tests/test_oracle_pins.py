"""Pins of the CPU oracle against what the paper and the mathematics fix.

The oracle is compared with things other than itself: hand-worked fixtures, exact
rational arithmetic, an exact fp64 model of fix_quant (paper Eq. 2 / Eq. 9), brute-force
loops written separately, library routines (numpy int64 matmul, torch fp64 conv2d and
max_pool2d) and structural identities.  No GPU is needed.
"""
import math
import os
from fractions import Fraction

import numpy as np
import pytest
import torch

from paper_2202_05239_amd import workloads as wl

GOLD = os.path.join(os.path.dirname(__file__), "golden")


class Q:
    """Plain parameter record for single-layer oracle calls."""

    def __init__(self, fl_x=0, fl_w=0, fl_y=0, lo=0, hi=255, x_type="u8", y_type="u8",
                 res_type="u8", fl_res=0):
        self.fl_x, self.fl_w, self.fl_y = fl_x, fl_w, fl_y
        self.clip_lo, self.clip_hi = lo, hi
        self.x_type, self.y_type = x_type, y_type
        self.res_type, self.fl_res = res_type, fl_res


def read_cases(name):
    rows = []
    with open(os.path.join(GOLD, name)) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if line:
                rows.append(line.split())
    return rows


def half_up(v: Fraction) -> int:
    """Exact round-half-up of a rational."""
    return math.floor(v + Fraction(1, 2))


# --------------------------------------------------------------------------- P1

def test_shift_round_golden(oracle):
    for a, s, want in read_cases("shift_round_cases.txt"):
        assert oracle.shift_round(int(a), int(s)) == int(want), (a, s)


def test_shift_round_exact_rational(oracle):
    rng = np.random.default_rng(1)
    for s in range(1, 25):
        span = list(range(-3 * 2 ** min(s, 6), 3 * 2 ** min(s, 6) + 1))
        span += [int(v) for v in rng.integers(-2 ** 31, 2 ** 31 - 2 ** 24, size=200)]
        span += [k * 2 ** (s - 1) for k in range(-9, 10)]          # every tie and integer
        for a in span:
            want = half_up(Fraction(a, 2 ** s))
            assert oracle.shift_round(a, s) == want, (a, s)
            assert want == math.floor(a / 2.0 ** s + 0.5)          # the fp64 form agrees


def test_shift_round_nonpositive_shift(oracle):
    for a in (-1000, -1, 0, 1, 77):
        assert oracle.shift_round(a, 0) == a
        for s in range(1, 9):
            assert oracle.shift_round(a, -s) == a * 2 ** s


# --------------------------------------------------------------------------- Eq. 2 / Eq. 9 fixtures

def test_fixquant_golden(oracle):
    """W = 0 leaves Y = fix_quant(bias); the bias carries the real value at FL 16."""
    for kind, val, fl, want in read_cases("fixquant_cases.txt"):
        fl = int(fl)
        b = np.array([round(float(val) * 2 ** 16)], np.int32)
        q = Q(8, 8, fl, 0, 255) if kind == "u" else Q(8, 8, fl, -127, 127, y_type="s8")
        y = oracle.gemm_fixed(np.array([[7]], np.uint8), np.zeros((1, 1), np.int8), b, q)
        assert int(y[0, 0]) == int(want), (kind, val, fl)


# --------------------------------------------------------------------------- P2 P3 P4 (GEMM)

def int_gemm(x, w, bias):
    return x.astype(np.int64) @ w.astype(np.int64).T + bias.astype(np.int64)


def fp64_requant(A, s, lo, hi):
    """Paper Eq. 2 / Eq. 9 evaluated in fp64: clip first, then round half up."""
    v = A.astype(np.float64) * 2.0 ** (-s)           # exact: power-of-two scaling
    return np.floor(np.clip(v, lo, hi) + 0.5).astype(np.int64)


@pytest.mark.parametrize("x_type,y_type", [("u8", "u8"), ("s8", "u8"), ("u8", "s8"), ("s8", "s8")])
def test_gemm_fp64_model(oracle, x_type, y_type):
    rng = np.random.default_rng(7)
    for trial in range(12):
        M, K, N = int(rng.integers(1, 20)), int(rng.integers(1, 70)), int(rng.integers(1, 20))
        x = wl.draw_u8(rng, (M, K)) if x_type == "u8" else rng.integers(-128, 128, (M, K), dtype=np.int8)
        w = rng.integers(-127, 128, (N, K), dtype=np.int8)
        fl_x, fl_w = int(rng.integers(0, 9)), int(rng.integers(0, 9))
        s = int(rng.integers(-3, 16))
        bias = rng.integers(-2 ** (max(s, 0) + 9), 2 ** (max(s, 0) + 9), N).astype(np.int32)
        lo, hi = (0, 255) if y_type == "u8" else (-127, 127)
        if trial % 3 == 0:
            hi = int(rng.integers(1, hi))
            lo = lo if y_type == "u8" else -int(rng.integers(1, 127))
        q = Q(fl_x, fl_w, fl_x + fl_w - s, lo, hi, x_type, y_type)
        y = oracle.gemm_fixed(x, w, bias, q).astype(np.int64)
        A = int_gemm(x, w, bias)
        want = fp64_requant(A, s, lo, hi)
        assert np.array_equal(y, want)
        assert y.min() >= lo and y.max() <= hi                      # P3
        raw = np.floor(A * 2.0 ** (-s) + 0.5)
        assert np.all(y[raw < lo] == lo) and np.all(y[raw > hi] == hi)
        inside = (raw >= lo) & (raw <= hi)
        a_real = A * 2.0 ** -(fl_x + fl_w)                          # error bound of Eq. 2
        err = np.abs(y * 2.0 ** -q.fl_y - a_real)
        assert np.all(err[inside] <= 2.0 ** -(q.fl_y + 1))


def test_pure_clip_when_no_shift(oracle):
    """FL_x + FL_w == FL_y: the output is the clipped accumulator."""
    rng = np.random.default_rng(11)
    x = wl.draw_u8(rng, (9, 5))
    w = rng.integers(-3, 4, (6, 5), dtype=np.int8)
    bias = rng.integers(-100, 100, 6).astype(np.int32)
    y = oracle.gemm_fixed(x, w, bias, Q(3, 4, 7, 0, 200))
    assert np.array_equal(y, np.clip(int_gemm(x, w, bias), 0, 200))
    y = oracle.gemm_fixed(x, w, bias, Q(3, 4, 7, -100, 90, y_type="s8"))
    assert np.array_equal(y, np.clip(int_gemm(x, w, bias), -100, 90))


def test_raw_int32_output(oracle):
    rng = np.random.default_rng(12)
    x = rng.integers(-128, 128, (5, 33), dtype=np.int8)
    w = rng.integers(-127, 128, (4, 33), dtype=np.int8)
    bias = rng.integers(-10 ** 6, 10 ** 6, 4).astype(np.int32)
    y = oracle.gemm_fixed(x, w, bias, Q(2, 3, 0, x_type="s8", y_type="s32"))
    assert y.dtype == np.int32 and np.array_equal(y, int_gemm(x, w, bias))
    y0 = oracle.gemm_fixed(x, w, None, Q(2, 3, 0, x_type="s8", y_type="s32"))
    assert np.array_equal(y0, int_gemm(x, w, np.zeros(4, np.int32)))


# --------------------------------------------------------------------------- P8 round / clip order

def test_round_and_clip_commute():
    """Eq. 2 clips before rounding; hardware rounds, then clips: same for integer bounds."""
    for lo, hi in ((0, 255), (-127, 127), (0, 192), (-5, 9)):
        v = np.arange(-600 * 256, 600 * 256 + 1, dtype=np.float64) / 256.0
        a = np.floor(np.clip(v, lo, hi) + 0.5)
        b = np.clip(np.floor(v + 0.5), lo, hi)
        assert np.array_equal(a, b)


# --------------------------------------------------------------------------- P9 PACT (Eq. 3, Eq. 4)

def test_pact_equals_scaled_fixquant(oracle):
    """PACT(x) = eta * fix_quant(x / eta), eta = 2^FL * alpha / (2^WL - 1)  (Eq. 4, Eq. 5),
    evaluated exactly with rationals; the oracle's full-range unsigned requantiser is the
    fix_quant on the right-hand side."""
    rng = np.random.default_rng(3)
    M = 255
    for _ in range(300):
        fl_y = int(rng.integers(0, 9))
        fl_acc = fl_y + int(rng.integers(0, 10))
        alpha = Fraction(int(rng.integers(1, 4000)), int(rng.integers(1, 200)))
        eta = Fraction(2 ** fl_y) * alpha / M
        A = int(rng.integers(-2 ** 12, 2 ** 20))
        u = Fraction(A, 2 ** fl_acc)               # the argument x / eta of fix_quant
        x = u * eta
        pact = alpha / M * half_up(Fraction(M) / alpha * min(max(x, 0), alpha))   # Eq. 3
        q = Q(0, fl_acc, fl_y, 0, 255)
        y = oracle.gemm_fixed(np.array([[1]], np.uint8), np.zeros((1, 1), np.int8),
                              np.array([A], np.int32), q)
        assert eta * Fraction(int(y[0, 0]), 2 ** fl_y) == pact


# --------------------------------------------------------------------------- P5 brute force conv

def brute_conv(x, w, bias, sh, sw, ph, pw, s, lo, hi, res=None, d=0, depthwise=False):
    """Direct convolution with every index written out; Python ints; padding by an
    explicitly zero-filled copy of the input (a different route from skipping taps)."""
    B, H, W, C = x.shape
    if depthwise:
        R, S, _ = w.shape
        N = C
    else:
        N, R, S, _ = w.shape
    xp = [[[[0] * C for _ in range(W + 2 * pw)] for _ in range(H + 2 * ph)] for _ in range(B)]
    for b in range(B):
        for i in range(H):
            for j in range(W):
                for c in range(C):
                    xp[b][i + ph][j + pw][c] = int(x[b, i, j, c])
    P = (H + 2 * ph - R) // sh + 1
    Qo = (W + 2 * pw - S) // sw + 1
    y = np.zeros((B, P, Qo, N), np.int64)
    for b in range(B):
        for p in range(P):
            for q in range(Qo):
                for n in range(N):
                    acc = int(bias[n])
                    for r in range(R):
                        for t in range(S):
                            if depthwise:
                                acc += xp[b][p * sh + r][q * sw + t][n] * int(w[r, t, n])
                            else:
                                for c in range(C):
                                    acc += xp[b][p * sh + r][q * sw + t][c] * int(w[n, r, t, c])
                    if res is not None:
                        rv = int(res[b, p, q, n])
                        acc += rv * 2 ** d if d >= 0 else half_up(Fraction(rv, 2 ** (-d)))
                    v = half_up(Fraction(acc, 2 ** s)) if s >= 0 else acc * 2 ** (-s)
                    y[b, p, q, n] = min(max(v, lo), hi)
    return y


CONV_SHAPES = [
    # B  H  W  C  N  R  S  sh sw ph pw
    (2, 5, 7, 3, 4, 3, 3, 1, 1, 1, 1),
    (1, 7, 6, 5, 2, 3, 3, 2, 2, 1, 1),
    (1, 7, 7, 2, 3, 7, 7, 2, 2, 3, 3),
    (2, 4, 6, 4, 3, 1, 1, 1, 1, 0, 0),
    (1, 6, 5, 3, 2, 1, 1, 2, 2, 0, 0),
    (1, 6, 7, 2, 3, 3, 1, 2, 1, 1, 0),      # asymmetric window, stride and padding
    (1, 5, 6, 3, 2, 1, 3, 1, 2, 0, 1),
    (1, 3, 3, 1, 1, 3, 3, 1, 1, 2, 2),      # padding wider than half the window
]


@pytest.mark.parametrize("shape", CONV_SHAPES)
def test_conv_brute_force(oracle, shape):
    B, H, W, C, N, R, S, sh, sw, ph, pw = shape
    rng = np.random.default_rng(sum(shape))
    for x_type, y_type in (("u8", "u8"), ("s8", "s8")):
        x = wl.draw_u8(rng, (B, H, W, C)) if x_type == "u8" else rng.integers(-128, 128, (B, H, W, C), dtype=np.int8)
        w = rng.integers(-20, 21, (N, R, S, C), dtype=np.int8)
        bias = rng.integers(-300, 300, N).astype(np.int32)
        s = int(rng.integers(3, 8))
        lo, hi = (0, 255) if y_type == "u8" else (-127, 127)
        q = Q(4, 4, 8 - s, lo, hi, x_type, y_type)
        y = oracle.conv2d_fixed(x, w, bias, q, (sh, sw), (ph, pw))
        assert np.array_equal(y, brute_conv(x, w, bias, sh, sw, ph, pw, s, lo, hi))
        # explicit zero padding of the input with pad = 0 gives the same result
        xpad = np.zeros((B, H + 2 * ph, W + 2 * pw, C), x.dtype)
        xpad[:, ph:ph + H, pw:pw + W] = x
        y2 = oracle.conv2d_fixed(xpad, w, bias, q, (sh, sw), (0, 0))
        assert np.array_equal(y, y2)


@pytest.mark.parametrize("shape", CONV_SHAPES[:3] + CONV_SHAPES[5:7])
def test_dwconv_brute_force(oracle, shape):
    B, H, W, C, _, R, S, sh, sw, ph, pw = shape
    rng = np.random.default_rng(100 + sum(shape))
    x = wl.draw_u8(rng, (B, H, W, C))
    w = rng.integers(-127, 128, (R, S, C), dtype=np.int8)
    bias = rng.integers(-3000, 3000, C).astype(np.int32)
    q = Q(5, 2, 1, 0, 255)
    y = oracle.dwconv_fixed(x, w, bias, q, (sh, sw), (ph, pw))
    assert np.array_equal(y, brute_conv(x, w, bias, sh, sw, ph, pw, 6, 0, 255, depthwise=True))


# --------------------------------------------------------------------------- P6 library cross-check

def torch_acc(x, w, bias, stride, pad, groups=1):
    """Accumulator through torch's fp64 conv2d (exact for these magnitudes)."""
    xt = torch.from_numpy(x.astype(np.float64)).permute(0, 3, 1, 2)
    wt = torch.from_numpy(w.astype(np.float64))
    wt = wt.permute(2, 0, 1).unsqueeze(1) if groups > 1 else wt.permute(0, 3, 1, 2)
    a = torch.nn.functional.conv2d(xt, wt, torch.from_numpy(bias.astype(np.float64)),
                                   stride=stride, padding=pad, groups=groups)
    return a.permute(0, 2, 3, 1).numpy().round().astype(np.int64)


@pytest.mark.parametrize("cfg", [
    (2, 14, 14, 16, 24, 3, 3, (1, 1), (1, 1)),
    (1, 15, 13, 8, 12, 3, 3, (2, 2), (1, 1)),
    (1, 18, 18, 3, 8, 7, 7, (2, 2), (3, 3)),
    (2, 9, 11, 32, 10, 1, 1, (1, 1), (0, 0)),
    (1, 9, 11, 6, 10, 1, 1, (2, 2), (0, 0)),
    (1, 10, 12, 5, 7, 3, 5, (1, 2), (1, 2)),
])
def test_conv_vs_torch_fp64(oracle, cfg):
    B, H, W, C, N, R, S, stride, pad = cfg
    rng = np.random.default_rng(H * W + C)
    x = wl.draw_u8(rng, (B, H, W, C))
    w = rng.integers(-127, 128, (N, R, S, C), dtype=np.int8)
    bias = rng.integers(-5000, 5000, N).astype(np.int32)
    A = torch_acc(x, w, bias, stride, pad)
    for s in (0, 5, 9, 12):
        q = Q(3, 6, 9 - s, 0, 255)
        y = oracle.conv2d_fixed(x, w, bias, q, stride, pad)
        assert np.array_equal(y, fp64_requant(A, s, 0, 255))
    y32 = oracle.conv2d_fixed(x, w, bias, Q(3, 6, 0, y_type="s32"), stride, pad)
    assert np.array_equal(y32, A)


def test_dwconv_vs_torch_fp64(oracle):
    rng = np.random.default_rng(5)
    for stride in ((1, 1), (2, 2)):
        x = wl.draw_u8(rng, (2, 11, 9, 12))
        w = rng.integers(-127, 128, (3, 3, 12), dtype=np.int8)
        bias = rng.integers(-5000, 5000, 12).astype(np.int32)
        A = torch_acc(x, w, bias, stride, (1, 1), groups=12)
        y = oracle.dwconv_fixed(x, w, bias, Q(4, 3, 2, 0, 255), stride, (1, 1))
        assert np.array_equal(y, fp64_requant(A, 5, 0, 255))


# --------------------------------------------------------------------------- P7 structural identities

def test_conv1x1_is_gemm(oracle):
    rng = np.random.default_rng(21)
    x = wl.draw_u8(rng, (2, 5, 6, 10))
    w = rng.integers(-127, 128, (7, 1, 1, 10), dtype=np.int8)
    bias = rng.integers(-999, 999, 7).astype(np.int32)
    q = Q(4, 5, 3, 0, 255)
    y = oracle.conv2d_fixed(x, w, bias, q)
    g = oracle.gemm_fixed(x.reshape(-1, 10), w.reshape(7, 10), bias, q)
    assert np.array_equal(y.reshape(-1, 7), g)
    ys = oracle.conv2d_fixed(x, w, bias, q, (2, 2))
    gs = oracle.gemm_fixed(np.ascontiguousarray(x[:, ::2, ::2]).reshape(-1, 10), w.reshape(7, 10), bias, q)
    assert np.array_equal(ys.reshape(-1, 7), gs)


def test_dwconv_is_block_diagonal_dense(oracle):
    rng = np.random.default_rng(22)
    C = 6
    x = wl.draw_u8(rng, (1, 7, 8, C))
    wd = rng.integers(-127, 128, (3, 3, C), dtype=np.int8)
    bias = rng.integers(-999, 999, C).astype(np.int32)
    dense = np.zeros((C, 3, 3, C), np.int8)
    for c in range(C):
        dense[c, :, :, c] = wd[:, :, c]
    q = Q(4, 5, 4, 0, 255)
    for stride in ((1, 1), (2, 2)):
        a = oracle.dwconv_fixed(x, wd, bias, q, stride, (1, 1))
        b = oracle.conv2d_fixed(x, dense, bias, q, stride, (1, 1))
        assert np.array_equal(a, b)


def test_identity_and_zero_weights(oracle):
    rng = np.random.default_rng(23)
    x = wl.draw_u8(rng, (12, 8))
    for fl_w in range(0, 7):                       # W = 2^FL_w * I is the real identity
        w = (np.eye(8) * 2 ** fl_w).astype(np.int8)
        y = oracle.gemm_fixed(x, w, None, Q(3, fl_w, 3, 0, 200))
        assert np.array_equal(y, np.clip(x, 0, 200))
    bias = rng.integers(-2 ** 14, 2 ** 14, 8).astype(np.int32)
    y = oracle.gemm_fixed(x, np.zeros((8, 8), np.int8), bias, Q(3, 4, 0, 0, 255))
    want = np.clip(np.floor(bias / 128.0 + 0.5), 0, 255)
    assert np.array_equal(y, np.broadcast_to(want, y.shape))


def test_transposed_operand_would_fail(oracle):
    """Non-square, non-symmetric operands: y[m][n] pairs row m of x with row n of w."""
    x = np.array([[1, 2, 3], [4, 5, 6]], np.uint8)
    w = np.array([[1, 0, 0], [0, 1, 0], [0, 0, 1], [1, 1, 1]], np.int8)
    y = oracle.gemm_fixed(x, w, np.array([0, 10, 20, 30], np.int32), Q(0, 0, 0, 0, 255))
    assert y.tolist() == [[1, 12, 23, 36], [4, 15, 26, 45]]


# --------------------------------------------------------------------------- residual (Sec. 4.3 reading)

def test_residual_fp64_model_and_scale_invariance(oracle):
    rng = np.random.default_rng(31)
    for res_type in ("u8", "s8", "s32"):
        for trial in range(10):
            B, H, W, C, N = 1, 5, 4, 6, 5
            x = wl.draw_u8(rng, (B, H, W, C))
            w = rng.integers(-127, 128, (N, 3, 3, C), dtype=np.int8)
            bias = rng.integers(-999, 999, N).astype(np.int32)
            fl_x, fl_w = int(rng.integers(0, 7)), int(rng.integers(0, 7))
            fl_r = int(rng.integers(0, fl_x + fl_w + 5))
            s = int(rng.integers(0, 12))
            if res_type == "u8":
                r = wl.draw_u8(rng, (B, H, W, N))
            elif res_type == "s8":
                r = rng.integers(-63, 64, (B, H, W, N), dtype=np.int8)
            else:
                r = rng.integers(-2 ** 18, 2 ** 18, (B, H, W, N), dtype=np.int32)
            q = Q(fl_x, fl_w, fl_x + fl_w - s, 0, 255, res_type=res_type, fl_res=fl_r)
            y = oracle.conv2d_fixed(x, w, bias, q, (1, 1), (1, 1), res=r)
            A = torch_acc(x, w, bias, (1, 1), (1, 1))
            d = fl_x + fl_w - fl_r
            # residual brought to the accumulator scale: exact when d >= 0, one
            # round-half-up when its format is finer than the accumulator's
            rr = r.astype(np.float64) * 2.0 ** d
            A = A + (rr if d >= 0 else np.floor(rr + 0.5)).astype(np.int64)
            assert np.array_equal(y, fp64_requant(A, s, 0, 255))
            if res_type == "s8":                  # (FL_r + 1, 2R) is the same real tensor
                q2 = Q(fl_x, fl_w, fl_x + fl_w - s, 0, 255, res_type="s8", fl_res=fl_r + 1)
                y2 = oracle.conv2d_fixed(x, w, bias, q2, (1, 1), (1, 1), res=(2 * r).astype(np.int8))
                assert np.array_equal(y, y2)


def test_residual_brute_force(oracle):
    rng = np.random.default_rng(32)
    x = wl.draw_u8(rng, (1, 4, 5, 3))
    w = rng.integers(-30, 31, (4, 3, 3, 3), dtype=np.int8)
    bias = rng.integers(-300, 300, 4).astype(np.int32)
    r = rng.integers(-127, 128, (1, 4, 5, 4), dtype=np.int8)
    for fl_r in (2, 6, 9):                           # d = 6 - fl_r: 4, 0, -3
        q = Q(3, 3, 2, 0, 255, res_type="s8", fl_res=fl_r)
        y = oracle.conv2d_fixed(x, w, bias, q, (1, 1), (1, 1), res=r)
        want = brute_conv(x, w, bias, 1, 1, 1, 1, 4, 0, 255, res=r, d=6 - fl_r)
        assert np.array_equal(y, want)


# --------------------------------------------------------------------------- pools

def test_maxpool_vs_torch_and_brute(oracle):
    rng = np.random.default_rng(41)
    for kind in ("u8", "s8"):
        for (H, W, k, st, pd) in ((9, 8, 3, 2, 1), (7, 7, 2, 2, 0), (6, 5, 3, 1, 1), (5, 5, 3, 2, 0)):
            x = wl.draw_u8(rng, (2, H, W, 5)) if kind == "u8" else rng.integers(-128, 0, (2, H, W, 5), dtype=np.int8)
            y = oracle.maxpool(x, kind, (k, k), (st, st), (pd, pd))
            t = torch.nn.functional.max_pool2d(torch.from_numpy(x.astype(np.float64)).permute(0, 3, 1, 2),
                                               k, st, pd).permute(0, 2, 3, 1).numpy()
            assert np.array_equal(y.astype(np.int64), t.astype(np.int64))
    x = wl.draw_u8(rng, (1, 4, 4, 1))
    y = oracle.maxpool(x, "u8", (3, 3), (2, 2), (1, 1))
    for p in range(2):
        for q in range(2):
            win = [int(x[0, i, j, 0]) for i in range(2 * p - 1, 2 * p + 2) for j in range(2 * q - 1, 2 * q + 2)
                   if 0 <= i < 4 and 0 <= j < 4]
            assert int(y[0, p, q, 0]) == max(win)


def test_global_pool_is_sum_then_fixquant(oracle):
    rng = np.random.default_rng(42)
    x = wl.draw_u8(rng, (3, 7, 7, 10))
    q = Q(4, 6, 4, 0, 255)                          # weights are 1 at FL 6: real 1/64
    y = oracle.global_pool_fixed(x, q)
    A = x.astype(np.int64).sum(axis=(1, 2))
    assert np.array_equal(y, fp64_requant(A, 6, 0, 255))
    ones = np.ones((7, 7, 10), np.int8)
    y2 = oracle.dwconv_fixed(x, ones, np.zeros(10, np.int32), q, (1, 1), (0, 0))
    assert np.array_equal(y2.reshape(3, 10), y)


# --------------------------------------------------------------------------- error paths

def test_second_output_format_is_one_rounding_of_the_accumulator(oracle):
    """Two formats of one layer (Sec. 4.3, private fractional lengths): each output is the exact
    fp64 fix_quant of the same accumulator; re-rounding the finer output into the coarser format
    is a different (double-rounded) function, so the oracle must not be doing that."""
    rng = np.random.default_rng(41)
    x = rng.integers(0, 256, (64, 48)).astype(np.uint8)
    w = np.clip(np.rint(rng.normal(0, 12, (40, 48))), -127, 127).astype(np.int8)
    b = rng.integers(-4000, 4000, 40).astype(np.int32)
    A = int_gemm(x, w, b)
    q = Q(4, 6, 3, 0, 255)
    q.fl_y2, q.clip_lo2, q.clip_hi2, q.y2_type = 1, 0, 200, "u8"
    y, y2 = oracle.conv2d_fixed_dual(x.reshape(1, 1, 64, 48), w.reshape(40, 1, 1, 48), b, q)
    assert np.array_equal(y.reshape(64, 40), fp64_requant(A, 7, 0, 255))
    assert np.array_equal(y2.reshape(64, 40), fp64_requant(A, 9, 0, 200))
    twice = np.clip(np.floor(y.reshape(64, 40).astype(np.float64) / 4 + 0.5), 0, 200)
    assert (twice != y2.reshape(64, 40)).sum() > 0
    # the same format twice gives the same tensor twice
    q.fl_y2, q.clip_lo2, q.clip_hi2 = 3, 0, 255
    y, y2 = oracle.conv2d_fixed_dual(x.reshape(1, 1, 64, 48), w.reshape(40, 1, 1, 48), b, q)
    assert np.array_equal(y, y2)


def test_oracle_rejects_bad_arguments(oracle):
    x = np.zeros((2, 4), np.uint8)
    w = np.zeros((3, 4), np.int8)
    for q, code in ((Q(0, 0, 9), 3), (Q(12, 13, 0), 3), (Q(4, 4, 4, 5, 3), 4), (Q(4, 4, 4, 0, 256), 4),
                    (Q(4, 4, 4, -128, 0, y_type="s8"), 4)):
        with pytest.raises(oracle.OracleError) as e:
            oracle.gemm_fixed(x, w, None, q)
        assert e.value.code == code
    big = np.full((1, 4), 255, np.uint8)
    with pytest.raises(oracle.OracleError) as e:
        oracle.gemm_fixed(big, np.full((1, 4), 127, np.int8), np.array([2 ** 31 - 1000], np.int32), Q(0, 0, 0))
    assert e.value.code == 6


# --------------------------------------------------------------------------- P10 signed-MFMA identity

def test_unsigned_via_signed_identity():
    """sum W*X == sum W*(X xor 0x80 read as int8) + 128*sum W: what lets a signed 8-bit
    matrix unit consume unsigned activations exactly."""
    rng = np.random.default_rng(51)
    x = wl.draw_u8(rng, (40, 77))
    w = rng.integers(-127, 128, (9, 77), dtype=np.int8)
    xs = (x ^ 0x80).view(np.int8)
    lhs = x.astype(np.int64) @ w.astype(np.int64).T
    rhs = xs.astype(np.int64) @ w.astype(np.int64).T + 128 * w.astype(np.int64).sum(axis=1)
    assert np.array_equal(lhs, rhs)


# --------------------------------------------------------------------------- whole networks are well formed

def test_config_generators_are_deterministic_and_valid(oracle):
    x0, L0 = wl.config0()
    x0b, L0b = wl.config0()
    assert np.array_equal(x0, x0b) and np.array_equal(L0.w, L0b.w)
    assert x0.shape == (256, 64) and L0.w.shape == (64, 1, 1, 64) and L0.fl_x + L0.fl_w - L0.fl_y == 7
    x1, L1 = wl.config1(batch=1)
    assert L1.clip_hi == 192 and L1.fl_x + L1.fl_w - L1.fl_y == 8
    _, net = wl.config3(batch=1, hw=32)
    assert sum(L.op == "conv" for L in net.layers) == 21            # 20 convs + FC
    _, net = wl.config4(batch=1, hw=32)
    assert sum(L.op == "conv" for L in net.layers) == 54            # 53 convs + FC
    x, net = wl.config4(batch=2, hw=64)
    out = oracle.run_network(net, x)
    assert out.shape == (2, 1, 1, 1000) and out.dtype == np.int32
    par = oracle.run_network_parallel(net, x, 2)
    assert np.array_equal(out, par)
    full = wl.config4(batch=1)[1]
    assert abs(full.macs_per_image / 1e9 - 4.089) < 0.01             # ResNet-50: 4.09 GMAC per image
    assert abs(wl.config3(batch=1)[1].macs_per_image / 1e9 - 1.814) < 0.01
