"""Pins of the floating-point side of the CPU oracle (fix_quant and PACT on real tensors, the
choice of a fractional length, the toy experiment, Conv-BN folding) against things other than
itself: hand-worked fixtures, exact rational arithmetic, a library fake-quantiser, closed forms,
the ranges the paper states for the toy experiment, and the step-by-step quantise / dequantise /
convolve / normalise pipeline that the folded form is derived from.  No GPU is needed.
"""
import math
import os
import statistics
from fractions import Fraction

import numpy as np
import pytest
import torch

from oracle import quant_ref as qr
from paper_2202_05239_amd import workloads as wl

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def read_cases(name):
    rows = []
    with open(os.path.join(GOLD, name)) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if line:
                rows.append(line.split())
    return rows


def half_up(v: Fraction) -> int:
    return math.floor(v + Fraction(1, 2))


# --------------------------------------------------------------------------- Eq. 2 / Eq. 9

def test_fix_quant_golden():
    for kind, val, fl, want in read_cases("fixquant_cases.txt"):
        code = qr.fix_quant_code(np.array([float(val)]), int(fl), kind == "s")
        assert int(code[0]) == int(want), (kind, val, fl)


def test_round_half_up_is_exact():
    v = np.array([0.49999999999999994, 0.5, -0.5, -0.50000000000000011, 1.5, 2.5, -1.5,
                  2.0 ** 52 + 1.0, -3.0, 0.0])
    want = [0, 1, 0, -1, 2, 3, -1, 2.0 ** 52 + 1.0, -3, 0]
    assert qr.round_half_up(v).tolist() == want
    v32 = np.array([0.49999997, 8388607.5, -0.49999997], np.float32)
    assert qr.round_half_up(v32).tolist() == [0.0, 8388608.0, 0.0]


@pytest.mark.parametrize("is_signed", [False, True])
def test_fix_quant_exact_rational(is_signed):
    rng = np.random.default_rng(11)
    lo, hi = (-127, 127) if is_signed else (0, 255)
    x = np.concatenate([rng.standard_normal(300) * 3, rng.standard_normal(100) * 300,
                        np.arange(-20, 20) / 16.0 + 1 / 32.0,      # exact ties
                        [0.0, 1e-30, -1e-30, 1e30, -1e30]])
    for fl in range(0, 8 if is_signed else 9):
        got = qr.fix_quant_code(x, fl, is_signed)
        for xi, g in zip(x, got):
            v = Fraction(float(xi)) * 2 ** fl
            assert int(g) == half_up(min(max(v, lo), hi)), (xi, fl)
        assert np.array_equal(qr.fix_quant(x, fl, is_signed), got * 2.0 ** -fl)


def test_fix_quant_vs_library_fake_quantiser():
    """Away from exact ties Eq. 2 / Eq. 9 is the affine fake-quantiser with scale 2^-FL and
    zero point 0 (the library rounds ties to even, so ties are kept out of the sample)."""
    rng = np.random.default_rng(12)
    x = (rng.standard_normal(20000) * 4).astype(np.float32)
    for fl in (0, 3, 5, 7):
        frac = np.abs((x.astype(np.float64) * 2 ** fl) % 1.0 - 0.5)
        keep = frac > 1e-6
        for is_signed, (lo, hi) in ((False, (0, 255)), (True, (-127, 127))):
            want = torch.fake_quantize_per_tensor_affine(torch.from_numpy(x), 2.0 ** -fl, 0, lo, hi)
            got = qr.fix_quant(x, fl, is_signed)
            assert np.array_equal(got[keep], want.numpy().astype(np.float64)[keep])


def test_fix_quant_nan_and_inf():
    x = np.array([np.nan, np.inf, -np.inf])
    assert qr.fix_quant_code(x, 3, False).tolist() == [0, 255, 0]
    assert qr.fix_quant_code(x, 3, True).tolist() == [-127, 127, -127]


# --------------------------------------------------------------------------- Eq. 3, 4, 5

def test_pact_exact_rational_and_identity():
    """Eq. 3 evaluated with rationals; Eq. 4 with eta_fix of Eq. 5 is the same function."""
    rng = np.random.default_rng(13)
    for _ in range(200):
        alpha = float(rng.uniform(0.5, 9.0))
        fl = int(rng.integers(0, 9))
        x = rng.standard_normal(8) * alpha
        a = Fraction(alpha)
        for xi, got, got4 in zip(x, qr.pact(x, alpha), qr.pact_as_fix_quant(x, alpha, fl)):
            t = Fraction(255) / a * min(max(Fraction(float(xi)), 0), a)
            if abs(t - math.floor(t) - Fraction(1, 2)) < Fraction(1, 10 ** 9):
                continue                                   # a tie decided by fp64 rounding
            want = a / 255 * half_up(t)
            assert abs(Fraction(float(got)) - want) <= abs(want) * Fraction(1, 10 ** 14)
            assert abs(got4 - got) <= 1e-13 * max(abs(got), 1e-300)
    assert qr.eta_fix(255.0, 0) == 1.0 and qr.eta_fix(3.0, 4) == 16 * 3.0 / 255


def test_pact_is_fix_quant_when_alpha_fills_the_format():
    """alpha = (2^WL - 1) / 2^FL makes eta_fix = 1: PACT is then the unsigned fix_quant."""
    x = np.random.default_rng(14).standard_normal(5000) * 6
    for fl in range(9):
        assert np.allclose(qr.pact(x, 255.0 / 2 ** fl), qr.fix_quant(x, fl, False), rtol=1e-14, atol=0)
        assert np.array_equal(qr.pact_as_fix_quant(x, 255.0 / 2 ** fl, fl), qr.fix_quant(x, fl, False))


def test_pact_float32_path_is_within_one_code_of_fp64():
    x = wl.fp_tensor(15, 20000, std=3.0)
    a = 4.7
    y32 = qr.pact(x, a, dtype=np.float32)
    y64 = qr.pact(x, a)
    assert y32.dtype == np.float32
    assert np.max(np.abs(y32 - y64)) <= a / 255 * 1.0001
    assert np.mean(np.abs(y32 - y64) > 1e-5) < 1e-3


def round_to_f32(fr):
    """A rational rounded to the nearest float32 (ties to even), returned as a rational: the
    IEEE-754 rounding every float32 operation applies to its exact result (normal range only)."""
    if fr == 0:
        return Fraction(0)
    sign, a = (-1 if fr < 0 else 1), abs(fr)
    e = 0
    while a >= Fraction(2) ** (e + 1):
        e += 1
    while a < Fraction(2) ** e:
        e -= 1
    assert -126 <= e <= 127
    ulp = Fraction(2) ** (e - 23)
    m = a / ulp
    lo = math.floor(m)
    if m - lo > Fraction(1, 2) or (m - lo == Fraction(1, 2) and lo % 2 == 1):
        lo += 1
    return sign * lo * ulp


def test_pact_float32_step_order_exact():
    """The float32 readings of Eq. 3 and Eq. 4 (every operation rounded to float32, in the order
    of the equation) against that order written out with rationals and an explicit model of
    float32 rounding: equality on every point, ties included (the value that is rounded to a
    code is itself a float32, so a tie is a well-defined input)."""
    rng = np.random.default_rng(151)
    f32 = lambda v: Fraction(float(np.float32(v)))
    for trial in range(60):
        alpha = float(rng.uniform(0.3, 9.0))
        fl = int(rng.integers(0, 9))
        x = np.concatenate([wl.fp_tensor(1000 + trial, 40, std=alpha),
                            np.float32(alpha) * (np.arange(0, 12, dtype=np.float32) + np.float32(0.5)) / np.float32(255)])
        a = f32(alpha)
        k_in = round_to_f32(Fraction(255) / a)
        k_out = round_to_f32(a / 255)
        eta = f32(2.0 ** fl * alpha / 255)                 # Eq. 5 in fp64, then one rounding to float32
        got3 = qr.pact(x, alpha, dtype=np.float32)
        got4 = qr.pact_as_fix_quant(x, alpha, fl, dtype=np.float32)
        assert got3.dtype == np.float32 and got4.dtype == np.float32
        for xi, g3, g4 in zip(x, got3, got4):
            xf = Fraction(float(xi))
            p3 = round_to_f32(min(max(xf, 0), a) * k_in)
            want3 = round_to_f32(half_up(p3) * k_out)
            assert Fraction(float(g3)) == want3, (alpha, float(xi))
            u = round_to_f32(xf / eta)
            v = min(max(u * 2 ** fl, 0), 255)               # power-of-two scaling and clip: exact
            want4 = round_to_f32(half_up(v) * Fraction(1, 2 ** fl) * eta)
            assert Fraction(float(g4)) == want4, (alpha, fl, float(xi))


# --------------------------------------------------------------------------- Eq. 1

def test_opt_fl_next_to_every_threshold():
    """Eq. 1 is the floor of the exact logarithm.  The neighbours of every threshold c / 2^k are
    where a floor of a rounded floating-point log2 goes wrong: at least one of these points must
    defeat that shortcut (so the pin is live), and none may defeat the oracle."""
    shortcut_fails = 0
    for is_signed, c, top in ((True, 40.0, 7), (False, 70.0, 8)):
        for k in range(-3, 12):
            t = c / 2.0 ** k                                 # exact: c has few bits
            for s in (np.nextafter(t, 0.0), t, np.nextafter(t, np.inf)):
                s = float(s)
                kk = -60
                while Fraction(s) * Fraction(2) ** (kk + 1) <= Fraction(c):
                    kk += 1
                want = min(max(kk, 0), top)
                assert qr.opt_fl(s, is_signed) == want, (s, is_signed)
                shortcut = min(max(math.floor(math.log2(c / s)), 0), top)
                shortcut_fails += shortcut != want
    assert shortcut_fails > 0


def test_opt_fl_is_the_largest_shift_that_keeps_sigma_under_the_constant():
    """floor(log2(c / sigma)) is the largest k with sigma * 2^k <= c; checked with rationals."""
    rng = np.random.default_rng(16)
    sig = np.concatenate([10 ** rng.uniform(-3, 3, 500), [40.0, 20.0, 10.0, 0.3125, 70.0, 35.0, 17.5,
                                                           np.nextafter(20.0, 30.0), np.nextafter(35.0, 40.0)]])
    for s in sig:
        for is_signed, c, top in ((True, 40, 7), (False, 70, 8)):
            k = -60
            while Fraction(float(s)) * Fraction(2) ** (k + 1) <= c:
                k += 1
            assert qr.opt_fl(float(s), is_signed) == min(max(k, 0), top), (s, is_signed)
    assert qr.opt_fl(40.0, True) == 0 and qr.opt_fl(20.0, True) == 1 and qr.opt_fl(20.000001, True) == 0
    assert qr.opt_fl(70.0 / 64, False) == 6 and qr.opt_fl(1e-9, False) == 8 and qr.opt_fl(1e9, False) == 0
    assert qr.opt_fl(0.0, True) == 7 and qr.opt_fl(0.0, False) == 8


def test_moments_closed_forms():
    n, d, a0 = 1001, 0.37, -5.0
    x = a0 + d * np.arange(n)
    m, s = qr.moments(x)
    assert abs(m - (a0 + d * (n - 1) / 2)) < 1e-12
    assert abs(s - d * math.sqrt((n * n - 1) / 12.0)) < 1e-12
    y = [0.5, -1.25, 3.0, 3.0, 7.75]
    m, s = qr.moments(np.array(y))
    assert abs(m - statistics.fmean(y)) < 1e-15 and abs(s - statistics.pstdev(y)) < 1e-15
    assert qr.moments(np.full(10, 2.5)) == (2.5, 0.0)


# --------------------------------------------------------------------------- toy experiment

SIGNED_GRID = [0.25, 0.5, 1, 2, 3, 5, 8, 10, 16, 20, 25, 40]
UNSIGNED_GRID = [0.13, 0.25, 0.5, 1, 2, 5, 10, 20, 40, 50, 70, 100]


def test_rel_error_closed_form_inside_the_representing_region():
    """With no clipping and many levels the rounding error is uniform on +-LSB/2: its mean
    magnitude is LSB/4, and E|x| = sigma * sqrt(2/pi) for a Gaussian."""
    z = wl.toy_samples().astype(np.float64)
    for sigma, fl in ((1.0, 5), (0.5, 6), (4.0, 3), (2.0, 4)):
        want = (2.0 ** -fl / 4) / (sigma * math.sqrt(2 / math.pi))
        got = qr.rel_quant_error(z * sigma, fl, True)
        assert abs(got / want - 1) < 0.03, (sigma, fl, got, want)
    # rectified: half the samples are exactly zero and exactly represented
    want = (2.0 ** -6 / 4 / 2) / (1.0 * math.sqrt(2 / math.pi) / 2)
    assert abs(qr.rel_quant_error(z, 6, False) / want - 1) < 0.03


def test_toy_experiment_ranges_of_the_paper():
    """Sec. 3.1: picking the best format keeps the relative error near or under 1 % for
    standard deviations up to about 40 (signed) and about 100 (unsigned), over a range of
    two to three orders of magnitude; outside those ranges it does not."""
    z = wl.toy_samples().astype(np.float64)
    for grid, is_signed, fls in ((SIGNED_GRID, True, range(8)), (UNSIGNED_GRID, False, range(9))):
        for sigma in grid:
            best = min(qr.rel_quant_error(z * sigma, fl, is_signed) for fl in fls)
            assert best < 0.0125, (sigma, is_signed, best)
    assert min(qr.rel_quant_error(z * 60.0, fl, True) for fl in range(8)) > 0.02
    assert min(qr.rel_quant_error(z * 150.0, fl, False) for fl in range(9)) > 0.03
    assert min(qr.rel_quant_error(z * 0.05, fl, True) for fl in range(8)) > 0.03
    assert min(qr.rel_quant_error(z * 0.03, fl, False) for fl in range(9)) > 0.03


def test_eq1_tracks_the_brute_force_optimum():
    """Eq. 1 is a fit to the jumps of the best fractional length: it is never more than one
    step from the brute-force optimum (one step costs about a factor two in error)."""
    z = wl.toy_samples().astype(np.float64)
    for is_signed, fls in ((True, list(range(8))), (False, list(range(9)))):
        agree = 0
        grid = 10 ** np.linspace(-0.6, 1.6 if is_signed else 2.0, 40)
        for sigma in grid:
            errs = [qr.rel_quant_error(z * sigma, fl, is_signed) for fl in fls]
            best = int(np.argmin(errs))
            pick = qr.opt_fl(float(sigma), is_signed)
            assert abs(pick - best) <= 1, (sigma, is_signed, pick, best)
            assert errs[pick] <= 2.2 * errs[best]
            agree += pick == best
        assert agree >= 0.6 * len(grid)


# --------------------------------------------------------------------------- Eq. 6

def appendix_pipeline(blk, x_prev):
    """The Conv-BN-ReLU block with the conventional quantise / dequantise PACT input, one step
    per line, and the next block's input quantiser (appendix on the effective weight)."""
    M = 255.0
    x_t = np.clip(x_prev, 0.0, blk.alpha_in)                         # nonlinearity
    q_hat = qr.round_half_up(M / blk.alpha_in * x_t)                 # integer input
    q_til = blk.alpha_in / M * q_hat                                 # dequantised input
    y = q_til @ blk.W.astype(np.float64).T                           # convolution (as a GEMM)
    g = blk.gamma.astype(np.float64)
    x_l = g * (y - blk.mu.astype(np.float64)) / blk.sigma.astype(np.float64) + blk.beta.astype(np.float64)
    x_t1 = np.clip(x_l, 0.0, blk.alpha_out)
    return q_hat, M / blk.alpha_out * x_t1                           # argument of the next round()


def test_effective_weight_reproduces_the_dequantise_conv_bn_pipeline():
    for seed, cout, k in ((21, 24, 40), (22, 7, 147), (23, 33, 9)):
        blk = wl.fp_conv_bn_block(seed, cout, k)
        rng = np.random.default_rng(seed + 100)
        x_prev = rng.standard_normal((50, k)) * blk.alpha_in * 0.6
        q_hat, want_arg = appendix_pipeline(blk, x_prev)
        eta_in = qr.eta_fix(blk.alpha_in, blk.fl_in)
        eta_out = qr.eta_fix(blk.alpha_out, blk.fl_out)
        W_eff, b_eff = qr.effective_weight_bias(blk.W, blk.gamma, blk.beta, blk.mu, blk.sigma, eta_in, eta_out)
        q = q_hat * 2.0 ** -blk.fl_in                                # fixed-point activation of Eq. 6
        v = q @ W_eff.T + b_eff                                      # argument of fix_quant
        got_arg = np.clip(v * 2.0 ** blk.fl_out, 0, 255)
        assert np.allclose(got_arg, want_arg, rtol=1e-12, atol=1e-10)
        # and the codes agree wherever fp64 rounding cannot move the argument across a tie
        safe = np.abs(want_arg % 1.0 - 0.5) > 1e-8
        assert np.array_equal(qr.round_half_up(got_arg)[safe], qr.round_half_up(want_arg)[safe])
        assert safe.mean() > 0.999 and (got_arg > 0).mean() > 0.2


def test_export_quantises_eq6_and_drives_the_integer_layer(oracle):
    """The exported integers are the nearest codes of Eq. 6 at FL_w / FL_x + FL_w, FL_w is the
    Eq. 1 choice, and the integer layer run on them stays within the bound that the weight and
    bias rounding allow from the unquantised pipeline."""
    from test_oracle_pins import Q
    for seed, cout, k in ((31, 16, 64), (32, 5, 27)):
        blk = wl.fp_conv_bn_block(seed, cout, k)
        eta_in = qr.eta_fix(blk.alpha_in, blk.fl_in)
        eta_out = qr.eta_fix(blk.alpha_out, blk.fl_out)
        W_eff, b_eff = qr.effective_weight_bias(blk.W, blk.gamma, blk.beta, blk.mu, blk.sigma, eta_in, eta_out)
        Wq, Bq, fl_w = qr.export_conv_bn(blk.W, blk.gamma, blk.beta, blk.mu, blk.sigma, eta_in, eta_out, blk.fl_in)
        assert Wq.dtype == np.int8 and Bq.dtype == np.int32
        sd = float(np.sqrt(np.mean((W_eff - W_eff.mean()) ** 2)))
        assert fl_w == min(max(math.floor(math.log2(40 / sd)), 0), 7)
        inside = np.abs(W_eff * 2 ** fl_w) <= 127
        assert np.all(np.abs(Wq[inside] - W_eff[inside] * 2 ** fl_w) <= 0.5)
        assert np.all(np.abs(Wq[~inside]) == 127) and inside.mean() > 0.95
        assert np.all(np.abs(Bq - b_eff * 2.0 ** (blk.fl_in + fl_w)) <= 0.5)
        # integer layer on the exported parameters
        rng = np.random.default_rng(seed + 100)
        codes = rng.integers(0, 256, (40, k)).astype(np.uint8)
        y = oracle.gemm_fixed(codes, Wq, Bq, Q(blk.fl_in, fl_w, blk.fl_out, 0, 255))
        v = (codes * 2.0 ** -blk.fl_in) @ W_eff.T + b_eff            # Eq. 6, unquantised parameters
        ideal = np.clip(v * 2.0 ** blk.fl_out, 0, 255)
        slack = (codes.astype(np.float64).sum(axis=1, keepdims=True) * 0.5 * 2.0 ** -(blk.fl_in + fl_w)
                 + 0.5 * 2.0 ** -(blk.fl_in + fl_w)) * 2.0 ** blk.fl_out
        # clipped weights add their own error; keep rows whose weights were all inside
        rows = np.all(inside, axis=1)
        assert np.all(np.abs(y.astype(np.float64) - ideal)[:, rows] <= (0.5 + slack + 1e-9))
        assert rows.sum() >= cout // 2
    # a given fractional length is used as it is
    assert qr.export_conv_bn(blk.W, blk.gamma, blk.beta, blk.mu, blk.sigma, eta_in, eta_out, 4, fl_w=3)[2] == 3


def test_export_saturates_the_bias():
    blk = wl.fp_conv_bn_block(33, 4, 8)
    beta = np.array([1e9, -1e9, 0.0, 1.0], np.float32)
    _, Bq, _ = qr.export_conv_bn(blk.W, blk.gamma, beta, blk.mu * 0, blk.sigma, 1.0, 1.0, 8, fl_w=7)
    assert Bq.tolist() == [2 ** 31 - 1, -2 ** 31, 0, 2 ** 15]
