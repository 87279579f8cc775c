"""CPU oracle for the steps just upstream of the integer layers (test infrastructure; never
on the product path): the floating-point fix_quant and PACT quantisers, the choice of a
fractional length from a standard deviation, the toy experiment on the representing region of
each format, and the folding of a Conv-BN block into 8-bit weights and a 32-bit bias.

Plain numpy in fp64, one function per equation of the paper, nothing blocked or fused.  Where
a floating-point value decides an integer code and the paper fixes no precision, the function
takes the precision of the data as a `dtype` argument and evaluates its steps in that
precision in the order written, so that a device kernel that follows the same steps must
reproduce the codes exactly.

`round` is round half up (floor(v + 1/2)), the same reading the integer oracle uses, written
so that it is exact for every finite v.
"""
import math

import numpy as np


def round_half_up(v):
    """floor(v + 1/2) without the double rounding the sum can suffer in floating point."""
    v = np.asarray(v)
    r = np.floor(v)
    return r + (v - r >= 0.5)


def code_bounds(is_signed, wl=8):
    """Integer range of a WL-bit code: Eq. 2 (unsigned) and Eq. 9 (signed, symmetric)."""
    if is_signed:
        return -(2 ** (wl - 1)) + 1, 2 ** (wl - 1) - 1
    return 0, 2 ** wl - 1


def fix_quant_code(x, fl, is_signed, wl=8):
    """The integer inside Eq. 2 / Eq. 9: round(clip(x * 2^FL, lo, hi)).  A NaN takes the lower
    bound (fmax/fmin semantics)."""
    lo, hi = code_bounds(is_signed, wl)
    v = np.asarray(x, dtype=np.float64) * 2.0 ** fl           # exact: power-of-two scaling
    v = np.fmin(np.fmax(v, lo), hi)
    return round_half_up(v).astype(np.int64)


def fix_quant(x, fl, is_signed, wl=8):
    """Eq. 2 / Eq. 9: the fixed-point value 2^-FL * round(clip(x * 2^FL, lo, hi))."""
    return fix_quant_code(x, fl, is_signed, wl) * 2.0 ** (-fl)


def pact(x, alpha, M=255, dtype=np.float64):
    """Eq. 3: (alpha / M) * round((M / alpha) * clip(x, 0, alpha)), every step in `dtype`."""
    t = dtype
    x = np.asarray(x, dtype=t)
    a = t(alpha)
    k_in = t(M) / a
    k_out = a / t(M)
    c = np.fmin(np.fmax(x, t(0)), a)
    return (round_half_up(c * k_in).astype(t) * k_out).astype(t)


def eta_fix(alpha, fl, wl=8):
    """Eq. 5: the fix scaling factor 2^FL * alpha / (2^WL - 1)."""
    return 2.0 ** fl * alpha / (2 ** wl - 1)


def pact_as_fix_quant(x, alpha, fl, wl=8, dtype=np.float64):
    """Eq. 4: eta_fix * fix_quant(x / eta_fix), unsigned; the division, the quantiser and the
    final product each in `dtype`.  eta_fix itself is formed in fp64 and rounded to `dtype`."""
    t = dtype
    eta = t(eta_fix(alpha, fl, wl))
    u = np.asarray(x, dtype=t) / eta
    lo, hi = code_bounds(False, wl)
    v = np.fmin(np.fmax(u * t(2.0 ** fl), t(lo)), t(hi))
    q = round_half_up(v).astype(t) * t(2.0 ** (-fl))
    return (q * eta).astype(t)


def moments(x):
    """Mean and population standard deviation of all elements (fp64)."""
    x = np.asarray(x, dtype=np.float64).ravel()
    return float(np.mean(x)), float(np.std(x))


def opt_fl(sigma, is_signed, wl=8):
    """Eq. 1: FL* = floor(log2(40 / sigma)) signed, floor(log2(70 / sigma)) unsigned, kept
    inside the range the format allows (0..WL-1 signed, 0..WL unsigned); sigma = 0 takes the
    largest."""
    top = wl - 1 if is_signed else wl
    if not sigma > 0.0:
        return top
    ratio = (40.0 if is_signed else 70.0) / sigma
    if math.isinf(ratio):
        return top
    k = math.floor(math.log2(ratio))
    # log2 of a value one rounding step below a power of two may come back as the integer
    # itself; the floor is taken of the exact logarithm
    if 2.0 ** k > ratio:
        k -= 1
    elif 2.0 ** (k + 1) <= ratio:
        k += 1
    return int(min(max(k, 0), top))


def rel_quant_error(x, fl, is_signed, wl=8):
    """Relative quantisation error of the toy experiment (Sec. 3.1, appendix on the statistical
    analysis): sum |v - fix_quant(v)| / sum |v|, where v = x for the signed format and
    v = relu(x) for the unsigned one."""
    v = np.asarray(x, dtype=np.float64)
    if not is_signed:
        v = np.maximum(v, 0.0)
    return float(np.sum(np.abs(v - fix_quant(v, fl, is_signed, wl))) / np.sum(np.abs(v)))


def effective_weight_bias(W, gamma, beta, mu, sigma, eta_in, eta_out):
    """Eq. 6 for one Conv-BN block: W is [Cout][...]; the four BN vectors have Cout entries.

        W_eff[i, ...] = (gamma_i / sigma_i) * (eta_in / eta_out) * W[i, ...]
        b_eff[i]      = (beta_i - (gamma_i / sigma_i) * mu_i) / eta_out
    """
    W = np.asarray(W, dtype=np.float64)
    g = np.asarray(gamma, np.float64) / np.asarray(sigma, np.float64)
    scale = g * (np.float64(eta_in) / np.float64(eta_out))
    W_eff = W * scale.reshape((-1,) + (1,) * (W.ndim - 1))
    b_eff = (np.asarray(beta, np.float64) - g * np.asarray(mu, np.float64)) / np.float64(eta_out)
    return W_eff, b_eff


def export_conv_bn(W, gamma, beta, mu, sigma, eta_in, eta_out, fl_x, fl_w=None, wl=8):
    """The integer parameters of a folded block: Eq. 6, then the weight fractional length by
    Eq. 1 from the standard deviation of the whole effective weight tensor (unless given), the
    weights by the signed fix_quant (Eq. 9) and the bias as a 32-bit integer at the
    accumulator's fractional length FL_x + FL_w (saturated)."""
    W_eff, b_eff = effective_weight_bias(W, gamma, beta, mu, sigma, eta_in, eta_out)
    if fl_w is None:
        fl_w = opt_fl(moments(W_eff)[1], True, wl)
    Wq = fix_quant_code(W_eff, fl_w, True, wl).astype(np.int8)
    v = np.fmin(np.fmax(b_eff * 2.0 ** (fl_x + fl_w), -2.0 ** 31), 2.0 ** 31 - 1)
    Bq = round_half_up(v).astype(np.int64).astype(np.int32)
    return Wq, Bq, int(fl_w)
