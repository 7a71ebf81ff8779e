"""The tables of the library's own log and exp (paper_1709_06416_amd/logexp_table.py), checked on the CPU.

The kernels' evaluation order is written out here step by step with every fused multiply-add rounded
once (exact rational arithmetic, then one rounding to f64), and compared with 60-digit decimal
logarithms and exponentials: the pins are the decimal values, not libm.  No GPU is needed.
"""
import decimal
import math
from fractions import Fraction

import numpy as np

from paper_1709_06416_amd import logexp_table as T

CTX = decimal.Context(prec=60)


def fma(a, b, c):
    if not (math.isfinite(a) and math.isfinite(b) and math.isfinite(c)):
        return a * b + c
    return float(Fraction(a) * Fraction(b) + Fraction(c))          # float(Fraction) rounds to nearest even


LOG = T.log_rows()
EXP = T.exp_rows()
K = T.constants()


def dev_log(x):
    """w_log of fused_prelude.hip.h, operation by operation."""
    if x != x:
        return x
    if x < 0.0:
        return math.nan
    if x == 0.0:
        return -math.inf
    if math.isinf(x):
        return x
    m, e = math.frexp(x)                                            # m in [0.5, 1), like v_frexp_mant / v_frexp_exp
    if m < 0.70703125:
        m, e = m * 2.0, e - 1
    i = min(max(int(m * 128.0) - 90, 0), 90)
    R, lhi, llo = LOG[i]
    r = fma(m, R, -1.0)
    p = K["W_LOG_C8"]
    for k in range(7, 1, -1):
        p = fma(p, r, K["W_LOG_C%d" % k])
    fe = float(e)
    hi = fma(fe, K["W_LN2_HI"], lhi)
    lo = fma(fe, K["W_LN2_LO"], llo)
    return hi + (r + fma(p, r * r, lo))


def dev_exp(x):
    """w_exp of fused_prelude.hip.h, operation by operation."""
    if x != x:
        return x
    xc = min(max(x, -1000.0), 1000.0)
    fn = float(round(xc * K["W_INV_L64"]))                          # round() of a float: ties to even, like v_rndne
    n = int(fn)
    r = fma(-fn, K["W_L64_HI"], xc)
    r = fma(-fn, K["W_L64_LO"], r)
    th, tl = EXP[n & 63]
    p = K["W_EXP_C6"]
    for k in range(5, 1, -1):
        p = fma(p, r, K["W_EXP_C%d" % k])
    p = fma(p, r * r, r)
    s = th + fma(th, p, tl)
    try:
        return math.ldexp(s, n >> 6)
    except OverflowError:
        return math.inf


def ulps(got, want_decimal):
    want = float(want_decimal)
    u = math.ulp(want)
    return abs(Fraction(got) - Fraction(str(want_decimal))) / Fraction(u)


def test_table_shapes_and_anchor_rows():
    assert len(LOG) == 91 and len(EXP) == 64
    assert LOG[37] == (1.0, 0.0, 0.0) and LOG[38] == (1.0, 0.0, 0.0)   # the intervals that touch 1: r = m - 1 exactly
    assert EXP[0] == (1.0, 0.0) and EXP[32][0] == math.sqrt(2.0)
    for i, (R, lhi, llo) in enumerate(LOG):
        c = (2 * (90 + i) + 1) / 256.0
        if i not in (37, 38):
            assert abs(R * c - 1.0) < 1e-15 and abs(lhi - math.log(c)) < 1e-15 and abs(llo) < 2e-16 * abs(lhi) + 1e-300
    # ln2 = high + low exactly to ~2^-95, and the high part times any binary exponent is exact in 53 bits
    ln2 = CTX.ln(decimal.Decimal(2))
    assert abs(decimal.Decimal(K["W_LN2_HI"]) + decimal.Decimal(K["W_LN2_LO"]) - ln2) < decimal.Decimal(2) ** -94
    assert Fraction(K["W_LN2_HI"]).denominator <= 2 ** 41
    assert all(float(Fraction(K["W_LN2_HI"]) * e) == K["W_LN2_HI"] * e and Fraction(K["W_LN2_HI"] * e) == Fraction(K["W_LN2_HI"]) * e
               for e in (-1074, -1022, -1, 1, 1023, 1024))


def test_log_against_decimal_logarithms():
    rnd = np.random.RandomState(3)
    xs = np.concatenate([
        rnd.uniform(0.1, 10.0, 1500),                       # price / strike of the option workload
        np.exp(rnd.uniform(-700, 700, 600)),
        1.0 + rnd.uniform(-1e-2, 1e-2, 300), 1.0 + rnd.uniform(-1e-9, 1e-9, 100),
        np.nextafter(np.arange(90, 182) / 128.0, 0), np.arange(90, 182) / 128.0,       # interval edges
        [1.0, np.nextafter(1.0, 0), np.nextafter(1.0, 2), 0.70703125, np.nextafter(0.70703125, 0), 2.0, 0.5,
         5e-324, 2.2250738585072014e-308, 1.7976931348623157e308]])
    worst = Fraction(0)
    for x in xs:
        x = float(x)
        got = dev_log(x)
        want = CTX.ln(decimal.Decimal(x))
        if x == 1.0:
            assert got == 0.0
            continue
        worst = max(worst, ulps(got, want))
    assert worst <= Fraction(3, 2), float(worst)            # within 1.5 units in the last place of the decimal value
    for x in (1.0 - 2.0 ** -30, 1.0 + 2.0 ** -40):          # relative accuracy where the result is tiny
        want = float(CTX.ln(decimal.Decimal(x)))
        assert abs(dev_log(x) - want) <= 2.3e-16 * abs(want)
    assert dev_log(0.0) == -math.inf and dev_log(-0.0) == -math.inf and math.isnan(dev_log(-1.0))
    assert dev_log(math.inf) == math.inf and math.isnan(dev_log(math.nan))


def test_exp_against_decimal_exponentials():
    rnd = np.random.RandomState(4)
    xs = np.concatenate([rnd.uniform(-0.05, 0.0, 800),      # -rate * t of the option workload
                         rnd.uniform(-700, 700, 1500), rnd.uniform(-1, 1, 500), rnd.uniform(-1e-9, 1e-9, 50),
                         (np.arange(-64, 65) + 0.5) * math.log(2) / 64,               # where n = rint(.) flips
                         [0.0, -0.0, 709.782712893384, -708.3964185322641, 1.0, -1.0, math.log(2)]])
    worst = Fraction(0)
    for x in xs:
        x = float(x)
        got = dev_exp(x)
        want = CTX.exp(decimal.Decimal(x))
        worst = max(worst, ulps(got, want))
    assert worst <= Fraction(3, 2), float(worst)
    assert dev_exp(0.0) == 1.0 and dev_exp(-0.0) == 1.0
    assert dev_exp(710.0) == math.inf and dev_exp(1e300) == math.inf and dev_exp(math.inf) == math.inf
    assert dev_exp(-746.0) == 0.0 and dev_exp(-1e300) == 0.0 and dev_exp(-math.inf) == 0.0
    assert math.isnan(dev_exp(math.nan))
    d = dev_exp(-740.0)                                      # a denormal result: within one denormal step
    assert abs(d - float(CTX.exp(decimal.Decimal(-740.0)))) <= 5e-324
