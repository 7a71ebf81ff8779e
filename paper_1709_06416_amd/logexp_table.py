"""Tables and constants of the library's own log and exp for f64 (build step; no GPU needed).

The device math library's log costs about 94 vector instructions and its exp about 38; the
Black-Scholes loop (Sec. 7.1 of the paper: "square roots, exponents and logarithms") issues more
instructions than its memory traffic gives it time for, so the run-time compiled kernels evaluate
both themselves, from small tables that this module computes in 80-digit decimal arithmetic.

log(x):  x = 2^e * m with m in [181/256, 362/256) (the binade is split at 181/256 ~ sqrt(1/2), so
    that arguments just below 1 are not the difference of -ln 2 and a number close to ln 2).
    m falls into one of 91 intervals of width 1/128, [(90+i)/128, (91+i)/128); the table holds, per
    interval, R = the double nearest 1/c (c the interval's centre) and -ln(R) as a high and a low
    double.  r = fma(m, R, -1) is small (|r| <= 2^-7) and m = (1 + r)/R holds exactly for the
    ROUNDED R, so  log(x) = e ln2 + (-ln R) + log1p(r),  log1p(r) = r - r^2/2 + ... - r^8/8
    (remainder |r|^9/9 < 1.3e-20).  The two intervals that touch 1 have R = 1 and -ln R = 0: there
    r = m - 1 exactly and the result keeps its relative accuracy as x -> 1.
exp(x):  n = rint(x * 64/ln2), r = x - n ln2/64 (|r| <= ln2/128, subtracted in two pieces),
    exp(x) = 2^(n >> 6) * 2^((n & 63)/64) * e^r, with 2^(j/64) from a table (high and low double)
    and e^r - 1 = r + r^2/2 + ... + r^6/720 (remainder < 3e-20).
ln2 and ln2/64 are split so that their high parts times any exponent / any n are exact.
"""
import decimal

LOG_INTERVALS = 91
LOG_FIRST = 90            # interval i covers m in [(LOG_FIRST + i)/128, (LOG_FIRST + i + 1)/128)
EXP_ENTRIES = 64


def _ctx():
    return decimal.Context(prec=80)


def _to_float(c, d):
    """The double nearest the decimal d (float() of a decimal string is correctly rounded)."""
    return float(str(c.plus(d)))


def _split(c, d, bits):
    """d as (hi, lo): hi has at most `bits` significant bits, lo is the double nearest d - hi."""
    hi = _to_float(c, d)
    m, e = __import__("math").frexp(hi)
    scale = 2.0 ** bits
    hi = __import__("math").ldexp(round(m * scale) / scale, e)
    lo = _to_float(c, c.subtract(d, decimal.Decimal(hi)))
    return hi, lo


def log_rows():
    """LOG_INTERVALS rows (R, -ln R high, -ln R low)."""
    c = _ctx()
    rows = []
    for i in range(LOG_INTERVALS):
        if LOG_FIRST + i in (127, 128):
            rows.append((1.0, 0.0, 0.0))
            continue
        centre = c.divide(decimal.Decimal(2 * (LOG_FIRST + i) + 1), decimal.Decimal(256))
        r = _to_float(c, c.divide(decimal.Decimal(1), centre))
        neg_ln = c.minus(c.ln(decimal.Decimal(r)))
        hi = _to_float(c, neg_ln)
        lo = _to_float(c, c.subtract(neg_ln, decimal.Decimal(hi)))
        rows.append((r, hi, lo))
    return rows


def exp_rows():
    """EXP_ENTRIES rows (2^(j/64) high, low)."""
    c = _ctx()
    ln2 = c.ln(decimal.Decimal(2))
    rows = []
    for j in range(EXP_ENTRIES):
        v = c.exp(c.divide(c.multiply(ln2, decimal.Decimal(j)), decimal.Decimal(EXP_ENTRIES)))
        hi = _to_float(c, v)
        lo = _to_float(c, c.subtract(v, decimal.Decimal(hi)))
        rows.append((hi, lo))
    return rows


def constants():
    c = _ctx()
    ln2 = c.ln(decimal.Decimal(2))
    ln2_hi, ln2_lo = _split(c, ln2, 41)                       # times |e| < 2^11: exact in 53 bits
    l64 = c.divide(ln2, decimal.Decimal(64))
    l64_hi, l64_lo = _split(c, l64, 35)                       # times |n| < 2^17: exact
    inv_l64 = _to_float(c, c.divide(decimal.Decimal(64), ln2))
    out = {"W_LN2_HI": ln2_hi, "W_LN2_LO": ln2_lo, "W_L64_HI": l64_hi, "W_L64_LO": l64_lo, "W_INV_L64": inv_l64}
    for k in range(2, 9):                                     # log1p: (-1)^(k+1) / k
        out["W_LOG_C%d" % k] = (1.0 if k % 2 else -1.0) / k
    f = 1
    for k in range(2, 7):                                     # e^r: 1 / k!
        f *= k
        out["W_EXP_C%d" % k] = 1.0 / f
    return out


def log_initialiser():
    return ",\n".join(", ".join(float.hex(v) for v in row) for row in log_rows())


def exp_initialiser():
    return ",\n".join(", ".join(float.hex(v) for v in row) for row in exp_rows())


def constant_defines():
    return "\n".join("#define %s %s" % (k, float.hex(v)) for k, v in constants().items())


if __name__ == "__main__":
    print(constant_defines())
    print(log_initialiser())
    print(exp_initialiser())
