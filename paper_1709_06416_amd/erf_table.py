"""Coefficient table of the library's own erf (build step; no GPU needed).

The run-time compiled kernels evaluate erf(x) for f64 as a piecewise Taylor polynomial: |x| is
cut into 96 intervals of width 1/16 on [0, 6); interval k >= 1 is expanded about its centre
(k + 1/2)/16, interval 0 about 0 (only odd terms there, so small arguments keep their
relative accuracy); beyond 6 the result is +-1, which is what erf rounds to in f64 from
5.93 on.  Degree 9: the remainder is (1/32)^10 / 10! * max|erf^(10)| < 4e-18 (interval 0:
the x^11 term, below 7e-16 relative), far below one rounding of the result.

The coefficients are erf^(j)(c) / j! with
    erf'(x) = 2/sqrt(pi) exp(-x^2),   erf^(n+1)(x) = 2/sqrt(pi) (-1)^n H_n(x) exp(-x^2),
H_n the physicists' Hermite polynomials (H_{n+1} = 2x H_n - 2n H_{n-1}), computed here in
80-digit decimal arithmetic and rounded once to f64.  erf(c) itself comes from its Maclaurin
series in the same arithmetic (alternating, terms up to e^36 at c = 6: 80 digits leave more
than 40 after the cancellation).
"""
import decimal

INTERVALS = 96
DEGREE = 9
WIDTH_INV = 16           # intervals per unit


def _ctx():
    c = decimal.Context(prec=80)
    return c


def _pi(c):
    # Machin: pi = 16 atan(1/5) - 4 atan(1/239)
    def atan_inv(n):
        x = c.divide(decimal.Decimal(1), decimal.Decimal(n))
        x2 = c.multiply(x, x)
        term, total, k = x, x, 1
        while abs(term) > decimal.Decimal(10) ** -78:
            term = c.multiply(term, x2)
            k += 2
            piece = c.divide(term, decimal.Decimal(k))
            total = c.subtract(total, piece) if (k // 2) % 2 else c.add(total, piece)
        return total
    return c.subtract(c.multiply(decimal.Decimal(16), atan_inv(5)), c.multiply(decimal.Decimal(4), atan_inv(239)))


def _erf(c, x, two_over_sqrt_pi):
    # erf(x) = 2/sqrt(pi) * sum_{n>=0} (-1)^n x^(2n+1) / (n! (2n+1))
    x2 = c.multiply(x, x)
    power, total, n = x, x, 0
    while True:
        n += 1
        power = c.divide(c.multiply(power, x2), decimal.Decimal(n))          # x^(2n+1) / n!
        piece = c.divide(power, decimal.Decimal(2 * n + 1))
        total = c.subtract(total, piece) if n % 2 else c.add(total, piece)
        if abs(piece) < decimal.Decimal(10) ** -76:
            break
    return c.multiply(two_over_sqrt_pi, total)


def coefficients():
    """INTERVALS rows of DEGREE + 1 Python floats: Taylor coefficients a_0 .. a_DEGREE."""
    c = _ctx()
    tosp = c.divide(decimal.Decimal(2), c.sqrt(_pi(c)))
    rows = []
    for k in range(INTERVALS):
        centre = decimal.Decimal(0) if k == 0 else c.divide(decimal.Decimal(2 * k + 1), decimal.Decimal(2 * WIDTH_INV))
        g = c.multiply(tosp, c.exp(c.minus(c.multiply(centre, centre))))       # erf'(centre)
        coef = [_erf(c, centre, tosp) if k else decimal.Decimal(0)]
        h_prev, h_cur = decimal.Decimal(0), decimal.Decimal(1)                 # H_{-1}, H_0
        fact = decimal.Decimal(1)
        for j in range(1, DEGREE + 1):
            n = j - 1                                                          # erf^(j) = (-1)^n H_n g
            fact = c.multiply(fact, decimal.Decimal(j))
            d = c.multiply(h_cur, g)
            if n % 2:
                d = c.minus(d)
            coef.append(c.divide(d, fact))
            h_prev, h_cur = h_cur, c.subtract(c.multiply(c.multiply(decimal.Decimal(2), centre), h_cur),
                                              c.multiply(decimal.Decimal(2 * n), h_prev))
        rows.append([float(v) for v in coef])
    return rows


def c_initialiser():
    """The table as the body of a C array initialiser (hex floats, row major)."""
    lines = []
    for row in coefficients():
        lines.append(", ".join(float.hex(v) for v in row))
    return ",\n".join(lines)


if __name__ == "__main__":
    print(c_initialiser())
