"""The coefficient table of the library's own erf (paper_1709_06416_amd/erf_table.py),
checked on the CPU against two independent evaluations: libm's erf and the decimal
Maclaurin series the oracle pins use.  The kernels evaluate the same polynomial with fused
multiply-adds; here plain f64 Horner steps are used, which can only be less accurate."""
import math

import numpy as np

from paper_1709_06416_amd import erf_table
from tests.test_oracle_pins import _dec_erf


def _poly(tab, x):
    a = abs(x)
    if a >= 6.0:
        return math.copysign(1.0, x)
    k = min(int(a * 16.0), 95)
    h = a - ((k + 0.5) * 0.0625 if k else 0.0)
    p = tab[k][9]
    for j in range(8, -1, -1):
        p = p * h + tab[k][j]
    return math.copysign(p, x)


def test_table_shape_and_first_rows():
    tab = erf_table.coefficients()
    assert len(tab) == 96 and all(len(r) == 10 for r in tab)
    two_over_sqrt_pi = 2.0 / math.sqrt(math.pi)
    assert tab[0][0] == 0.0 and tab[0][2] == 0.0 and tab[0][4] == 0.0          # odd function about 0
    assert tab[0][1] == two_over_sqrt_pi and tab[0][3] == -two_over_sqrt_pi / 3.0
    assert tab[1][0] == math.erf(1.5 / 16)                                      # value at the centre
    assert abs(tab[95][0] - 1.0) < 1e-15


def test_polynomial_against_libm_and_decimal_series():
    tab = erf_table.coefficients()
    rnd = np.random.RandomState(2)
    xs = np.concatenate([rnd.uniform(-6.5, 6.5, 100_000), rnd.uniform(-0.07, 0.07, 10_000),
                         10.0 ** rnd.uniform(-300, -1, 1_000), np.arange(0, 97) / 16.0,
                         np.nextafter(np.arange(1, 97) / 16.0, 0), [-0.0, 0.0, 5.99999, 6.0, 7.5, -7.5, 1e300]])
    for x in xs:
        got, want = _poly(tab, float(x)), math.erf(float(x))
        assert abs(got - want) <= 2.3e-16 and abs(got - want) <= 1e-15 * abs(want), (x, got, want)
    assert math.copysign(1.0, _poly(tab, -0.0)) == -1.0
    for x in (1e-8, 0.03, 0.0625, 0.1, 0.5, 1.0, 2.5, 4.0, 5.5):
        assert abs(_poly(tab, x) - float(_dec_erf(x))) <= 1e-15 * float(_dec_erf(x)), x
