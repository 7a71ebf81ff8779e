"""Pins for every operator of the oracle's expression language (Sec. 3.2 of the paper: arithmetic,
comparisons, boolean operators, select, casts, math functions).

Two kinds of pin, neither of which is the oracle's own formula typed again:
  * hand-worked tables: the operands and the expected results are literals written out below
    (truth tables, truncating casts of negative fractions, min/max of mixed signs, wrapping);
  * the operator-at-a-time interpreter (numpy columns) against the per-row pure-Python loop, which
    share no code, on seeded random programs: EVERY expression column is compared, not only what
    reaches a builder, so an operator that is wrong in one of them fails here even where a
    program's builders would mask it.
No GPU is needed.
"""
import math

import numpy as np
import pytest

from oracle import interp, rowwise
from workloads import random_programs
from workloads.ir import Program

NP = {"bool": np.bool_, "i8": np.int8, "i32": np.int32, "i64": np.int64, "f64": np.float64}


def _map(columns, build):
    """Run `for(zip(columns), vecbuilder, x => merge(b, build(p, x...)))` through both oracle forms;
    returns (operator-at-a-time result, per-row result) as Python lists."""
    types = [t for t, _ in columns]
    p = Program(types)
    v = build(p, *[p.col(k) for k in range(len(types))])
    p.merge(p.vecbuilder(p.type_of(v)), v)
    a = interp.run(p, [np.array(c, dtype=NP[t]) for t, c in columns])[0]
    b = rowwise.run(p, [list(c) for _, c in columns])[0]
    return a.tolist(), b


def _both(columns, build, expected):
    a, b = _map(columns, build)
    assert a == expected, ("operator at a time", a, expected)
    assert b == expected, ("per row", b, expected)
    for x, y, e in zip(a, b, expected):
        assert type(x) is type(e) and type(y) is type(e), (x, y, e)


# ----------------------------------------------------------------------
# a scalar defined outside the loop (Sec. 3.2: the loop's function is a closure): every row reads it
# ----------------------------------------------------------------------
def test_scalar_from_outside_the_loop_is_read_by_every_row():
    p = Program(["i64", "i64", "f64"])
    x, s, f = p.col(0), p.scalar(1), p.scalar(2)
    p.merge(p.vecbuilder("i64"), p.bin("sub", p.bin("mul", x, s), p.const("i64", 1)))
    p.merge(p.merger("i64", "add"), s, pred=p.bin("gt", x, s))
    p.merge(p.vecbuilder("f64"), p.bin("add", p.un("cast", x, "f64"), f))
    cols = [[1, 5, 2, 9], [3], [0.5]]
    want = [[2, 14, 5, 26], 6, [1.5, 5.5, 2.5, 9.5]]             # 3x - 1; s counted where x > 3: twice; x + 0.5
    a = interp.run(p, [np.array(cols[0]), np.array(cols[1]), np.array(cols[2])])
    b = rowwise.run(p, cols)
    assert a[0].tolist() == want[0] and int(a[1]) == want[1] and a[2].tolist() == want[2]
    assert b[0] == want[0] and b[1] == want[1] and b[2] == want[2]
    # the loop's length is that of its vectors, wherever the scalar stands in the list
    q = Program(["i64", "i64"])
    q.merge(q.vecbuilder("i64"), q.bin("add", q.scalar(0), q.col(1)))
    assert interp.run(q, [np.array([10]), np.array([1, 2, 3])])[0].tolist() == [11, 12, 13]
    assert rowwise.run(q, [[10], [1, 2, 3]])[0] == [11, 12, 13]
    assert interp.run(q, [np.array([10]), np.array([], dtype=np.int64)])[0].tolist() == []
    assert rowwise.run(q, [[10], []])[0] == []


# ----------------------------------------------------------------------
# boolean operators: complete truth tables
# ----------------------------------------------------------------------
def _bool_cols():
    # two i64 columns compared with 0 give every pair of truth values
    return [("i64", [0, 0, 1, 1]), ("i64", [0, 1, 0, 1])]


def _truth(p, x):
    return p.bin("ne", x, p.const("i64", 0))


def test_not_truth_table():
    _both([("i64", [0, 1, -7])], lambda p, x: p.un("not", _truth(p, x)), [True, False, False])


def test_and_truth_table():
    _both(_bool_cols(), lambda p, x, y: p.bin("and", _truth(p, x), _truth(p, y)), [False, False, False, True])


def test_or_truth_table():
    _both(_bool_cols(), lambda p, x, y: p.bin("or", _truth(p, x), _truth(p, y)), [False, True, True, True])


def test_select_takes_second_operand_where_true():
    _both([("i64", [1, 0, 1, 0]), ("i32", [10, 20, 30, 40]), ("i32", [-1, -2, -3, -4])],
          lambda p, c, a, b: p.select(_truth(p, c), a, b), [10, -2, 30, -4])


# ----------------------------------------------------------------------
# binary min / max, mixed signs, every numeric type
# ----------------------------------------------------------------------
MINMAX = {
    "i8": ([-128, -3, 5, 127, 0, -1], [127, 4, -6, 126, 0, 1],
           [-128, -3, -6, 126, 0, -1], [127, 4, 5, 127, 0, 1]),
    "i32": ([-2147483648, -3, 5, 70000], [2147483647, 4, -6, 69999],
            [-2147483648, -3, -6, 69999], [2147483647, 4, 5, 70000]),
    "i64": ([-2 ** 63, -3, 5, 2 ** 40], [2 ** 63 - 1, 4, -6, -2 ** 40],
            [-2 ** 63, -3, -6, -2 ** 40], [2 ** 63 - 1, 4, 5, 2 ** 40]),
    "f64": ([-2.5, -0.25, 3.0, 1e300, -1e-300], [2.5, -0.5, -3.0, 1e299, 1e-300],
            [-2.5, -0.5, -3.0, 1e299, -1e-300], [2.5, -0.25, 3.0, 1e300, 1e-300]),
}


@pytest.mark.parametrize("t", sorted(MINMAX))
def test_binary_min_and_max(t):
    a, b, lo, hi = MINMAX[t]
    _both([(t, a), (t, b)], lambda p, x, y: p.bin("min", x, y), lo)
    _both([(t, a), (t, b)], lambda p, x, y: p.bin("max", x, y), hi)
    # and with the operands exchanged: neither is "take the first" or "take the second"
    _both([(t, b), (t, a)], lambda p, x, y: p.bin("min", x, y), lo)
    _both([(t, b), (t, a)], lambda p, x, y: p.bin("max", x, y), hi)


# ----------------------------------------------------------------------
# casts
# ----------------------------------------------------------------------
FRACTIONS = [-2.7, -0.5, 2.7, 0.5, -0.0, -1.0, 1000.9, -1000.9, 2.0 ** 31 - 0.5]


@pytest.mark.parametrize("t,expected", [
    ("i64", [-2, 0, 2, 0, 0, -1, 1000, -1000, 2 ** 31 - 1]),
    ("i32", [-2, 0, 2, 0, 0, -1, 1000, -1000, 2 ** 31 - 1]),
])
def test_cast_f64_to_integer_truncates_toward_zero(t, expected):
    _both([("f64", FRACTIONS)], lambda p, x: p.un("cast", x, to=t), expected)


def test_cast_f64_to_i8_truncates_toward_zero():
    _both([("f64", [-2.7, -0.5, 2.7, 0.5, -127.9, 127.9])], lambda p, x: p.un("cast", x, to="i8"),
          [-2, 0, 2, 0, -127, 127])


def test_cast_to_bool_is_not_equal_zero():
    _both([("i64", [-3, 0, 5, -2 ** 63, 256])], lambda p, x: p.un("cast", x, to="bool"),
          [True, False, True, True, True])
    _both([("i8", [-3, 0, 5])], lambda p, x: p.un("cast", x, to="bool"), [True, False, True])
    _both([("f64", [-0.5, 0.0, 0.25, -0.0, -3.0])], lambda p, x: p.un("cast", x, to="bool"),
          [True, False, True, False, True])


def test_cast_between_integers_wraps():
    _both([("i64", [300, -129, 127, -128, 2 ** 40 + 7])], lambda p, x: p.un("cast", x, to="i8"),
          [44, 127, 127, -128, 7])
    _both([("i64", [2 ** 31, -2 ** 31 - 1, 5])], lambda p, x: p.un("cast", x, to="i32"),
          [-2 ** 31, 2 ** 31 - 1, 5])
    _both([("i8", [-128, -1, 127])], lambda p, x: p.un("cast", x, to="i64"), [-128, -1, 127])


def test_cast_to_f64_and_from_bool():
    _both([("i64", [-3, 0, 2 ** 53 + 1, -2 ** 63])], lambda p, x: p.un("cast", x, to="f64"),
          [-3.0, 0.0, 9007199254740992.0, -9223372036854775808.0])      # 2^53+1 rounds to even
    _both([("i64", [0, 9, -9])], lambda p, x: p.un("cast", _truth(p, x), to="i64"), [0, 1, 1])
    _both([("i64", [0, 9])], lambda p, x: p.un("cast", _truth(p, x), to="f64"), [0.0, 1.0])


# ----------------------------------------------------------------------
# arithmetic: signs, wrapping, truncation (literal expectations)
# ----------------------------------------------------------------------
def test_neg_sub_and_wrapping():
    _both([("i8", [-128, 127, 0, 5])], lambda p, x: p.un("neg", x), [-128, -127, 0, -5])
    _both([("f64", [-2.5, 0.0, 3.0])], lambda p, x: p.un("neg", x), [2.5, -0.0, -3.0])
    _both([("i32", [5, -2147483648, 7]), ("i32", [7, 1, -2147483647])], lambda p, x, y: p.bin("sub", x, y),
          [-2, 2147483647, -2147483642])
    _both([("i8", [100, -100, 16]), ("i8", [100, -100, 16])], lambda p, x, y: p.bin("add", x, y), [-56, 56, 32])
    _both([("i8", [16, -16, 127])], lambda p, x: p.bin("mul", x, x), [0, 0, 1])


def test_integer_div_and_mod_truncate_toward_zero():
    a = [7, -7, 7, -7, 0, -9, 9]
    b = [2, 2, -2, -2, 5, 3, -3]
    for t in ("i8", "i32", "i64"):
        _both([(t, a), (t, b)], lambda p, x, y: p.bin("div", x, y), [3, -3, -3, 3, 0, -3, -3])
        _both([(t, a), (t, b)], lambda p, x, y: p.bin("mod", x, y), [1, -1, 1, -1, 0, 0, 0])


def test_edge_values_where_the_paper_is_silent():
    """The readings both oracle forms (and the kernels) follow: x / 0 = 0 and x % 0 = 0, the most negative
    value over -1 wraps to itself with remainder 0, min / max with a NaN is NaN, a cast of NaN to an
    integer is 0 and values beyond the 64-bit range cast to its nearest end (narrower types then wrap)."""
    lo8, lo32, lo64 = -128, -2 ** 31, -2 ** 63
    for t, lo in (("i8", lo8), ("i32", lo32), ("i64", lo64)):
        _both([(t, [7, -7, 0, lo, lo, 5]), (t, [0, 0, 0, -1, 1, -1])], lambda p, x, y: p.bin("div", x, y), [0, 0, 0, lo, lo, -5])
        _both([(t, [7, -7, 0, lo, lo, 5]), (t, [0, 0, 0, -1, 1, -1])], lambda p, x, y: p.bin("mod", x, y), [0, 0, 0, 0, 0, 0])
    nan, inf = math.nan, math.inf
    for op in ("min", "max"):
        a, b = _map([("f64", [nan, 1.0, nan, -inf]), ("f64", [1.0, nan, nan, inf])], lambda p, x, y, op=op: p.bin(op, x, y))
        for got in (a, b):
            assert all(math.isnan(v) for v in got[:3]) and got[3] == (-inf if op == "min" else inf)
    big = [nan, 1e30, -1e30, 9.3e18, -9.3e18, 9.2e18, inf, -inf]
    _both([("f64", big)], lambda p, x: p.un("cast", x, to="i64"),
          [0, 2 ** 63 - 1, lo64, 2 ** 63 - 1, lo64, 9200000000000000000, 2 ** 63 - 1, lo64])
    _both([("f64", big)], lambda p, x: p.un("cast", x, to="i32"),
          [0, -1, 0, -1, 0, -1650982912, -1, 0])       # 2^63 - 1 and -2^63 wrapped to 32 bits; 9.2e18 mod 2^32 as a signed value
    # merge functions: a NaN among the merged values makes a min / max merger NaN
    for func in ("min", "max"):
        p = Program(["f64"])
        p.merge(p.merger("f64", func), p.col(0))
        vals = [3.0, nan, -2.0, 7.5]
        assert math.isnan(float(interp.run(p, [np.array(vals)])[0])) and math.isnan(rowwise.run(p, [vals])[0])


def test_f64_arithmetic_and_compares():
    x = [0.1, -0.75, 1e16, 3.0]
    y = [0.2, 0.5, 1.0, -2.0]
    _both([("f64", x), ("f64", y)], lambda p, a, b: p.bin("add", a, b), [0.30000000000000004, -0.25, 1e16, 1.0])
    _both([("f64", x), ("f64", y)], lambda p, a, b: p.bin("sub", a, b), [-0.1, -1.25, 1e16, 5.0])
    _both([("f64", x), ("f64", y)], lambda p, a, b: p.bin("mul", a, b), [0.020000000000000004, -0.375, 1e16, -6.0])
    _both([("f64", x), ("f64", y)], lambda p, a, b: p.bin("div", a, b), [0.5, -1.5, 1e16, -1.5])
    _both([("f64", [7.5, -7.5, 7.5]), ("f64", [2.0, 2.0, -2.0])], lambda p, a, b: p.bin("mod", a, b), [1.5, -1.5, 1.5])
    for op, want in (("lt", [True, True, False, False]), ("le", [True, True, False, False]),
                     ("gt", [False, False, True, True]), ("ge", [False, False, True, True]),
                     ("eq", [False, False, False, False]), ("ne", [True, True, True, True])):
        _both([("f64", x), ("f64", y)], lambda p, a, b, op=op: p.bin(op, a, b), want)
    _both([("i64", [1, 2, 3]), ("i64", [2, 2, 2])], lambda p, a, b: p.bin("le", a, b), [True, True, False])
    _both([("i64", [1, 2, 3]), ("i64", [2, 2, 2])], lambda p, a, b: p.bin("ge", a, b), [False, True, True])
    _both([("i64", [1, 2, 3]), ("i64", [2, 2, 2])], lambda p, a, b: p.bin("eq", a, b), [False, True, False])


def test_math_functions_at_points_with_known_values():
    # exact by the functions' definitions: exp(0) = 1, log(1) = 0, sqrt of squares, erf(0) = 0;
    # elsewhere against digits worked out by hand from the series (20 significant digits shown)
    _both([("f64", [0.0])], lambda p, x: p.un("exp", x), [1.0])
    _both([("f64", [1.0])], lambda p, x: p.un("log", x), [0.0])
    _both([("f64", [0.0, 6.25, 1e-300 * 1e-300])], lambda p, x: p.un("sqrt", x), [0.0, 2.5, 0.0])
    _both([("f64", [0.0])], lambda p, x: p.un("erf", x), [0.0])
    known = {"exp": (1.0, 2.7182818284590452354), "log": (2.0, 0.69314718055994530942),
             "sqrt": (2.0, 1.4142135623730950488), "erf": (0.5, 0.52049987781304653768)}
    for op, (arg, want) in known.items():
        a, b = _map([("f64", [arg, -arg if op == "erf" else arg])], lambda p, x, op=op: p.un(op, x))
        for got in (a, b):
            assert abs(got[0] - want) <= 2e-16 * want, (op, got)
        if op == "erf":                                   # odd function
            assert a[1] == -a[0] and b[1] == -b[0]


# ----------------------------------------------------------------------
# every expression column of seeded random programs: numpy columns vs the per-row loop
# ----------------------------------------------------------------------
ROWS = 160


def _rows_of(program, cols):
    """Every expression of `program` for every row, by the per-row evaluator."""
    lists = [c.tolist() for c in cols]
    return [rowwise._body(program, i, [c[i] for c in lists]) for i in range(len(lists[0]))]


@pytest.mark.parametrize("seed", range(120))
def test_every_expression_column_of_a_random_program(seed):
    prog, cols, inits = random_programs.make(seed)
    cols = [c[:ROWS] for c in cols]
    n = len(cols[0])
    columns = interp.eval_columns(prog, cols)
    rows = _rows_of(prog, cols)
    for k, op in enumerate(prog.ops):
        got = columns[k].tolist()
        want = [rows[i][k] for i in range(n)]
        if op[1] == "f64":
            # + - * / sqrt neg min max select casts: one correctly rounded operation each on both
            # sides, so the doubles are identical (compared by bits: -0.0 is not +0.0)
            assert [math.copysign(1.0, x) for x in got] == [math.copysign(1.0, x) for x in want], (k, op)
        assert got == want, (seed, k, op)
    # the builders on top, in the literal fold order
    a = interp.run(prog, cols, sums="fold", inits=inits)
    b = rowwise.run(prog, [c.tolist() for c in cols], inits={k: v.tolist() for k, v in inits.items()})
    for spec, ra, rb in zip(prog.builders, a, b):
        kind = spec["kind"]
        if kind == "merger":
            assert ra.item() == rb, (seed, spec)
        elif kind in ("vecbuilder", "vecmerger"):
            assert ra.tolist() == list(rb), (seed, spec)
        elif kind == "dictmerger":
            keys, vals = ra
            got = {tuple(k[i].item() for k in keys): [v[i].item() for v in vals] for i in range(len(keys[0]))}
            assert got == {k: list(v) for k, v in rb.items()}, (seed, spec)
        else:
            keys, offsets, values = ra
            got = {tuple(k[g].item() for k in keys): values[offsets[g]:offsets[g + 1]].tolist()
                   for g in range(len(keys[0]))}
            assert got == {k: list(v) for k, v in rb.items()}, (seed, spec)


def test_the_random_programs_cover_the_operators_pinned_here():
    seen = set()
    for seed in range(120):
        prog, _, _ = random_programs.make(seed)
        for op in prog.ops:
            seen.add(op[0] if op[0] != "cast" else "cast:%s>%s" % (prog.ops[op[2]][1], op[1]))
    for code in ("not", "and", "or", "min", "max", "select", "neg", "sub", "div", "mod",
                 "cast:f64>i64", "cast:f64>i32", "cast:f64>i8", "cast:bool>i64", "cast:i64>i8"):
        assert code in seen, code
