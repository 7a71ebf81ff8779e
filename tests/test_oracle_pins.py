"""Pins for the CPU oracle: it is checked against things other than itself.

  * the results the paper prints (tests/golden/paper_builder_examples.txt)
  * the fused == unfused equivalence of Sec. 4.5 (per-row loop vs operator at a time)
  * closed forms, exact sums, brute force on tiny inputs, numpy library routines
  * a decimal-arithmetic evaluation of the option formula, put-call parity, bounds
No GPU is needed for any of these.
"""
import decimal
import math
import os
import random

import numpy as np
import pytest

from oracle import interp, rowwise
from workloads import configs
from workloads.ir import Program

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "paper_builder_examples.txt")


def _golden_cases():
    cases = []
    for line in open(GOLDEN):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        name, ins, outs = [s.strip() for s in line.split("|")]
        vecs = [[int(x) for x in v.split()] for v in ins.split(";")]
        exp = [[int(x) for x in v.split()] for v in outs.split(";")]
        cases.append((name, vecs, exp))
    return cases


@pytest.mark.parametrize("name,vecs,exp", _golden_cases())
def test_paper_printed_results(name, vecs, exp):
    prog = configs.EXAMPLES[name]()
    res = interp.run(prog, [np.array(v, dtype=np.int32) for v in vecs])
    res_rw = rowwise.run(prog, vecs)
    for spec, r, rr, e in zip(prog.builders, res, res_rw, exp):
        if spec["kind"] == "vecbuilder":
            assert r.tolist() == e
            assert rr == e
        else:
            assert [int(r)] == e
            assert [rr] == e


def test_filter_sum_equals_reduce_of_filter():
    # Sec. 4.5: reduce(filter(v0, x > 500000), 0, +) == the single fused loop.
    rnd = random.Random(7)
    pop = [rnd.randrange(0, 1_000_000) for _ in range(500)]
    expected = sum(x for x in pop if x > 500000)
    prog = configs.example_filter_sum()
    assert int(interp.run(prog, [np.array(pop, dtype=np.int64)])[0]) == expected
    assert rowwise.run(prog, [pop])[0] == expected


# ----------------------------------------------------------------------
# fused (per-row) == unfused (operator at a time), on every config
# ----------------------------------------------------------------------
def _as_lists(cols):
    return [c.tolist() for c in cols]


def _compare_interp_rowwise(prog, cols, f64_rel=0.0):
    a = interp.run(prog, cols, sums="fold")
    b = rowwise.run(prog, _as_lists(cols))
    for spec, ra, rb in zip(prog.builders, a, b):
        if spec["kind"] == "merger":
            if spec["type"] == "f64":
                assert ra == pytest.approx(rb, rel=f64_rel, abs=0.0)
            else:
                assert int(ra) == rb
        elif spec["kind"] == "vecbuilder":
            if spec["type"] == "f64":
                np.testing.assert_allclose(ra, np.array(rb, dtype=np.float64), rtol=f64_rel, atol=0)
            else:
                assert ra.tolist() == rb
        else:
            keys, vals = ra
            got = {tuple(int(k[i]) for k in keys): [v[i] for v in vals] for i in range(len(keys[0]))}
            assert set(got) == set(rb)
            for k, vs in rb.items():
                for t, x, y in zip(spec["val_types"], got[k], vs):
                    if t == "f64":
                        assert x == pytest.approx(y, rel=f64_rel, abs=0.0)
                    else:
                        assert int(x) == y


@pytest.mark.parametrize("name", ["C1", "C3", "C4", "C5"])
def test_fused_equals_unfused_bit_exact(name):
    n = 3000
    cols = [c.numpy() for c in configs.make_columns(name, n)]
    # arithmetic is +,-,*,/ and compares only: both forms must agree to the bit when
    # both fold in index order
    _compare_interp_rowwise(configs.PROGRAMS[name](), cols, f64_rel=0.0)


def test_fused_equals_unfused_black_scholes():
    cols = [c.numpy() for c in configs.make_columns("C2", 2000)]
    # erf comes from two different libraries here (scipy vs libm): a few ulp on the
    # erf value, amplified by cancellation in deep out-of-the-money prices, hence an
    # absolute floor like the one used against the GPU
    prog = configs.program_c2()
    a = interp.run(prog, cols)
    b = rowwise.run(prog, _as_lists(cols))
    for ra, rb in zip(a, b):
        rb = np.array(rb)
        assert np.all(np.abs(ra - rb) <= 1e-12 * np.maximum(np.abs(rb), 1.0))


# ----------------------------------------------------------------------
# mergers: closed forms, exact sums, order independence
# ----------------------------------------------------------------------
def _index_sum_program(func="add", t="i64"):
    p = Program(["i64"])
    p.merge(p.merger(t, func), p.index() if t == "i64" else p.un("cast", p.index(), to=t))
    return p


def test_sum_of_indices_closed_form():
    n = 100_003
    res = interp.run(_index_sum_program(), [np.zeros(n, dtype=np.int64)])
    assert int(res[0]) == n * (n - 1) // 2


def test_count_multiples_of_three_closed_form():
    n = 100_001
    p = Program(["i64"])
    i = p.index()
    pred = p.bin("eq", p.bin("mod", i, p.const("i64", 3)), p.const("i64", 0))
    p.merge(p.merger("i64", "add"), p.const("i64", 1), pred=pred)
    res = interp.run(p, [np.zeros(n, dtype=np.int64)])
    assert int(res[0]) == (n + 2) // 3


def test_integer_wrap_and_truncation():
    p = Program(["i32", "i32"])
    a, b = p.col(0), p.col(1)
    p.merge(p.vecbuilder("i32"), p.bin("add", a, b))
    p.merge(p.vecbuilder("i32"), p.bin("mul", a, b))
    p.merge(p.vecbuilder("i32"), p.bin("mod", a, b))
    p.merge(p.vecbuilder("i32"), p.bin("div", a, b))
    av = np.array([2147483647, -7, 7, -7, 65536], dtype=np.int32)
    bv = np.array([1, 3, -3, -3, 65536], dtype=np.int32)
    r = interp.run(p, [av, bv])
    assert r[0].tolist() == [-2147483648, -4, 4, -10, 131072]
    assert r[1].tolist() == [2147483647, -21, -21, 21, 0]
    assert r[2].tolist() == [0, -1, 1, -1, 0]          # sign of the dividend (C)
    assert r[3].tolist() == [2147483647, -2, -2, 2, 1]  # toward zero (C)
    assert rowwise.run(p, [av.tolist(), bv.tolist()]) == [x.tolist() for x in r]


def test_i8_sum_wraps():
    p = Program(["i8"])
    p.merge(p.merger("i8", "add"), p.col(0))
    v = np.full(300, 1, dtype=np.int8)
    assert int(interp.run(p, [v])[0]) == 300 - 256


def test_exact_sum_is_exact_where_fold_is_not():
    v = np.array([1e16] + [1.0] * 1000 + [-1e16], dtype=np.float64)
    assert float(interp.exact_sum(v)) == 1000.0
    assert float(np.cumsum(v)[-1]) != 1000.0
    ones = np.ones(1 << 20)
    assert float(interp.exact_sum(ones)) == float(1 << 20)
    pw = np.array([2.0 ** -k for k in range(40)])
    assert float(interp.exact_sum(pw)) == 2.0 - 2.0 ** -39


def test_extended_sum_matches_fsum():
    rnd = np.random.RandomState(3)
    v = rnd.uniform(900.0, 105000.0, size=2_000_000)
    ext = np.float64(np.sum(v, dtype=np.longdouble))
    assert ext == math.fsum(v.tolist())


def test_fold_close_to_exact_on_c1():
    cols = [c.numpy() for c in configs.make_columns("C1", 200_000)]
    prog = configs.program_c1()
    ex = interp.run(prog, cols, sums="exact")
    fo = interp.run(prog, cols, sums="fold")
    assert abs(float(ex[0]) - float(fo[0])) <= 1e-10 * abs(float(ex[0]))
    assert int(ex[1]) == int(fo[1]) == int(np.count_nonzero(cols[0] > 0.5))
    # sanity band: E[x*y+1 | x>0.5] = 0.75*0.5+1 = 1.375
    assert float(ex[0]) / int(ex[1]) == pytest.approx(1.375, rel=5e-3)


@pytest.mark.parametrize("func", ["add", "mul", "min", "max"])
@pytest.mark.parametrize("t", ["i32", "i64", "f64"])
def test_merger_brute_force_and_permutation(func, t):
    rnd = np.random.RandomState(11)
    if t == "f64":
        v = rnd.choice([0.5, 1.0, 2.0, 4.0, -1.0, 0.25], size=60).astype(np.float64)
    else:
        v = rnd.randint(-5, 6, size=60).astype(interp.NP_TYPE[t])
        v[v == 0] = 3
    p = Program([t])
    p.merge(p.merger(t, func), p.col(0), pred=p.bin("ne", p.col(0), p.const(t, 4)))
    r = interp.run(p, [v], sums="fold")[0]
    kept = [x for x in v.tolist() if x != 4]
    if func == "add":
        want = sum(kept)
    elif func == "mul":
        want = math.prod(kept)
    elif func == "min":
        want = min(kept)
    else:
        want = max(kept)
    if t != "f64":
        w = {"i32": 32, "i64": 64}[t]
        want = (want + (1 << (w - 1))) % (1 << w) - (1 << (w - 1))
    assert r == want                      # values chosen so that f64 results are exact
    perm = rnd.permutation(len(v))
    assert interp.run(p, [v[perm]], sums="fold")[0] == r
    assert rowwise.run(p, [v.tolist()])[0] == want


def test_untouched_builders_return_identity():
    p = Program(["f64"])
    never = p.bin("lt", p.col(0), p.const("f64", -1.0))
    p.merge(p.merger("f64", "add"), p.col(0), pred=never)
    p.merge(p.merger("f64", "min"), p.col(0), pred=never)
    p.merge(p.merger("f64", "max"), p.col(0), pred=never)
    p.merge(p.merger("f64", "mul"), p.col(0), pred=never)
    p.merge(p.vecbuilder("f64"), p.col(0), pred=never)
    r = interp.run(p, [np.linspace(0, 1, 17)])
    assert (float(r[0]), float(r[1]), float(r[2]), float(r[3])) == (0.0, math.inf, -math.inf, 1.0)
    assert r[4].size == 0
    r0 = interp.run(p, [np.zeros(0)])
    assert float(r0[0]) == 0.0 and r0[4].size == 0


# ----------------------------------------------------------------------
# vecbuilder
# ----------------------------------------------------------------------
@pytest.mark.parametrize("pattern", ["random", "all", "none", "single", "empty"])
def test_vecbuilder_is_boolean_mask_in_index_order(pattern):
    rnd = np.random.RandomState(5)
    n = 0 if pattern == "empty" else 4099
    x = rnd.randint(0, 100, size=n).astype(np.int64)
    if pattern == "all":
        x[:] = 99
    elif pattern == "none":
        x[:] = 0
    elif pattern == "single":
        x[:] = 0
        x[1234] = 77
    p = Program(["i64"])
    pred = p.bin("gt", p.col(0), p.const("i64", 49))
    p.merge(p.vecbuilder("i64"), p.index(), pred=pred)
    p.merge(p.vecbuilder("i64"), p.col(0), pred=pred)
    p.merge(p.merger("i64", "add"), p.const("i64", 1), pred=pred)
    idx, vals, cnt = interp.run(p, [x])
    assert len(idx) == int(cnt) == int(np.count_nonzero(x > 49))
    assert np.all(np.diff(idx) > 0)                       # strictly increasing source rows
    assert np.array_equal(vals, x[x > 49])
    assert np.array_equal(idx, np.flatnonzero(x > 49))


# ----------------------------------------------------------------------
# dictmerger
# ----------------------------------------------------------------------
def test_dictmerger_c4_invariants():
    n = 50_000
    cols = [c.numpy() for c in configs.make_columns("C4", n)]
    prog = configs.program_c4()
    (keys, vals), = interp.run(prog, cols, sums="exact")
    flag, status, day, qty, price, disc, tax = cols
    keep = day <= 2400
    assert len(keys[0]) == 6
    pairs = sorted(set(zip(flag[keep].tolist(), status[keep].tolist())))
    assert list(zip(keys[0].tolist(), keys[1].tolist())) == pairs
    assert int(vals[4].sum()) == int(keep.sum())          # sum of group counts == filtered count
    tot_qty = math.fsum(qty[keep].tolist())
    assert math.fsum(vals[0].tolist()) == pytest.approx(tot_qty, rel=1e-14)
    tot_dp = math.fsum((price * (1.0 - disc))[keep].tolist())
    assert math.fsum(vals[2].tolist()) == pytest.approx(tot_dp, rel=1e-14)
    # one group by brute force
    sel = keep & (flag == 1) & (status == 0)
    g = pairs.index((1, 0))
    assert int(vals[4][g]) == int(sel.sum())
    assert float(vals[1][g]) == math.fsum(price[sel].tolist())
    ch = (price * (1.0 - disc)) * (1.0 + tax)
    assert float(vals[3][g]) == math.fsum(ch[sel].tolist())
    # selectivity band: 2401/2557
    assert keep.mean() == pytest.approx(2401 / 2557, abs=0.01)


def test_dictmerger_c5_invariants():
    n = 200_000
    code, = [c.numpy() for c in configs.make_columns("C5", n)]
    prog = configs.program_c5()
    cleaned, (keys, vals) = interp.run(prog, [code])
    valid = code > 0
    assert len(cleaned) == int(valid.sum())
    assert valid.mean() == pytest.approx(0.90, abs=0.01)
    assert np.array_equal(cleaned, code[valid] % 100000)   # positive operands: % == C remainder
    uk, uc = np.unique(cleaned, return_counts=True)
    assert np.array_equal(keys[0], uk)
    assert np.array_equal(vals[0], uc)
    assert int(vals[0].sum()) == len(cleaned)
    assert keys[0].min() >= 0 and keys[0].max() < 100000
    # skew: the most frequent key carries roughly 1/H(1e5, 1.1) of the merges
    assert uc.max() / len(cleaned) == pytest.approx(0.13, abs=0.03)


@pytest.mark.parametrize("func", ["add", "min", "max", "mul"])
def test_dictmerger_brute_force(func):
    rnd = random.Random(23)
    n = 400
    k1 = [rnd.randrange(-2, 3) for _ in range(n)]
    k2 = [rnd.randrange(0, 2) for _ in range(n)]
    a = [rnd.randrange(-3, 4) or 1 for _ in range(n)]
    f = [rnd.choice([0.5, 1.0, 2.0]) for _ in range(n)]
    p = Program(["i8", "i32", "i64", "f64"])
    pred = p.bin("ne", p.col(2), p.const("i64", 2))
    d = p.dictmerger(["i8", "i32"], ["i64", "f64"], func, 16)
    p.merge(d, [p.col(2), p.col(3)], keys=[p.col(0), p.col(1)], pred=pred)
    cols = [np.array(k1, np.int8), np.array(k2, np.int32), np.array(a, np.int64), np.array(f)]
    (keys, vals), = interp.run(p, cols, sums="fold")
    want = {}
    for i in range(n):
        if a[i] == 2:
            continue
        key = (k1[i], k2[i])
        if key not in want:
            want[key] = [a[i], f[i]]
        else:
            c = want[key]
            if func == "add":
                want[key] = [c[0] + a[i], c[1] + f[i]]
            elif func == "mul":
                want[key] = [c[0] * a[i], c[1] * f[i]]
            elif func == "min":
                want[key] = [min(c[0], a[i]), min(c[1], f[i])]
            else:
                want[key] = [max(c[0], a[i]), max(c[1], f[i])]
    got = {(int(keys[0][i]), int(keys[1][i])): [int(vals[0][i]), float(vals[1][i])]
           for i in range(len(keys[0]))}
    if func == "mul":
        want = {k: [(v[0] + (1 << 63)) % (1 << 64) - (1 << 63), v[1]] for k, v in want.items()}
    assert got == want
    assert list(got) == sorted(got)
    rw = rowwise.run(p, [k1, k2, a, f])[0]
    assert {k: list(v) for k, v in rw.items()} == want


# ----------------------------------------------------------------------
# selective filter-reduce (C3)
# ----------------------------------------------------------------------
def test_c3_against_direct_numpy_and_selectivity():
    n = 400_000
    cols = [c.numpy() for c in configs.make_columns("C3", n)]
    day, disc, qty, price = cols
    # discount columns hold exactly the doubles the literals parse to
    assert set(np.unique(disc).tolist()) == {k / 100.0 for k in range(11)}
    assert 0.05 in disc and 0.07 in disc
    keep = (day >= 365) & (day < 730) & (disc >= 0.05) & (disc <= 0.07) & (qty < 24.0)
    want = math.fsum((price * disc)[keep].tolist())
    got = interp.run(configs.program_c3(), cols, sums="exact")[0]
    assert float(got) == want
    assert keep.mean() == pytest.approx(365 / 2557 * 3 / 11 * 23 / 50, rel=0.1)


# ----------------------------------------------------------------------
# Black-Scholes map (C2)
# ----------------------------------------------------------------------
_PI = decimal.Decimal("3.14159265358979323846264338327950288419716939937510582097494")


def _dec_erf(x):
    decimal.getcontext().prec = 60
    x = decimal.Decimal(x)
    term = x
    total = x
    k = 0
    while abs(term) > decimal.Decimal(10) ** -55:
        k += 1
        term = -term * x * x / k
        total += term / (2 * k + 1)
    return 2 * total / _PI.sqrt()


def _dec_black_scholes(S, K, T, vol, r):
    decimal.getcontext().prec = 60
    D = decimal.Decimal
    S, K, T, vol, r = D(S), D(K), D(T), D(vol), D(r)
    st = vol * T.sqrt()
    d1 = ((S / K).ln() + (r + vol * vol / 2) * T) / st
    d2 = d1 - st
    N = lambda z: (1 + _dec_erf(z / D(2).sqrt())) / 2
    disc = (-r * T).exp()
    call = S * N(d1) - K * disc * N(d2)
    put = K * disc * N(-d2) - S * N(-d1)
    return float(d1), float(d2), float(call), float(put)


def test_erf_spot_values_against_decimal_series():
    xs = np.array([0.0, 1e-3, 0.1, 0.5, 0.84375, 1.0, 1.25, 2.0, 2.857, 3.5, -0.3, -2.2])
    p = Program(["f64"])
    p.merge(p.vecbuilder("f64"), p.un("erf", p.col(0)))
    got = interp.run(p, [xs])[0]
    for x, g in zip(xs.tolist(), got.tolist()):
        want = float(_dec_erf(x))
        assert g == pytest.approx(want, rel=4e-16, abs=0.0)
        assert math.erf(x) == pytest.approx(want, rel=4e-16, abs=0.0)
    assert got[0] == 0.0
    assert np.array_equal(interp.run(p, [-xs])[0], -got)       # odd function


def test_black_scholes_against_decimal_formula():
    rows = [(100.0, 100.0, 1.0, 0.2), (50.0, 60.0, 0.5, 0.3), (90.0, 45.0, 2.0, 0.45),
            (80.0, 99.0, 0.5, 0.4), (37.25, 36.5, 1.75, 0.125)]
    cols = [np.array([r[k] for r in rows]) for k in range(4)]
    prog = configs.program_c2()
    val = interp.eval_columns(prog, cols)
    call, put = interp.run(prog, cols)
    for i, (S, K, T, vol) in enumerate(rows):
        d1, d2, c, p_ = _dec_black_scholes(S, K, T, vol, configs.RATE)
        assert val[prog.named["d1"]][i] == pytest.approx(d1, rel=1e-13)
        assert val[prog.named["d2"]][i] == pytest.approx(d2, rel=1e-13)
        assert abs(call[i] - c) <= 1e-13 * max(S, K)
        assert abs(put[i] - p_) <= 1e-13 * max(S, K)


def test_black_scholes_parity_and_bounds():
    cols = [c.numpy() for c in configs.make_columns("C2", 20_000)]
    S, K, T, vol = cols
    call, put = interp.run(configs.program_c2(), cols)
    kd = K * np.exp(-configs.RATE * T)
    assert np.all(np.abs((call - put) - (S - kd)) <= 1e-12 * np.maximum(S, K))
    eps = 1e-12 * np.maximum(S, K)
    assert np.all(call >= np.maximum(S - kd, 0.0) - eps) and np.all(call <= S + eps)
    assert np.all(put >= -eps) and np.all(put <= kd + eps)
    # monotone in volatility
    call_hi, _ = interp.run(configs.program_c2(), [S, K, T, vol + 0.05])
    assert np.all(call_hi >= call - eps)
    # recipe ranges
    assert S.min() >= 10 and S.max() < 100 and T.min() >= 0.1 and T.max() < 2.0
    assert vol.min() >= 0.1 and vol.max() < 0.5


# ----------------------------------------------------------------------
# generators
# ----------------------------------------------------------------------
def test_generators_are_reproducible_and_chunk_independent():
    from workloads import rng
    a = rng.bits64(9, 2, 0, 1000)
    b = rng.bits64(9, 2, 500, 500)
    assert np.array_equal(a[500:].numpy(), b.numpy())
    assert configs.checksum(configs.make_columns("C3", 1000)[3]) == \
        configs.checksum(configs.make_columns("C3", 1000)[3])
    u = rng.unit_f64(1, 0, 0, 100_000).numpy()
    assert 0.0 <= u.min() and u.max() < 1.0 and abs(u.mean() - 0.5) < 0.01
    k = rng.uniform_int(1, 1, 0, 100_000, 0, 10).numpy()
    assert k.min() == 0 and k.max() == 10
    assert np.all(np.abs(np.bincount(k) / 100_000 - 1 / 11) < 0.01)


# ----------------------------------------------------------------------
# vecmerger (Table 1; Sec. 7.7 counts occurrences of keys with it)
# ----------------------------------------------------------------------
def _vecmerger_count_program(m):
    p = Program(["i32"])
    p.merge(p.vecmerger("i64", "add", m), [p.const("i64", 1)], keys=[p.un("cast", p.col(0), to="i64")])
    return p


def test_vecmerger_counts_match_bincount_and_closed_form():
    m, n = 37, 10_000
    keys = (np.arange(n) % m).astype(np.int32)
    got = interp.run(_vecmerger_count_program(m), [keys])[0]
    assert got.tolist() == [n // m + (1 if c < n % m else 0) for c in range(m)]     # closed form
    rnd = np.random.RandomState(2)
    keys = rnd.randint(0, m, size=n).astype(np.int32)
    got = interp.run(_vecmerger_count_program(m), [keys])[0]
    assert np.array_equal(got, np.bincount(keys, minlength=m))
    assert rowwise.run(_vecmerger_count_program(m), [keys.tolist()])[0] == got.tolist()
    perm = rnd.permutation(n)
    assert np.array_equal(interp.run(_vecmerger_count_program(m), [keys[perm]])[0], got)


@pytest.mark.parametrize("func", ["add", "mul", "min", "max"])
def test_vecmerger_brute_force_with_initial_vector(func):
    rnd = random.Random(5)
    n, m = 300, 11
    idx = [rnd.randrange(m) for _ in range(n)]
    v = [rnd.choice([1, 2, -1, 3]) for _ in range(n)]
    init = [rnd.randrange(-3, 4) for _ in range(m)]
    p = Program(["i64", "i64"])
    pred = p.bin("ne", p.col(0), p.const("i64", 4))
    p.merge(p.vecmerger("i64", func, m), [p.col(1)], keys=[p.col(0)], pred=pred)
    want = list(init)
    for i, x in zip(idx, v):
        if i == 4:
            continue
        want[i] = {"add": want[i] + x, "mul": want[i] * x, "min": min(want[i], x), "max": max(want[i], x)}[func]
    want = [(w + (1 << 63)) % (1 << 64) - (1 << 63) for w in want]
    got = interp.run(p, [np.array(idx, np.int64), np.array(v, np.int64)], inits={0: np.array(init, np.int64)})[0]
    assert got.tolist() == want and want[4] == init[4]
    assert rowwise.run(p, [idx, v], inits={0: init})[0] == want
    fresh = interp.run(p, [np.array(idx, np.int64), np.array(v, np.int64)])[0]      # no init: identities
    assert fresh[4] == interp.identity(func, "i64")


# ----------------------------------------------------------------------
# groupbuilder (Table 1): dict[K, vec[V]] by grouping {K, V} pairs by key
# ----------------------------------------------------------------------
def _group_program(key_types, t, with_pred):
    p = Program(list(key_types) + [t])
    keys = [p.col(i) for i in range(len(key_types))]
    v = p.col(len(key_types))
    pred = p.bin("ne", keys[0], p.const(key_types[0], 3)) if with_pred else None
    p.merge(p.groupbuilder(key_types, t, 64), v, keys=keys, pred=pred)
    return p


def test_groupbuilder_hand_worked_example():
    # pairs (k, v): (2,10) (1,20) (2,30) (7,40) (1,50) (2,60)  ->  1:[20,50]  2:[10,30,60]  7:[40]
    k = np.array([2, 1, 2, 7, 1, 2], dtype=np.int32)
    v = np.array([10, 20, 30, 40, 50, 60], dtype=np.int64)
    keys, off, vals = interp.run(_group_program(["i32"], "i64", False), [k, v])[0]
    assert keys[0].tolist() == [1, 2, 7] and off.tolist() == [0, 2, 5, 6]
    assert vals.tolist() == [20, 50, 10, 30, 60, 40]
    assert rowwise.run(_group_program(["i32"], "i64", False), [k.tolist(), v.tolist()])[0] == \
        {(1,): [20, 50], (2,): [10, 30, 60], (7,): [40]}


@pytest.mark.parametrize("with_pred", [False, True])
@pytest.mark.parametrize("t", ["i8", "i32", "i64", "f64"])
def test_groupbuilder_against_per_row_loop_and_pandas(t, with_pred):
    import pandas as pd
    rnd = np.random.RandomState(4)
    n = 700
    k1 = rnd.randint(-2, 6, size=n).astype(np.int8)
    k2 = rnd.randint(0, 5, size=n).astype(np.int64) * 1_000_000_007
    v = (rnd.uniform(-5, 5, size=n) if t == "f64" else rnd.randint(-100, 100, size=n)).astype(interp.NP_TYPE[t])
    prog = _group_program(["i8", "i64"], t, with_pred)
    keys, off, vals = interp.run(prog, [k1, k2, v])[0]
    want = rowwise.run(prog, [k1.tolist(), k2.tolist(), v.tolist()])[0]
    assert len(keys[0]) == len(want) and off[0] == 0 and off[-1] == len(vals) == sum(len(x) for x in want.values())
    for g in range(len(keys[0])):
        assert vals[off[g]:off[g + 1]].tolist() == want[(int(keys[0][g]), int(keys[1][g]))]     # index order inside a group
    # a library group-by over the same filtered pairs
    mask = k1 != 3 if with_pred else np.ones(n, dtype=bool)
    df = pd.DataFrame({"a": k1[mask], "b": k2[mask], "v": v[mask]})
    lib = df.groupby(["a", "b"], sort=True)["v"].apply(list)
    assert [tuple(ix) for ix in lib.index] == list(zip(keys[0].tolist(), keys[1].tolist()))
    assert [vals[off[g]:off[g + 1]].tolist() for g in range(len(lib))] == list(lib.values)


def test_groupbuilder_relations_to_the_other_builders():
    # group sizes are the dictmerger's counts; the groups' concatenation is the vecbuilder's output
    # reordered; one key -> exactly the vecbuilder's output; all keys distinct -> singletons
    cols = [c.numpy() for c in configs.make_columns("C5", 20_000)]
    code = cols[0]
    p = Program(["i64"])
    c = p.col(0)
    pred = p.bin("gt", c, p.const("i64", 0))
    key = p.bin("mod", c, p.const("i64", 100_000))
    p.merge(p.groupbuilder(["i64"], "i64", 100_000), c, keys=[key], pred=pred)
    p.merge(p.dictmerger(["i64"], ["i64"], "add", 100_000), [p.const("i64", 1)], keys=[key], pred=pred)
    p.merge(p.vecbuilder("i64"), c, pred=pred)
    (gk, off, vals), (dk, dv), vec = interp.run(p, [code])
    assert np.array_equal(gk[0], dk[0]) and np.array_equal(np.diff(off), dv[0])
    assert np.array_equal(np.sort(vals), np.sort(vec))
    assert all(np.all(vals[off[g]:off[g + 1]] % 100_000 == gk[0][g]) for g in range(len(off) - 1))
    q = Program(["i64"])
    q.merge(q.groupbuilder(["i64"], "i64", 4), q.col(0), keys=[q.const("i64", 5)], pred=q.bin("gt", q.col(0), q.const("i64", 0)))
    gk, off, vals = interp.run(q, [code])[0]
    assert gk[0].tolist() == [5] and np.array_equal(vals, vec)
    r = Program(["i64"])
    r.merge(r.groupbuilder(["i64"], "i64", 30_000), r.col(0), keys=[r.index()])
    gk, off, vals = interp.run(r, [code])[0]
    assert np.array_equal(gk[0], np.arange(len(code))) and np.array_equal(off, np.arange(len(code) + 1)) and np.array_equal(vals, code)


# ----------------------------------------------------------------------
# dictionaries as inputs of a later loop: keyexists / dictlookup (a hash join's probe side)
# ----------------------------------------------------------------------
def _join_programs():
    """build: dict[{i32 id} -> {i64 weight, f64 price}] over the build side's rows with id % 3 != 0;
    probe: rows whose id is in the dictionary contribute price * qty to a sum and are grouped
    by the looked-up weight."""
    b = Program(["i32", "i64", "f64"])
    b.merge(b.dictmerger(["i32"], ["i64", "f64"], "add", 1000), [b.col(1), b.col(2)], keys=[b.col(0)],
            pred=b.bin("ne", b.bin("mod", b.col(0), b.const("i32", 3)), b.const("i32", 0)))
    p = Program(["i32", "f64"], dicts=[{"key_types": ["i32"], "val_types": ["i64", "f64"]}])
    hit = p.keyexists(0, [p.col(0)])
    w = p.dictlookup(0, 0, [p.col(0)])
    price = p.dictlookup(0, 1, [p.col(0)])
    p.merge(p.merger("f64", "add"), p.bin("mul", price, p.col(1)), pred=hit)
    p.merge(p.dictmerger(["i64"], ["i64"], "add", 64), [p.const("i64", 1)], keys=[w], pred=hit)
    p.merge(p.vecbuilder("i64"), w)                                     # absent keys look up 0
    return b, p


def test_dictionary_probe_hand_worked_example():
    b, p = _join_programs()
    ids = np.array([1, 2, 3, 4, 2], dtype=np.int32)                     # id 3 is filtered out, id 2 occurs twice
    weight = np.array([10, 20, 30, 40, 5], dtype=np.int64)
    price = np.array([1.0, 2.0, 3.0, 4.0, 0.5])
    table = interp.run(b, [ids, weight, price])[0]
    assert table[0][0].tolist() == [1, 2, 4] and table[1][0].tolist() == [10, 25, 40] and table[1][1].tolist() == [1.0, 2.5, 4.0]
    probe_ids = np.array([2, 3, 9, 4, 2, 1], dtype=np.int32)
    qty = np.array([1.0, 1.0, 1.0, 2.0, 3.0, 10.0])
    total, (gk, gv), looked = interp.run(p, [probe_ids, qty], dicts=[table])
    assert float(total) == 2.5 * 1 + 4.0 * 2 + 2.5 * 3 + 1.0 * 10
    assert gk[0].tolist() == [10, 25, 40] and gv[0].tolist() == [1, 2, 1]
    assert looked.tolist() == [25, 0, 0, 40, 25, 10]


def test_dictionary_probe_against_per_row_loop_and_pandas_merge():
    import pandas as pd
    rnd = np.random.RandomState(8)
    b, p = _join_programs()
    nb, npr = 900, 3000
    ids = rnd.randint(0, 700, size=nb).astype(np.int32)
    weight = rnd.randint(0, 20, size=nb).astype(np.int64)
    price = rnd.randint(1, 9, size=nb).astype(np.float64)
    table = interp.run(b, [ids, weight, price])[0]
    table_rows = rowwise.run(b, [ids.tolist(), weight.tolist(), price.tolist()])[0]
    probe_ids = rnd.randint(0, 800, size=npr).astype(np.int32)
    qty = rnd.randint(1, 5, size=npr).astype(np.float64)
    total, (gk, gv), looked = interp.run(p, [probe_ids, qty], dicts=[table])
    w_total, w_groups, w_looked = rowwise.run(p, [probe_ids.tolist(), qty.tolist()], dicts=[table_rows])
    assert float(total) == w_total and looked.tolist() == w_looked
    assert dict(zip(gk[0].tolist(), gv[0].tolist())) == {k[0]: v[0] for k, v in w_groups.items()}
    # the same join with a library: aggregate the build side, inner-merge, aggregate
    keep = ids % 3 != 0
    build = pd.DataFrame({"id": ids[keep], "w": weight[keep], "price": price[keep]}).groupby("id", as_index=False).sum()
    joined = pd.DataFrame({"id": probe_ids, "qty": qty}).merge(build, on="id", how="inner")
    assert float(total) == float((joined["price"] * joined["qty"]).sum())
    assert joined.groupby("w").size().to_dict() == dict(zip(gk[0].tolist(), gv[0].tolist()))
