"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle.

Every case runs the same seeded columns through weld_fused_for and through
oracle/interp.py and compares builder by builder under the rules of
tests/parity.py.  Sizes span several tiles (a tile is 2048 rows by default) and
a ragged tail.
"""
import math
import os

import numpy as np
import pytest
import torch

from tests import parity

from workloads import configs
from workloads.ir import Program

pytestmark = pytest.mark.gpu

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "paper_builder_examples.txt")


@pytest.fixture(scope="module")
def wb():
    from paper_1709_06416_amd import binding
    return binding


def _run(wb, prog, cols, **kw):
    return wb.fused_for(prog, cols, **kw)


def _check(wb, prog, cols, map_floor=0.0, label="", **kw):
    from tests import parity
    want = parity.oracle_results(prog, cols, kw.get("inits"))
    res = _run(wb, prog, cols, **kw)
    try:
        parity.assert_matches(prog, res, want, map_floor=map_floor, label=label)
    finally:
        res.free()


def _dev(arr):
    return torch.from_numpy(np.ascontiguousarray(arr)).cuda()


# ----------------------------------------------------------------------
# results printed in the paper
# ----------------------------------------------------------------------
def _golden_cases():
    cases = []
    for line in open(GOLDEN):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        name, ins, outs = [s.strip() for s in line.split("|")]
        cases.append((name, [[int(x) for x in v.split()] for v in ins.split(";")],
                      [[int(x) for x in v.split()] for v in outs.split(";")]))
    return cases


@pytest.mark.parametrize("name,vecs,exp", _golden_cases())
def test_paper_printed_results(wb, name, vecs, exp):
    prog = configs.EXAMPLES[name]()
    cols = [_dev(np.array(v, dtype=np.int32)) for v in vecs]
    res = _run(wb, prog, cols).check()
    for b, (spec, e) in enumerate(zip(prog.builders, exp)):
        if spec["kind"] == "vecbuilder":
            assert res.vec_host(b).tolist() == e
        else:
            assert [int(res.merger(b))] == e
    res.free()


def test_filter_sum_listing(wb):
    rnd = np.random.RandomState(7)
    pop = rnd.randint(0, 1_000_000, size=5000).astype(np.int64)
    res = _run(wb, configs.example_filter_sum(), [_dev(pop)]).check()
    assert int(res.merger(0)) == int(pop[pop > 500000].sum())
    res.free()


# ----------------------------------------------------------------------
# the five benchmark loops
# ----------------------------------------------------------------------
@pytest.mark.parametrize("name,n", [("C1", 1_000_000), ("C3", 1_000_003), ("C4", 700_001), ("C5", 1_000_003)])
def test_config(wb, name, n):
    cols = configs.make_columns(name, n, device="cuda")
    _check(wb, configs.PROGRAMS[name](), cols, label=name)


def test_config_c2_black_scholes(wb):
    # a deep out-of-the-money price is ~1e-16 while N(d) = 1/2 + 1/2 erf(.) is formed from an
    # O(1) erf value: one ulp of erf is an O(1) relative change of such a price.  Prices live in
    # [0, 100], so the element bound is 1e-12 * max(|price|, 1.0)
    cols = configs.make_columns("C2", 300_007, device="cuda")
    _check(wb, configs.program_c2(), cols, map_floor=1.0, label="C2")


def test_c2_intermediates_strict_relative(wb):
    # d1, d2 are well conditioned: strict 1e-12 relative, no floor
    base = configs.program_c2()
    p = Program(base.columns)
    p.ops = list(base.ops)
    p.merge(p.vecbuilder("f64"), base.named["d1"])
    p.merge(p.vecbuilder("f64"), base.named["d2"])
    cols = configs.make_columns("C2", 100_003, device="cuda")
    _check(wb, p, cols, label="C2-d1d2")


def test_erf_map_against_the_oracle(wb):
    # the library evaluates erf itself (piecewise polynomial, table built with the library):
    # relative 1e-12 everywhere, tiny arguments and the interval ends included; +-1 beyond 6
    rnd = np.random.RandomState(9)
    x = np.concatenate([rnd.uniform(-6.5, 6.5, 150_000), rnd.uniform(-0.07, 0.07, 20_000),
                        10.0 ** rnd.uniform(-300, -1, 2_000), -(10.0 ** rnd.uniform(-300, -1, 2_000)),
                        np.arange(0, 97) / 16.0, np.nextafter(np.arange(1, 97) / 16.0, 0),
                        [-0.0, 0.0, 5.99999, 6.0, 7.5, -7.5, 1e300, -1e300, np.inf, -np.inf]])
    p = Program(["f64"])
    p.merge(p.vecbuilder("f64"), p.un("erf", p.col(0)))
    _check(wb, p, [_dev(x)], label="erf map")


def test_log_and_exp_maps_against_the_oracle(wb):
    # the library evaluates log and exp itself (tables + polynomials): maps over wide ranges, the
    # neighbourhood of 1 where log loses its leading digits, table-interval edges, special values
    rnd = np.random.RandomState(32)
    x = np.concatenate([rnd.uniform(0.1, 10.0, 150_000), np.exp(rnd.uniform(-700, 700, 100_000)),
                        1.0 + rnd.uniform(-1e-2, 1e-2, 20_000), 1.0 + rnd.uniform(-1e-10, 1e-10, 1_000),
                        np.arange(90, 182) / 128.0, np.nextafter(np.arange(90, 182) / 128.0, 0),
                        [1.0, 0.5, 2.0, 5e-324, 2.2250738585072014e-308, 1.7976931348623157e308, 0.70703125]])
    p = Program(["f64"])
    p.merge(p.vecbuilder("f64"), p.un("log", p.col(0)))
    _check(wb, p, [_dev(x)], label="log map")                 # strict 1e-12 relative, no floor
    y = np.concatenate([rnd.uniform(-0.05, 0.0, 100_000), rnd.uniform(-700, 700, 150_000), rnd.uniform(-1, 1, 20_000),
                        (np.arange(-64, 65) + 0.5) * np.log(2) / 64, [0.0, -0.0, 709.782712893384, -708.0, 1.0, -1.0]])
    q = Program(["f64"])
    q.merge(q.vecbuilder("f64"), q.un("exp", q.col(0)))
    _check(wb, q, [_dev(y)], label="exp map")
    # special values, as the C library has them
    sp = np.array([0.0, -0.0, -1.0, np.inf, np.nan, -np.inf, 1.0])
    res = wb.fused_for(p, [_dev(sp)]).check()
    got = res.vec_host(0)
    res.free()
    assert got[0] == -np.inf and got[1] == -np.inf and np.isnan(got[2]) and got[3] == np.inf and np.isnan(got[4])
    assert np.isnan(got[5]) and got[6] == 0.0
    se = np.array([710.0, 1e300, np.inf, -746.0, -1e300, -np.inf, np.nan, -740.0])
    res = wb.fused_for(q, [_dev(se)]).check()
    got = res.vec_host(0)
    res.free()
    assert np.all(got[:3] == np.inf) and np.all(got[3:6] == 0.0) and np.isnan(got[6])
    assert abs(got[7] - np.exp(-740.0)) <= 5e-324            # a denormal result: within one denormal step


def test_plain_arithmetic_maps_are_bit_exact(wb):
    # +,-,*,/ and sqrt are correctly rounded on both sides and nothing is contracted
    p = Program(["f64", "f64"])
    x, y = p.col(0), p.col(1)
    one = p.const("f64", 1.0)
    e = p.bin("div", p.bin("add", p.bin("mul", x, y), one), p.bin("sub", p.un("sqrt", y), p.const("f64", 3.0)))
    p.merge(p.vecbuilder("f64"), e)
    cols = configs.make_columns("C1", 50_001, device="cuda")
    from oracle import interp
    want = interp.run(p, [c.cpu().numpy() for c in cols])[0]
    res = _run(wb, p, cols).check()
    assert np.array_equal(res.vec_host(0), want)
    res.free()


# ----------------------------------------------------------------------
# sizes around the tile boundary, empty input
# ----------------------------------------------------------------------
@pytest.mark.parametrize("n", [0, 1, 2, 63, 64, 127, 2047, 2048, 2049, 4096, 6143, 20_481])
@pytest.mark.parametrize("name", ["C1", "C5"])
def test_ragged_sizes(wb, name, n):
    cols = configs.make_columns(name, n, device="cuda")
    _check(wb, configs.PROGRAMS[name](), cols, label="%s n=%d" % (name, n))


@pytest.mark.parametrize("pattern", ["all", "none", "single", "first", "last"])
def test_compaction_patterns(wb, pattern):
    n = 10_007
    x = np.zeros(n, dtype=np.int64)
    if pattern == "all":
        x[:] = 99
    elif pattern == "single":
        x[4321] = 77
    elif pattern == "first":
        x[0] = 5
    elif pattern == "last":
        x[-1] = 5
    p = Program(["i64"])
    pred = p.bin("gt", p.col(0), p.const("i64", 0))
    p.merge(p.vecbuilder("i64"), p.index(), pred=pred)
    p.merge(p.vecbuilder("i64"), p.col(0), pred=pred)
    p.merge(p.merger("i64", "add"), p.const("i64", 1), pred=pred)
    res = _run(wb, p, [_dev(x)]).check()
    idx = res.vec_host(0)
    assert np.array_equal(idx, np.flatnonzero(x > 0))
    assert np.array_equal(res.vec_host(1), x[x > 0])
    assert int(res.merger(2)) == len(idx)          # compaction length == predicate count
    res.free()


def test_two_compactions_with_different_predicates(wb):
    n = 50_003
    cols = configs.make_columns("C3", n, device="cuda")
    p = Program(["i32", "f64", "f64", "f64"])
    day, disc, qty, price = p.col(0), p.col(1), p.col(2), p.col(3)
    p1 = p.bin("lt", day, p.const("i32", 1000))
    p2 = p.bin("ge", qty, p.const("f64", 25.0))
    p.merge(p.vecbuilder("i32"), day, pred=p1)
    p.merge(p.vecbuilder("f64"), p.bin("mul", price, disc), pred=p2)
    p.merge(p.vecbuilder("i64"), p.index())
    p.merge(p.merger("f64", "max"), price, pred=p1)
    _check(wb, p, cols, label="two compactions")


@pytest.mark.parametrize("n", [0, 1, 16_383, 50_003, 700_001])
@pytest.mark.parametrize("with_dict", [False, True])
def test_filtered_table_columns_share_their_predicate(wb, n, with_dict):
    """The columns of a filtered table: several vecbuilders under ONE predicate (one count and one look-back per
    tile serves them all), one under another predicate in between, with and without an LDS dictionary in the loop
    (the overlapped tile loop).  Every vector has its own length word."""
    cols = configs.make_columns("C3", n, device="cuda")
    p = Program(["i32", "f64", "f64", "f64"])
    day, disc, qty, price = p.col(0), p.col(1), p.col(2), p.col(3)
    keep = p.bin("and", p.bin("lt", day, p.const("i32", 1200)), p.bin("ge", qty, p.const("f64", 10.0)))
    other = p.bin("ge", disc, p.const("f64", 0.05))
    p.merge(p.vecbuilder("i32"), day, pred=keep)
    p.merge(p.vecbuilder("f64"), p.bin("mul", price, disc), pred=keep)
    p.merge(p.vecbuilder("f64"), qty, pred=other)
    p.merge(p.vecbuilder("i64"), p.index(), pred=keep)
    if with_dict:
        p.merge(p.dictmerger(["i64"], ["i64"], "add", 50_000), [p.const("i64", 1)],
                keys=[p.bin("mod", p.un("cast", p.bin("mul", price, p.const("f64", 7.0)), to="i64"), p.const("i64", 40_000))], pred=keep)
    res = _run(wb, p, cols).check()
    lens = [len(res.vec_host(b)) for b in (0, 1, 2, 3)]
    res.free()
    assert lens[0] == lens[1] == lens[3]
    _check(wb, p, cols, label="filtered table, %d rows" % n)


# ----------------------------------------------------------------------
# mergers
# ----------------------------------------------------------------------
@pytest.mark.parametrize("func", ["add", "mul", "min", "max"])
@pytest.mark.parametrize("t", ["i8", "i32", "i64", "f64"])
def test_merger_matrix(wb, func, t):
    rnd = np.random.RandomState(11)
    n = 30_011
    if t == "f64":
        v = rnd.choice([0.5, 1.0, 2.0, 1.0, 1.0, -1.0], size=n).astype(np.float64) if func == "mul" \
            else rnd.uniform(-3, 3, size=n)
    else:
        v = rnd.randint(-5, 6, size=n).astype(wb.TYPE_NP[t])
        if func == "mul":
            v[v == 0] = 3
    p = Program([t])
    p.merge(p.merger(t, func), p.col(0), pred=p.bin("ne", p.col(0), p.const(t, 4)))
    _check(wb, p, [_dev(v)], label="%s %s" % (func, t))


def test_unmerged_builders_return_identity(wb):
    p = Program(["f64"])
    never = p.bin("lt", p.col(0), p.const("f64", -1.0))
    for f in ("add", "min", "max", "mul"):
        p.merge(p.merger("f64", f), p.col(0), pred=never)
    p.merge(p.vecbuilder("f64"), p.col(0), pred=never)
    p.merger("i64", "min")           # declared, never merged
    cols = [configs.make_columns("C1", 5000, device="cuda")[0]]
    res = _run(wb, p, cols).check()
    assert [float(res.merger(k)) for k in range(4)] == [0.0, np.inf, -np.inf, 1.0]
    assert res.vec_len(4) == 0
    assert int(res.merger(5)) == np.iinfo(np.int64).max
    res.free()


def test_f64_sum_is_reproducible_and_inputs_untouched(wb):
    cols = configs.make_columns("C1", 300_001, device="cuda")
    before = [configs.checksum(c) for c in cols]
    prog = configs.program_c1()
    bits = set()
    for _ in range(3):
        res = _run(wb, prog, cols).check()
        bits.add(np.float64(res.merger(0)).tobytes())
        res.free()
    assert len(bits) == 1
    assert [configs.checksum(c) for c in cols] == before


# ----------------------------------------------------------------------
# loops whose builders are all mergers finish in one launch: the work-group that arrives last
# combines the partials and writes results and status
# ----------------------------------------------------------------------
def _merger_only_programs():
    progs = {"C1": configs.program_c1(), "C3": configs.program_c3()}
    p = Program(["i32", "i8", "f64"])
    keep = p.bin("ne", p.col(0), p.const("i32", 7))
    p.merge(p.merger("i32", "min"), p.col(0), pred=keep)
    p.merge(p.merger("i8", "max"), p.col(1))
    p.merge(p.merger("i64", "add"), p.un("cast", p.col(0), to="i64"), pred=keep)
    p.merge(p.merger("f64", "max"), p.col(2))
    p.merge(p.merger("i32", "add"), p.col(0))          # wraps
    progs["narrow integers, four functions"] = p
    return progs


def _merger_only_columns(name, n):
    if name in ("C1", "C3"):
        return configs.make_columns(name, n, device="cuda")
    rnd = np.random.RandomState(n % 997)
    return [_dev(rnd.randint(-2 ** 31, 2 ** 31, size=n).astype(np.int32)), _dev(rnd.randint(-128, 128, size=n).astype(np.int8)),
            _dev(rnd.normal(size=n))]


@pytest.mark.parametrize("name", sorted(_merger_only_programs()))
@pytest.mark.parametrize("n", [0, 1, 255, 4097, 300_001, 5_000_011])
def test_single_launch_merger_loops(wb, name, n):
    """One launch, the oracle's results, and bit for bit the results of the three-launch form run with
    the same grid (both combine the same partials; integer results are exact in any order, f64 sums are
    compared with the oracle inside `_check` and with each other to 1e-12 relative)."""
    prog = _merger_only_programs()[name]
    cols = _merger_only_columns(name, n)
    _check(wb, prog, cols, label="%s n=%d" % (name, n), n=n)
    one = _run(wb, prog, cols, n=n).check()
    three = _run(wb, prog, cols, n=n, tune={"single_launch": -1}).check()
    try:
        assert one.kernel_count() == 1 and three.kernel_count() == 3
        for b, spec in enumerate(prog.builders):
            x, y = one.merger(b), three.merger(b)
            if spec["type"] == "f64":
                assert x == y or abs(x - y) <= 1e-12 * abs(y), (name, n, b, x, y)
            else:
                assert int(x) == int(y), (name, n, b, x, y)
    finally:
        one.free()
        three.free()


def test_single_launch_calls_back_to_back_and_on_two_streams(wb):
    """The arrival words are shared by the calls of a stream and must be back at zero after each; two
    streams have their own and may run at once."""
    prog = configs.program_c1()
    sizes = [1_000_003, 10, 70_001, 0, 2_000_000, 4097]
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    from tests import parity
    cols = {n: configs.make_columns("C1", n, device="cuda") for n in sizes}
    want = {n: parity.oracle_results(prog, cols[n], None) for n in sizes}
    torch.cuda.synchronize()
    results = []
    for rep in range(3):
        for k, n in enumerate(sizes):
            st = streams[(k + rep) % 2]
            results.append((n, wb.fused_for(prog, cols[n], stream=st.cuda_stream)))
    try:
        for n, res in results:
            res.check()
            assert res.kernel_count() == 1
            parity.assert_matches(prog, res, want[n], label="n=%d" % n)
    finally:
        for _, res in results:
            res.free()


# ----------------------------------------------------------------------
# dictmerger
# ----------------------------------------------------------------------
@pytest.mark.parametrize("strategy", [1, 2, 3, 4])
def test_c4_every_dictionary_strategy(wb, strategy):
    cols = configs.make_columns("C4", 200_003, device="cuda")
    _check(wb, configs.program_c4(), cols, label="C4 strategy %d" % strategy, tune={"dict_strategy": strategy})


@pytest.mark.parametrize("strategy", [2, 3])
def test_c5_dictionary_strategies(wb, strategy):
    cols = configs.make_columns("C5", 400_009, device="cuda")
    _check(wb, configs.program_c5(), cols, label="C5 strategy %d" % strategy, tune={"dict_strategy": strategy})


def test_small_lds_table_overflows_into_global(wb):
    cols = configs.make_columns("C5", 300_007, device="cuda")
    _check(wb, configs.program_c5(), cols, label="C5 tiny LDS", tune={"dict_strategy": 2, "lds_dict_slots": 64})


@pytest.mark.parametrize("spill", [0, -1, 3, 40])
def test_c5_spill_queue_variants(wb, spill):
    # misses of the LDS table: queued and aggregated per key partition (0: queues sized for
    # every row), straight to the global table (-1), or queues so short that most merges
    # overflow them and take the global road after all (3, 40)
    cols = configs.make_columns("C5", 400_009, device="cuda")
    _check(wb, configs.program_c5(), cols, label="C5 spill %d" % spill, tune={"dict_spill": spill})


def test_spill_queues_shrink_to_the_memory_limit(wb):
    cols = configs.make_columns("C5", 400_009, device="cuda")
    _check(wb, configs.program_c5(), cols, label="C5 spill under a limit", memory_limit=12_000_000)
    with pytest.raises(wb.WeldError) as e:
        _run(wb, configs.program_c5(), cols, memory_limit=5_000_000)
    assert e.value.status == wb.ERR_OOM


def test_large_dictionary_of_mostly_distinct_keys(wb):
    # nearly every merge misses the LDS table; includes the key equal to the free-slot marker
    rnd = np.random.RandomState(5)
    n = 300_011
    keys = rnd.randint(0, 150_000, size=n).astype(np.int64) * 7_919 - 500_000_000
    keys[::1001] = np.iinfo(np.int64).min
    vals = rnd.uniform(-1, 1, size=n)
    p = Program(["i64", "f64"])
    p.merge(p.dictmerger(["i64"], ["f64", "i64", "f64"], "add", 160_000),
            [p.col(1), p.const("i64", 1), p.bin("mul", p.col(1), p.col(1))], keys=[p.col(0)])
    for spill in (0, -1, 5):
        _check(wb, p, [_dev(keys), _dev(vals)], label="distinct keys spill %d" % spill, tune={"dict_spill": spill})


@pytest.mark.parametrize("func", ["add", "min", "max", "mul"])
def test_dictmerger_functions_and_struct_keys(wb, func):
    rnd = np.random.RandomState(23)
    n = 40_009
    k1 = rnd.randint(-2, 3, size=n).astype(np.int8)
    k2 = rnd.randint(-1000, 1000, size=n).astype(np.int32) * 1000
    a = rnd.randint(-3, 4, size=n).astype(np.int64)
    a[a == 0] = 1
    f = rnd.choice([0.5, 1.0, 2.0, 1.0], size=n) if func == "mul" else rnd.uniform(-2, 2, size=n)
    if func == "mul":
        a = rnd.choice([1, -1, 1, 1], size=n).astype(np.int64)
        k2 = (k2 // 100000).astype(np.int32)
    p = Program(["i8", "i32", "i64", "f64"])
    pred = p.bin("ne", p.col(2), p.const("i64", 2))
    d = p.dictmerger(["i8", "i32"], ["i64", "f64"], func, 12_000)
    p.merge(d, [p.col(2), p.col(3)], keys=[p.col(0), p.col(1)], pred=pred)
    _check(wb, p, [_dev(k1), _dev(k2), _dev(a), _dev(f)], label="dict " + func)


@pytest.mark.parametrize("tune", [None, {"dict_compact": -1}, {"dict_spill": -1}, {"dict_spill": 3}, {"lds_dict_slots": 256}])
@pytest.mark.parametrize("shape", ["i32 key", "i8 i8 key", "narrow i64 key", "i32 sums", "compaction too"])
def test_compact_dictionary_cells(wb, shape, tune):
    """dictmerger[K,V,+] under a key that fits 32 bits, counting or summing 32-bit integers: 8-byte cells in
    LDS and 8-byte queue entries.  Keys of both signs, the key whose low half is the free-slot marker
    (-2^31), sums that wrap in 32 bits, more keys than the table holds."""
    rnd = np.random.RandomState(41)
    n = 300_011
    if shape == "i32 key":
        k = (rnd.randint(0, 60_000, size=n) * 71_567 - 2_000_000_000).astype(np.int32)
        k[::997] = np.iinfo(np.int32).min
        p = Program(["i32"])
        p.merge(p.dictmerger(["i32"], ["i64"], "add", 70_000), [p.const("i64", 3)], keys=[p.col(0)])
        cols = [_dev(k)]
    elif shape == "i8 i8 key":
        a = rnd.randint(-128, 128, size=n).astype(np.int8)
        b = rnd.randint(-128, 128, size=n).astype(np.int8)
        p = Program(["i8", "i8"])
        pred = p.bin("ne", p.col(0), p.const("i8", 5))
        p.merge(p.dictmerger(["i8", "i8"], ["i64"], "add", 65_536), [p.const("i64", -1)], keys=[p.col(0), p.col(1)], pred=pred)
        cols = [_dev(a), _dev(b)]
    elif shape == "narrow i64 key":
        x = rnd.randint(-10 ** 12, 10 ** 12, size=n).astype(np.int64)           # x mod 40000 takes both signs
        p = Program(["i64"])
        p.merge(p.dictmerger(["i64"], ["i64"], "add", 80_000), [p.const("i64", 1)], keys=[p.bin("mod", p.col(0), p.const("i64", 40_000))])
        cols = [_dev(x)]
    elif shape == "i32 sums":
        k = rnd.randint(0, 30_000, size=n).astype(np.int32)
        v = rnd.randint(-2 ** 31, 2 ** 31, size=n).astype(np.int32)              # sums wrap modulo 2^32
        p = Program(["i32", "i32"])
        pred = p.bin("gt", p.col(1), p.const("i32", -2_000_000_000))
        p.merge(p.dictmerger(["i32"], ["i32"], "add", 30_000), [p.col(1)], keys=[p.col(0)], pred=pred)
        cols = [_dev(k), _dev(v)]
    else:
        x = rnd.randint(-10 ** 6, 10 ** 9, size=n).astype(np.int64)
        p = Program(["i64"])
        pred = p.bin("gt", p.col(0), p.const("i64", 0))
        key = p.bin("mod", p.col(0), p.const("i64", 50_000))
        p.merge(p.vecbuilder("i64"), key, pred=pred)
        p.merge(p.dictmerger(["i64"], ["i64"], "add", 50_000), [p.const("i64", 2)], keys=[key], pred=pred)
        cols = [_dev(x)]
    if tune is None:
        src = wb.generated_source(p)
        assert "w_compact_entry(kb" in src or "w_lds_add32" in src, "this shape should take compact cells"
    _check(wb, p, cols, label="compact %s %s" % (shape, tune), tune=tune)


def test_compact_cells_are_flushed_before_a_partial_sum_overflows(wb):
    # one work-group, a constant of 1000 per merge into a handful of keys: a 32-bit partial sum would pass
    # 2^31 after 2.1 million rows; the work-group sends its table's contents on before that and goes on
    n = 5_000_003
    x = torch.arange(n, dtype=torch.int64, device="cuda")
    p = Program(["i64"])
    p.merge(p.dictmerger(["i64"], ["i64"], "add", 20_000), [p.const("i64", 1000)], keys=[p.bin("mod", p.col(0), p.const("i64", 3))])
    assert "flush_d0(); wg_rows = 0;" in wb.generated_source(p)
    res = wb.fused_for(p, [x], tune={"grid_blocks": 1, "dict_strategy": 2}).check()
    keys, vals = parity.sorted_dict(res, 0)
    res.free()
    assert keys[0].tolist() == [0, 1, 2]
    assert vals[0].tolist() == [1000 * ((n + 2 - r) // 3) for r in range(3)]       # closed form, far above 2^31


def test_dictmerger_extreme_i64_keys(wb):
    # the key whose bits equal the table's free-slot marker, and its neighbours
    lo = np.iinfo(np.int64).min
    keys = np.array([lo, lo + 1, -1, 0, 1, np.iinfo(np.int64).max, lo, lo, 0, -1] * 501, dtype=np.int64)
    p = Program(["i64"])
    p.merge(p.dictmerger(["i64"], ["i64"], "add", 16), [p.const("i64", 1)], keys=[p.col(0)])
    _check(wb, p, [_dev(keys)], label="extreme keys")
    _check(wb, p, [_dev(keys)], label="extreme keys global", tune={"dict_strategy": 3})


@pytest.mark.parametrize("tune", [None, {"dict_spill": 2}, {"dict_spill": -1}, {"lds_dict_slots": 1024}])
@pytest.mark.parametrize("func,vts", [("add", ["i64"]), ("max", ["f64", "i32"]), ("min", ["i8", "i64", "f64", "i64"])])
def test_dictionary_of_millions_of_keys_built_slice_by_slice(wb, func, vts, tune):
    """Capacity beyond what 256 LDS tables hold: the queues are partitioned by slice of the global
    table and the table is built slice by slice (one, two and four value fields: 8192-, 4096- and
    2048-slot slices); tiny queue segments send most merges down the direct path instead, which the
    slice kernel then finds in the table; keys repeat, some probe past the end of their slice."""
    rnd = np.random.RandomState(len(vts) * 7 + len(func))
    n = 400_003
    capacity = 2_000_000
    keys = rnd.randint(0, 150_000, size=n).astype(np.int64) * 2_654_435_761 % (2**40)
    keys[::1000] = -2**63                                   # the marker key
    cols = [_dev(keys)]
    p = Program(["i64"] + vts)
    vals = []
    for k, t in enumerate(vts):
        c = rnd.uniform(-3, 3, size=n) if t == "f64" else rnd.randint(-100, 100, size=n).astype(
            {"i8": np.int8, "i32": np.int32, "i64": np.int64}[t])
        cols.append(_dev(c))
        vals.append(p.col(1 + k))
    p.merge(p.dictmerger(["i64"], vts, func, capacity), vals, keys=[p.col(0)], pred=p.bin("ne", p.col(0), p.const("i64", 7)))
    _check(wb, p, cols, label="slices %s %s %s" % (func, vts, tune), tune=tune)


@pytest.mark.parametrize("repeat", [1, 2])
def test_slices_filled_the_way_a_join_build_fills_them(wb, repeat):
    """3e6 distinct keys with a stride of four (order numbers), every one once or twice, in a table of 2^23
    slots: 1024 slices that each merge some 2900 (5900) queue entries - a second round of 4096 for most of
    them when keys repeat - with the table's second hash (a table this size takes it; under the first,
    three of these keys share a home slot)."""
    from oracle import interp
    from tests import parity
    from workloads import joins
    orders, _ = joins.make_tables(3_000_000, 10, device="cuda")
    if repeat == 2:
        g = torch.Generator(device="cpu").manual_seed(5)
        order = torch.randperm(6_000_000, generator=g).cuda()
        orders = [torch.cat([c, c])[order].contiguous() for c in orders]
    build = joins.program_build(3_000_000)
    want = interp.run(build, [c.cpu().numpy() for c in orders])
    res = _run(wb, build, orders)
    try:
        parity.assert_matches(build, res, want, label="dense slices x%d" % repeat)
    finally:
        res.free()


def test_dictmerger_capacity_error(wb):
    keys = np.arange(5000, dtype=np.int64)
    p = Program(["i64"])
    p.merge(p.dictmerger(["i64"], ["i64"], "add", 100), [p.const("i64", 1)], keys=[p.col(0)])
    res = _run(wb, p, [_dev(keys)])
    assert res.status() == wb.ERR_CAPACITY
    res.free()
    p4 = configs.program_c4(capacity=4)          # six groups into four register slots
    res = _run(wb, p4, configs.make_columns("C4", 10_000, device="cuda"))
    assert res.status() == wb.ERR_CAPACITY
    res.free()


# ----------------------------------------------------------------------
# boundary behaviour
# ----------------------------------------------------------------------
def test_unaligned_columns_take_the_scalar_load_variant(wb):
    n = 30_001
    full = configs.make_columns("C1", n + 1, device="cuda")
    cols = [c[1:] for c in full]                       # 8-byte aligned only
    assert cols[0].data_ptr() % 16 == 8
    _check(wb, configs.program_c1(), cols, label="unaligned")


def test_memory_limit_is_enforced_before_launch(wb):
    cols = configs.make_columns("C2", 100_000, device="cuda")
    with pytest.raises(wb.WeldError) as e:
        _run(wb, configs.program_c2(), cols, memory_limit=1_000_000)
    assert e.value.status == wb.ERR_OOM
    res = _run(wb, configs.program_c2(), cols, memory_limit=4_000_000).check()
    res.free()


def test_tuning_variants_agree(wb):
    cols = configs.make_columns("C5", 123_457, device="cuda")
    for tune in ({"block_threads": 64, "units_per_thread": 1}, {"block_threads": 512, "units_per_thread": 2},
                 {"block_threads": 1024, "units_per_thread": 4, "grid_blocks": 3}, {"grid_blocks": 1}):
        _check(wb, configs.program_c5(), cols, label=str(tune), tune=tune)
    cols = configs.make_columns("C3", 123_457, device="cuda")
    for tune in ({"block_threads": 128, "units_per_thread": 8}, {"grid_blocks": 7}, {"block_threads": 1024}):
        _check(wb, configs.program_c3(), cols, label=str(tune), tune=tune)


def test_bounded_wait_reports_instead_of_hanging(wb):
    # a spin limit of one poll: tiles that find a predecessor unpublished give up, the
    # kernel still terminates, and the call reports a device error (or succeeds if no
    # tile ever had to wait)
    cols = configs.make_columns("C5", 2_000_003, device="cuda")
    res = _run(wb, configs.program_c5(), cols, tune={"spin_limit": 1})
    assert res.status() in (wb.OK, wb.ERR_DEVICE)
    res.free()
    _check(wb, configs.program_c5(), cols, label="after bounded wait")


def test_other_stream(wb):
    s = torch.cuda.Stream()
    cols = configs.make_columns("C3", 200_001, device="cuda")
    torch.cuda.synchronize()
    with torch.cuda.stream(s):
        _check(wb, configs.program_c3(), cols, label="side stream")


def _mixed_memory_builders():
    """Compaction + struct-key dictmerger with two value fields + vecmerger, under different predicates."""
    p = Program(["i8", "i32", "f64", "i64"])
    k1, k2, x, y = p.col(0), p.col(1), p.col(2), p.col(3)
    pa = p.bin("gt", x, p.const("f64", 0.0))
    pb = p.bin("ne", k1, p.const("i8", 1))
    p.merge(p.vecbuilder("f64"), x, pred=pa)
    p.merge(p.dictmerger(["i8", "i32"], ["f64", "i64"], "add", 40_000), [x, y], keys=[k1, k2], pred=pb)
    p.merge(p.vecmerger("i64", "add", 5000), p.const("i64", 2),
            keys=[p.bin("mod", p.bin("mul", y, y), p.const("i64", 5000))], pred=pa)
    return p


@pytest.mark.parametrize("tune", [None, {"dict_defer": -1}, {"dict_defer": -1, "merge_loop": 1}, {"units_per_thread": 2},
                                  {"units_per_thread": 1}, {"block_threads": 256, "grid_blocks": 3}, {"lds_dict_slots": 256}])
def test_merge_phase_variants_of_compacting_loops(wb, tune):
    """Loops that compact and merge into builders held in memory: merges unrolled or as one loop
    over the lane's rows, LDS-table misses walked in place or queued per wavefront - every variant
    gives the oracle's result."""
    for n in (0, 1, 4097, 300_007):
        _check(wb, configs.program_c5(), configs.make_columns("C5", n, device="cuda"), label="C5 %d %s" % (n, tune), tune=tune)
    _check(wb, _group_on_c5(), configs.make_columns("C5", 120_001, device="cuda"), label="groups %s" % tune, tune=tune)
    rnd = np.random.RandomState(5)
    n = 200_003
    cols = [_dev(a) for a in (rnd.randint(-2, 3, size=n).astype(np.int8), (rnd.zipf(1.3, size=n) % 30000).astype(np.int32) * 3,
                              rnd.uniform(-1, 3, size=n), rnd.randint(-1000, 1000, size=n).astype(np.int64))]
    _check(wb, _mixed_memory_builders(), cols, label="mixed %s" % tune, tune=tune)


def test_division_by_a_constant_takes_the_same_value_on_both_paths(wb):
    """i64 / and % by a small constant use 32-bit arithmetic when a wavefront's operands fit and
    the 64-bit form otherwise: columns that fit, columns that do not, and mixtures (also with
    negative values and values only the predicate excludes) agree with the oracle bit for bit."""
    rnd = np.random.RandomState(11)
    n = 100_003
    small = rnd.randint(0, 2**32, size=n, dtype=np.int64)
    wide = rnd.randint(-2**62, 2**62, size=n, dtype=np.int64)
    mixed = np.where(rnd.uniform(size=n) < 0.01, wide, small)
    edge = np.array([0, 1, 2**32 - 1, 2**32, 2**32 + 1, -1, -2**32, 2**63 - 1, -2**63, 99_999, 100_000, 100_001] * 10, dtype=np.int64)
    for d in (2, 7, 100_000, 2**31 - 1):
        p = Program(["i64"])
        x = p.col(0)
        p.merge(p.vecbuilder("i64"), p.bin("mod", x, p.const("i64", d)))
        p.merge(p.vecbuilder("i64"), p.bin("div", x, p.const("i64", d)))
        p.merge(p.vecbuilder("i64"), p.bin("mod", x, p.const("i64", d)), pred=p.bin("gt", x, p.const("i64", 0)))
        p.merge(p.merger("i64", "add"), p.bin("div", x, p.const("i64", d)), pred=p.bin("lt", x, p.const("i64", 5)))
        for name, col in (("small", small), ("wide", wide), ("mixed", mixed), ("edge", edge)):
            _check(wb, p, [_dev(col)], label="div/mod by %d, %s" % (d, name))


@pytest.mark.parametrize("t", ["i8", "i32"])
def test_narrow_integer_arithmetic_over_all_operand_pairs(wb, t):
    """Products, sums and differences of narrow integers wrap to their width before they are
    divided, compared or cast: every pair of i8 values (and i32 pairs around the type's limits),
    bit-exact.  (x * x) % 2 on an i8 column once came back as 89: the compiler had merged the 8-bit
    product and the remainder's rounding term into a byte dot product.)"""
    if t == "i8":
        v = np.arange(-128, 128, dtype=np.int8)
        a, b = np.repeat(v, 256), np.tile(v, 256)
    else:
        rnd = np.random.RandomState(8)
        edge = np.array([-2**31, -2**31 + 1, -65537, -65536, -46341, -3, -2, -1, 0, 1, 2, 3, 46340, 46341, 65535, 65536,
                         2**31 - 2, 2**31 - 1], dtype=np.int64)
        v = np.concatenate([edge, rnd.randint(-2**31, 2**31, size=238)]).astype(np.int32)
        a, b = np.repeat(v, 256), np.tile(v, 256)
    for ops in ((("mul", "mod", 2), ("mul", "div", 2), ("mul", "mod", 7)),            # a call has eight builders at most
                (("mul", "div", -3), ("add", "mod", 2), ("sub", "div", 5)),
                (("mul", "mod", -2), ("mul", "div", 16), ("add", "div", -2)),
                (("sub", "mod", 16), ("mul", "mod", 100), ("mul", None, 0))):
        p = Program([t, t])
        for first, second, c in ops:
            x = p.bin(first, p.col(0), p.col(1))
            if second:
                x = p.bin(second, x, p.const(t, c))
            p.merge(p.vecbuilder(t), x)
            p.merge(p.vecbuilder("i64"), p.un("cast", p.un("neg", x), to="i64"), pred=p.bin("lt", x, p.const(t, 1)))
        sq = p.bin("mul", p.col(0), p.col(0))
        p.merge(p.dictmerger([t], ["i64"], "add", 16), [p.const("i64", 1)], keys=[p.bin("mod", sq, p.const(t, 2))])
        _check(wb, p, [_dev(a), _dev(b)], label="%s arithmetic %s" % (t, ops[0]))


def test_edge_values_follow_the_documented_readings(wb):
    """Where the paper is silent the library fixes one behaviour (include/weld_hip.h) and the oracle follows the
    same reading: x / 0 = x % 0 = 0, the most negative value over -1 wraps, min / max with a NaN is NaN (operator and
    merge function), a cast of NaN is 0 and of a value beyond the 64-bit range its nearest end."""
    for t, np_t in (("i8", np.int8), ("i32", np.int32), ("i64", np.int64)):
        lo = np.iinfo(np_t).min
        a = np.array([7, -7, 0, lo, lo, 5, lo, 100] * 300, dtype=np_t)
        b = np.array([0, 0, 0, -1, 1, -1, 0, 7] * 300, dtype=np_t)
        p = Program([t, t])
        p.merge(p.vecbuilder(t), p.bin("div", p.col(0), p.col(1)))
        p.merge(p.vecbuilder(t), p.bin("mod", p.col(0), p.col(1)))
        p.merge(p.vecbuilder(t), p.bin("div", p.col(0), p.const(t, -1)))
        p.merge(p.merger(t, "add"), p.bin("mod", p.col(0), p.const(t, -1)))
        _check(wb, p, [_dev(a), _dev(b)], label="integer division edges " + t)
    nan, inf = np.nan, np.inf
    x = np.array([nan, 1.0, nan, -inf, 2.0, -0.0] * 500)
    y = np.array([1.0, nan, nan, inf, 3.0, 0.0] * 500)
    q = Program(["f64", "f64"])
    q.merge(q.vecbuilder("f64"), q.bin("min", q.col(0), q.col(1)))
    q.merge(q.vecbuilder("f64"), q.bin("max", q.col(0), q.col(1)))
    res = wb.fused_for(q, [_dev(x), _dev(y)]).check()
    mn, mx = res.vec_host(0), res.vec_host(1)
    res.free()
    assert np.all(np.isnan(mn.reshape(-1, 6)[:, :3])) and np.all(np.isnan(mx.reshape(-1, 6)[:, :3]))
    assert np.all(mn.reshape(-1, 6)[:, 3] == -inf) and np.all(mx.reshape(-1, 6)[:, 3] == inf)
    assert np.all(mn.reshape(-1, 6)[:, 4] == 2.0) and np.all(mx.reshape(-1, 6)[:, 4] == 3.0)
    for func in ("min", "max"):                                     # one NaN among 70001 merged values
        v = np.random.RandomState(3).uniform(-5, 5, size=70_001)
        v[31_337] = nan
        m = Program(["f64"])
        m.merge(m.merger("f64", func), m.col(0))
        m.merge(m.dictmerger(["i64"], ["f64"], func, 4), [m.col(0)], keys=[m.bin("mod", m.index(), m.const("i64", 3))])
        res = wb.fused_for(m, [_dev(v)]).check()
        assert np.isnan(float(res.merger(0)))
        keys, vals = parity.sorted_dict(res, 1)
        res.free()
        assert keys[0].tolist() == [0, 1, 2] and np.isnan(vals[0][31_337 % 3]) and not np.isnan(vals[0][(31_337 + 1) % 3])
    big = np.array([nan, 1e30, -1e30, 9.3e18, -9.3e18, 9.2e18, inf, -inf, 2.5, -2.5] * 300)
    c = Program(["f64"])
    for t in ("i64", "i32", "i8"):
        c.merge(c.vecbuilder(t), c.un("cast", c.col(0), to=t))
    _check(wb, c, [_dev(big)], label="casts of NaN and of values beyond the 64-bit range")


def test_prepared_loop_runs_repeatedly_on_different_inputs(wb):
    """A loop description marshalled once (prepare) and run on inputs of different sizes, with
    a tuning that differs from the default, matches the oracle every time."""
    from tests import parity
    for name, tune in (("C4", {"dict_strategy": 2}), ("C5", None), ("C2", None)):
        prog = configs.PROGRAMS[name]()
        loop = wb.prepare(prog, tune=tune)
        for n in (70_001, 0, 5_003, 70_001):
            cols = configs.make_columns(name, n, device="cuda", seed=n + 1)
            want = parity.oracle_results(prog, cols, None)
            res = wb.fused_for(loop, cols)
            try:
                parity.assert_matches(prog, res, want, map_floor=1.0 if name == "C2" else 0.0, label="%s prepared %d" % (name, n))
            finally:
                res.free()


def test_pipelined_calls_are_checked_one_by_one(wb):
    """Several calls enqueued back to back on one stream; each result is looked at while later
    calls may still be running (the evaluation point waits for its own call only), freed, and its
    memory is reused by the next round.  Every result of every round matches the oracle."""
    from tests import parity
    names = ("C5", "C1", "C4", "C2", "C3")
    progs = {c: configs.PROGRAMS[c]() for c in names}
    loops = {c: wb.prepare(progs[c]) for c in names}
    sizes = {"C5": 1_200_007, "C1": 50_001, "C4": 2_000_003, "C2": 300_001, "C3": 1_500_001}
    cols = {c: configs.make_columns(c, sizes[c], device="cuda", seed=5) for c in names}
    want = {c: parity.oracle_results(progs[c], cols[c], None) for c in names}
    pending = None
    for rnd in range(3):
        cur = [(c, wb.fused_for(loops[c], cols[c])) for c in names]
        for c, res in (pending or []):
            try:
                parity.assert_matches(progs[c], res, want[c], map_floor=1.0 if c == "C2" else 0.0, label="%s pipelined" % c)
            finally:
                res.free()
        pending = cur
    for c, res in reversed(pending):      # and the last round from its end
        try:
            parity.assert_matches(progs[c], res, want[c], map_floor=1.0 if c == "C2" else 0.0, label="%s pipelined, last round" % c)
        finally:
            res.free()


_RANDOM_TUNES = (None, None, {"units_per_thread": 1}, {"block_threads": 256, "grid_blocks": 3}, {"lds_dict_slots": 256},
                 {"dict_defer": -1}, {"merge_loop": 1}, {"dict_strategy": 2}, {"dict_spill": -1}, {"tile_pipeline": 1},
                 {"tile_pipeline": 1, "units_per_thread": 2})


@pytest.mark.parametrize("group", range(16))
def test_random_programs_match_the_oracle(wb, group):
    """Differential test: seeded random expression graphs over random column types, merged into
    random builders under random predicates (workloads/random_programs.py), evaluated by the
    generated kernel and by the oracle.  Integer results bit-exact, f64 to the usual bounds."""
    from tests import parity
    from workloads import random_programs
    for seed in range(1000 + 10 * group, 1010 + 10 * group):
        prog, cols, inits = random_programs.make(seed)
        dev_inits = {b: _dev(v) for b, v in inits.items()}
        tune = _RANDOM_TUNES[seed % len(_RANDOM_TUNES)]
        label = "random program, seed %d (%d ops, %s, %d rows, tune %s)" % (
            seed, len(prog.ops), "+".join(b["kind"] for b in prog.builders), len(cols[0]), tune)
        print(label, flush=True)
        dev = [_dev(c) for c in cols]
        if seed % 7 == 3:            # columns that start one element past an aligned address: the scalar-load variant
            dev = [torch.cat([d[:1], d])[1:] for d in dev]
        _check(wb, prog, dev, label=label, inits=dev_inits or None, tune=tune)


def test_random_programs_operator_at_a_time(wb):
    """The same kind of random programs through the operator-at-a-time mode (every intermediate
    a vector in HBM): it shares the row code generator with the fused loop but none of its
    tiling, so the two modes check each other through the oracle."""
    from workloads import random_programs
    for seed in range(3000, 3012):
        prog, cols, inits = random_programs.make(seed)
        dev_inits = {b: _dev(v) for b, v in inits.items()}
        label = "random program, unfused, seed %d (%d ops, %s, %d rows)" % (
            seed, len(prog.ops), "+".join(b["kind"] for b in prog.builders), len(cols[0]))
        print(label, flush=True)
        _check(wb, prog, [_dev(c) for c in cols], label=label, inits=dev_inits or None, mode="unfused")


def test_launch_tuning_returns_a_record_that_gives_the_same_results(wb):
    """weld_tune_launch times the loop on its own columns over several grid sizes; whatever it
    returns is a tuning record like any other: the loop run with it matches the oracle, and the
    times it reports are those of real runs."""
    from tests import parity
    for name, n in (("C3", 3_000_001), ("C4", 2_000_003), ("C5", 1_000_003)):
        prog = configs.PROGRAMS[name]()
        cols = configs.make_columns(name, n, device="cuda", seed=9)
        tune, best_ms, default_ms = wb.tune_launch(prog, cols)
        assert set(tune) <= {"grid_blocks"} and 0 < best_ms <= default_ms, (tune, best_ms, default_ms)
        want = parity.oracle_results(prog, cols, None)
        res = wb.fused_for(wb.prepare(prog, tune=tune), cols)
        try:
            parity.assert_matches(prog, res, want, label="%s tuned %s" % (name, tune))
        finally:
            res.free()
    p = Program(["f64"])
    p.merge(p.dictmerger(["i64"], ["i64"], "add", 4), [p.const("i64", 1)], keys=[p.un("cast", p.col(0), to="i64")])
    with pytest.raises(wb.WeldError):                 # more keys than the declared capacity: the tuner reports the loop's error
        wb.tune_launch(p, [_dev(np.arange(100, dtype=np.float64))])


@pytest.mark.parametrize("words", [4, 4 * 14 * 256 * 3 + 4 * 77, 40_000_004])
def test_memory_probes_touch_every_byte_once(wb, words):
    """The read probe's checksum is the sum of the 32-bit words it was given (whole 56 KB tiles and
    a ragged rest), and the copy probe copies them: the two kernels the bench line's attainable read
    rate and the scaling of the HBM counters rest on."""
    rnd = np.random.RandomState(words % 1000)
    host = rnd.randint(0, 256, size=words).astype(np.int32)        # small: a thread sums its words in 32 bits
    src = _dev(host)
    assert int(wb.probe_read(src).item()) == int(host.astype(np.int64).sum())
    dst = torch.zeros_like(src)
    wb.probe_copy(dst, src)
    torch.cuda.synchronize()
    assert torch.equal(dst, src)


def test_single_library_instance_loaded():
    # the library must bind to the HIP runtime torch already loaded, not a second copy
    libs = set()
    for line in open("/proc/self/maps"):
        if "libamdhip64" in line:
            libs.add(line.split()[-1])
    assert len(libs) == 1, libs


# ----------------------------------------------------------------------
# operator-at-a-time mode (every intermediate materialised in HBM)
# ----------------------------------------------------------------------
@pytest.mark.parametrize("name,n", [("C1", 200_003), ("C3", 300_001), ("C4", 200_001), ("C5", 300_007)])
def test_unfused_config(wb, name, n):
    cols = configs.make_columns(name, n, device="cuda")
    _check(wb, configs.PROGRAMS[name](), cols, label=name + " unfused", mode="unfused")


def test_unfused_black_scholes(wb):
    cols = configs.make_columns("C2", 100_003, device="cuda")
    _check(wb, configs.program_c2(), cols, map_floor=1.0, label="C2 unfused", mode="unfused")


@pytest.mark.parametrize("name,vecs,exp", _golden_cases())
def test_unfused_paper_printed_results(wb, name, vecs, exp):
    prog = configs.EXAMPLES[name]()
    cols = [_dev(np.array(v, dtype=np.int32)) for v in vecs]
    res = _run(wb, prog, cols, mode="unfused").check()
    for b, (spec, e) in enumerate(zip(prog.builders, exp)):
        if spec["kind"] == "vecbuilder":
            assert res.vec_host(b).tolist() == e
        else:
            assert [int(res.merger(b))] == e
    res.free()


def test_fused_equals_unfused_on_the_gpu(wb):
    # Sec. 4.5: the combined program and the loop after fusion return the same value.
    # Integer results, compaction order and f64 maps agree to the bit between the modes.
    cols = configs.make_columns("C5", 150_001, device="cuda")
    prog = configs.program_c5()
    a = _run(wb, prog, cols).check()
    b = _run(wb, prog, cols, mode="unfused").check()
    assert np.array_equal(a.vec_host(0), b.vec_host(0))
    ka, va = parity.sorted_dict(a, 1)
    kb, vb = parity.sorted_dict(b, 1)
    assert np.array_equal(ka[0], kb[0]) and np.array_equal(va[0], vb[0])
    assert b.kernel_count() > 2 * a.kernel_count()
    a.free()
    b.free()
    cols = configs.make_columns("C2", 50_001, device="cuda")
    prog = configs.program_c2()
    a = _run(wb, prog, cols).check()
    b = _run(wb, prog, cols, mode="unfused").check()
    assert np.array_equal(a.vec_host(0), b.vec_host(0)) and np.array_equal(a.vec_host(1), b.vec_host(1))
    a.free()
    b.free()


@pytest.mark.parametrize("n", [0, 1, 63, 8191, 8193])
def test_unfused_ragged_sizes(wb, n):
    for name in ("C1", "C5"):
        cols = configs.make_columns(name, n, device="cuda")
        _check(wb, configs.PROGRAMS[name](), cols, label="%s unfused n=%d" % (name, n), mode="unfused")


def test_unfused_index_constants_and_unmerged_builders(wb):
    p = Program(["i64"])
    pred = p.bin("gt", p.col(0), p.const("i64", 49))
    p.merge(p.vecbuilder("i64"), p.index(), pred=pred)
    p.merge(p.vecbuilder("i64"), p.col(0))
    p.merge(p.merger("i64", "add"), p.const("i64", 1), pred=pred)
    p.merge(p.vecbuilder("i64"), p.bin("add", p.index(), p.col(0)))
    p.merger("f64", "max")
    rnd = np.random.RandomState(5)
    x = rnd.randint(0, 100, size=20_011).astype(np.int64)
    _check(wb, p, [_dev(x)], label="unfused misc", mode="unfused")


# ----------------------------------------------------------------------
# vecmerger (Table 1; the count-occurrences program of Sec. 7.7)
# ----------------------------------------------------------------------
def _count_program(length, t="i64", func="add"):
    p = Program(["i32"])
    idx = p.un("cast", p.col(0), to="i64")
    one = p.const(t, 1) if t == "i64" else p.const(t, 1.0)
    p.merge(p.vecmerger(t, func, length), [one], keys=[idx])
    return p


@pytest.mark.parametrize("strategy", [-1, 0, 1, 2, 3, 4, 5, 6])
@pytest.mark.parametrize("length", [1, 5, 8, 9, 1000, 8192, 8193, 20_000, 300_000])
def test_vecmerger_counts_occurrences(wb, length, strategy):
    rnd = np.random.RandomState(length)
    n = 200_003
    keys = rnd.randint(0, length, size=n).astype(np.int32)
    keys[: n // 4] = keys[0]                                   # one hot cell
    p = _count_program(length)
    res = _run(wb, p, [_dev(keys)], tune={"vecmerger_strategy": strategy}).check()
    got = res.vec_host(0)
    res.free()
    assert np.array_equal(got, np.bincount(keys, minlength=length))     # library routine
    _check(wb, p, [_dev(keys)], label="vecmerger %d/%d" % (length, strategy), tune={"vecmerger_strategy": strategy})


@pytest.mark.parametrize("func", ["add", "mul", "min", "max"])
@pytest.mark.parametrize("t", ["i64", "f64"])
def test_vecmerger_functions_with_initial_vector(wb, func, t):
    rnd = np.random.RandomState(3)
    n, m = 50_021, 777
    idx = rnd.randint(0, m, size=n).astype(np.int64)
    if t == "f64":
        v = rnd.choice([0.5, 1.0, 2.0, 1.0], size=n) if func == "mul" else rnd.randint(-50, 50, size=n).astype(np.float64)
        init = rnd.randint(-5, 5, size=m).astype(np.float64)
    else:
        v = rnd.choice([1, -1, 1, 1], size=n).astype(np.int64) if func == "mul" else rnd.randint(-50, 50, size=n).astype(np.int64)
        init = rnd.randint(-5, 5, size=m).astype(np.int64)
    p = Program(["i64", t])
    pred = p.bin("ne", p.col(0), p.const("i64", 13))           # cell 13 keeps its initial value
    p.merge(p.vecmerger(t, func, m), [p.col(1)], keys=[p.col(0)], pred=pred)
    p.merge(p.merger("i64", "add"), p.const("i64", 1), pred=pred)
    inits = {0: _dev(init)}
    for strategy in (2, 3, 4):
        _check(wb, p, [_dev(idx), _dev(v)], label="vecmerger %s %s" % (func, t), inits=inits,
               tune={"vecmerger_strategy": strategy})
    _check(wb, p, [_dev(idx), _dev(v)], label="vecmerger unfused", inits=inits, mode="unfused")
    res = _run(wb, p, [_dev(idx), _dev(v)], inits=inits).check()
    assert res.vec_host(0)[13] == init[13]
    assert np.array_equal(inits[0].cpu().numpy(), init)        # the caller's vector is not written
    res.free()


def test_vecmerger_index_out_of_range_is_reported(wb):
    keys = np.array([0, 1, 2, 70, 3], dtype=np.int32)
    for strategy in (1, 2, 3):
        res = _run(wb, _count_program(8), [_dev(keys)], tune={"vecmerger_strategy": strategy})
        assert res.status() == wb.ERR_INVALID_ARG
        res.free()
    keys = np.array([0, 1, 2, 70_000, -1, 3], dtype=np.int32)
    res = _run(wb, _count_program(20_000), [_dev(keys)], tune={"vecmerger_strategy": 5})
    assert res.status() == wb.ERR_INVALID_ARG
    res.free()


@pytest.mark.parametrize("func", ["add", "mul", "min", "max"])
@pytest.mark.parametrize("t", ["i64", "f64"])
def test_vecmerger_queued_by_range_of_cells(wb, func, t):
    """Vectors beyond what one LDS copy holds: the merges are queued by range of cells and a second kernel merges
    every range in LDS.  Values from a column (10-byte entries) and constants (2-byte entries), an initial
    vector, a predicate, a second builder beside it, lengths that end inside a range and inside a tile of ranges,
    and indices so skewed that segments fill up and the rest of their merges goes to the result directly."""
    rnd = np.random.RandomState(len(func) + len(t))
    n = 400_009
    for m in (8193, 70_001, 2_100_000):
        idx = rnd.randint(0, m, size=n).astype(np.int64)
        idx[: n // 3] = idx[0]                                       # one cell takes a third of the merges
        idx[n // 3: n // 2] = m - 1                                   # the last cell
        if t == "f64":
            v = rnd.choice([0.5, 1.0, 2.0, 1.0], size=n) if func == "mul" else rnd.randint(-50, 50, size=n).astype(np.float64)
            init = rnd.randint(-5, 5, size=m).astype(np.float64)
        else:
            v = rnd.choice([1, -1, 1, 1], size=n).astype(np.int64) if func == "mul" else rnd.randint(-50, 50, size=n).astype(np.int64)
            init = rnd.randint(-5, 5, size=m).astype(np.int64)
        p = Program(["i64", t])
        pred = p.bin("ne", p.col(0), p.const("i64", 13))             # cell 13 keeps its initial value
        p.merge(p.vecmerger(t, func, m), [p.col(1)], keys=[p.col(0)], pred=pred)
        p.merge(p.merger("i64", "add"), p.const("i64", 1), pred=pred)
        inits = {0: _dev(init)}
        _check(wb, p, [_dev(idx), _dev(v)], label="queued vecmerger %s %s %d" % (func, t, m), inits=inits,
               tune={"vecmerger_strategy": 5})
        res = _run(wb, p, [_dev(idx), _dev(v)], inits=inits, tune={"vecmerger_strategy": 5}).check()
        assert res.vec_host(0)[13] == init[13]
        res.free()
        c = Program(["i64", t])
        two = c.const(t, 2) if t == "i64" else c.const(t, -1.0 if func == "mul" else 2.0)    # (a product of 1e5 twos is inf)
        c.merge(c.vecmerger(t, func, m), [two], keys=[c.col(0)])
        _check(wb, c, [_dev(idx), _dev(v)], label="queued vecmerger of a constant %s %s %d" % (func, t, m),
               tune={"vecmerger_strategy": 5})


@pytest.mark.parametrize("n", [0, 1, 63, 5_000, 16_384, 16_385])
def test_vecmerger_queued_with_few_rows(wb, n):
    """No row at all, fewer rows than one tile (every merge then takes the one-row-per-thread path behind the tiles),
    exactly one tile, one tile and a row."""
    rnd = np.random.RandomState(n + 1)
    m = 100_000
    keys = rnd.randint(0, m, size=n).astype(np.int64)
    init = rnd.randint(-5, 5, size=m).astype(np.int64)
    p = Program(["i64"])
    p.merge(p.vecmerger("i64", "add", m), [p.const("i64", 3)], keys=[p.col(0)])
    _check(wb, p, [_dev(keys)], label="queued vecmerger, %d rows" % n, inits={0: _dev(init)}, tune={"vecmerger_strategy": 5})
    v = Program(["i64"])
    v.merge(v.vecmerger("i64", "min", m), [v.col(0)], keys=[v.col(0)])
    _check(wb, v, [_dev(keys)], label="queued vecmerger with values, %d rows" % n, inits={0: _dev(init)}, tune={"vecmerger_strategy": 5})


def test_two_large_vecmergers_in_one_loop(wb):
    """One vecmerger per loop is queued by range, the other merges with device atomics; a merger and a filtered
    vector share the loop."""
    rnd = np.random.RandomState(77)
    n = 300_017
    a = rnd.randint(0, 50_000, size=n).astype(np.int64)
    b = rnd.randint(0, 90_000, size=n).astype(np.int64)
    w = rnd.randint(-9, 9, size=n).astype(np.int64)
    p = Program(["i64", "i64", "i64"])
    pred = p.bin("ne", p.col(2), p.const("i64", 0))
    p.merge(p.vecmerger("i64", "add", 50_000), [p.col(2)], keys=[p.col(0)], pred=pred)
    p.merge(p.vecmerger("i64", "max", 90_000), [p.col(2)], keys=[p.col(1)])
    p.merge(p.merger("i64", "add"), p.col(2))
    p.merge(p.vecbuilder("i64"), p.col(1), pred=pred)
    _check(wb, p, [_dev(a), _dev(b), _dev(w)], label="two large vecmergers")
    src = wb.generated_source(p)
    assert "v0_qn" in src and "v1_qn" not in src and "w_atomic<3>(a.b1_out + ix" in src


def test_vecmerger_queues_under_a_memory_limit(wb):
    """A memory limit shrinks the queues' segments (down to nothing): the merges that find no room go to the result
    with device atomics; the counts are the same."""
    rnd = np.random.RandomState(5)
    n, m = 600_011, 100_000
    keys = rnd.randint(0, m, size=n).astype(np.int32)
    p = _count_program(m)
    want = np.bincount(keys, minlength=m)
    for limit in (0, 4_000_000, 1_000_000):          # room for every entry, for about half of them, for none
        res = wb.fused_for(p, [_dev(keys)], tune={"vecmerger_strategy": 5}, memory_limit=limit).check()
        assert np.array_equal(res.vec_host(0), want), limit
        res.free()


def test_vecmerger_agrees_with_dictmerger(wb):
    # the same counts through two different builders
    cols = configs.make_columns("C5", 300_011, device="cuda")
    base = configs.program_c5()
    p = Program(["i64"])
    p.ops = list(base.ops)
    m = base.merges[1]
    p.merge(p.vecmerger("i64", "add", 100_000), m["vals"], keys=m["keys"], pred=m["pred"])
    p.merge(p.dictmerger(["i64"], ["i64"], "add", 100_000), m["vals"], keys=m["keys"], pred=m["pred"])
    res = _run(wb, p, cols).check()
    counts = res.vec_host(0)
    keys, vals = parity.sorted_dict(res, 1)
    res.free()
    assert np.array_equal(np.flatnonzero(counts), keys[0])
    assert np.array_equal(counts[keys[0]], vals[0])


# ----------------------------------------------------------------------
# lazy objects + fusion pass (Sec. 4.1, 4.5): library-style programs evaluated as one loop
# ----------------------------------------------------------------------
def test_lazy_pandas_numpy_example(wb):
    from paper_1709_06416_amd import lazy
    rnd = np.random.RandomState(7)
    pop = rnd.randint(0, 1_000_000, size=123_457).astype(np.int64)
    data = lazy.Vec.from_tensor(_dev(pop))
    total = data[data > 500000].sum()                      # filtered = data[data > 500000]; numpy.sum(filtered)
    for mode in ("fused", "unfused"):
        res = lazy.evaluate(total, mode=mode).check()
        assert int(res.merger(0)) == int(pop[pop > 500000].sum())
        launches = res.kernel_count()
        res.free()
        # fused: one loop, which (its one builder being a merger) is one launch; unfused: a kernel per operator
        assert (launches == 1) if mode == "fused" else (launches >= 5), (mode, launches)


def test_lazy_c1_and_c3_match_the_oracle(wb):
    from oracle import interp
    from paper_1709_06416_amd import lazy
    cols = configs.make_columns("C1", 400_003, device="cuda")
    x, y = [lazy.Vec.from_tensor(c) for c in cols]
    keep = x > 0.5
    v = x * y + 1.0
    res = lazy.evaluate(v[keep].sum(), v[keep].count()).check()
    want = interp.run(configs.program_c1(), [c.cpu().numpy() for c in cols])
    assert abs(float(res.merger(0)) - float(want[0])) <= 1e-9 * abs(float(want[0]))
    assert int(res.merger(1)) == int(want[1])
    res.free()

    cols = configs.make_columns("C3", 500_009, device="cuda")
    day, disc, qty, price = [lazy.Vec.from_tensor(c) for c in cols]
    keep = (day >= 365) & (day < 730) & (disc >= 0.05) & (disc <= 0.07) & (qty < 24.0)
    res = lazy.evaluate((price * disc)[keep].sum()).check()
    want = interp.run(configs.program_c3(), [c.cpu().numpy() for c in cols])
    assert abs(float(res.merger(0)) - float(want[0])) <= 1e-9 * abs(float(want[0]))
    assert res.kernel_count() == 1                        # one fused loop (and one launch), not one kernel per operator
    res.free()


def _trunc_div(a, b):
    r = np.fmod(a, b)
    return (a - r) // b


@pytest.mark.parametrize("seed", range(48))
def test_random_lazy_graphs_fuse_into_one_loop_with_numpy_results(wb, seed):
    """Random expression graphs built through the lazy object API over shared inputs, with filters
    (also chained) and several roots: reductions, counts and one materialised vector.  Every root
    is mirrored in NumPy while the graph is built; the roots are evaluated together (one fused
    loop: at most three kernels) and compared (integers and order-preserving vectors bit-exact, f64
    sums of non-negative values at 1e-9)."""
    from paper_1709_06416_amd import lazy
    rnd = np.random.RandomState(900 + seed)
    n = int(rnd.choice([1, 4_097, 123_457, 300_007]))
    pool = {"i64": [], "f64": [], "i32": []}                     # (lazy vector, numpy mirror) of full length
    for t in ("i64", "f64", "i32")[: int(rnd.randint(1, 4))]:
        host = {"i64": lambda: rnd.randint(-10 ** 9, 10 ** 9, size=n).astype(np.int64),
                "f64": lambda: np.round(rnd.uniform(-3, 3, size=n), 6),
                "i32": lambda: rnd.randint(-30_000, 30_000, size=n).astype(np.int32)}[t]()
        pool[t].append((lazy.Vec.from_tensor(_dev(host)), host))
    types = [t for t in pool if pool[t]]
    masks = []
    np_t = {"i64": np.int64, "f64": np.float64, "i32": np.int32}
    with np.errstate(all="ignore"):
        for _ in range(int(rnd.randint(3, 10))):
            t = str(rnd.choice(types))
            (la, ha) = pool[t][int(rnd.randint(len(pool[t])))]
            other_is_vec = rnd.rand() < 0.5
            (lb, hb) = pool[t][int(rnd.randint(len(pool[t])))] if other_is_vec else (None, None)
            c = float(np.round(rnd.uniform(-2, 2), 2)) if t == "f64" else int(rnd.randint(2, 50))
            op = str(rnd.choice(["add", "sub", "mul", "cmp", "cmp", "neg", "divc", "modc"] if t != "f64" else
                                ["add", "sub", "mul", "cmp", "cmp", "neg", "sqrt2"]))
            rhs_l, rhs_h = (lb, hb) if other_is_vec else (c, np_t[t](c))
            if op == "add":
                pool[t].append((la + rhs_l, ha + rhs_h))
            elif op == "sub":
                pool[t].append((la - rhs_l, ha - rhs_h))
            elif op == "mul":
                if t == "f64" and np.max(np.abs(ha), initial=0) * np.max(np.abs(rhs_h), initial=0) > 1e100:
                    continue
                pool[t].append((la * rhs_l, ha * rhs_h))
            elif op == "neg":
                pool[t].append((-la, -ha))
            elif op == "divc":
                pool[t].append((la / c, _trunc_div(ha, np_t[t](c))))
            elif op == "modc":
                pool[t].append((la % c, np.fmod(ha, np_t[t](c))))
            elif op == "sqrt2":
                pool[t].append(((la * la).sqrt(), np.sqrt(ha * ha)))
            else:
                which = str(rnd.choice(["lt", "le", "gt", "ge"]))
                lm = {"lt": la < rhs_l, "le": la <= rhs_l, "gt": la > rhs_l, "ge": la >= rhs_l}[which]
                hm = {"lt": ha < rhs_h, "le": ha <= rhs_h, "gt": ha > rhs_h, "ge": ha >= rhs_h}[which]
                masks.append((lm, hm))
                if len(masks) >= 2 and rnd.rand() < 0.4:
                    (l1, h1), (l2, h2) = masks[-1], masks[int(rnd.randint(len(masks) - 1))]
                    masks.append((l1 & l2, h1 & h2) if rnd.rand() < 0.5 else (l1 | l2, h1 | h2))
    roots, wants = [], []
    for _ in range(int(rnd.randint(1, 5))):
        t = str(rnd.choice(types))
        lv, hv = pool[t][int(rnd.randint(len(pool[t])))]
        kind = str(rnd.choice(["sum", "min", "max", "count", "vec"]))
        if kind == "sum" and t == "f64":
            lv, hv = lv * lv, hv * hv                          # non-negative: the tolerance is relative to the sum
        if masks and rnd.rand() < 0.7:
            lm, hm = masks[int(rnd.randint(len(masks)))]
            lv, hv = lv[lm], hv[hm]
            if masks and rnd.rand() < 0.3 and kind != "vec":      # a filter of a filtered vector
                lm2, hm2 = masks[int(rnd.randint(len(masks)))]
                lv, hv = lv[lm2[lm]], hv[hm2[hm]]
        if kind == "sum":
            roots.append(lv.sum()); wants.append(("sum", t, hv))
        elif kind == "min":
            roots.append(lv.min()); wants.append(("min", t, hv))
        elif kind == "max":
            roots.append(lv.max()); wants.append(("max", t, hv))
        elif kind == "count":
            roots.append(lv.count()); wants.append(("count", "i64", hv))
        elif not any(w[0] == "vec" for w in wants):
            roots.append(lv); wants.append(("vec", t, hv))
    if not roots:
        lv, hv = pool[types[0]][0]
        roots.append(lv.count()); wants.append(("count", "i64", hv))
    res = lazy.evaluate(*roots).check()
    try:
        assert res.kernel_count() <= 3, res.kernel_count()          # one fused loop: fill, loop, final combination
        for i, (kind, t, hv) in enumerate(wants):
            tag = "seed %d root %d (%s %s)" % (seed, i, kind, t)
            if kind == "vec":
                assert np.array_equal(res.vec_host(i), hv), tag
            elif kind == "count":
                assert int(res.merger(i)) == len(hv), tag
            elif kind == "sum":
                if t == "f64":
                    want = math.fsum(hv.tolist())
                    assert abs(float(res.merger(i)) - want) <= 1e-9 * abs(want), (tag, res.merger(i), want)
                else:
                    assert int(res.merger(i)) == int(np.add.reduce(hv, dtype=hv.dtype)), tag
            elif len(hv):
                want = hv.min() if kind == "min" else hv.max()
                assert res.merger(i) == want, (tag, res.merger(i), want)
    finally:
        res.free()


def test_lazy_groupby_and_materialised_vector(wb):
    from oracle import interp
    from paper_1709_06416_amd import lazy
    cols = configs.make_columns("C4", 300_007, device="cuda")
    flag, status, day, qty, price, disc, tax = [lazy.Vec.from_tensor(c) for c in cols]
    keep = day <= 2400
    dp = price * (1.0 - disc)
    charge = dp * (1.0 + tax)
    ones = (day * 0).cast("i64") + 1
    d = lazy.groupby([flag[keep], status[keep]], [qty[keep], price[keep], dp[keep], charge[keep], ones[keep]], "add", 8)
    res = lazy.evaluate(d, charge[keep]).check()
    (wkeys, wvals), = interp.run(configs.program_c4(), [c.cpu().numpy() for c in cols])
    keys, vals = parity.sorted_dict(res, 0)
    assert np.array_equal(keys[0], wkeys[0]) and np.array_equal(keys[1], wkeys[1])
    for k in range(4):
        assert np.all(np.abs(vals[k] - wvals[k]) <= 1e-9 * np.abs(wvals[k]))
    assert np.array_equal(vals[4], wvals[4])
    host = [c.cpu().numpy() for c in cols]
    m = host[2] <= 2400
    want_vec = ((host[4] * (1.0 - host[5])) * (1.0 + host[6]))[m]
    assert np.array_equal(res.vec_host(1), want_vec)      # order-preserving, bit-exact
    res.free()


# ----------------------------------------------------------------------
# compacting loops with the next tile's columns loaded ahead (two tiles of one work-group overlap)
# ----------------------------------------------------------------------
def _pipelined_programs():
    progs = {}
    p = Program(["i64"])                                          # the C5 shape: the library's own choice is the pipelined form
    pred = p.bin("gt", p.col(0), p.const("i64", 0))
    key = p.bin("mod", p.col(0), p.const("i64", 30_000))
    p.merge(p.vecbuilder("i64"), key, pred=pred)
    p.merge(p.dictmerger(["i64"], ["i64"], "add", 30_000), [p.const("i64", 1)], keys=[key], pred=pred)
    progs["filter, vector and count"] = p
    p = Program(["i32", "f64", "i64"])                            # several columns, two compacted vectors, an f64 dictionary
    pred = p.bin("lt", p.col(1), p.const("f64", 0.75))
    p.merge(p.vecbuilder("i32"), p.col(0), pred=pred)
    p.merge(p.vecbuilder("f64"), p.bin("mul", p.col(1), p.const("f64", 3.0)), pred=pred)
    p.merge(p.dictmerger(["i64"], ["f64", "i64"], "add", 10_000), [p.col(1), p.const("i64", 1)],
            keys=[p.bin("mod", p.col(2), p.const("i64", 5_000))], pred=pred)
    p.merge(p.merger("i64", "max"), p.col(2))
    progs["three columns, two vectors"] = p
    p = Program(["i64"])                                          # compaction alone (no merge phase between loads and stores)
    p.merge(p.vecbuilder("i64"), p.col(0), pred=p.bin("ne", p.bin("mod", p.col(0), p.const("i64", 3)), p.const("i64", 0)))
    progs["compaction alone"] = p
    return progs


@pytest.mark.parametrize("name", sorted(_pipelined_programs()))
@pytest.mark.parametrize("n", [0, 1, 16_383, 16_384, 16_385, 1_000_003])
def test_pipelined_tile_loop_matches_the_oracle(wb, name, n):
    """Forced on and forced off, on sizes around one tile (16384 rows of a 1024-thread work-group),
    a ragged last tile and many tiles per work-group; order-preserving vectors are compared element by element."""
    prog = _pipelined_programs()[name]
    rnd = np.random.RandomState(n % 1000 + len(name))
    host = {"i64": rnd.randint(-50_000, 10 ** 9, size=n).astype(np.int64), "i32": rnd.randint(-2 ** 31, 2 ** 31, size=n).astype(np.int32),
            "f64": rnd.uniform(0, 1, size=n)}
    cols = [_dev(host[t]) for t in prog.columns]
    for form in (1, -1):
        _check(wb, prog, cols, label="%s n=%d tile_pipeline=%d" % (name, n, form), tune={"tile_pipeline": form}, n=n)


# ----------------------------------------------------------------------
# scalars defined outside the loop as operands of its body (Sec. 3.2: the loop's function is a
# closure; Sec. 4.1: objects depend on the results of other objects)
# ----------------------------------------------------------------------
def _scalar_program(t):
    """Every builder kind fed by expressions of a vector element x and an outside scalar s."""
    p = Program([t, t])
    x, s = p.col(0), p.scalar(1)
    p.merge(p.merger(t, "add"), p.bin("mul", x, s))
    p.merge(p.vecbuilder(t), p.bin("sub", x, s), pred=p.bin("gt", x, s))
    if t != "f64":
        key = p.bin("mod", p.bin("add", x, s), p.const(t, 7))
        p.merge(p.dictmerger([t], [t], "add", 16), [s], keys=[key])
    p.merge(p.merger(t, "max"), s, pred=p.bin("lt", x, s))         # a scalar merged directly
    return p


@pytest.mark.parametrize("t", ["i32", "i64", "f64"])
@pytest.mark.parametrize("mode", ["fused", "unfused"])
def test_scalar_operand_of_a_loop_body(wb, t, mode):
    from oracle import interp
    from tests import parity
    rnd = np.random.RandomState(11)
    prog = _scalar_program(t)
    for n in (0, 1, 5000, 70_001):
        if t == "f64":
            x, s = rnd.uniform(-50, 50, n), np.array([3.25])
        else:
            x, s = rnd.randint(-1000, 1000, n).astype(wb.TYPE_NP[t]), np.array([17], dtype=wb.TYPE_NP[t])
        want = interp.run(prog, [x, s], sums="exact")
        res = wb.fused_for(prog, [_dev(x), _dev(s)], mode=mode, n=n)
        try:
            parity.assert_matches(prog, res, want, label="%s %s n=%d" % (t, mode, n))
        finally:
            res.free()


def test_scalar_operands_are_checked_on_the_host(wb):
    p = Program(["i64", "i64"])
    x = p.col(0)
    p.merge(p.merger("i64", "add"), p.bin("add", x, p.scalar(1)))
    with pytest.raises(wb.WeldError):                              # two elements where one is expected
        wb.fused_for(p, [_dev(np.arange(4)), _dev(np.arange(2))])
    with pytest.raises(wb.WeldError) as e:                         # the same entry as vector and as scalar
        q = Program(["i64"])
        q.merge(q.merger("i64", "add"), q.bin("add", q.col(0), q.scalar(0)))
        wb.fused_for(q, [_dev(np.arange(1))])
    assert "scalar" in str(e.value) or "vector" in str(e.value)


def test_a_reduction_feeds_the_next_loop_without_a_host_wait(wb):
    """sum and count in one loop; the second loop reads both from device memory (x * count - sum:
    integers, so every stage is exact) while nothing has waited for the first."""
    from oracle import interp
    rnd = np.random.RandomState(5)
    x = rnd.randint(-10_000, 10_000, 300_007).astype(np.int64)
    first = Program(["i64"])
    c = first.col(0)
    first.merge(first.merger("i64", "add"), c)
    first.merge(first.merger("i64", "add"), first.const("i64", 1))
    second = Program(["i64", "i64", "i64"])
    v, total, count = second.col(0), second.scalar(1), second.scalar(2)
    centred = second.bin("sub", second.bin("mul", v, count), total)
    second.merge(second.vecbuilder("i64"), centred)
    second.merge(second.merger("i64", "max"), centred)
    second.merge(second.vecbuilder("i64"), v, pred=second.bin("gt", centred, second.const("i64", 0)))
    w1 = interp.run(first, [x])
    w2 = interp.run(second, [x, np.array([w1[0]]), np.array([w1[1]])])
    dx = _dev(x)
    r1 = wb.fused_for(first, [dx])
    r2 = wb.fused_for(second, [dx, r1.scalar_ref(0), r1.scalar_ref(1)], n=len(x))      # enqueued behind r1, no wait between
    r2.check()
    assert np.array_equal(r2.vec_host(0), w2[0]) and int(r2.merger(1)) == int(w2[1])
    assert np.array_equal(r2.vec_host(2), w2[2])
    assert int(r1.merger(0)) == int(w1[0]) and int(r1.merger(1)) == int(w1[1])
    r2.free()
    r1.free()


@pytest.mark.parametrize("mode", ["fused", "unfused"])
def test_lazy_scalars_feed_later_objects_in_stages(wb, mode):
    """Standardisation as a library would write it (z = (x - mean) / std): the mean needs a sum and
    a count, the variance needs the mean, z needs both: three loops, the later ones reading the
    earlier ones' results on the device.  The oracle runs the same three loops, each fed with the
    ORACLE's results of the one before."""
    from oracle import interp
    from paper_1709_06416_amd import lazy
    rnd = np.random.RandomState(21)
    x = rnd.normal(40.0, 12.0, 200_003)
    lx = lazy.Vec.from_tensor(_dev(x))
    n = lx.count().cast("f64")
    total = lx.sum()
    mean = total / n
    d = lx - mean
    var = (d * d).sum() / lx.count().cast("f64")                   # a second count(): folded into the first
    z = d / var.sqrt()
    text = lazy.describe(z, total, z.max())
    assert text.count("for(") == 3 and "let {s0, s1} =" in text and "let {s2} =" in text

    s1 = Program(["f64"])
    s1.merge(s1.merger("f64", "add"), s1.col(0))
    s1.merge(s1.merger("i64", "add"), s1.const("i64", 1))
    w_sum, w_cnt = interp.run(s1, [x], sums="exact")

    def centred(p):
        v, t, c = p.col(0), p.scalar(1), p.scalar(2)
        return p.bin("sub", v, p.bin("div", t, p.un("cast", c, "f64")))
    s2 = Program(["f64", "f64", "i64"])
    dd = centred(s2)
    s2.merge(s2.merger("f64", "add"), s2.bin("mul", dd, dd))
    scal = [np.array([w_sum]), np.array([w_cnt])]
    w_ss, = interp.run(s2, [x] + scal, sums="exact")
    s3 = Program(["f64", "f64", "i64", "f64"])
    dd = centred(s3)
    std = s3.un("sqrt", s3.bin("div", s3.scalar(3), s3.un("cast", s3.scalar(2), "f64")))
    zz = s3.bin("div", dd, std)
    s3.merge(s3.vecbuilder("f64"), zz)
    s3.merge(s3.merger("f64", "max"), zz)
    w_z, w_max = interp.run(s3, [x] + scal + [np.array([w_ss])], sums="exact")

    res = lazy.evaluate(z, total, z.max(), mode=mode).check()
    got = res.vec_host(0)
    # the scalars are sums, equal to the oracle's to 1e-9 of their value (in practice a few ulp); an
    # error e in the mean moves every z by e / std: an absolute bound, not one relative to z
    assert len(got) == len(w_z) and np.all(np.abs(got - w_z) <= 1e-9 * 40.0 / 12.0)
    assert np.all(np.abs(got - w_z) <= 1e-12)                       # what is actually seen: rounding only
    assert abs(float(res.merger(1)) - float(w_sum)) <= 1e-9 * abs(float(w_sum))       # a root an earlier stage computed
    assert abs(float(res.merger(2)) - float(w_max)) <= 1e-9
    if mode == "fused":
        assert res.kernel_count() <= 9                              # three loops (each: loop kernel + finish), not one per operator
    res.free()


# ----------------------------------------------------------------------
# groupbuilder (Table 1): dict[K, vec[V]]
# ----------------------------------------------------------------------
def _group_on_c5(capacity=100_000):
    p = Program(["i64"])
    c = p.col(0)
    pred = p.bin("gt", c, p.const("i64", 0))
    key = p.bin("mod", c, p.const("i64", 100_000))
    p.merge(p.groupbuilder(["i64"], "i64", capacity), c, keys=[key], pred=pred)
    return p


@pytest.mark.parametrize("n", [0, 1, 63, 4096, 4097, 300_007])
def test_groupbuilder_on_the_zip_code_column(wb, n):
    cols = configs.make_columns("C5", n, device="cuda")
    _check(wb, _group_on_c5(), cols, label="groups %d" % n)


@pytest.mark.parametrize("t", ["i8", "i32", "i64", "f64"])
def test_groupbuilder_struct_keys_value_types_and_other_builders(wb, t):
    rnd = np.random.RandomState(31)
    n = 150_001
    k1 = rnd.randint(-2, 3, size=n).astype(np.int8)
    k2 = (rnd.zipf(1.5, size=n) % 3000).astype(np.int32) * 7
    v = (rnd.uniform(-5, 5, size=n) if t == "f64" else rnd.randint(-100, 100, size=n)).astype(
        {"i8": np.int8, "i32": np.int32, "i64": np.int64, "f64": np.float64}[t])
    p = Program(["i8", "i32", t])
    pred = p.bin("ne", p.col(1), p.const("i32", 14))
    p.merge(p.merger("i64", "add"), p.un("cast", p.col(1), to="i64"))
    p.merge(p.groupbuilder(["i8", "i32"], t, 20_000), p.col(2), keys=[p.col(0), p.col(1)], pred=pred)
    p.merge(p.vecbuilder(t), p.col(2), pred=pred)
    _check(wb, p, [_dev(k1), _dev(k2), _dev(v)], label="groups " + t)


def test_groupbuilder_one_group_all_distinct_and_the_marker_key(wb):
    n = 50_000
    x = np.arange(n, dtype=np.int64) * 3 - 70_000
    p = Program(["i64"])
    p.merge(p.groupbuilder(["i64"], "i64", 4), p.col(0), keys=[p.const("i64", 5)])
    _check(wb, p, [_dev(x)], label="one group")
    q = Program(["i64"])
    q.merge(q.groupbuilder(["i64"], "i64", n), q.col(0), keys=[q.col(0)])
    _check(wb, q, [_dev(x)], label="all distinct")
    lo = np.iinfo(np.int64).min
    keys = np.array([lo, lo + 1, -1, 0, lo, 5, lo] * 300, dtype=np.int64)
    vals = np.arange(len(keys), dtype=np.int64)
    r = Program(["i64", "i64"])
    r.merge(r.groupbuilder(["i64"], "i64", 16), r.col(1), keys=[r.col(0)])
    _check(wb, r, [_dev(keys), _dev(vals)], label="marker key")


def test_groupbuilder_capacity_error_and_unfused_mode(wb):
    cols = configs.make_columns("C5", 100_003, device="cuda")
    res = _run(wb, _group_on_c5(capacity=100), cols)
    assert res.status() == wb.ERR_CAPACITY
    res.free()
    _check(wb, _group_on_c5(), cols, label="groups unfused", mode="unfused")


@pytest.mark.parametrize("capacity", [1_024, 1_025, 40_000, 131_073, 1_048_576, 2_000_000])
@pytest.mark.parametrize("vt", ["i8", "f64"])
def test_groupbuilder_placement_paths(wb, capacity, vt):
    """Few groups are placed by one kernel, many by partitioning into ranges of groups first (1024
    to 4096 groups a range by capacity), very many by the one kernel again; keys whose packed
    bits are the table's marker, capacities one past a power of two, 1- and 8-byte values."""
    rnd = np.random.RandomState(capacity % 1000 + len(vt))
    n = 180_001
    distinct = min(capacity, 900) if capacity < 2_000 else 30_000
    keys = (rnd.zipf(1.2, size=n) % distinct).astype(np.int64) * 1_000_003 - 77
    keys[::5000] = -2**63                                   # the marker key
    vals = rnd.randint(-100, 100, size=n).astype(np.int8) if vt == "i8" else rnd.uniform(-1, 1, size=n)
    p = Program(["i64", vt])
    p.merge(p.groupbuilder(["i64"], vt, capacity), p.col(1), keys=[p.col(0)], pred=p.bin("ne", p.col(0), p.const("i64", 5)))
    _check(wb, p, [_dev(keys), _dev(vals)], label="groups cap %d %s" % (capacity, vt))


@pytest.mark.parametrize("capacity", [1_024, 40_000])
@pytest.mark.parametrize("vt", ["i8", "i64"])
def test_groupbuilder_keys_that_provably_fit_32_bits(wb, capacity, vt):
    """A 64-bit key that the body bounds (a remainder by a constant, a cast from i32) travels to the placement
    kernels as its low half: negative keys, -1 and both ends of the range must come back as themselves."""
    rnd = np.random.RandomState(capacity % 97 + len(vt))
    n = 170_003
    x = rnd.randint(-2**40, 2**40, size=n).astype(np.int64)
    x[:4] = [-499, 499, -1, 0]
    y = rnd.randint(0, 700, size=n).astype(np.int64) * 6_000_011 - 2**31 + 5      # few distinct values over the whole 32-bit range
    y[:4] = [-2**31, 2**31 - 1, -1, 0]
    y = y.astype(np.int32)
    vals = rnd.randint(-100, 100, size=n).astype(np.int8 if vt == "i8" else np.int64)
    p = Program(["i64", "i32", vt])
    p.merge(p.groupbuilder(["i64"], vt, capacity), p.col(2), keys=[p.bin("mod", p.col(0), p.const("i64", 500))])
    _check(wb, p, [_dev(x), _dev(y), _dev(vals)], label="groups, remainder keys %d %s" % (capacity, vt))
    q = Program(["i64", "i32", vt])
    q.merge(q.groupbuilder(["i64"], vt, capacity), q.col(2), keys=[q.un("cast", q.col(1), to="i64")],
            pred=q.bin("ne", q.col(0), q.const("i64", 7)))
    _check(wb, q, [_dev(x), _dev(y), _dev(vals)], label="groups, cast keys %d %s" % (capacity, vt))


def test_groupbuilder_offsets_over_more_rounds_than_work_groups(wb):
    """2.2e6 groups: the offsets are scanned 8192 groups a round by at most one work-group per compute
    unit, so here every work-group takes a second round and looks back at rounds of other work-groups."""
    n = 2_200_000
    rnd = np.random.RandomState(12)
    keys = rnd.permutation(n).astype(np.int64) * 7 - 3
    keys[:200_000] = keys[200_000:400_000]                    # some groups of two, some keys absent
    vals = np.arange(n, dtype=np.int64)
    p = Program(["i64", "i64"])
    p.merge(p.groupbuilder(["i64"], "i64", n), p.col(1), keys=[p.col(0)])
    _check(wb, p, [_dev(keys), _dev(vals)], label="groups, 269 rounds of offsets")


def test_groupbuilder_without_room_for_the_partition_scratch(wb):
    """Under a memory limit that leaves no room for 10 bytes of scratch per row the one-kernel
    placement is used; the result is the same."""
    cols = configs.make_columns("C5", 300_007, device="cuda")
    prog = _group_on_c5()
    from tests import parity
    want = parity.oracle_results(prog, cols, None)
    free = wb.fused_for(prog, cols)
    limited = wb.fused_for(prog, cols, memory_limit=16_500_000)      # the loop itself needs about 15 MB here
    try:
        parity.assert_matches(prog, free, want, label="groups, no limit")
        parity.assert_matches(prog, limited, want, label="groups, limit")
        assert limited.kernel_count() < free.kernel_count()             # one placement kernel instead of two
    finally:
        free.free()
        limited.free()


# ----------------------------------------------------------------------
# dictionaries of earlier calls probed by a later loop (hash join: build, then probe)
# ----------------------------------------------------------------------
def _join_case(rnd, n_build, n_probe, two_keys):
    kt = ["i32", "i8"] if two_keys else ["i32"]
    b = Program(kt + ["i64", "f64"])
    bk = [b.col(i) for i in range(len(kt))]
    b.merge(b.dictmerger(kt, ["i64", "f64"], "add", max(64, n_build)), [b.col(len(kt)), b.col(len(kt) + 1)], keys=bk,
            pred=b.bin("ne", b.bin("mod", b.col(0), b.const("i32", 3)), b.const("i32", 0)))
    p = Program(kt + ["f64"], dicts=[{"key_types": kt, "val_types": ["i64", "f64"]}])
    pk = [p.col(i) for i in range(len(kt))]
    hit = p.keyexists(0, pk)
    w = p.dictlookup(0, 0, pk)
    price = p.dictlookup(0, 1, pk)
    p.merge(p.merger("f64", "add"), p.bin("mul", price, p.col(len(kt))), pred=hit)
    p.merge(p.dictmerger(["i64"], ["i64"], "add", 4096), [p.const("i64", 1)], keys=[w], pred=hit)
    p.merge(p.vecbuilder("i64"), w)
    p.merge(p.vecbuilder("f64"), price, pred=p.un("not", hit))
    span = max(4, n_build)
    mk = lambda m: [rnd.randint(-span, span, size=m).astype(np.int32)] + ([rnd.randint(-2, 3, size=m).astype(np.int8)] if two_keys else [])
    build_cols = mk(n_build) + [rnd.randint(0, 50, size=n_build).astype(np.int64), rnd.randint(1, 9, size=n_build).astype(np.float64)]
    probe_cols = mk(n_probe) + [rnd.randint(1, 5, size=n_probe).astype(np.float64)]
    return b, p, build_cols, probe_cols


@pytest.mark.parametrize("two_keys", [False, True])
@pytest.mark.parametrize("n_build,n_probe", [(0, 1000), (1, 1), (5_000, 0), (5_000, 200_003), (150_000, 70_001)])
def test_probe_of_a_dictionary_built_by_an_earlier_call(wb, n_build, n_probe, two_keys):
    from oracle import interp
    from tests import parity
    rnd = np.random.RandomState(n_build + n_probe)
    b, p, build_cols, probe_cols = _join_case(rnd, n_build, n_probe, two_keys)
    table = interp.run(b, build_cols)[0]
    want = interp.run(p, probe_cols, dicts=[table])
    built = _run(wb, b, [_dev(c) for c in build_cols])            # not waited for: the probe is enqueued behind it
    res = _run(wb, p, [_dev(c) for c in probe_cols], dicts=[(built, 0)])
    try:
        parity.assert_matches(p, res, want, label="probe %d %d" % (n_build, n_probe))
        built.check()
    finally:
        res.free()
        built.free()


@pytest.mark.parametrize("group", range(5))
def test_random_joins_match_the_oracle(wb, group):
    """Differential test of dictionaries as loop inputs: a seeded random build loop (one dictmerger
    over one or two reduced integer keys, one to three value fields) and a random probe loop that
    computes key structs, asks whether they exist, looks value fields up and computes on with the
    answers (workloads/random_programs.py), against the oracle's Python-dict probe."""
    from oracle import interp
    from tests import parity
    from workloads import random_programs
    for seed in range(4000 + 8 * group, 4008 + 8 * group):
        b, build_cols, p, probe_cols, inits = random_programs.make_probe(seed)
        label = "random join, seed %d (%d build rows, %d probe rows, keys %s)" % (
            seed, len(build_cols[0]), len(probe_cols[0]), b.builders[0]["key_types"])
        print(label, flush=True)
        table = interp.run(b, build_cols)[0]
        want = interp.run(p, probe_cols, dicts=[table], sums="exact", inits=inits)
        dev_inits = {k: _dev(v) for k, v in inits.items()}
        built = _run(wb, b, [_dev(c) for c in build_cols])
        res = _run(wb, p, [_dev(c) for c in probe_cols], dicts=[(built, 0)], inits=dev_inits or None)
        try:
            parity.assert_matches(p, res, want, label=label)
            parity.assert_matches(b, built, [table], label=label + ", build side")
        finally:
            res.free()
            built.free()


def test_probe_argument_errors(wb):
    rnd = np.random.RandomState(1)
    b, p, build_cols, probe_cols = _join_case(rnd, 100, 100, False)
    built = _run(wb, b, [_dev(c) for c in build_cols]).check()
    dev = [_dev(c) for c in probe_cols]
    with pytest.raises(wb.WeldError) as e:                          # probe ops without a dictionary
        _run(wb, p, dev)
    assert e.value.status == wb.ERR_INVALID_ARG
    other = _run(wb, configs.program_c1(), configs.make_columns("C1", 1000, device="cuda")).check()
    with pytest.raises(wb.WeldError) as e:                          # a merger is not a dictionary
        _run(wb, p, dev, dicts=[(other, 0)])
    assert e.value.status == wb.ERR_INVALID_ARG
    q = Program(["i64", "f64"], dicts=[{"key_types": ["i64"], "val_types": ["i64", "f64"]}])
    q.merge(q.merger("i64", "add"), q.dictlookup(0, 0, [q.col(0)]))
    with pytest.raises(wb.WeldError) as e:                          # i64 key against an i32-keyed dictionary
        _run(wb, q, [_dev(np.zeros(10, np.int64)), _dev(np.zeros(10))], dicts=[(built, 0)])
    assert e.value.status == wb.ERR_TYPE
    with pytest.raises(wb.WeldError) as e:
        _run(wb, p, dev, dicts=[(built, 0)], mode="unfused")
    assert e.value.status == wb.ERR_UNSUPPORTED
    other.free()
    built.free()


def test_join_shaped_like_q12(wb):
    from oracle import interp
    from tests import parity
    from workloads import joins
    orders, lines = joins.make_tables(40_000, 160_001, device="cuda")
    build, probe = joins.program_build(40_000), joins.program_probe()
    table = interp.run(build, [c.cpu().numpy() for c in orders])[0]
    want = interp.run(probe, [c.cpu().numpy() for c in lines], dicts=[table])
    built = _run(wb, build, orders)
    res = _run(wb, probe, lines, dicts=[(built, 0)])
    try:
        parity.assert_matches(probe, res, want, label="q12")
        parity.assert_matches(build, built, [table], label="q12 build side")
    finally:
        res.free()
        built.free()
