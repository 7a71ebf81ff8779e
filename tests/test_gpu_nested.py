"""GPU parity of weld_nested_for (a `for` nested in a `for`, run by un-nesting) against the
CPU oracle, through the C ABI.

Tolerances: integer results bit-exact; an f64 result that is a sum over an inner range is
compared at 1e-9 relative to the correctly rounded sum (the order of the merges is free), on
data without cancellation; min / max bit-exact.
"""
import numpy as np
import pytest
import torch

from workloads import graphs
from workloads.ir import NestedProgram

pytestmark = pytest.mark.gpu

NP = {"i64": np.int64, "f64": np.float64}
TT = {"i32": torch.int32, "i64": torch.int64, "f64": torch.float64}


@pytest.fixture(scope="module")
def wb():
    from paper_1709_06416_amd import binding
    return binding


def _dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def _compare(prog, res, want, label):
    res.check()
    for b, spec in enumerate(prog.builders):
        tag = "%s builder %d" % (label, b)
        if spec["kind"] == "merger":
            got = res.merger(b)
            if spec["type"] == "f64" and spec.get("func") in ("add", "mul"):
                assert abs(float(got) - float(want[b])) <= 1e-9 * abs(float(want[b])), (tag, got, want[b])
            else:
                assert got == want[b], (tag, got, want[b])
        else:
            got = res.vec_host(b)
            assert len(got) == len(want[b]), tag
            if spec["type"] == "f64":
                bad = np.flatnonzero(~(np.abs(got - want[b]) <= 1e-9 * np.abs(want[b])) & ~(got == want[b]))
                assert bad.size == 0, (tag, bad[:5], got[bad[:5]], want[b][bad[:5]])
            else:
                assert np.array_equal(got, want[b]), tag


def _check(wb, prog, outer, inner, gather, label="", **kw):
    from oracle import interp
    want = interp.run_nested(prog, outer, inner, gather, sums="exact")
    res = wb.nested_for(prog, [_dev(c) for c in outer], [_dev(c) for c in inner], [_dev(g) for g in gather], **kw)
    try:
        _compare(prog.outer, res, want, label)
    finally:
        res.free()


def _graph(n, offsets="i64", **kw):
    rowptr, src, weight, outdeg = [t.numpy() for t in graphs.make_graph(n, offsets=offsets, **kw)]
    return rowptr, src, weight, outdeg


@pytest.mark.parametrize("offsets", ["i64", "i32"])
@pytest.mark.parametrize("n", [1, 700, 60_001])
def test_spmv(wb, n, offsets):
    rowptr, src, weight, _ = _graph(n, offsets)
    x = np.random.RandomState(n).uniform(0.5, 1.5, size=n)
    _check(wb, graphs.program_spmv(offsets), [rowptr[:-1].copy(), rowptr[1:].copy()], [src, weight], [x], label="spmv %d" % n)


@pytest.mark.parametrize("n", [5, 40_003])
def test_pagerank_iteration(wb, n):
    from oracle import interp
    rowptr, src, _, outdeg = _graph(n)
    rank = np.full(n, 1.0 / n)
    contrib = interp.run(graphs.program_contrib(), [rank, outdeg])[0]
    _check(wb, graphs.program_pagerank(n), [rowptr[:-1].copy(), rowptr[1:].copy()], [src], [contrib], label="pagerank %d" % n)


def test_two_pagerank_iterations_through_the_library(wb):
    """contrib (a fused map loop) and the nested loop, twice, all on the GPU; the oracle does the same."""
    from oracle import interp
    n = 30_011
    rowptr, src, _, outdeg = _graph(n)
    start, end = _dev(rowptr[:-1].copy()), _dev(rowptr[1:].copy())
    d_src, d_deg = _dev(src), _dev(outdeg)
    rank = torch.full((n,), 1.0 / n, dtype=torch.float64, device="cuda")
    want = np.full(n, 1.0 / n)
    for _ in range(2):
        r1 = wb.fused_for(graphs.program_contrib(), [rank, d_deg]).check()
        contrib = r1.vec(0)
        r2 = wb.nested_for(graphs.program_pagerank(n), [start, end], [d_src], [contrib]).check()
        rank = r2.vec(0)
        r1.free()
        r2.free()
        c = interp.run(graphs.program_contrib(), [want, outdeg])[0]
        want = interp.run_nested(graphs.program_pagerank(n), [rowptr[:-1], rowptr[1:]], [src], [c])[0]
    got = rank.cpu().numpy()
    assert np.all(np.abs(got - want) <= 1e-9 * np.abs(want))


def _random_nested(rnd, func, t, with_pred, n_outer, n_inner, empty_share=0.3):
    cuts = np.sort(rnd.randint(0, n_inner + 1, size=max(n_outer - 1, 0)))
    if empty_share > 0 and cuts.size:                    # runs of empty ranges: repeat the previous cut
        repeat = rnd.uniform(size=cuts.size) < empty_share
        cuts = np.maximum.accumulate(np.where(repeat, 0, cuts))
    if n_outer == 0:
        start = end = np.zeros(0, dtype=np.int64)
    else:
        start = np.concatenate([[0], cuts]).astype(np.int64)
        end = np.concatenate([cuts, [n_inner]]).astype(np.int64)
    scale = rnd.randint(-3, 4, size=n_outer).astype(np.int64)
    idx = rnd.randint(0, 1000, size=n_inner).astype(np.int32)
    if t == "i64":
        a = rnd.randint(-4, 5, size=n_inner).astype(np.int64)
        g = rnd.randint(-5, 6, size=1000).astype(np.int64)
    else:
        a = rnd.uniform(0.5, 2.0, size=n_inner)
        g = rnd.uniform(0.5, 2.0, size=1000)
    if func == "mul":                                    # products stay exact and finite
        a = np.where(rnd.uniform(size=n_inner) < 0.5, 1, -1).astype(NP[t])
        g = np.where(rnd.uniform(size=1000) < 0.5, 1, -1).astype(NP[t])
    p = NestedProgram(["i64", "i64", "i64"], 0, 1, ["i32", t], [t], t, func)
    q = p.inner
    v = q.bin("mul", q.col(1), q.lookup(0, q.col(0)))
    if t == "i64":
        v = q.bin("add", v, q.outer(2))                  # the current outer element, inside the inner loop
    pred = q.bin("ne", q.bin("mod", q.col(0), q.const("i32", 7)), q.const("i32", 3)) if with_pred else None
    q.merge(0, v, pred=pred)
    o = p.outer
    o.merge(o.vecbuilder(t), o.inner())
    o.merge(o.merger(t, "max" if func == "mul" else func), o.inner(), pred=o.bin("gt", o.col(2), o.const("i64", -2)))
    o.merge(o.vecbuilder("i64"), o.bin("add", o.index(), o.col(2)), pred=o.bin("lt", o.col(0), o.col(1)))
    return p, [start, end, scale], [idx, a], [g]


@pytest.mark.parametrize("with_pred", [False, True])
@pytest.mark.parametrize("t", ["i64", "f64"])
@pytest.mark.parametrize("func", ["add", "mul", "min", "max"])
def test_functions_predicates_and_outer_access(wb, func, t, with_pred):
    rnd = np.random.RandomState(17)
    p, outer, inner, gather = _random_nested(rnd, func, t, with_pred, n_outer=7_001, n_inner=150_003)
    _check(wb, p, outer, inner, gather, label="%s %s %s" % (func, t, with_pred))


@pytest.mark.parametrize("n_outer,n_inner", [(0, 0), (1, 0), (5, 0), (1, 1), (1, 70_000), (3, 9_000), (2_000, 2_047),
                                             (2_000, 2_048), (2_000, 2_049), (90_000, 30_001), (300_000, 5_000)])
def test_shapes(wb, n_outer, n_inner):
    """Empty inputs, one range spanning many tiles, tile-sized inputs with a ragged end, and
    many more outer than inner elements (more range boundaries in a tile than LDS stages)."""
    rnd = np.random.RandomState(n_outer + n_inner)
    p, outer, inner, gather = _random_nested(rnd, "add", "f64", False, n_outer, n_inner, empty_share=0.0)
    _check(wb, p, outer, inner, gather, label="shape %d %d" % (n_outer, n_inner))


def test_one_huge_range_among_small_ones(wb):
    rowptr, src, weight, _ = _graph(200_000)
    deg = np.diff(rowptr)
    assert deg.max() > 3 * 2048                                            # spans several tiles
    x = np.random.RandomState(1).uniform(0.5, 1.5, size=200_000)
    _check(wb, graphs.program_spmv(), [rowptr[:-1].copy(), rowptr[1:].copy()], [src, weight], [x], label="huge row")


def test_ranges_that_are_not_consecutive_are_rejected(wb):
    rowptr, src, weight, _ = _graph(5_000)
    x = np.ones(5_000)
    start, end = rowptr[:-1].copy(), rowptr[1:].copy()
    bad_end = end.copy()
    bad_end[100] -= 1 if bad_end[100] > start[100] else -1                # a gap / an overlap
    for s, e in ((start, bad_end), (start + 1, end + 1), (start, np.minimum(end, end[-1] - 5))):
        res = wb.nested_for(graphs.program_spmv(), [_dev(s), _dev(e)], [_dev(src), _dev(weight)], [_dev(x)])
        assert res.status() == wb.ERR_INVALID_ARG and "consecutive" in res.error()
        res.free()


def _column_sums(offsets="i64"):
    p = NestedProgram([offsets] * 3, 0, 1, ["f64"], [], "f64", "add", stride_col=2, ranges="any")
    p.inner.merge(0, p.inner.col(0))
    p.outer.merge(p.outer.vecbuilder("f64"), p.outer.inner())
    p.outer.merge(p.outer.merger("f64", "add"), p.outer.inner())
    return p


def test_strided_ranges_hand_worked_and_matrix_columns(wb):
    # the 3 x 4 matrix 0..11 stored row by row: column j is start = j, end = 12, stride = 4 (Sec. 3.2: a loop's
    # start, end and stride per vector); the sums are written out, not computed
    m = np.arange(12, dtype=np.float64)
    outer = [np.array(c, dtype=np.int64) for c in ([0, 1, 2, 3], [12, 12, 12, 12], [4, 4, 4, 4])]
    res = wb.nested_for(_column_sums(), [_dev(c) for c in outer], [_dev(m)], []).check()
    assert res.vec_host(0).tolist() == [12.0, 15.0, 18.0, 21.0] and float(res.merger(1)) == 66.0
    res.free()
    # overlapping, empty, gapped, stride past the end: elements [1,4,7], [2], [], [0,2,4,6,8], [5]
    outer = [np.array(c, dtype=np.int64) for c in ([1, 2, 6, 0, 5], [8, 3, 6, 9, 7], [3, 7, 2, 2, 100])]
    res = wb.nested_for(_column_sums(), [_dev(c) for c in outer], [_dev(m)], []).check()
    assert res.vec_host(0).tolist() == [12.0, 2.0, 0.0, 20.0, 5.0]
    res.free()
    # every column of a 700 x 1300 matrix (columns of 700 elements, each a 1300-element stride apart) and
    # every row (stride 1) in one call, against the oracle and against numpy's own axis sums
    rows, cols = 700, 1300
    a = np.random.RandomState(8).uniform(0.5, 1.5, size=(rows, cols))
    start = np.concatenate([np.arange(cols), np.arange(rows) * cols])
    end = np.concatenate([np.full(cols, rows * cols), (np.arange(rows) + 1) * cols])
    stride = np.concatenate([np.full(cols, cols), np.ones(rows, dtype=np.int64)])
    for offsets in ("i64", "i32"):
        dt = np.int64 if offsets == "i64" else np.int32
        outer = [start.astype(dt), end.astype(dt), stride.astype(dt)]
        _check(wb, _column_sums(offsets), outer, [a.reshape(-1)], [], label="matrix " + offsets)
        res = wb.nested_for(_column_sums(offsets), [_dev(c) for c in outer], [_dev(a.reshape(-1))], []).check()
        got = res.vec_host(0)
        res.free()
        assert np.allclose(got[:cols], a.sum(axis=0), rtol=1e-12) and np.allclose(got[cols:], a.sum(axis=1), rtol=1e-12)


@pytest.mark.parametrize("n_outer,n_inner,span", [(0, 0, 0), (1, 1, 1), (7, 0, 0), (5_000, 300, 40), (3, 500_000, 400_000),
                                                  (60_000, 100_000, 9), (400_000, 50, 0), (2_000, 70_000, 5_000)])
def test_any_ranges_shapes(wb, n_outer, n_inner, span):
    """Ranges drawn independently (overlaps, gaps, empty ranges, one range longer than many tiles, far more
    outer elements than positions so that a tile holds more boundaries than LDS stages), with and
    without a stride vector; `index` and the current outer element are visible in the inner body."""
    rnd = np.random.RandomState(n_outer * 7 + n_inner)
    for with_stride in (False, True):
        start = rnd.randint(0, max(n_inner, 1), size=n_outer).astype(np.int64)
        length = rnd.randint(0, span + 1, size=n_outer)
        stride = rnd.choice([1, 2, 5, 64, 999], size=n_outer).astype(np.int64)
        end = np.minimum(n_inner, start + length * (stride if with_stride else 1)).astype(np.int64)
        start = np.minimum(start, end)
        scale = rnd.randint(-3, 4, size=n_outer).astype(np.int64)
        a = rnd.randint(-4, 5, size=n_inner).astype(np.int64)
        cols = ["i64", "i64", "i64", "i64"] if with_stride else ["i64", "i64", "i64"]
        p = NestedProgram(cols, 0, 1, ["i64"], [], "i64", "add", stride_col=3 if with_stride else None, ranges="any")
        q = p.inner
        v = q.bin("add", q.bin("mul", q.col(0), q.outer(2)), q.bin("mod", q.index(), q.const("i64", 11)))
        q.merge(0, v, pred=q.bin("ne", q.col(0), q.const("i64", 3)))
        o = p.outer
        o.merge(o.vecbuilder("i64"), o.inner())
        o.merge(o.merger("i64", "max"), o.inner(), pred=o.bin("lt", o.col(0), o.col(1)))
        outer = [start, end, scale] + ([stride] if with_stride else [])
        _check(wb, p, outer, [a], [], label="any ranges %d %d stride %s" % (n_outer, n_inner, with_stride))


def test_invalid_ranges_fail_the_call(wb):
    m = _dev(np.arange(100, dtype=np.float64))
    for bad in (([0, -1], [5, 5], [1, 1]), ([0, 7], [5, 6], [1, 1]), ([0, 1], [5, 101], [1, 1]), ([0, 1], [5, 5], [1, 0])):
        outer = [_dev(np.array(c, dtype=np.int64)) for c in bad]
        with pytest.raises(wb.WeldError) as e:
            wb.nested_for(_column_sums(), outer, [m], [])
        assert e.value.status == wb.ERR_INVALID_ARG and "range" in str(e.value)
    q = NestedProgram(["i64", "i64", "i32"], 0, 1, ["f64"], [], "f64", "add", ranges="any")
    q.stride_col = 2                                                   # a stride vector of another type than start / end
    q.inner.merge(0, q.inner.col(0))
    q.outer.merge(q.outer.vecbuilder("f64"), q.outer.inner())
    st, text = wb.nested_validate(q)
    assert st == wb.ERR_TYPE, text


@pytest.mark.parametrize("group", range(3))
def test_random_nested_programs_over_any_ranges(wb, group):
    from workloads import random_programs
    for seed in range(3000 + 8 * group, 3008 + 8 * group):
        nested, outer, inner, gather = random_programs.make_nested(seed, any_ranges=True)
        label = "random nested program over any ranges, seed %d (%d outer, %d inner rows, %s %s, stride %s)" % (
            seed, len(outer[0]), len(inner[0]), nested.inner_type, nested.inner_func, nested.stride_col)
        print(label, flush=True)
        _check(wb, nested, outer, inner, gather, label=label)


def test_lookup_outside_its_vector_is_reported(wb):
    rowptr, src, weight, _ = _graph(5_000)
    x = np.ones(4_000)                                                     # shorter than the vertex count
    res = wb.nested_for(graphs.program_spmv(), [_dev(rowptr[:-1].copy()), _dev(rowptr[1:].copy())],
                        [_dev(src), _dev(weight)], [_dev(x)])
    assert res.status() == wb.ERR_INVALID_ARG and "lookup" in res.error()
    res.free()


def test_validation_errors(wb):
    p = graphs.program_spmv()
    p.inner.merges.append(dict(p.inner.merges[0]))
    st, text = wb.nested_validate(p)
    assert st == wb.ERR_LINEARITY, text
    q = NestedProgram(["i64", "i64"], 0, 1, ["i32"], ["f64"], "f64", "add")
    q.inner.merge(0, q.inner.un("cast", q.inner.col(0), to="f64"))
    q.outer.merge(q.outer.vecbuilder("i64"), q.outer.inner())          # f64 result into an i64 vecbuilder
    st, text = wb.nested_validate(q)
    assert st == wb.ERR_TYPE, text
    from workloads.ir import Program
    plain = Program(["i64"], gather=["f64"])
    plain.merge(plain.merger("f64", "add"), plain.lookup(0, plain.col(0)))
    st, text = wb.validate(plain)                                       # lookup outside a nested loop
    assert st == wb.ERR_UNSUPPORTED, text


@pytest.mark.parametrize("group", range(5))
def test_random_nested_programs_match_the_oracle(wb, group):
    """Differential test: seeded random nested loops (workloads/random_programs.py): random inner
    bodies over random column types that read the current outer element and look values up in
    gather vectors, folded per inner range (empty, short and long ranges mixed; i32 or i64
    offsets), and random outer bodies over the results."""
    from workloads import random_programs
    for seed in range(2000 + 8 * group, 2008 + 8 * group):
        nested, outer, inner, gather = random_programs.make_nested(seed)
        label = "random nested program, seed %d (%d outer, %d inner rows, %s %s)" % (
            seed, len(outer[0]), len(inner[0]), nested.inner_type, nested.inner_func)
        print(label, flush=True)
        _check(wb, nested, outer, inner, gather, label=label)
