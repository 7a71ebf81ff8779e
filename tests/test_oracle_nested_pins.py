"""Pins for the nested-loop part of the CPU oracle (oracle.interp.run_nested and
oracle.rowwise.run_nested): checked against things other than themselves.

  * a three-row example worked by hand
  * the sparse matrix-vector product of a library (scipy.sparse) and a dense matmul
  * the literal nested loops (pure Python) against the operator-at-a-time form on small
    random inputs: empty ranges, predicates, every merger function, ranges that overlap
  * closed forms of PageRank: the uniform vector is a fixed point on a cycle and on a
    complete graph; one iteration keeps total rank when no vertex lacks out-edges
No GPU is needed for any of these.
"""
import numpy as np
import pytest
import scipy.sparse as sp

from oracle import interp, rowwise
from workloads import graphs
from workloads.ir import NestedProgram


def _np(t):
    return t.numpy() if hasattr(t, "numpy") else np.asarray(t)


def test_hand_worked_example():
    # rows: [0,2) -> 2*x[1] + 3*x[0] = 2*10 + 3*1 = 23 ; [2,2) empty -> 0 ; [2,5) -> 1*x[2] + 1*x[2] + 4*x[1] = 100+100+40
    rowptr = np.array([0, 2, 2, 5], dtype=np.int64)
    col = np.array([1, 0, 2, 2, 1], dtype=np.int32)
    w = np.array([2.0, 3.0, 1.0, 1.0, 4.0])
    x = np.array([1.0, 10.0, 100.0])
    p = graphs.program_spmv()
    for run in (lambda: interp.run_nested(p, [rowptr[:-1], rowptr[1:]], [col, w], [x]),
                lambda: rowwise.run_nested(p, [rowptr[:-1].tolist(), rowptr[1:].tolist()], [col.tolist(), w.tolist()], [x.tolist()])):
        y = run()[0]
        assert list(y) == [23.0, 0.0, 240.0]


@pytest.mark.parametrize("offsets", ["i64", "i32"])
def test_spmv_against_scipy_and_dense(offsets):
    rowptr, src, weight, _ = [_np(t) for t in graphs.make_graph(3000, offsets=offsets)]
    n = len(rowptr) - 1
    x = np.random.RandomState(3).uniform(-1, 1, size=n)
    y = interp.run_nested(graphs.program_spmv(offsets), [rowptr[:-1], rowptr[1:]], [src, weight], [x])[0]
    a = sp.csr_matrix((weight, src.astype(np.int64), rowptr.astype(np.int64)), shape=(n, n))
    want = a @ x
    assert np.allclose(y, want, rtol=1e-12, atol=1e-12)
    dense = a[:200].toarray() @ x
    assert np.allclose(y[:200], dense, rtol=1e-12, atol=1e-12)


def _random_nested(rnd, func, t, with_pred, overlapping):
    n_outer, n_inner = 23, 90
    if overlapping:
        start = rnd.randint(0, n_inner, size=n_outer)
        end = np.minimum(n_inner, start + rnd.randint(0, 9, size=n_outer))
    else:
        cuts = np.sort(rnd.randint(0, n_inner + 1, size=n_outer - 1))
        start = np.concatenate([[0], cuts])
        end = np.concatenate([cuts, [n_inner]])
    scale = rnd.randint(-3, 4, size=n_outer).astype(np.int64)
    idx = rnd.randint(0, 40, size=n_inner).astype(np.int32)
    a = (rnd.randint(-4, 5, size=n_inner).astype(np.int64) if t == "i64" else rnd.uniform(-2, 2, size=n_inner))
    g = (rnd.randint(-5, 6, size=40).astype(np.int64) if t == "i64" else rnd.uniform(-2, 2, size=40))
    if func == "mul":          # keep products exact and far from overflow
        a = np.sign(a) + (a == 0)
        g = np.sign(g) + (g == 0)
        a, g = a.astype(NP[t]), g.astype(NP[t])
    p = NestedProgram(["i64", "i64", "i64"], 0, 1, ["i32", t], [t], t, func)
    q = p.inner
    v = q.bin("mul", q.col(1), q.lookup(0, q.col(0)))
    if t == "i64":
        v = q.bin("add", v, q.outer(2))                       # the outer element is visible inside
    pred = q.bin("ne", q.col(0), q.const("i32", 7)) if with_pred else None
    q.merge(0, v, pred=pred)
    o = p.outer
    o.merge(o.vecbuilder(t), o.inner())
    o.merge(o.merger(t, func), o.inner(), pred=o.bin("gt", o.col(2), o.const("i64", -2)))
    return p, [start.astype(np.int64), end.astype(np.int64), scale], [idx, a], [g]


NP = {"i64": np.int64, "f64": np.float64}


@pytest.mark.parametrize("overlapping", [False, True])
@pytest.mark.parametrize("with_pred", [False, True])
@pytest.mark.parametrize("t", ["i64", "f64"])
@pytest.mark.parametrize("func", ["add", "mul", "min", "max"])
def test_operator_at_a_time_equals_literal_nested_loops(func, t, with_pred, overlapping):
    rnd = np.random.RandomState(11)
    p, outer, inner, gather = _random_nested(rnd, func, t, with_pred, overlapping)
    got = interp.run_nested(p, outer, inner, gather, sums="fold")
    want = rowwise.run_nested(p, [c.tolist() for c in outer], [c.tolist() for c in inner], [g.tolist() for g in gather])
    if t == "i64":
        assert got[0].tolist() == want[0]
        assert int(got[1]) == want[1]
    else:
        assert np.allclose(got[0], np.array(want[0]), rtol=1e-13, atol=0.0, equal_nan=True)
        assert float(got[1]) == pytest.approx(want[1], rel=1e-13) or (np.isinf(got[1]) and np.isinf(want[1]))


def _column_program(with_index=False):
    """for every column j of a row-major matrix: sum of the column (Sec. 3.2: a loop takes a start, an end
    and a stride per vector, which is how the paper iterates over matrices) - and, with_index, the sum of
    the positions the inner loop visited."""
    p = NestedProgram(["i64", "i64", "i64"], 0, 1, ["i64"], [], "i64", "add", stride_col=2, ranges="any")
    q = p.inner
    q.merge(0, q.index() if with_index else q.col(0))
    p.outer.merge(p.outer.vecbuilder("i64"), p.outer.inner())
    return p


def test_strided_ranges_hand_worked_matrix_columns():
    # the 3 x 4 matrix [[0,1,2,3],[4,5,6,7],[8,9,10,11]] stored row by row; column j is start = j,
    # end = 12, stride = 4: sums 0+4+8, 1+5+9, 2+6+10, 3+7+11
    m = list(range(12))
    start, end, stride = [0, 1, 2, 3], [12, 12, 12, 12], [4, 4, 4, 4]
    want = [12, 15, 18, 21]
    p = _column_program()
    assert interp.run_nested(p, [np.array(c, dtype=np.int64) for c in (start, end, stride)], [np.array(m, dtype=np.int64)], [])[0].tolist() == want
    assert rowwise.run_nested(p, [start, end, stride], [m], [])[0] == want
    # ends that are not start + k * stride, ranges that overlap, an empty one, a gap (elements 9..11 unread),
    # stride larger than the range: elements [1,4,7], [2], [], [0,2,4,6,8], [5]
    start, end, stride = [1, 2, 6, 0, 5], [8, 3, 6, 9, 7], [3, 7, 2, 2, 100]
    want = [1 + 4 + 7, 2, 0, 0 + 2 + 4 + 6 + 8, 5]
    assert interp.run_nested(p, [np.array(c, dtype=np.int64) for c in (start, end, stride)], [np.array(m, dtype=np.int64)], [])[0].tolist() == want
    assert rowwise.run_nested(p, [start, end, stride], [m], [])[0] == want
    # `index` in the inner body is the position in the inner vector, not the iteration count
    pi = _column_program(with_index=True)
    vals = [100 + v for v in m]
    assert interp.run_nested(pi, [np.array(c, dtype=np.int64) for c in (start, end, stride)], [np.array(vals, dtype=np.int64)], [])[0].tolist() == want
    assert rowwise.run_nested(pi, [start, end, stride], [vals], [])[0] == want


@pytest.mark.parametrize("seed", range(12))
def test_strided_ranges_operator_at_a_time_equals_literal_loops(seed):
    rnd = np.random.RandomState(100 + seed)
    n_outer, n_inner = 31, 200
    t = "i64" if seed % 2 else "f64"
    func = ["add", "min", "max", "add"][seed % 4]
    start = rnd.randint(0, n_inner, size=n_outer)
    end = np.minimum(n_inner, start + rnd.randint(0 if func == "add" else 1, 60, size=n_outer))
    stride = rnd.choice([1, 2, 3, 7, 50], size=n_outer)
    a = rnd.randint(-9, 10, size=n_inner).astype(np.int64) if t == "i64" else np.round(rnd.uniform(-2, 2, size=n_inner), 3)
    p = NestedProgram(["i64", "i64", "i64"], 0, 1, [t], [], t, func, stride_col=2, ranges="any")
    q = p.inner
    v = q.col(0)
    if t == "i64":
        v = q.bin("add", v, q.bin("mul", q.index(), q.outer(2)))          # position and outer element both visible
    q.merge(0, v, pred=q.bin("ne", q.bin("mod", q.index(), q.const("i64", 5)), q.const("i64", 0)) if seed % 3 == 0 else None)
    p.outer.merge(p.outer.vecbuilder(t), p.outer.inner())
    outer = [start.astype(np.int64), end.astype(np.int64), stride.astype(np.int64)]
    got = interp.run_nested(p, outer, [a], [], sums="fold")[0]
    want = rowwise.run_nested(p, [c.tolist() for c in outer], [a.tolist()], [])[0]
    if t == "i64":
        assert got.tolist() == want
    else:
        assert np.array_equal(got, np.array(want))          # same fold order on both sides: identical doubles
    # brute force per range with numpy slicing (a library routine): start:end:stride
    if seed % 3 != 0 and t == "f64":
        red = {"add": np.sum, "min": np.min, "max": np.max}[func]
        for i in range(n_outer):
            sl = a[start[i]:end[i]:stride[i]]
            assert (len(sl) == 0 and func == "add" and got[i] == 0.0) or np.isclose(got[i], red(sl), rtol=1e-12)


def _pagerank_once(rowptr, src, outdeg, rank):
    contrib = interp.run(graphs.program_contrib(), [rank, outdeg])[0]
    new_rank, total = interp.run_nested(graphs.program_pagerank(len(rank)), [rowptr[:-1], rowptr[1:]], [src], [contrib])
    return new_rank, float(total)


def test_pagerank_uniform_is_a_fixed_point_on_a_cycle_and_a_complete_graph():
    n = 50
    rank = np.full(n, 1.0 / n)
    # cycle: the one edge into i comes from i - 1
    rowptr = np.arange(n + 1, dtype=np.int64)
    src = ((np.arange(n) - 1) % n).astype(np.int32)
    new_rank, total = _pagerank_once(rowptr, src, np.ones(n, dtype=np.int64), rank)
    assert np.allclose(new_rank, rank, rtol=1e-14) and total == pytest.approx(1.0, rel=1e-14)
    # complete graph without self loops
    rowptr = np.arange(n + 1, dtype=np.int64) * (n - 1)
    src = np.concatenate([[j for j in range(n) if j != i] for i in range(n)]).astype(np.int32)
    new_rank, total = _pagerank_once(rowptr, src, np.full(n, n - 1, dtype=np.int64), rank)
    assert np.allclose(new_rank, rank, rtol=1e-14) and total == pytest.approx(1.0, rel=1e-14)


def test_pagerank_keeps_total_rank_without_dangling_vertices_and_matches_matrix_form():
    rowptr, src, _, outdeg = [_np(t) for t in graphs.make_graph(2000)]
    n = len(rowptr) - 1
    rnd = np.random.RandomState(5)
    rank = rnd.uniform(0.5, 1.5, size=n)
    rank /= rank.sum()
    new_rank, total = _pagerank_once(rowptr, src, outdeg, rank)
    # matrix form: d * A D^-1 rank + (1 - d) / n with A[i, j] = number of edges j -> i
    a = sp.csr_matrix((np.ones(len(src)), src.astype(np.int64), rowptr), shape=(n, n))
    inv = np.where(outdeg > 0, 1.0 / np.maximum(outdeg, 1), 0.0)
    want = graphs.DAMPING * (a @ (rank * inv)) + (1.0 - graphs.DAMPING) / n
    assert np.allclose(new_rank, want, rtol=1e-12)
    assert total == pytest.approx(float(np.sum(want)), rel=1e-12)
    # every vertex that has out-edges hands all of its rank on; the others' rank is dropped
    kept = rank[outdeg > 0].sum()
    assert total == pytest.approx(graphs.DAMPING * kept + (1.0 - graphs.DAMPING), rel=1e-12)


def test_graph_generator_shape_and_reproducibility():
    rowptr, src, weight, outdeg = [_np(t) for t in graphs.make_graph(50_000)]
    deg = np.diff(rowptr)
    assert rowptr[0] == 0 and np.all(deg >= 0) and rowptr[-1] == len(src) == len(weight)
    assert 0.2 < np.mean(deg == 0) < 0.3 and 9 < deg.mean() < 14 and deg.max() > 1000
    assert src.min() >= 0 and src.max() < 50_000 and outdeg.sum() == len(src)
    again = [_np(t) for t in graphs.make_graph(50_000)]
    assert all(np.array_equal(a, b) for a, b in zip((rowptr, src, weight, outdeg), again))
