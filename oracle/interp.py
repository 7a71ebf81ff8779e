"""CPU oracle: operator-at-a-time evaluation of one `for` loop over zipped columns.

TEST INFRASTRUCTURE ONLY.  This file is the slow, plain statement of what the
fused loop must return.  It is imported by the tests, by the smoke check and by
the benchmark's cpu_baseline leg, never by the product library, and it shares
no code with the HIP path.

What it follows (paper, Sec. 3.2 and Table 1; Sec. 3.3 for the macros):
  * `for(vectors, builders, func)` applies func to every index i and the
    struct of the i-th elements of the zipped vectors.
  * each expression of the body is evaluated here for ALL rows before the next
    one starts, producing a full intermediate column: this is the unfused
    `map` / `filter` / `reduce` form which the fused loop must equal
    (Listing "combined program" == Listing "after loop fusion", Sec. 4.5).
  * `if (p) merge(b, v) else b`  ==  merge of the rows where column p is true.
  * merger[T,func,id]: fold of the merged values with func, starting at id.
  * vecbuilder[T]: the merged values appended, i.e. the selected subsequence
    in index order (all three printed examples keep index order).
  * dictmerger[K,V,func]: first merge of a key stores the value, later ones
    combine with func, field by field when V is a struct.
  * vecmerger[T,func] (Table 1, Sec. 7.7): starts from a copy of an input vector and
    merges each {index, value} pair into the cell at that index with func.
  * groupbuilder[K,V] (Table 1): groups the merged {key, value} pairs by key; the result
    maps each key to the vector of its values (here: in index order, the order a
    sequential loop appends them in; a parallel loop may return any order inside a group).

  * nested loops (Sec. 3.2: loops nest arbitrarily; a loop may take a start and an end
    index per vector): `run_nested` evaluates the inner body over every (outer element,
    inner element) pair, folds each outer element's pairs with the inner merger, and
    runs the outer body over the outer elements with those results as a column.

Readings where the paper is silent: integers wrap modulo 2^w; integer div/mod
truncate toward zero (C), a zero divisor gives quotient 0 and remainder 0, the most
negative value over -1 wraps to itself (remainder 0); min / max (operator and merge
function) of anything with a NaN is NaN; a cast of f64 to an integer truncates, NaN gives
0 and values beyond the 64-bit range its nearest end (narrower types then wrap); no
implicit promotion (a `cast` op is required); f64
is IEEE round-to-nearest with one rounding per operator and no contraction;
dictionary entries are returned sorted by key (the paper leaves them
unordered, so callers compare sorted).

Parity pins live in tests/test_oracle_pins.py (paper-printed results, closed
forms, brute force against oracle/rowwise.py, library routines, exact sums), in
tests/test_oracle_operator_pins.py (every operator of the expression language against
hand-worked tables, and every expression column of seeded random programs against the
per-row loop) and, for
nested loops, tests/test_oracle_nested_pins.py (a hand-worked example, scipy's sparse
product, the literal nested loops, PageRank fixed points and rank conservation).
Black-Scholes prices have no printed value in the paper: they are pinned by
put-call parity, bounds and a decimal-arithmetic evaluation of the formula;
agreement of erf/exp/log with higher precision is checked on samples only.
"""
import math

import numpy as np
from scipy import special as _special

NP_TYPE = {"bool": np.bool_, "i8": np.int8, "i32": np.int32, "i64": np.int64,
           "f64": np.float64}
INT_TYPES = ("i8", "i32", "i64")

_COMPARE = {"lt": np.less, "le": np.less_equal, "gt": np.greater,
            "ge": np.greater_equal, "eq": np.equal, "ne": np.not_equal}


def identity(func, t):
    """Identity element of a merger function for type t (Sec. 3.2: merger[T,func,id])."""
    dt = NP_TYPE[t]
    if func == "add":
        return dt(0)
    if func == "mul":
        return dt(1)
    if t == "f64":
        return dt(np.inf) if func == "min" else dt(-np.inf)
    info = np.iinfo(dt)
    return dt(info.max) if func == "min" else dt(info.min)


def _trunc_div(a, b):
    """Integer quotient rounded toward zero, exact in the operand type.  Where the paper is
    silent: a zero divisor gives quotient 0; the most negative value over -1 wraps to itself."""
    safe = np.where(b == 0, 1, b)
    r = np.fmod(a, safe)
    q = np.where(safe == -1, np.negative(a), (a - r) // np.where(safe == -1, 1, safe))   # -a wraps for the most negative a
    return np.where(b == 0, 0, q).astype(a.dtype)


def _trunc_mod(a, b):
    """Integer remainder with the sign of the dividend (C); 0 for a zero divisor and for -1."""
    safe = np.where((b == 0) | (b == -1), 1, b)
    return np.where((b == 0) | (b == -1), 0, np.fmod(a, safe)).astype(a.dtype)


def _minmax(code, a, b):
    """min / max; a NaN operand gives NaN (numpy's minimum / maximum do that for floats)."""
    return np.minimum(a, b) if code == "min" else np.maximum(a, b)


def _f64_to_i64(x):
    """Truncation toward zero; where the paper is silent: NaN gives 0, values beyond the 64-bit range
    the nearest end of it."""
    t = np.trunc(x)
    inside = (t >= -9.223372036854775808e18) & (t < 9.223372036854775808e18)
    out = np.where(inside, t, 0.0).astype(np.int64)
    out = np.where(t >= 9.223372036854775808e18, np.iinfo(np.int64).max, out)
    out = np.where(t < -9.223372036854775808e18, np.iinfo(np.int64).min, out)
    return out


def _probe(table, key_cols):
    """Position of each probed key struct in a dictionary result `table` = (key columns, value
    columns), -1 where the key is absent (a hash join's probe, written with a Python dict)."""
    index = {key: pos for pos, key in enumerate(zip(*[c.tolist() for c in table[0]]))}
    n = len(key_cols[0]) if key_cols else 0
    probe = zip(*[c.tolist() for c in key_cols])
    return np.fromiter((index.get(key, -1) for key in probe), dtype=np.int64, count=n)


def scalar_columns(program):
    """Entries of the column list that hold one element: scalars defined outside the loop."""
    return {op[2] for op in program.ops if op[0] == "scalar"}


def row_count(program, columns):
    """Rows of the loop: the length of its zipped vectors (scalars from outside do not count)."""
    scalars = scalar_columns(program)
    lengths = [len(c) for k, c in enumerate(columns) if k not in scalars]
    return lengths[0] if lengths else 0


def eval_columns(program, columns, n=None, gather=None, outer=None, inner=None, dicts=None, index=None):
    """Materialise every body expression as a full column (one operator at a time).

    gather / outer / inner give meaning to the operators of nested loops: the vectors
    `lookup` reads, the outer vectors already expanded to one element per row of this
    (inner) loop, and the column of inner-loop results seen by an outer body; index: the
    position of each row's element in the inner vectors (an inner loop over ranges).
    """
    scalars = scalar_columns(program)
    if n is None:
        n = row_count(program, columns)
    for k, c in enumerate(columns):
        assert c.dtype == NP_TYPE[program.columns[k]], (k, c.dtype)
        assert len(c) == (1 if k in scalars else n)
    val = []
    with np.errstate(all="ignore"):
        for op in program.ops:
            code, t = op[0], op[1]
            dt = NP_TYPE[t]
            a = ([val[j] for j in op[2:]]
                 if code not in ("col", "scalar", "const", "index", "lookup", "outer", "inner", "keyexists", "dictlookup")
                 else None)
            if code == "col":
                out = columns[op[2]]
            elif code == "scalar":                  # a value from outside the loop: the same for every row
                out = np.full(n, columns[op[2]][0], dtype=dt)
            elif code == "lookup":
                vec, idx = gather[op[2]], val[op[3]].astype(np.int64)
                assert idx.size == 0 or (idx.min() >= 0 and idx.max() < len(vec)), "lookup out of range"
                out = vec[idx]
            elif code == "keyexists":
                out = _probe(dicts[op[2]], [val[j] for j in op[3:]]) >= 0
            elif code == "dictlookup":
                pos = _probe(dicts[op[2]], [val[j] for j in op[4:]])
                field = dicts[op[2]][1][op[3]]
                out = np.where(pos >= 0, field[np.maximum(pos, 0)] if len(field) else dt(0), dt(0)).astype(dt)
            elif code == "outer":
                out = outer[op[2]]
            elif code == "inner":
                out = inner
            elif code == "const":
                out = np.full(n, op[2], dtype=dt)
            elif code == "index":
                out = np.arange(n, dtype=np.int64) if index is None else index
            elif code == "neg":
                out = np.negative(a[0])
            elif code == "not":
                out = np.logical_not(a[0])
            elif code == "cast":
                src = a[0]
                if src.dtype == np.float64 and t in INT_TYPES:
                    out = _f64_to_i64(src).astype(dt)
                else:
                    out = src.astype(dt)
            elif code == "exp":
                out = np.exp(a[0])
            elif code == "log":
                out = np.log(a[0])
            elif code == "sqrt":
                out = np.sqrt(a[0])
            elif code == "erf":
                out = _special.erf(a[0])
            elif code == "add":
                out = np.add(a[0], a[1])
            elif code == "sub":
                out = np.subtract(a[0], a[1])
            elif code == "mul":
                out = np.multiply(a[0], a[1])
            elif code == "div":
                out = np.divide(a[0], a[1]) if t == "f64" else _trunc_div(a[0], a[1])
            elif code == "mod":
                out = np.fmod(a[0], a[1]) if t == "f64" else _trunc_mod(a[0], a[1])
            elif code in ("min", "max"):
                out = _minmax(code, a[0], a[1])
            elif code in _COMPARE:
                assert a[0].dtype == a[1].dtype, "compare needs equal types"
                out = _COMPARE[code](a[0], a[1])
            elif code == "and":
                out = np.logical_and(a[0], a[1])
            elif code == "or":
                out = np.logical_or(a[0], a[1])
            elif code == "select":
                out = np.where(a[0], a[1], a[2])
            else:
                raise ValueError("unknown op " + code)
            out = np.asarray(out)
            assert out.dtype == dt, (code, t, out.dtype)
            val.append(out)
    return val


def exact_sum(v):
    """The real-number sum of the doubles in v, rounded once to f64.

    math.fsum is exactly rounded.  For very long inputs an extended-precision
    (x87 80-bit) pairwise sum is used instead; its error, about log2(n) * 2^-64
    relative to sum|v|, is far below one f64 rounding for the positive data used
    here (pinned against math.fsum in the tests).
    """
    if v.size <= 20_000_000:
        return np.float64(math.fsum(v.tolist() if v.size < 1_000_000 else v))
    return np.float64(np.sum(v, dtype=np.longdouble))


def _fold(func, t, v, sums):
    """merger: acc = func(acc, v[i]) over the merged values in index order."""
    ident = identity(func, t)
    if v.size == 0:
        return ident
    with np.errstate(all="ignore"):
        if func == "add":
            if t == "f64":
                if sums == "exact":
                    return exact_sum(v)
                return np.float64(np.cumsum(v)[-1])
            return np.add.reduce(v, dtype=v.dtype)
        if func == "mul":
            return np.multiply.accumulate(v, dtype=v.dtype)[-1]
        if func == "min":
            return np.minimum.reduce(v)
        return np.maximum.reduce(v)


_REDUCEAT = {"add": np.add, "mul": np.multiply, "min": np.minimum, "max": np.maximum}


def _group(func, key_cols, val_cols, val_types, sums):
    """dictmerger: combine values of equal keys; entries returned sorted by key."""
    m = len(key_cols[0])
    if m == 0:
        return ([k[:0] for k in key_cols], [v[:0] for v in val_cols])
    order = np.lexsort(tuple(reversed(key_cols)))          # stable: index order within a key
    ks = [k[order] for k in key_cols]
    change = np.zeros(m, dtype=bool)
    change[0] = True
    for k in ks:
        change[1:] |= k[1:] != k[:-1]
    starts = np.flatnonzero(change)
    ends = np.append(starts[1:], m)
    out_keys = [k[starts] for k in ks]
    out_vals = []
    with np.errstate(all="ignore"):
        for v, t in zip(val_cols, val_types):
            vs = v[order]
            if func == "add" and t == "f64":
                if sums == "exact":
                    out_vals.append(np.array([exact_sum(vs[s:e]) for s, e in zip(starts, ends)],
                                             dtype=np.float64))
                else:
                    out_vals.append(np.array([np.cumsum(vs[s:e])[-1] for s, e in zip(starts, ends)],
                                             dtype=np.float64))
            else:
                out_vals.append(_REDUCEAT[func].reduceat(vs, starts, dtype=v.dtype))
    return (out_keys, out_vals)


_AT = {"add": np.add, "mul": np.multiply, "min": np.minimum, "max": np.maximum}


def _groups(key_cols, v):
    """groupbuilder: (key columns of the distinct keys sorted by key, offsets, values): the
    values of key g are values[offsets[g]:offsets[g+1]], in index order."""
    m = len(v)
    if m == 0:
        return ([k[:0] for k in key_cols], np.zeros(1, dtype=np.int64), v[:0].copy())
    order = np.lexsort(tuple(reversed(key_cols)))          # stable: index order within a key
    ks = [k[order] for k in key_cols]
    change = np.zeros(m, dtype=bool)
    change[0] = True
    for k in ks:
        change[1:] |= k[1:] != k[:-1]
    starts = np.flatnonzero(change)
    return ([k[starts] for k in ks], np.append(starts, m).astype(np.int64), v[order].copy())


def _vecmerge(spec, init, idx, v):
    """vecmerger: out = copy(init); out[idx[j]] = func(out[idx[j]], v[j]) for j in index order."""
    dt = NP_TYPE[spec["type"]]
    out = (np.full(spec["length"], identity(spec["func"], spec["type"]), dtype=dt) if init is None
           else np.array(init, dtype=dt, copy=True))
    assert out.shape == (spec["length"],)
    assert idx.size == 0 or (idx.min() >= 0 and idx.max() < spec["length"]), "index out of range"
    with np.errstate(all="ignore"):
        _AT[spec["func"]].at(out, idx, v)          # unbuffered: applied pair by pair, in order
    return out


def run(program, columns, sums="exact", inits=None, dicts=None):
    """Evaluate the loop; returns one result per builder, in builder order.

    merger      -> numpy scalar of its type
    vecbuilder  -> 1-d numpy array
    dictmerger  -> (list of key columns, list of value columns), sorted by key

    vecmerger   -> 1-d numpy array (inits: {builder index: initial vector})
    groupbuilder-> (list of key columns sorted by key, offsets, values)

    dicts: the dictionaries `keyexists` / `dictlookup` probe, each the (key columns, value
    columns) result of an earlier `run` (a hash join's build side).

    sums = "exact": an f64 `add` returns the correctly rounded real sum (any
    merge order is legal, Sec. 3.2, so this is the value every order
    approximates);  sums = "fold": the literal left-to-right f64 fold.
    """
    val = eval_columns(program, columns, dicts=dicts)
    n = row_count(program, columns)
    return _results(program, val, n, sums, inits)


def _results(program, val, n, sums, inits):
    """The builders' results, given every body expression as a column."""
    results = [None] * len(program.builders)
    merged = set()
    for m in program.merges:
        b = m["builder"]
        assert b not in merged, "a builder may be merged once per control path"
        merged.add(b)
        spec = program.builders[b]
        mask = val[m["pred"]] if m["pred"] is not None else np.ones(n, dtype=bool)
        assert mask.dtype == np.bool_
        if spec["kind"] == "merger":
            v = val[m["vals"][0]][mask]
            assert v.dtype == NP_TYPE[spec["type"]]
            results[b] = _fold(spec["func"], spec["type"], v, sums)
        elif spec["kind"] == "vecbuilder":
            v = val[m["vals"][0]]
            assert v.dtype == NP_TYPE[spec["type"]]
            results[b] = v[mask].copy()
        elif spec["kind"] == "dictmerger":
            kc = [val[k][mask] for k in m["keys"]]
            vc = [val[v][mask] for v in m["vals"]]
            for c, t in zip(kc, spec["key_types"]):
                assert c.dtype == NP_TYPE[t]
            for c, t in zip(vc, spec["val_types"]):
                assert c.dtype == NP_TYPE[t]
            results[b] = _group(spec["func"], kc, vc, spec["val_types"], sums)
        elif spec["kind"] == "vecmerger":
            idx = val[m["keys"][0]][mask]
            v = val[m["vals"][0]][mask]
            assert idx.dtype == np.int64 and v.dtype == NP_TYPE[spec["type"]]
            results[b] = _vecmerge(spec, (inits or {}).get(b), idx, v)
        elif spec["kind"] == "groupbuilder":
            kc = [val[k][mask] for k in m["keys"]]
            v = val[m["vals"][0]][mask]
            for c, t in zip(kc, spec["key_types"]):
                assert c.dtype == NP_TYPE[t]
            assert v.dtype == NP_TYPE[spec["type"]]
            results[b] = _groups(kc, v)
        else:
            raise ValueError(spec["kind"])
    for b, spec in enumerate(program.builders):
        if results[b] is None:                      # never merged: result(b) of a fresh builder
            if spec["kind"] == "merger":
                results[b] = identity(spec["func"], spec["type"])
            elif spec["kind"] == "vecbuilder":
                results[b] = np.zeros(0, dtype=NP_TYPE[spec["type"]])
            elif spec["kind"] == "vecmerger":
                results[b] = _vecmerge(spec, (inits or {}).get(b), np.zeros(0, np.int64),
                                       np.zeros(0, NP_TYPE[spec["type"]]))
            elif spec["kind"] == "groupbuilder":
                results[b] = _groups([np.zeros(0, NP_TYPE[t]) for t in spec["key_types"]],
                                     np.zeros(0, NP_TYPE[spec["type"]]))
            else:
                results[b] = ([np.zeros(0, NP_TYPE[t]) for t in spec["key_types"]],
                              [np.zeros(0, NP_TYPE[t]) for t in spec["val_types"]])
    return results


def run_nested(nested, outer_columns, inner_columns, gather, sums="exact"):
    """A `for` nested in a `for` (Sec. 3.2: loops nest arbitrarily; a loop takes an
    optional start and end index per vector), evaluated one operator at a time:

      1. every (outer element i, inner element j = start[i], start[i] + stride[i], ... below
         end[i]) pair becomes one row (stride 1 unless the loop names a stride vector): the
         inner body is evaluated over all pairs, `outer` reading element i of an outer vector,
         `col` element j of an inner vector and `index` being j;
      2. the pairs of one outer element are folded with the inner merger's function
         (f64 sums: the correctly rounded real sum when sums == "exact"): one result per
         outer element, the identity for an empty range;
      3. the outer body is the ordinary loop of `run` over the outer elements, with that
         column of results as the value of `inner`.

    Ranges may overlap or leave gaps: nothing here assumes they are consecutive.
    Returns one result per builder of the outer program, like `run`.
    """
    n_outer = len(outer_columns[0]) if outer_columns else 0
    start = outer_columns[nested.start_col].astype(np.int64)
    end = outer_columns[nested.end_col].astype(np.int64)
    n_inner = len(inner_columns[0]) if inner_columns else None
    assert np.all(start <= end) and (n_outer == 0 or start.min() >= 0)
    if n_inner is not None and n_outer:
        assert end.max() <= n_inner
    stride_col = getattr(nested, "stride_col", None)
    stride = (outer_columns[stride_col].astype(np.int64) if stride_col is not None
              else np.ones(n_outer, dtype=np.int64))
    assert np.all(stride >= 1)
    length = (end - start + stride - 1) // stride                    # elements start, start + stride, ... < end
    seg = np.repeat(np.arange(n_outer, dtype=np.int64), length)      # outer element of each pair
    first = np.cumsum(length) - length                               # pairs before each outer element
    step = np.arange(int(length.sum()), dtype=np.int64) - np.repeat(first, length)
    j = np.repeat(start, length) + step * np.repeat(stride, length)
    prog = nested.inner
    val = eval_columns(prog, [c[j] for c in inner_columns], n=len(j), gather=gather,
                       outer=[c[seg] for c in outer_columns], index=j)
    assert len(prog.merges) == 1 and prog.merges[0]["builder"] == 0
    m = prog.merges[0]
    mask = val[m["pred"]] if m["pred"] is not None else np.ones(len(j), dtype=bool)
    v = val[m["vals"][0]]
    assert v.dtype == NP_TYPE[nested.inner_type]
    r = np.empty(n_outer, dtype=NP_TYPE[nested.inner_type])
    bounds = np.append(first, len(j))
    for i in range(n_outer):
        lo, hi = bounds[i], bounds[i + 1]
        r[i] = _fold(nested.inner_func, nested.inner_type, v[lo:hi][mask[lo:hi]], sums)
    # step 3: the outer loop, `inner` bound to r
    outer_prog = nested.outer
    oval = eval_columns(outer_prog, outer_columns, n=n_outer, inner=r)
    return _results(outer_prog, oval, n_outer, sums, None)
