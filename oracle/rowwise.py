"""CPU oracle, second form: the literal per-row `for` loop (pure Python).

TEST INFRASTRUCTURE ONLY; for tiny inputs.  Shares no code with the HIP path
and none with oracle/interp.py either: integers are Python ints wrapped by
hand, doubles are Python floats, math functions come from `math` (libm).

Follows Sec. 3.2 of the paper to the letter: for i = 0..n-1, call func with
(builders, i, struct of the i-th elements); func evaluates its whole body for
that one row and merges into each builder at most once.  Builders are kept as
mutable state, which the linearity rule of Sec. 3.2 makes legal.

It is used (a) as brute force against which interp.py is pinned, and (b) for the
fused == unfused invariant (one pass over rows here, one pass per operator
there; Sec. 4.5, the combined program versus the loop after fusion).
"""
import math

BITS = {"i8": 8, "i32": 32, "i64": 64}


def _wrap(x, t):
    w = BITS[t]
    x &= (1 << w) - 1
    return x - (1 << w) if x >> (w - 1) else x


def _tdiv(a, b):
    if b == 0:
        return 0                            # reading: a zero divisor gives quotient 0 (and remainder 0)
    q = abs(a) // abs(b)
    return q if (a < 0) == (b < 0) else -q


def _tmod(a, b):
    if b == 0:
        return 0
    return a - _tdiv(a, b) * b


def _isnan(x):
    return isinstance(x, float) and x != x


def _apply(code, t, a):
    isint = t in BITS
    if code == "neg":
        return _wrap(-a[0], t) if isint else -a[0]
    if code == "not":
        return not a[0]
    if code == "exp":
        return math.exp(a[0])
    if code == "log":
        return math.log(a[0])
    if code == "sqrt":
        return math.sqrt(a[0])
    if code == "erf":
        return math.erf(a[0])
    if code == "add":
        return _wrap(a[0] + a[1], t) if isint else a[0] + a[1]
    if code == "sub":
        return _wrap(a[0] - a[1], t) if isint else a[0] - a[1]
    if code == "mul":
        return _wrap(a[0] * a[1], t) if isint else a[0] * a[1]
    if code == "div":
        return _wrap(_tdiv(a[0], a[1]), t) if isint else a[0] / a[1]
    if code == "mod":
        return _tmod(a[0], a[1]) if isint else math.fmod(a[0], a[1])
    if code in ("min", "max") and (_isnan(a[0]) or _isnan(a[1])):
        return math.nan                     # reading: NaN in, NaN out
    if code == "min":
        return a[0] if a[0] <= a[1] else a[1]
    if code == "max":
        return a[0] if a[0] >= a[1] else a[1]
    if code == "lt":
        return a[0] < a[1]
    if code == "le":
        return a[0] <= a[1]
    if code == "gt":
        return a[0] > a[1]
    if code == "ge":
        return a[0] >= a[1]
    if code == "eq":
        return a[0] == a[1]
    if code == "ne":
        return a[0] != a[1]
    if code == "and":
        return bool(a[0]) and bool(a[1])
    if code == "or":
        return bool(a[0]) or bool(a[1])
    if code == "select":
        return a[1] if a[0] else a[2]
    raise ValueError(code)


def _cast(x, src, dst):
    if dst == "bool":
        return bool(x)
    if dst == "f64":
        return float(x)
    if src == "f64":
        if x != x:
            return 0                        # reading: NaN casts to 0
        if x >= 9.223372036854775808e18:
            return _wrap((1 << 63) - 1, dst)   # beyond the 64-bit range: its nearest end, then wrapped to dst
        if x < -9.223372036854775808e18:
            return _wrap(-(1 << 63), dst)
        return _wrap(int(x), dst)          # int() truncates toward zero
    return _wrap(int(x), dst)


def _combine(func, t, acc, v):
    if func == "add":
        return _wrap(acc + v, t) if t in BITS else acc + v
    if func == "mul":
        return _wrap(acc * v, t) if t in BITS else acc * v
    if _isnan(v) or _isnan(acc):
        return math.nan
    if func == "min":
        return v if v < acc else acc
    return v if v > acc else acc


def _identity(func, t):
    if func == "add":
        return 0 if t in BITS else 0.0
    if func == "mul":
        return 1 if t in BITS else 1.0
    if t in BITS:
        w = BITS[t]
        return (1 << (w - 1)) - 1 if func == "min" else -(1 << (w - 1))
    return math.inf if func == "min" else -math.inf


def _typed(x, t):
    return float(x) if t == "f64" else (bool(x) if t == "bool" else int(x))


def _body(program, i, elem, gather=None, outer_elem=None, inner_value=None, dicts=None, scalars=None):
    """Every expression of the body for ONE row: index i, `elem` = this row's element of each
    zipped vector.  Nested loops: `gather` are the vectors lookup may read, `outer_elem` the
    current outer element (inner bodies), `inner_value` the inner loop's result (outer bodies)."""
    val = []
    for op in program.ops:
        code, t = op[0], op[1]
        if code == "col":
            val.append(_typed(elem[op[2]], t))
        elif code == "scalar":
            val.append(_typed(scalars[op[2]], t))
        elif code == "const":
            val.append(_typed(op[2], t))
        elif code == "index":
            val.append(i)
        elif code == "cast":
            val.append(_cast(val[op[2]], program.ops[op[2]][1], t))
        elif code == "lookup":
            ix = val[op[3]]
            assert 0 <= ix < len(gather[op[2]]), "lookup out of range"
            val.append(_typed(gather[op[2]][ix], t))
        elif code == "keyexists":
            val.append(tuple(val[j] for j in op[3:]) in dicts[op[2]])
        elif code == "dictlookup":
            entry = dicts[op[2]].get(tuple(val[j] for j in op[4:]))
            val.append(_typed(entry[op[3]] if entry is not None else 0, t))
        elif code == "outer":
            val.append(_typed(outer_elem[op[2]], t))
        elif code == "inner":
            val.append(inner_value)
        else:
            val.append(_apply(code, t, [val[j] for j in op[2:]]))
    return val


def run_nested(nested, outer_columns, inner_columns, gather):
    """The nested loop written out: for every outer element, run its inner `for` over
    start, start + stride, ... below end with a fresh merger, take result(), then evaluate the
    outer body and merge.
    Returns the outer builders like `run` (merger -> number, vecbuilder -> list, ...)."""
    n_outer = len(outer_columns[0]) if outer_columns else 0
    inner_results = []
    for i in range(n_outer):
        x = [c[i] for c in outer_columns]
        acc = _identity(nested.inner_func, nested.inner_type)        # a new merger per outer element
        m = nested.inner.merges[0]
        stride_col = getattr(nested, "stride_col", None)
        stride = int(x[stride_col]) if stride_col is not None else 1
        assert stride >= 1
        for j in range(int(x[nested.start_col]), int(x[nested.end_col]), stride):
            val = _body(nested.inner, j, [c[j] for c in inner_columns], gather=gather, outer_elem=x)
            if m["pred"] is None or val[m["pred"]]:
                acc = _combine(nested.inner_func, nested.inner_type, acc, val[m["vals"][0]])
        inner_results.append(acc)                                    # result(inner builder)
    return run(nested.outer, outer_columns, inner_results=inner_results)


def run(program, columns, inits=None, inner_results=None, dicts=None):
    """columns: list of Python lists (ints / floats).  Returns Python values:
    merger -> number, vecbuilder -> list, dictmerger -> {key tuple: [values]},
    vecmerger -> list (inits: {builder index: list}), groupbuilder -> {key tuple: list of values}.
    dicts: dictionaries probed by keyexists / dictlookup, each {key tuple: [values]} as returned
    for a dictmerger by an earlier run."""
    # entries of the column list read by `scalar` hold one element, defined outside the loop
    scalars = {op[2]: columns[op[2]][0] for op in program.ops if op[0] == "scalar"}
    lengths = [len(c) for k, c in enumerate(columns) if k not in scalars]
    n = lengths[0] if lengths else 0
    state = []
    for b, spec in enumerate(program.builders):
        if spec["kind"] == "merger":
            state.append(_identity(spec["func"], spec["type"]))
        elif spec["kind"] == "vecbuilder":
            state.append([])
        elif spec["kind"] == "groupbuilder":
            state.append({})
        elif spec["kind"] == "vecmerger":
            init = (inits or {}).get(b)
            state.append(list(init) if init is not None
                         else [_identity(spec["func"], spec["type"])] * spec["length"])
        else:
            state.append({})
    for i in range(n):
        val = _body(program, i, [None if k in scalars else c[i] for k, c in enumerate(columns)],
                    inner_value=None if inner_results is None else inner_results[i], dicts=dicts, scalars=scalars)
        for m in program.merges:
            if m["pred"] is not None and not val[m["pred"]]:
                continue                            # `else b`: builder returned untouched
            b = m["builder"]
            spec = program.builders[b]
            if spec["kind"] == "merger":
                state[b] = _combine(spec["func"], spec["type"], state[b], val[m["vals"][0]])
            elif spec["kind"] == "vecbuilder":
                state[b].append(val[m["vals"][0]])
            elif spec["kind"] == "groupbuilder":
                state[b].setdefault(tuple(val[k] for k in m["keys"]), []).append(val[m["vals"][0]])
            elif spec["kind"] == "vecmerger":
                ix = val[m["keys"][0]]
                state[b][ix] = _combine(spec["func"], spec["type"], state[b][ix], val[m["vals"][0]])
            else:
                key = tuple(val[k] for k in m["keys"])
                vs = [val[v] for v in m["vals"]]
                if key not in state[b]:
                    state[b][key] = vs
                else:
                    cur = state[b][key]
                    state[b][key] = [_combine(spec["func"], t, c, v)
                                     for c, v, t in zip(cur, vs, spec["val_types"])]
    return state
