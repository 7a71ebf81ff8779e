"""Plain-data description of one fused `for` loop over zipped columns.

This module is *input plumbing only*: it records which operator is applied to
which earlier value, which builder a value is merged into and under which
predicate.  It performs no arithmetic of the method itself.  The CPU oracle and
the HIP binding each read a `Program` and give it meaning on their own.

The loop described is the paper's parallel `for(vectors, builders, func)`
(Sec. 3.2): `func` sees the row index and one element of every zipped vector,
and returns the builders after zero or one `merge` into each of them.

A `Program` holds
  columns  : list of type names, one per zipped input vector
  ops      : SSA list; entry k is a tuple (opcode, result_type, *args)
             'col'   -> args = (column_index,)
             'const' -> args = (python number,)
             'index' -> args = ()            (row index, i64)
             unary   -> args = (a,)          neg not cast exp log sqrt erf
             binary  -> args = (a, b)        add sub mul div mod min max
                                             lt le gt ge eq ne and or
             'select'-> args = (cond, a, b)
             'lookup'-> args = (gather_vector_index, index_value)   element of a
                        vector read at a computed position (nested loops only)
             'outer' -> args = (outer_column_index,)   inner body of a nested loop:
                        the current OUTER element of that vector
             'inner' -> args = ()   outer body of a nested loop: the result of this
                        outer element's inner loop
             'keyexists' -> args = (dict_index, *key_values)   whether a dictionary that an
                        earlier loop built (an input of this loop) holds the key struct
             'dictlookup'-> args = (dict_index, value_field, *key_values)   that field of
                        the key's value struct (0 if the key is absent)
           operand references are indices of earlier entries.
  builders : list of dicts
             {'kind': 'merger',     'type': T, 'func': f}
             {'kind': 'vecbuilder', 'type': T}
             {'kind': 'dictmerger', 'key_types': [..], 'val_types': [..],
              'func': f, 'capacity': hint}
             {'kind': 'vecmerger', 'type': T, 'func': f, 'length': m}
               (merges {index, value} pairs into a vector of m cells; the
                initial vector is an input of the call, not of the program)
             {'kind': 'groupbuilder', 'key_types': [..], 'type': T, 'capacity': hint}
               (groups merged {key, value} pairs by key: one vector of values per key)
  merges   : list of dicts {'builder': b, 'pred': op or None,
                            'keys': [ops], 'vals': [ops]}
             (Sec. 3.2: `if (p) merge(b, v) else b` is a merge under predicate p.)
"""

TYPES = ("bool", "i8", "i32", "i64", "f64")
UNARY = ("neg", "not", "cast", "exp", "log", "sqrt", "erf")
BINARY = ("add", "sub", "mul", "div", "mod", "min", "max",
          "lt", "le", "gt", "ge", "eq", "ne", "and", "or")
COMPARE = ("lt", "le", "gt", "ge", "eq", "ne")
FUNCS = ("add", "mul", "min", "max")


class Program:
    """Builder for the plain-data loop description (no evaluation here)."""

    def __init__(self, columns, gather=(), outer=(), inner_type=None, dicts=()):
        for t in list(columns) + list(gather) + list(outer):
            assert t in TYPES, t
        # dictionaries built by earlier loops that this loop may probe:
        # [{'key_types': [...], 'val_types': [...]}, ...]
        self.dicts = [dict(d) for d in dicts]
        self.columns = list(columns)
        self.gather = list(gather)        # element types of the vectors `lookup` may read
        self.outer_columns = list(outer)  # an inner body's view of the outer vectors
        self.inner_type = inner_type      # an outer body's view of the inner loop's result
        self.ops = []
        self.builders = []
        self.merges = []

    # ---- values -----------------------------------------------------
    def _push(self, entry):
        self.ops.append(tuple(entry))
        return len(self.ops) - 1

    def type_of(self, v):
        return self.ops[v][1]

    def col(self, k):
        return self._push(("col", self.columns[k], k))

    def scalar(self, k):
        """Entry k of the column list holds ONE element: a scalar defined outside the loop (say an
        earlier loop's merger result) that every row reads; never also read with col(k)."""
        return self._push(("scalar", self.columns[k], k))

    def const(self, t, value):
        assert t in TYPES
        return self._push(("const", t, value))

    def index(self):
        return self._push(("index", "i64"))

    def un(self, opcode, a, to=None):
        assert opcode in UNARY
        if opcode == "cast":
            assert to in TYPES
            t = to
        else:
            t = self.type_of(a)
        return self._push((opcode, t, a))

    def bin(self, opcode, a, b):
        assert opcode in BINARY
        t = "bool" if opcode in COMPARE else self.type_of(a)
        return self._push((opcode, t, a, b))

    def select(self, c, a, b):
        return self._push(("select", self.type_of(a), c, a, b))

    def lookup(self, k, idx):
        assert self.type_of(idx) in ("i8", "i32", "i64")
        return self._push(("lookup", self.gather[k], k, idx))

    def keyexists(self, d, keys):
        assert [self.type_of(k) for k in keys] == self.dicts[d]["key_types"]
        return self._push(("keyexists", "bool", d) + tuple(keys))

    def dictlookup(self, d, field, keys):
        assert [self.type_of(k) for k in keys] == self.dicts[d]["key_types"]
        return self._push(("dictlookup", self.dicts[d]["val_types"][field], d, field) + tuple(keys))

    def outer(self, k):
        return self._push(("outer", self.outer_columns[k], k))

    def inner(self):
        assert self.inner_type is not None
        return self._push(("inner", self.inner_type))

    # ---- builders ---------------------------------------------------
    def merger(self, t, func):
        assert func in FUNCS
        self.builders.append({"kind": "merger", "type": t, "func": func})
        return len(self.builders) - 1

    def vecbuilder(self, t):
        self.builders.append({"kind": "vecbuilder", "type": t})
        return len(self.builders) - 1

    def dictmerger(self, key_types, val_types, func, capacity):
        assert func in FUNCS
        self.builders.append({"kind": "dictmerger", "key_types": list(key_types),
                              "val_types": list(val_types), "func": func,
                              "capacity": int(capacity)})
        return len(self.builders) - 1

    def vecmerger(self, t, func, length):
        assert func in FUNCS
        self.builders.append({"kind": "vecmerger", "type": t, "func": func, "length": int(length)})
        return len(self.builders) - 1

    def groupbuilder(self, key_types, t, capacity):
        self.builders.append({"kind": "groupbuilder", "key_types": list(key_types), "type": t,
                              "capacity": int(capacity)})
        return len(self.builders) - 1

    def merge(self, builder, vals, keys=(), pred=None):
        if isinstance(vals, int):
            vals = [vals]
        self.merges.append({"builder": builder, "pred": pred,
                            "keys": list(keys), "vals": list(vals)})


class NestedProgram:
    """A `for` nested in a `for` (Sec. 3.2 of the paper: loops nest; a loop may take a
    start and an end index per input vector):

        for(zip(outer...), builders, (bs, i, x) =>
            let r = result(for(iter(zip(inner...), x.start, x.end), merger[T, func], inner_body));
            outer_body(x, r, i))

    `inner` is a Program over the inner vectors with exactly one merger (builder 0) and may
    use `lookup` and `outer`; `outer` is a Program over the outer vectors that may use
    `inner()`; start_col / end_col name the outer columns that hold each outer element's
    inner range [start, end).  stride_col (optional) names the outer column with each range's
    stride: the inner loop then visits start, start + stride, ... below end (the paper's
    per-vector start, end and stride: a column of a row-major matrix is start = j,
    end = rows * cols, stride = cols).  ranges = "csr": the ranges are consecutive with stride 1
    (end[i] == start[i+1], a CSR row-pointer array); "any": they may overlap, leave gaps and
    carry strides.  In an inner body `index` is the position of the element in the inner vectors.
    Plain data, no evaluation.
    """

    def __init__(self, outer_columns, start_col, end_col, inner_columns, gather, inner_type, inner_func,
                 stride_col=None, ranges="csr"):
        assert inner_func in FUNCS and inner_type in ("i64", "f64")
        assert outer_columns[start_col] == outer_columns[end_col] and outer_columns[start_col] in ("i32", "i64")
        assert ranges in ("csr", "any") and (stride_col is None or ranges == "any")
        assert stride_col is None or outer_columns[stride_col] == outer_columns[start_col]
        self.stride_col, self.ranges = stride_col, ranges
        self.start_col, self.end_col = start_col, end_col
        self.inner_type, self.inner_func = inner_type, inner_func
        self.inner = Program(inner_columns, gather=gather, outer=outer_columns)
        self.inner.merger(inner_type, inner_func)
        self.outer = Program(outer_columns, inner_type=inner_type)
        self.gather = list(gather)
