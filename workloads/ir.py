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
           operand references are indices of earlier entries.
  builders : list of dicts
             {'kind': 'merger',     'type': T, 'func': f}
             {'kind': 'vecbuilder', 'type': T}
             {'kind': 'dictmerger', 'key_types': [..], 'val_types': [..],
              'func': f, 'capacity': hint}
             {'kind': 'vecmerger', 'type': T, 'func': f, 'length': m}
               (merges {index, value} pairs into a vector of m cells; the
                initial vector is an input of the call, not of the program)
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

    def __init__(self, columns):
        for t in columns:
            assert t in TYPES, t
        self.columns = list(columns)
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

    def merge(self, builder, vals, keys=(), pred=None):
        if isinstance(vals, int):
            vals = [vals]
        self.merges.append({"builder": builder, "pred": pred,
                            "keys": list(keys), "vals": list(vals)})
