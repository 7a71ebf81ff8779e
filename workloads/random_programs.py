"""Seeded random loop bodies and inputs for differential tests (input plumbing only).

`make(seed)` returns (Program, columns as numpy arrays, initial vectors of the vecmergers):
a random expression graph over one to five zipped columns of random types, merged into one
to three random builders (merger, vecbuilder, dictmerger, vecmerger, groupbuilder) under random
predicates.  Nothing here evaluates a program: the
CPU oracle and the HIP library each give it meaning on their own, and the tests compare them.

The graphs stay inside what both sides define and what the comparison rules can judge:
  * no operator whose result depends on a library's last bit (exp, log, erf): a predicate
    that flips on such a bit changes counts; those operators have tests of their own;
  * an upper bound on |value| is carried along for every f64 value, and operators that would
    take it past 1e100 are not generated (no inf - inf);
  * f64 -> integer casts are clamped into the target's range first; integer divisors are
    constants of magnitude >= 2; f64 divisors are of the form x*x + 1;
  * f64 values merged with `add` are squares: a sum of mixed signs can cancel to nothing,
    and then no relative tolerance is meaningful;
  * dictionary keys and vecmerger indices are reduced modulo small constants, so capacities
    and lengths are known.
"""
import numpy as np

from workloads.ir import NestedProgram, Program

INTS = ("i8", "i32", "i64")
INT_MAX = {"i8": 127.0, "i32": 2147483647.0, "i64": 9.3e18}
CLAMP = {"i8": 100.0, "i32": 1.0e9, "i64": 1.0e15}
NP = {"i8": np.int8, "i32": np.int32, "i64": np.int64, "f64": np.float64}
SIZES = (1, 63, 4_097, 70_001, 70_001, 300_007, 300_007)


COL_MAG = {"i8": 128.0, "i32": 2.0e6, "i64": 1.0e12, "f64": 3.0}


def random_column(rnd, t, n):
    if t == "f64":
        return np.round(rnd.uniform(-3, 3, size=n), 6)
    if t == "i8":
        return rnd.randint(-128, 128, size=n).astype(np.int8)
    if t == "i32":
        c = rnd.randint(-1_000_000, 1_000_001, size=n).astype(np.int32)
        c[rnd.rand(n) < 0.01] = np.int32(2147483647)
        return c
    c = rnd.randint(-10 ** 12, 10 ** 12, size=n).astype(np.int64)
    c[rnd.rand(n) < 0.01] = np.int64(-2 ** 63)
    return c


class _Gen:
    def __init__(self, rnd, program=None, skip_columns=()):
        self.rnd = rnd
        if program is None:
            ncols = int(self.rnd.randint(1, 6))
            program = Program([str(self.rnd.choice(["i8", "i32", "i64", "f64"])) for _ in range(ncols)])
        self.col_types = list(program.columns)
        self.p = program
        self.pool = {"bool": [], "i8": [], "i32": [], "i64": [], "f64": []}
        self.mag = {}
        for k, t in enumerate(self.col_types):
            if k not in skip_columns:
                self._add(self.p.col(k), COL_MAG[t])
        if self.rnd.rand() < 0.4:
            self._add(self.p.index(), 1.0e6)

    def _add(self, v, mag):
        t = self.p.type_of(v)
        self.pool[t].append(v)
        self.mag[v] = min(mag, INT_MAX[t]) if t in INTS else mag
        return v

    def pick(self, t):
        vs = self.pool[t]
        return vs[int(self.rnd.randint(len(vs)))] if vs else None

    def const(self, t, value):
        v = self.p.const(t, value)
        self.mag[v] = abs(float(value))
        return v

    def some(self, t):
        """A value of type t: an earlier one, else a constant."""
        v = self.pick(t)
        if v is not None and self.rnd.rand() < 0.85:
            return v
        if t == "f64":
            return self.const(t, float(np.round(self.rnd.uniform(-4, 4), 3)))
        if t == "bool":
            c = self.const("i64", 0)
            return self._add(self.p.bin("eq", c, c), 1.0)
        return self.const(t, int(self.rnd.randint(-100, 101)))

    def square(self, v):
        return self._add(self.p.bin("mul", v, v), self.mag[v] ** 2)

    def grow(self):
        rnd, p = self.rnd, self.p
        kind = rnd.choice(["iarith", "iarith", "idiv", "farith", "farith", "fdiv", "sqrt", "neg", "cmp", "cmp",
                           "logic", "select", "cast", "cast"])
        if kind == "iarith":
            t = str(rnd.choice(INTS))
            a, b = self.some(t), self.some(t)
            op = str(rnd.choice(["add", "sub", "mul", "min", "max"]))
            m = {"add": self.mag[a] + self.mag[b], "sub": self.mag[a] + self.mag[b], "mul": self.mag[a] * self.mag[b]}.get(
                op, max(self.mag[a], self.mag[b]))
            self._add(p.bin(op, a, b), m)
        elif kind == "idiv":
            t = str(rnd.choice(INTS))
            a = self.some(t)
            d = int(rnd.choice([2, 3, 5, 7, 10, 11, 16, 60, 100, 127])) * (-1 if rnd.rand() < 0.25 else 1)
            op = str(rnd.choice(["div", "mod"]))
            self._add(p.bin(op, a, self.const(t, d)), self.mag[a] if op == "div" else abs(d))
        elif kind == "farith":
            a, b = self.some("f64"), self.some("f64")
            op = str(rnd.choice(["add", "sub", "mul", "min", "max"]))
            m = self.mag[a] * self.mag[b] if op == "mul" else self.mag[a] + self.mag[b]
            if m < 1e100:
                self._add(p.bin(op, a, b), m)
        elif kind == "fdiv":
            a, b = self.some("f64"), self.some("f64")
            if self.mag[b] ** 2 < 1e100:
                den = self._add(p.bin("add", self.square(b), self.const("f64", 1.0)), self.mag[b] ** 2 + 1)
                self._add(p.bin("div", a, den), self.mag[a])
        elif kind == "sqrt":
            a = self.some("f64")
            if self.mag[a] ** 2 < 1e100:
                self._add(p.un("sqrt", self.square(a)), self.mag[a])
        elif kind == "neg":
            t = str(rnd.choice(INTS + ("f64",)))
            a = self.some(t)
            self._add(p.un("neg", a), self.mag[a])
        elif kind == "cmp":
            t = str(rnd.choice(INTS + ("f64",)))
            a, b = self.some(t), self.some(t)
            self._add(p.bin(str(rnd.choice(["lt", "le", "gt", "ge", "eq", "ne"])), a, b), 1.0)
        elif kind == "logic":
            a = self.some("bool")
            if rnd.rand() < 0.3:
                self._add(p.un("not", a), 1.0)
            else:
                self._add(p.bin(str(rnd.choice(["and", "or"])), a, self.some("bool")), 1.0)
        elif kind == "select":
            t = str(rnd.choice(INTS + ("f64",)))
            a, b = self.some(t), self.some(t)
            self._add(p.select(self.some("bool"), a, b), max(self.mag[a], self.mag[b]))
        else:
            src = str(rnd.choice(["bool"] + list(INTS) + ["f64"]))
            dst = str(rnd.choice([t for t in INTS + ("f64",) if t != src]))
            a = self.some(src)
            if src == "f64" and dst in INTS and self.mag[a] >= CLAMP[dst]:
                lo, hi = self.const("f64", -CLAMP[dst]), self.const("f64", CLAMP[dst])
                a = self._add(p.bin("min", self._add(p.bin("max", a, lo), CLAMP[dst]), hi), CLAMP[dst])
            self._add(p.un("cast", a, to=dst), self.mag[a])

    # ---- values fit for merging -------------------------------------
    def summand(self, t, func):
        v = self.some(t)
        if t == "f64" and func == "add":
            if self.mag[v] ** 2 >= 1e100:
                v = self.const("f64", 1.5)
            v = self.square(v)
        return v

    def reduced(self, v, modulus):
        """v mod modulus, in (-modulus, modulus)."""
        t = self.p.type_of(v)
        return self._add(self.p.bin("mod", v, self.const(t, modulus)), modulus)

    def pred(self):
        return self.some("bool") if self.rnd.rand() < 0.7 else None


def _add_builders(g):
    """One to three random builders with their merges; returns the vecmergers' initial vectors."""
    rnd, p = g.rnd, g.p
    inits = {}
    for _ in range(int(rnd.randint(1, 4))):
        kind = str(rnd.choice(["merger", "merger", "vecbuilder", "vecbuilder", "dictmerger", "dictmerger", "vecmerger",
                               "groupbuilder"]))
        if kind == "groupbuilder" and any(b["kind"] == "groupbuilder" for b in p.builders):
            kind = "vecbuilder"              # one a program: it stands for three builders inside the library
        if kind == "merger":
            t = str(rnd.choice(INTS + ("f64",)))
            func = str(rnd.choice(["add", "min", "max"] if t == "f64" else ["add", "mul", "min", "max"]))
            p.merge(p.merger(t, func), g.summand(t, func), pred=g.pred())
        elif kind == "vecbuilder":
            t = str(rnd.choice(INTS + ("f64",)))
            p.merge(p.vecbuilder(t), g.some(t), pred=g.pred())
        elif kind == "dictmerger":
            keys, capacity = [], 1
            nkeys = int(rnd.randint(1, 3))
            for _k in range(nkeys):
                t = str(rnd.choice(INTS if nkeys == 1 else ("i8", "i32")))      # a key struct has 64 bits at most
                modulus = int(rnd.choice([2, 3, 7, 50, 120])) if t == "i8" or len(keys) else int(rnd.choice([3, 40, 900, 20_000]))
                keys.append(g.reduced(g.some(t), modulus))
                capacity *= 2 * modulus - 1
            func = str(rnd.choice(["add", "add", "min", "max", "mul"]))
            vts = [str(rnd.choice(INTS if func == "mul" else INTS + ("f64",))) for _v in range(int(rnd.randint(1, 4)))]
            vals = [g.summand(t, func) for t in vts]
            p.merge(p.dictmerger([p.type_of(k) for k in keys], vts, func, capacity), vals, keys=keys, pred=g.pred())
        elif kind == "groupbuilder":
            keys, capacity = [], 1
            nkeys = int(rnd.randint(1, 3))
            for _k in range(nkeys):
                t = str(rnd.choice(INTS if nkeys == 1 else ("i8", "i32")))
                modulus = int(rnd.choice([2, 3, 7, 50, 120])) if t == "i8" or len(keys) else int(rnd.choice([3, 40, 900, 20_000]))
                keys.append(g.reduced(g.some(t), modulus))
                capacity *= 2 * modulus - 1
            t = str(rnd.choice(INTS + ("f64",)))
            p.merge(p.groupbuilder([p.type_of(k) for k in keys], t, capacity), [g.some(t)], keys=keys, pred=g.pred())
        else:
            t = str(rnd.choice(["i64", "f64"]))
            func = str(rnd.choice(["add", "min", "max"]))
            length = int(rnd.choice([1, 17, 1_000, 50_000]))
            src = g.some(str(rnd.choice(INTS)))
            if p.type_of(src) != "i64":
                src = g._add(p.un("cast", src, to="i64"), g.mag[src])
            r = g.reduced(src, length) if length > 1 else g.const("i64", 0)
            if length > 1:   # into [0, length)
                r = g.reduced(g._add(p.bin("add", r, g.const("i64", length)), 2 * length), length)
            b = p.vecmerger(t, func, length)
            p.merge(b, [g.summand(t, func)], keys=[r], pred=g.pred())
            if rnd.rand() < 0.5:
                inits[b] = (rnd.uniform(0, 2, size=length) if t == "f64" else rnd.randint(-5, 6, size=length)).astype(
                    np.float64 if t == "f64" else np.int64)
    return inits


def make(seed):
    g = _Gen(np.random.RandomState(seed))
    rnd, p = g.rnd, g.p
    for _ in range(int(rnd.randint(3, 15))):
        g.grow()
    inits = _add_builders(g)
    n = int(rnd.choice(SIZES))
    cols = [random_column(rnd, t, n) for t in g.col_types]
    return p, cols, inits


def make_probe(seed):
    """A random build side and probe side of a hash join: (build Program, build columns, probe Program,
    probe columns, initial vectors of the probe's vecmergers).  The build loop merges into one
    dictmerger (builder 0); the probe loop computes key structs of the same types (reduced with a
    modulus of its own, so some keys are absent), asks whether they exist and looks fields of their
    values up, and goes on computing with the answers."""
    rnd = np.random.RandomState(seed)
    gb = _Gen(rnd)
    for _ in range(int(rnd.randint(1, 6))):
        gb.grow()
    nkeys = int(rnd.randint(1, 3))
    key_types = [str(rnd.choice(INTS if nkeys == 1 else ("i8", "i32"))) for _ in range(nkeys)]
    build_mod = [int(rnd.choice([2, 7, 50, 120])) if t == "i8" or k else int(rnd.choice([3, 40, 900, 20_000, 300_000]))
                 for k, t in enumerate(key_types)]
    keys = [gb.reduced(gb.some(t), m) for t, m in zip(key_types, build_mod)]
    capacity = 1
    for m in build_mod:
        capacity *= 2 * m - 1
    # an f64 sum in the dictionary would depend on merge order in its last bits, and the probe side
    # compares and casts what it looks up
    func = str(rnd.choice(["add", "min", "max"]))
    val_types = [str(rnd.choice(INTS if func == "add" else INTS + ("f64",))) for _ in range(int(rnd.randint(1, 4)))]
    vals = [gb.summand(t, func) for t in val_types]
    gb.p.merge(gb.p.dictmerger(key_types, val_types, func, capacity), vals, keys=keys, pred=gb.pred())
    n_build = int(rnd.choice([1, 500, 70_001, 300_007]))
    build_cols = [random_column(rnd, t, n_build) for t in gb.col_types]

    ncols = int(rnd.randint(1, 5))
    probe = Program([str(rnd.choice(["i8", "i32", "i64", "f64"])) for _ in range(ncols)],
                    dicts=[{"key_types": key_types, "val_types": val_types}])
    gp = _Gen(rnd, probe)
    for _ in range(int(rnd.randint(0, 4))):
        gp.grow()
    for _ in range(int(rnd.randint(1, 3))):
        pk = [gp.reduced(gp.some(t), min(int(m * rnd.choice([1, 1, 2])), 127 if t == "i8" else 2 ** 30))
              for t, m in zip(key_types, build_mod)]
        gp._add(probe.keyexists(0, pk), 1.0)
        for f in range(len(val_types)):
            if rnd.rand() < 0.7:
                gp._add(probe.dictlookup(0, f, pk), INT_MAX[val_types[f]] if val_types[f] in INTS else 1.0e99)
    for _ in range(int(rnd.randint(1, 8))):
        gp.grow()
    inits = _add_builders(gp)
    n_probe = int(rnd.choice([1, 63, 4_097, 70_001, 300_007]))
    probe_cols = [random_column(rnd, t, n_probe) for t in gp.col_types]
    return gb.p, build_cols, probe, probe_cols, inits


def make_nested(seed, any_ranges=False):
    """A random `for` nested in a `for`: (NestedProgram, outer columns, inner columns, gather vectors).
    Inner ranges are consecutive (a CSR row-pointer array split into its start and end columns),
    with empty, short and long ranges mixed; the inner body may read the current outer element and
    look values up in the gather vectors at reduced (in-range) positions.
    any_ranges: the ranges are drawn independently instead - they overlap, leave gaps, some are
    empty - and (two times in three) every range carries a stride of its own."""
    rnd = np.random.RandomState(seed)
    n_outer = int(rnd.choice([1, 50, 3_000, 40_000]))
    inner_type = str(rnd.choice(["i64", "f64"]))
    inner_func = str(rnd.choice(["add", "min", "max"] if inner_type == "f64" else ["add", "mul", "min", "max"]))
    never_empty = inner_type == "f64" and inner_func != "add"      # an empty range gives the identity: +-inf
    lengths = rnd.randint(0, 9, size=n_outer)
    long_rows = rnd.rand(n_outer) < 0.01
    lengths[long_rows] = rnd.randint(100, 5_000, size=int(long_rows.sum()))
    if never_empty:
        lengths = np.maximum(lengths, 1)
    offsets_type = str(rnd.choice(["i32", "i64"]))
    rowptr = np.concatenate([[0], np.cumsum(lengths)]).astype(NP[offsets_type])
    n_inner = int(rowptr[-1])
    extra_outer = [str(rnd.choice(["i8", "i32", "i64", "f64"])) for _ in range(int(rnd.randint(0, 3)))]
    inner_cols = [str(rnd.choice(["i8", "i32", "i64", "f64"])) for _ in range(int(rnd.randint(1, 4)))]
    gather_types = [str(rnd.choice(["i32", "i64", "f64"])) for _ in range(int(rnd.randint(0, 3)))]
    gather_len = [int(rnd.choice([1, 7, 1_000, 5_000])) for _ in gather_types]
    with_stride = any_ranges and seed % 3 != 0
    first_extra = 3 if with_stride else 2
    nested = NestedProgram([offsets_type] * first_extra + extra_outer, 0, 1, inner_cols, gather_types, inner_type, inner_func,
                           stride_col=2 if with_stride else None, ranges="any" if any_ranges else "csr")
    ranges = [rowptr[:-1].copy(), rowptr[1:].copy()]
    if any_ranges:
        n_inner = max(n_inner, 1)
        strides = rnd.choice([1, 1, 2, 3, 17, 1000], size=n_outer) if with_stride else np.ones(n_outer, dtype=np.int64)
        start = rnd.randint(0, n_inner, size=n_outer)
        span = lengths * strides                                   # about `lengths` elements each, whatever the stride
        end = np.minimum(n_inner, start + span)
        if never_empty:
            start = np.minimum(start, n_inner - 1)
            end = np.maximum(end, start + 1)
        ranges = [start.astype(NP[offsets_type]), end.astype(NP[offsets_type])]
        if with_stride:
            ranges.append(strides.astype(NP[offsets_type]))

    gi = _Gen(rnd, nested.inner)
    for k, t in enumerate(extra_outer):
        gi._add(nested.inner.outer(first_extra + k), COL_MAG[t])
    for k, t in enumerate(gather_types):
        src = gi.some(str(rnd.choice(INTS)))
        wide = src if nested.inner.type_of(src) == "i64" else gi._add(nested.inner.un("cast", src, to="i64"), gi.mag[src])
        if gather_len[k] > 1:      # into [0, length): reduced, shifted up by the length, reduced again
            pos = gi.reduced(gi._add(nested.inner.bin("add", gi.reduced(wide, gather_len[k]), gi.const("i64", gather_len[k])),
                                     2.0 * gather_len[k]), gather_len[k])
        else:
            pos = gi.const("i64", 0)
        gi._add(nested.inner.lookup(k, pos), COL_MAG[t])
    for _ in range(int(rnd.randint(2, 9))):
        gi.grow()
    v = gi.summand(inner_type, inner_func)
    nested.inner.merge(0, v, pred=None if never_empty else gi.pred())

    go = _Gen(rnd, nested.outer, skip_columns=())
    inner_mag = gi.mag[v] * 5_000 if inner_func == "add" else gi.mag[v]
    inner_value = nested.outer.inner()
    # an f64 sum depends on the order of its merges in the last bits: it is merged as it is (and
    # compared with a tolerance), never compared, cast or combined further, where a last bit decides
    order_dependent = inner_type == "f64" and inner_func == "add"
    if not order_dependent:
        go._add(inner_value, min(inner_mag, 9.9e99) if inner_type == "f64" else inner_mag)
    for _ in range(int(rnd.randint(1, 7))):
        go.grow()
    if order_dependent:
        if rnd.rand() < 0.5:
            nested.outer.merge(nested.outer.vecbuilder("f64"), inner_value, pred=go.pred())
        else:
            nested.outer.merge(nested.outer.merger("f64", "add"), inner_value, pred=go.pred())
    for _ in range(int(rnd.randint(1, 3))):
        if rnd.rand() < 0.5:
            t = str(rnd.choice(INTS + ("f64",)))
            func = str(rnd.choice(["add", "min", "max"] if t == "f64" else ["add", "mul", "min", "max"]))
            nested.outer.merge(nested.outer.merger(t, func), go.summand(t, func), pred=go.pred())
        else:
            t = str(rnd.choice(INTS + ("f64",)))
            nested.outer.merge(nested.outer.vecbuilder(t), go.some(t), pred=go.pred())
    outer = ranges + [random_column(rnd, t, n_outer) for t in extra_outer]
    inner = [random_column(rnd, t, n_inner) for t in inner_cols]
    gather = [random_column(rnd, t, m) for t, m in zip(gather_types, gather_len)]
    return nested, outer, inner, gather
