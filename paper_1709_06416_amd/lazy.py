"""A NumPy/Pandas-flavoured front end over the lazy object API (include/weld_object.h).

This is what a library integration looks like (paper Sec. 4.5, Sec. 6): every operator
of the library builds one small lazy object (`a * b`, `x > 0.5`, `v[mask]`, `v.sum()`);
nothing runs until `evaluate`, which lets the runtime fuse the whole DAG into one loop.
Marshalling only: expressions are handed to the C library as operator lists.
"""
import ctypes as C

import torch

from . import binding as wb

_lib = wb.lib
_lib.weld_object_new_data.argtypes = [C.c_void_p, C.c_int32, C.c_int64, C.POINTER(C.c_void_p)]
_lib.weld_object_new_map.argtypes = [C.POINTER(C.c_void_p), C.c_int32, C.POINTER(wb.Op), C.c_int32, C.POINTER(C.c_void_p)]
_lib.weld_object_new_filter.argtypes = [C.c_void_p, C.c_void_p, C.POINTER(C.c_void_p)]
_lib.weld_object_new_reduce.argtypes = [C.c_void_p, C.c_int32, C.POINTER(C.c_void_p)]
_lib.weld_object_new_groupby.argtypes = [C.POINTER(C.c_void_p), C.c_int32, C.POINTER(C.c_void_p), C.c_int32,
                                         C.c_int32, C.c_int64, C.POINTER(C.c_void_p)]
_lib.weld_object_evaluate.argtypes = [C.POINTER(C.c_void_p), C.c_int32, C.POINTER(wb.Conf), C.POINTER(C.c_void_p)]
_lib.weld_object_describe.argtypes = [C.POINTER(C.c_void_p), C.c_int32, C.c_char_p, C.c_int64]
_lib.weld_object_describe.restype = C.c_int64
_lib.weld_object_free.argtypes = [C.c_void_p]
_lib.weld_object_free.restype = None
_lib.weld_object_kind.argtypes = [C.c_void_p]
_lib.weld_object_elem_type.argtypes = [C.c_void_p]
for _f in ("weld_object_new_data", "weld_object_new_map", "weld_object_new_filter", "weld_object_new_reduce",
           "weld_object_new_groupby", "weld_object_evaluate", "weld_object_kind", "weld_object_elem_type"):
    getattr(_lib, _f).restype = C.c_int

_TYPE_NAME = {v: k for k, v in wb.TYPE_ID.items()}
_COMPARE = ("lt", "le", "gt", "ge", "eq", "ne")


def _check(st):
    if st != wb.OK:
        raise wb.WeldError(st, _lib.weld_last_error().decode())


class Obj:
    """One lazy object; keeps its dependencies (and their tensors) alive."""

    def __init__(self, handle, dtype, keep=()):
        self._h = handle
        self.dtype = dtype            # "i8" / "i32" / "i64" / "f64" / "bool", None for dictionaries
        self._keep = keep

    def __del__(self):
        try:
            if self._h:
                _lib.weld_object_free(self._h)
        except Exception:
            pass


def _map(deps, ops, dtype):
    arr = (wb.Op * len(ops))()
    for i, (code, t, a, b, c, imm) in enumerate(ops):
        o = arr[i]
        o.opcode, o.type, o.a, o.b, o.c = wb.OPCODE[code], wb.TYPE_ID[t], a, b, c
        if code == "const":
            if t == "f64":
                o.imm.f64 = float(imm)
            else:
                o.imm.i64 = int(imm)
    handles = (C.c_void_p * max(len(deps), 1))(*[d._h for d in deps])
    out = C.c_void_p()
    _check(_lib.weld_object_new_map(handles, len(deps), arr, len(ops), C.byref(out)))
    return Vec(out, dtype, tuple(deps))


class Vec(Obj):
    """A lazily evaluated vector."""

    @staticmethod
    def from_tensor(t):
        assert t.is_cuda and t.is_contiguous()
        dtype = wb.TORCH_TYPE[t.dtype]
        out = C.c_void_p()
        _check(_lib.weld_object_new_data(t.data_ptr(), wb.TYPE_ID[dtype], t.numel(), C.byref(out)))
        return Vec(out, dtype, (t,))

    @staticmethod
    def from_pointer(ptr, dtype, n, keep=()):
        """Wrap `n` elements of `dtype` at device address `ptr` (the caller keeps them alive)."""
        out = C.c_void_p()
        _check(_lib.weld_object_new_data(ptr, wb.TYPE_ID[dtype], n, C.byref(out)))
        return Vec(out, dtype, keep)

    # ---- elementwise operators: one object per library call
    def _binary(self, code, other, reflect=False):
        rt = "bool" if code in _COMPARE else self.dtype
        if isinstance(other, (Scalar, ScalarExpr)):
            return _with_scalars(self, code, other, reflect, rt)
        if isinstance(other, Vec):
            assert other.dtype == self.dtype, "no implicit casts: use .cast()"
            a, b = (1, 0) if reflect else (0, 1)
            return _map([self, other], [("col", self.dtype, 0, -1, -1, 0), ("col", other.dtype, 1, -1, -1, 0),
                                        (code, rt, a, b, -1, 0)], rt)
        a, b = (1, 0) if reflect else (0, 1)
        return _map([self], [("col", self.dtype, 0, -1, -1, 0), ("const", self.dtype, -1, -1, -1, other),
                             (code, rt, a, b, -1, 0)], rt)

    def __add__(self, o): return self._binary("add", o)
    def __radd__(self, o): return self._binary("add", o, True)
    def __sub__(self, o): return self._binary("sub", o)
    def __rsub__(self, o): return self._binary("sub", o, True)
    def __mul__(self, o): return self._binary("mul", o)
    def __rmul__(self, o): return self._binary("mul", o, True)
    def __truediv__(self, o): return self._binary("div", o)
    def __rtruediv__(self, o): return self._binary("div", o, True)
    def __mod__(self, o): return self._binary("mod", o)
    def __lt__(self, o): return self._binary("lt", o)
    def __le__(self, o): return self._binary("le", o)
    def __gt__(self, o): return self._binary("gt", o)
    def __ge__(self, o): return self._binary("ge", o)
    def eq(self, o): return self._binary("eq", o)
    def ne(self, o): return self._binary("ne", o)
    def __and__(self, o): return self._binary("and", o)
    def __or__(self, o): return self._binary("or", o)

    def _unary(self, code, dtype=None):
        return _map([self], [("col", self.dtype, 0, -1, -1, 0), (code, dtype or self.dtype, 0, -1, -1, 0)],
                    dtype or self.dtype)

    def __neg__(self): return self._unary("neg")
    def __invert__(self): return self._unary("not")
    def exp(self): return self._unary("exp")
    def log(self): return self._unary("log")
    def sqrt(self): return self._unary("sqrt")
    def erf(self): return self._unary("erf")
    def cast(self, dtype): return self._unary("cast", dtype)

    # ---- filter, reductions
    def __getitem__(self, mask):
        assert isinstance(mask, Vec) and mask.dtype == "bool"
        out = C.c_void_p()
        _check(_lib.weld_object_new_filter(self._h, mask._h, C.byref(out)))
        return Vec(out, self.dtype, (self, mask))

    def _reduce(self, func):
        out = C.c_void_p()
        _check(_lib.weld_object_new_reduce(self._h, wb.FUNC[func], C.byref(out)))
        return Scalar(out, self.dtype, (self,))

    def sum(self): return self._reduce("add")
    def prod(self): return self._reduce("mul")
    def min(self): return self._reduce("min")
    def max(self): return self._reduce("max")

    def count(self):
        ones = _map([self], [("const", "i64", -1, -1, -1, 1)], "i64")
        return ones._reduce("add")


class ScalarExpr:
    """Arithmetic over lazily evaluated scalars and constants (`s.sum() / s.count()`): nothing of
    its own to evaluate; it becomes part of the map that combines it with a vector, in which every
    scalar it mentions is a dependency."""

    def __init__(self, dtype, tree):
        self.dtype, self.tree = dtype, tree          # tree: ("scalar", Scalar) | ("const", v) | (code, dtype, args...)

    @staticmethod
    def of(x, dtype):
        if isinstance(x, ScalarExpr):
            return x
        if isinstance(x, Scalar):
            return ScalarExpr(x.dtype, ("scalar", x))
        return ScalarExpr(dtype, ("const", x))

    def _bin(self, code, other, reflect=False):
        o = ScalarExpr.of(other, self.dtype)
        assert o.dtype == self.dtype, "no implicit casts: use .cast()"
        a, b = (o, self) if reflect else (self, o)
        return ScalarExpr(self.dtype, (code, self.dtype, a, b))

    def __add__(self, o): return self._bin("add", o)
    def __radd__(self, o): return self._bin("add", o, True)
    def __sub__(self, o): return self._bin("sub", o)
    def __rsub__(self, o): return self._bin("sub", o, True)
    def __mul__(self, o): return self._bin("mul", o)
    def __rmul__(self, o): return self._bin("mul", o, True)
    def __truediv__(self, o): return self._bin("div", o)
    def __rtruediv__(self, o): return self._bin("div", o, True)
    def __neg__(self): return ScalarExpr(self.dtype, ("neg", self.dtype, self))
    def sqrt(self): return ScalarExpr(self.dtype, ("sqrt", self.dtype, self))
    def cast(self, dtype): return ScalarExpr(dtype, ("cast", dtype, self))


class Scalar(Obj):
    """A lazily evaluated scalar (the result of a reduction).  It can be evaluated, and it can be an
    operand of elementwise operators on vectors (`x - x.sum() / x.count()`): evaluation then runs
    the loop that computes it first and the loop that reads it afterwards, on the device."""

    def _e(self): return ScalarExpr.of(self, self.dtype)
    def __add__(self, o): return self._e() + o
    def __radd__(self, o): return o + self._e()
    def __sub__(self, o): return self._e() - o
    def __rsub__(self, o): return o - self._e()
    def __mul__(self, o): return self._e() * o
    def __rmul__(self, o): return o * self._e()
    def __truediv__(self, o): return self._e() / o
    def __rtruediv__(self, o): return o / self._e()
    def __neg__(self): return -self._e()
    def sqrt(self): return self._e().sqrt()
    def cast(self, dtype): return self._e().cast(dtype)


def _with_scalars(vec, code, other, reflect, rt):
    """`vec <code> expression over scalars` as one map whose dependencies are the vector and every
    scalar the expression mentions."""
    expr = ScalarExpr.of(other, vec.dtype)
    assert expr.dtype == vec.dtype, "no implicit casts: use .cast()"
    deps, ops = [vec], [("col", vec.dtype, 0, -1, -1, 0)]

    def emit(e):
        t = e.tree
        if t[0] == "scalar":
            for k, d in enumerate(deps):
                if d is t[1]:
                    break
            else:
                deps.append(t[1])
                k = len(deps) - 1
            ops.append(("col", e.dtype, k, -1, -1, 0))
        elif t[0] == "const":
            ops.append(("const", e.dtype, -1, -1, -1, t[1]))
        else:
            args = [emit(a) for a in t[2:]] + [-1, -1]
            ops.append((t[0], t[1], args[0], args[1], -1, 0))
        return len(ops) - 1

    s = emit(expr)
    a, b = (s, 0) if reflect else (0, s)
    ops.append((code, rt, a, b, -1, 0))
    return _map(deps, ops, rt)


class Dict(Obj):
    def __init__(self, handle, key_types, val_types, func, capacity, keep):
        super().__init__(handle, None, keep)
        self.key_types, self.val_types, self.func, self.capacity = key_types, val_types, func, capacity


def groupby(keys, vals, func="add", capacity=1024):
    kh = (C.c_void_p * len(keys))(*[k._h for k in keys])
    vh = (C.c_void_p * len(vals))(*[v._h for v in vals])
    out = C.c_void_p()
    _check(_lib.weld_object_new_groupby(kh, len(keys), vh, len(vals), wb.FUNC[func], capacity, C.byref(out)))
    return Dict(out, [k.dtype for k in keys], [v.dtype for v in vals], func, capacity, tuple(keys) + tuple(vals))


class _Shape:
    """Builder descriptions of the roots, in the form binding.Result reads results back with."""

    def __init__(self, roots):
        self.builders = []
        for r in roots:
            if isinstance(r, Vec):
                self.builders.append({"kind": "vecbuilder", "type": r.dtype})
            elif isinstance(r, Scalar):
                self.builders.append({"kind": "merger", "type": r.dtype})
            else:
                self.builders.append({"kind": "dictmerger", "key_types": r.key_types, "val_types": r.val_types,
                                      "func": r.func, "capacity": r.capacity})


def evaluate(*roots, mode="fused", stream=None, memory_limit=0, tune=None):
    """Fuse everything below `roots` into one loop and run it; returns a binding.Result whose
    entry i belongs to roots[i]."""
    if stream is None:
        stream = torch.cuda.current_stream().cuda_stream
    conf = wb.Conf()
    conf.stream = stream
    conf.mode = wb.MODE[mode]
    conf.memory_limit = memory_limit
    for k, v in (tune or {}).items():
        setattr(conf.tune, k, int(v))
    handles = (C.c_void_p * len(roots))(*[r._h for r in roots])
    out = C.c_void_p()
    _check(_lib.weld_object_evaluate(handles, len(roots), C.byref(conf), C.byref(out)))
    return wb.Result(out, _Shape(roots), (roots,))


def describe(*roots):
    """The fused loop in the notation of the paper's listings (no GPU needed)."""
    handles = (C.c_void_p * len(roots))(*[r._h for r in roots])
    need = _lib.weld_object_describe(handles, len(roots), None, 0)
    if need < 0:
        raise wb.WeldError(wb.ERR_INVALID_ARG, _lib.weld_last_error().decode())
    buf = C.create_string_buffer(need)
    _lib.weld_object_describe(handles, len(roots), buf, need)
    return buf.value.decode()
