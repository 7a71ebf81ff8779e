"""ctypes binding of libweldhip.so: argument marshalling only.

Every step of the loop runs inside the library's kernels; this module turns a
plain-data loop description (columns / ops / builders / merges, see
include/weld_hip.h for their meaning) into the C structs, and copies results
out.  torch is used for device memory and the current stream, nothing else.
There is no CPU fallback: if the library is missing, importing fails loudly.
"""
import ctypes as C
import os

import numpy as np
import torch  # noqa: F401  (imported first: it loads the HIP runtime the library binds to)

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libweldhip.so")
if not os.path.exists(_LIB_PATH):
    raise ImportError("libweldhip.so is not built; run `python -m paper_1709_06416_amd.build` "
                      "(there is no fallback path)")
lib = C.CDLL(_LIB_PATH)

# ---- enums (include/weld_hip.h)
OK, ERR_INVALID_ARG, ERR_TYPE, ERR_LINEARITY, ERR_UNSUPPORTED, ERR_OOM, ERR_CAPACITY, ERR_DEVICE, ERR_NOT_READY = range(9)
STATUS_NAME = ["OK", "INVALID_ARG", "TYPE", "LINEARITY", "UNSUPPORTED", "OOM", "CAPACITY", "DEVICE", "NOT_READY"]
TYPE_ID = {"bool": 0, "i8": 1, "i32": 2, "i64": 3, "f64": 4}
TYPE_NP = {"bool": np.bool_, "i8": np.int8, "i32": np.int32, "i64": np.int64, "f64": np.float64}
TYPE_TORCH = {"i8": torch.int8, "i32": torch.int32, "i64": torch.int64, "f64": torch.float64}
TORCH_TYPE = {v: k for k, v in TYPE_TORCH.items()}
OPCODE = {"col": 0, "const": 1, "index": 2, "neg": 3, "not": 4, "cast": 5, "exp": 6, "log": 7, "sqrt": 8,
          "erf": 9, "add": 10, "sub": 11, "mul": 12, "div": 13, "mod": 14, "min": 15, "max": 16, "lt": 17,
          "le": 18, "gt": 19, "ge": 20, "eq": 21, "ne": 22, "and": 23, "or": 24, "select": 25,
          "lookup": 26, "outer": 27, "inner": 28,      # these three: include/weld_nested.h
          "keyexists": 29, "dictlookup": 30, "scalar": 31}
KIND = {"merger": 0, "vecbuilder": 1, "dictmerger": 2, "vecmerger": 3, "groupbuilder": 4}
FUNC = {"add": 0, "mul": 1, "min": 2, "max": 3}
MODE = {"fused": 0, "unfused": 1}

MAX_KEY, MAX_VAL = 4, 8


class _Imm(C.Union):
    _fields_ = [("i64", C.c_int64), ("f64", C.c_double)]


class Op(C.Structure):
    _fields_ = [("opcode", C.c_int32), ("type", C.c_int32), ("a", C.c_int32), ("b", C.c_int32),
                ("c", C.c_int32), ("reserved", C.c_int32), ("imm", _Imm)]


class Merge(C.Structure):
    _fields_ = [("builder", C.c_int32), ("pred", C.c_int32), ("nkeys", C.c_int32),
                ("key", C.c_int32 * MAX_KEY), ("nvals", C.c_int32), ("val", C.c_int32 * MAX_VAL)]


class Body(C.Structure):
    _fields_ = [("nops", C.c_int32), ("ops", C.POINTER(Op)), ("nmerges", C.c_int32),
                ("merges", C.POINTER(Merge))]


class Col(C.Structure):
    _fields_ = [("data", C.c_void_p), ("type", C.c_int32)]


class Cols(C.Structure):
    _fields_ = [("ncols", C.c_int32), ("col", C.POINTER(Col))]


class BuilderSpec(C.Structure):
    _fields_ = [("kind", C.c_int32), ("func", C.c_int32), ("nkeys", C.c_int32),
                ("key_type", C.c_int32 * MAX_KEY), ("nvals", C.c_int32),
                ("val_type", C.c_int32 * MAX_VAL), ("capacity", C.c_int64), ("length", C.c_int64),
                ("init", C.c_void_p)]


class Tuning(C.Structure):
    _fields_ = [("block_threads", C.c_int32), ("units_per_thread", C.c_int32), ("grid_blocks", C.c_int32),
                ("dict_strategy", C.c_int32), ("lds_dict_slots", C.c_int32), ("spin_limit", C.c_int32),
                ("vecmerger_strategy", C.c_int32), ("lds_filter_words", C.c_int32), ("dict_spill", C.c_int32),
                ("merge_loop", C.c_int32), ("dict_defer", C.c_int32), ("dict_compact", C.c_int32), ("device_math", C.c_int32), ("tile_pipeline", C.c_int32),
                ("single_launch", C.c_int32)]


class Conf(C.Structure):
    _fields_ = [("stream", C.c_void_p), ("mode", C.c_int32), ("flags", C.c_int32),
                ("memory_limit", C.c_int64), ("tune", Tuning)]


class Builder(C.Structure):
    _fields_ = [("count", C.c_int32), ("spec", C.POINTER(BuilderSpec)), ("conf", Conf)]


class Vec(C.Structure):
    _fields_ = [("len", C.c_int64), ("ptr", C.c_void_p)]


class Dict(C.Structure):
    _fields_ = [("keys", Vec), ("values", Vec)]


class Groups(C.Structure):
    _fields_ = [("keys", Vec), ("offsets", Vec), ("values", Vec)]


lib.weld_fused_for.argtypes = [C.POINTER(Cols), C.c_int64, C.POINTER(Body), C.POINTER(Builder),
                               C.POINTER(C.c_void_p)]
lib.weld_fused_for.restype = C.c_int
class DictRef(C.Structure):
    _fields_ = [("result", C.c_void_p), ("builder", C.c_int32)]


lib.weld_fused_for_probe.argtypes = [C.POINTER(Cols), C.c_int64, C.POINTER(DictRef), C.c_int32, C.POINTER(Body),
                                     C.POINTER(Builder), C.POINTER(C.c_void_p)]
lib.weld_fused_for_probe.restype = C.c_int
class Out(C.Structure):
    _fields_ = [("data", C.c_void_p), ("data2", C.c_void_p), ("capacity", C.c_int64)]


lib.weld_fused_for_static.argtypes = [C.POINTER(Cols), C.c_int64, C.POINTER(Body), C.POINTER(Builder), C.POINTER(Out),
                                      C.c_void_p]
lib.weld_fused_for_static.restype = C.c_int
STATIC_SCRATCH_BYTES = 32 << 20
MAX_BUILDERS = 8
lib.weld_result_status.argtypes = [C.c_void_p]
lib.weld_result_status.restype = C.c_int
lib.weld_result_error.argtypes = [C.c_void_p]
lib.weld_result_error.restype = C.c_char_p
lib.weld_result_data.argtypes = [C.c_void_p, C.c_int32]
lib.weld_result_data.restype = C.c_void_p
lib.weld_result_scalar.argtypes = [C.c_void_p, C.c_int32]
lib.weld_result_scalar.restype = C.c_void_p
lib.weld_result_fetch.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_int64, C.c_int64, C.c_int32]
lib.weld_result_fetch.restype = C.c_int
lib.weld_result_elapsed_ms.argtypes = [C.c_void_p, C.POINTER(C.c_float)]
lib.weld_result_elapsed_ms.restype = C.c_int
lib.weld_result_busy_ms.argtypes = [C.c_void_p, C.POINTER(C.c_float)]
lib.weld_result_busy_ms.restype = C.c_int
lib.weld_result_kernel_ms.argtypes = [C.c_void_p, C.POINTER(C.c_float)]
lib.weld_result_kernel_ms.restype = C.c_int
lib.weld_result_kernel_name.argtypes = [C.c_void_p]
lib.weld_result_kernel_name.restype = C.c_char_p
lib.weld_result_kernel_count.argtypes = [C.c_void_p]
lib.weld_result_kernel_count.restype = C.c_int32
lib.weld_result_grid.argtypes = [C.c_void_p]
lib.weld_result_grid.restype = C.c_int64
lib.weld_result_free.argtypes = [C.c_void_p]
lib.weld_result_free.restype = None
lib.weld_precompile.argtypes = [C.POINTER(C.c_int32), C.c_int32, C.POINTER(Body), C.POINTER(Builder)]
lib.weld_precompile.restype = C.c_int
lib.weld_tune_launch.argtypes = [C.POINTER(Cols), C.c_int64, C.POINTER(Body), C.POINTER(Builder), C.POINTER(Tuning),
                                 C.POINTER(C.c_float), C.POINTER(C.c_float)]
lib.weld_tune_launch.restype = C.c_int
lib.weld_set_cache_dir.argtypes = [C.c_char_p]
lib.weld_set_cache_dir.restype = C.c_int
lib.weld_validate.argtypes = [C.POINTER(C.c_int32), C.c_int32, C.POINTER(Body), C.POINTER(Builder),
                              C.c_char_p, C.c_size_t]
lib.weld_validate.restype = C.c_int
lib.weld_generated_source.argtypes = [C.POINTER(C.c_int32), C.c_int32, C.POINTER(Body), C.POINTER(Builder),
                                      C.c_char_p, C.c_int64]
lib.weld_generated_source.restype = C.c_int64
lib.weld_pool_trim.argtypes = []
lib.weld_pool_trim.restype = None
lib.weld_pool_bytes.argtypes = []
lib.weld_pool_bytes.restype = C.c_int64
lib.weld_last_error.argtypes = []
lib.weld_last_error.restype = C.c_char_p
lib.weld_probe_read.argtypes = [C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p]
lib.weld_probe_read.restype = C.c_int
lib.weld_probe_copy.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p]
lib.weld_probe_copy.restype = C.c_int
lib.weld_version.argtypes = []
lib.weld_version.restype = C.c_char_p


class Nested(C.Structure):
    _fields_ = [("n_outer", C.c_int64), ("outer", Cols), ("start_col", C.c_int32), ("end_col", C.c_int32),
                ("n_inner", C.c_int64), ("inner", Cols), ("ngather", C.c_int32), ("gather", C.POINTER(Col)),
                ("gather_len", C.POINTER(C.c_int64)), ("inner_body", Body), ("inner_type", C.c_int32),
                ("inner_func", C.c_int32), ("outer_body", Body), ("range_kind", C.c_int32), ("stride_col", C.c_int32)]


lib.weld_nested_for.argtypes = [C.POINTER(Nested), C.POINTER(Builder), C.POINTER(C.c_void_p)]
lib.weld_nested_for.restype = C.c_int
lib.weld_nested_validate.argtypes = [C.POINTER(Nested), C.POINTER(Builder), C.c_char_p, C.c_size_t]
lib.weld_nested_validate.restype = C.c_int
lib.weld_nested_precompile.argtypes = [C.POINTER(Nested), C.POINTER(Builder)]
lib.weld_nested_precompile.restype = C.c_int


class WeldError(RuntimeError):
    def __init__(self, status, text):
        super().__init__("WELD_ERR_%s: %s" % (STATUS_NAME[status], text))
        self.status = status


class Marshalled:
    """C structs of one loop description; keeps the backing arrays alive."""

    def __init__(self, program, mode="fused", stream=0, memory_limit=0, tune=None, inits=None):
        self.program = program
        nops = len(program.ops)
        inits = inits or {}
        self.inits = inits                               # kept alive with the description
        self.ops = (Op * max(nops, 1))()
        for i, op in enumerate(program.ops):
            o = self.ops[i]
            o.opcode = OPCODE[op[0]]
            o.type = TYPE_ID[op[1]]
            o.a = o.b = o.c = -1
            if op[0] == "const":
                if op[1] == "f64":
                    o.imm.f64 = float(op[2])
                else:
                    o.imm.i64 = int(op[2])
            elif op[0] == "dictlookup":                 # (dict, value field, key fields...)
                o.a, o.reserved = int(op[2]), int(op[3])
                keys = list(op[4:])
                if len(keys) > 2:
                    raise WeldError(ERR_UNSUPPORTED, "probes take dictionaries of one or two key fields")
                o.b = int(keys[0])
                o.c = int(keys[1]) if len(keys) > 1 else -1
            else:
                args = list(op[2:])
                if op[0] == "keyexists" and len(args) > 3:
                    raise WeldError(ERR_UNSUPPORTED, "probes take dictionaries of one or two key fields")
                if len(args) > 0:
                    o.a = int(args[0])
                if len(args) > 1:
                    o.b = int(args[1])
                if len(args) > 2:
                    o.c = int(args[2])
        nm = len(program.merges)
        self.merges = (Merge * max(nm, 1))()
        for i, m in enumerate(program.merges):
            g = self.merges[i]
            g.builder = int(m["builder"])
            g.pred = -1 if m["pred"] is None else int(m["pred"])
            g.nkeys = len(m["keys"])
            g.nvals = len(m["vals"])
            if g.nkeys > MAX_KEY or g.nvals > MAX_VAL:
                raise WeldError(ERR_INVALID_ARG, "too many key/value fields")
            for k, v in enumerate(m["keys"]):
                g.key[k] = int(v)
            for k, v in enumerate(m["vals"]):
                g.val[k] = int(v)
        self.body = Body(nops, self.ops, nm, self.merges)
        nb = len(program.builders)
        self.specs = (BuilderSpec * max(nb, 1))()
        for i, b in enumerate(program.builders):
            s = self.specs[i]
            s.kind = KIND[b["kind"]]
            s.func = FUNC[b.get("func", "add")]
            if b["kind"] == "dictmerger":
                s.nkeys = len(b["key_types"])
                s.nvals = len(b["val_types"])
                if s.nkeys > MAX_KEY or s.nvals > MAX_VAL:
                    raise WeldError(ERR_INVALID_ARG, "too many key/value fields")
                for k, t in enumerate(b["key_types"]):
                    s.key_type[k] = TYPE_ID[t]
                for k, t in enumerate(b["val_types"]):
                    s.val_type[k] = TYPE_ID[t]
                s.capacity = int(b["capacity"])
            elif b["kind"] == "groupbuilder":
                s.nkeys = len(b["key_types"])
                if s.nkeys > MAX_KEY:
                    raise WeldError(ERR_INVALID_ARG, "too many key fields")
                for k, t in enumerate(b["key_types"]):
                    s.key_type[k] = TYPE_ID[t]
                s.nvals = 1
                s.val_type[0] = TYPE_ID[b["type"]]
                s.capacity = int(b["capacity"])
            elif b["kind"] == "vecmerger":
                s.nkeys = 1
                s.key_type[0] = TYPE_ID["i64"]
                s.nvals = 1
                s.val_type[0] = TYPE_ID[b["type"]]
                s.length = int(b["length"])
                t = inits.get(i)
                if t is not None:
                    if (not t.is_cuda or not t.is_contiguous() or t.numel() != s.length
                            or TORCH_TYPE.get(t.dtype) != b["type"]):
                        raise WeldError(ERR_INVALID_ARG, "vecmerger init must be a contiguous CUDA tensor of its type and length")
                    s.init = t.data_ptr()
            else:
                s.nkeys = 0
                s.nvals = 1
                s.val_type[0] = TYPE_ID[b["type"]]
                s.capacity = 0
        self.builder = Builder()
        self.builder.count = nb
        self.builder.spec = self.specs
        self.builder.conf.stream = stream
        self.builder.conf.mode = MODE[mode]
        self.builder.conf.memory_limit = int(memory_limit)
        for k, v in (tune or {}).items():
            setattr(self.builder.conf.tune, k, int(v))
        ncols = len(program.columns)
        self.col_types = (C.c_int32 * max(ncols, 1))(*[TYPE_ID[t] for t in program.columns])
        self.ncols = ncols


class Result:
    """Handle of one evaluated loop (the paper's WeldResult); free() returns its memory."""

    def __init__(self, handle, program, keep):
        self._h = handle
        self._program = program
        self._keep = keep

    def status(self):
        return lib.weld_result_status(self._h)

    def check(self):
        st = self.status()
        if st != OK:
            raise WeldError(st, lib.weld_result_error(self._h).decode())
        return self

    def error(self):
        return lib.weld_result_error(self._h).decode()

    def elapsed_ms(self):
        ms = C.c_float()
        lib.weld_result_elapsed_ms(self._h, C.byref(ms))
        return ms.value

    def kernel_ms(self):
        ms = C.c_float()
        lib.weld_result_kernel_ms(self._h, C.byref(ms))
        return ms.value

    def busy_ms(self):
        ms = C.c_float()
        lib.weld_result_busy_ms(self._h, C.byref(ms))
        return ms.value

    def kernel_name(self):
        return lib.weld_result_kernel_name(self._h).decode()

    def kernel_count(self):
        return lib.weld_result_kernel_count(self._h)

    def grid(self):
        return lib.weld_result_grid(self._h)

    def _fetch_host(self, idx, part, nbytes):
        buf = np.empty(nbytes, dtype=np.uint8)
        if nbytes:
            st = lib.weld_result_fetch(self._h, idx, part, buf.ctypes.data, 0, nbytes, 0)
            if st != OK:
                raise WeldError(st, self.error())
        return buf

    def merger(self, idx):
        self.check()
        t = self._program.builders[idx]["type"]
        return self._fetch_host(idx, 0, np.dtype(TYPE_NP[t]).itemsize).view(TYPE_NP[t])[0]

    def scalar_ref(self, idx):
        """The merger result idx where it lies in device memory, without waiting for it."""
        p = lib.weld_result_scalar(self._h, idx)
        if not p:
            raise WeldError(ERR_INVALID_ARG, "result %d is not a merger" % idx)
        return DevScalar(p, self._program.builders[idx]["type"], self)

    def vec_len(self, idx):
        self.check()
        p = lib.weld_result_data(self._h, idx)
        return C.cast(p, C.POINTER(Vec)).contents.len

    def vec(self, idx):
        """vecbuilder result as a new torch tensor on the GPU (device-to-device copy)."""
        n = self.vec_len(idx)
        t = self._program.builders[idx]["type"]
        out = torch.empty(n, dtype=TYPE_TORCH[t], device="cuda")
        if n:
            st = lib.weld_result_fetch(self._h, idx, 0, out.data_ptr(), 0, n * out.element_size(), 1)
            if st != OK:
                raise WeldError(st, self.error())
        return out

    def vec_host(self, idx):
        n = self.vec_len(idx)
        t = self._program.builders[idx]["type"]
        return self._fetch_host(idx, 0, n * np.dtype(TYPE_NP[t]).itemsize).view(TYPE_NP[t])

    def dict(self, idx):
        """dictmerger result as (key columns, value columns), in the order the library stores them (unspecified)."""
        self.check()
        spec = self._program.builders[idx]
        p = lib.weld_result_data(self._h, idx)
        d = C.cast(p, C.POINTER(Dict)).contents
        n = d.keys.len
        kdt = np.dtype({"names": ["k%d" % i for i in range(len(spec["key_types"]))],
                        "formats": [TYPE_NP[t] for t in spec["key_types"]]}, align=False)
        vdt = np.dtype({"names": ["v%d" % i for i in range(len(spec["val_types"]))],
                        "formats": [TYPE_NP[t] for t in spec["val_types"]]}, align=False)
        keys = self._fetch_host(idx, 0, n * kdt.itemsize).view(kdt)
        vals = self._fetch_host(idx, 1, n * vdt.itemsize).view(vdt)
        kcols = [np.ascontiguousarray(keys[name]) for name in kdt.names]
        vcols = [np.ascontiguousarray(vals[name]) for name in vdt.names]
        return kcols, vcols

    def groups(self, idx):
        """groupbuilder result as (key columns, offsets, values): the values of group g are
        values[offsets[g]:offsets[g+1]]; the order of the groups and of the values inside a group is
        the library's (unspecified)."""
        self.check()
        spec = self._program.builders[idx]
        p = lib.weld_result_data(self._h, idx)
        g = C.cast(p, C.POINTER(Groups)).contents
        ng, nv = g.keys.len, g.values.len
        kdt = np.dtype({"names": ["k%d" % i for i in range(len(spec["key_types"]))],
                        "formats": [TYPE_NP[t] for t in spec["key_types"]]}, align=False)
        vt = TYPE_NP[spec["type"]]
        keys = self._fetch_host(idx, 0, ng * kdt.itemsize).view(kdt)
        offsets = self._fetch_host(idx, 1, (ng + 1) * 8).view(np.int64)
        values = self._fetch_host(idx, 2, nv * np.dtype(vt).itemsize).view(vt)
        kcols = [np.ascontiguousarray(keys[name]) for name in kdt.names]
        return kcols, offsets, values

    def free(self):
        if self._h:
            lib.weld_result_free(self._h)
            self._h = None

    def __del__(self):
        try:
            self.free()
        except Exception:
            pass


class DevScalar:
    """One element in device memory that a later loop reads with the `scalar` operator: the merger
    result of an earlier call (Result.scalar_ref), used in stream order without a host wait."""

    def __init__(self, ptr, dtype, keep=None):
        self.ptr, self.dtype, self._keep = ptr, dtype, keep


def _zipped_columns(program, columns):
    if len(columns) != len(program.columns):
        raise WeldError(ERR_INVALID_ARG, "column count mismatch")
    cols = (Col * max(len(columns), 1))()
    rows = None
    scalars = {op[2] for op in program.ops if op[0] == "scalar"}
    for k, t in enumerate(columns):
        if k in scalars:                          # one element: a DevScalar or a one-element CUDA tensor
            if isinstance(t, DevScalar):
                ptr, dt = t.ptr, t.dtype
            else:
                if not t.is_cuda or t.numel() != 1:
                    raise WeldError(ERR_INVALID_ARG, "a scalar operand is one element in device memory")
                ptr, dt = t.data_ptr(), TORCH_TYPE.get(t.dtype)
            if dt != program.columns[k]:
                raise WeldError(ERR_TYPE, "scalar %d: has type %s, declared %s" % (k, dt, program.columns[k]))
            cols[k].data = ptr
            cols[k].type = TYPE_ID[program.columns[k]]
            continue
        if not t.is_cuda or not t.is_contiguous():
            raise WeldError(ERR_INVALID_ARG, "columns must be contiguous CUDA tensors")
        if TORCH_TYPE.get(t.dtype) != program.columns[k]:
            raise WeldError(ERR_TYPE, "column %d: tensor dtype %s, declared %s" % (k, t.dtype, program.columns[k]))
        if rows is None:
            rows = t.numel()
        elif rows != t.numel():
            raise WeldError(ERR_INVALID_ARG, "columns differ in length")
        cols[k].data = t.data_ptr()
        cols[k].type = TYPE_ID[program.columns[k]]
    return cols, rows


def tune_launch(program, columns, tune=None, memory_limit=0, inits=None, stream=None):
    """weld_tune_launch: times the loop on these columns with several persistent-grid sizes and
    returns (tuning dict to pass as `tune=`, loop-kernel ms of the winner, ms of the library's own choice)."""
    if stream is None:
        stream = torch.cuda.current_stream().cuda_stream
    m = Marshalled(program, stream=stream, memory_limit=memory_limit, tune=tune, inits=inits)
    cols, rows = _zipped_columns(program, columns)
    cs = Cols(len(columns), cols)
    best = Tuning()
    best_ms, default_ms = C.c_float(-1.0), C.c_float(-1.0)
    st = lib.weld_tune_launch(C.byref(cs), rows or 0, C.byref(m.body), C.byref(m.builder), C.byref(best),
                              C.byref(best_ms), C.byref(default_ms))
    if st != OK:
        raise WeldError(st, lib.weld_last_error().decode())
    out = {name: getattr(best, name) for name, _ in Tuning._fields_ if getattr(best, name) != 0}
    return out, best_ms.value, default_ms.value


def fused_for(program, columns, mode="fused", stream=None, memory_limit=0, tune=None, n=None, inits=None, dicts=None):
    """weld_fused_for over torch CUDA tensors; returns a Result (work is only enqueued).
    inits: {builder index: CUDA tensor} initial vectors of vecmergers.
    dicts: [(Result, builder index), ...] dictionaries of earlier calls that the body probes
    (weld_fused_for_probe); the Results are kept alive by the returned one."""
    if stream is None:
        stream = torch.cuda.current_stream().cuda_stream
    if isinstance(program, Marshalled):
        m, program = program, program.program
        if inits:
            raise WeldError(ERR_INVALID_ARG, "a prepared loop carries its initial vectors; pass them to prepare()")
        m.builder.conf.stream = stream
    else:
        m = Marshalled(program, mode=mode, stream=stream, memory_limit=memory_limit, tune=tune, inits=inits)
    cols, rows = _zipped_columns(program, columns)
    if n is None:
        n = rows if rows is not None else 0
    cs = Cols(len(columns), cols)
    out = C.c_void_p()
    if dicts:
        refs = (DictRef * len(dicts))()
        for k, (res, b) in enumerate(dicts):
            refs[k].result = res._h
            refs[k].builder = int(b)
        st = lib.weld_fused_for_probe(C.byref(cs), n, refs, len(dicts), C.byref(m.body), C.byref(m.builder), C.byref(out))
    else:
        st = lib.weld_fused_for(C.byref(cs), n, C.byref(m.body), C.byref(m.builder), C.byref(out))
    if st != OK:
        raise WeldError(st, lib.weld_last_error().decode())
    return Result(out, program, (m, cols, list(columns), inits, dicts))


def fused_for_static(program, columns, outs, status, stream=None, tune=None, n=None, inits=None):
    """weld_fused_for_static: the loop enqueued with the caller's output tensors and no allocation by
    the library.  outs: per builder a CUDA tensor (merger: one 8-byte element; vecbuilder / vecmerger:
    room for the elements) or, for a dictmerger, a pair of uint8 CUDA tensors (packed keys, packed
    values); status: int64 CUDA tensor of 1 + MAX_BUILDERS elements.  Returns nothing: the caller
    waits for the stream and reads `status` and the outputs."""
    if stream is None:
        stream = torch.cuda.current_stream().cuda_stream
    if isinstance(program, Marshalled):
        m, program = program, program.program
        m.builder.conf.stream = stream
    else:
        m = Marshalled(program, stream=stream, tune=tune, inits=inits)
    cols, rows = _zipped_columns(program, columns)
    if n is None:
        n = rows if rows is not None else 0
    cs = Cols(len(columns), cols)
    if status.dtype != torch.int64 or not status.is_cuda or status.numel() < 1 + MAX_BUILDERS:
        raise WeldError(ERR_INVALID_ARG, "status must be an int64 CUDA tensor of 1 + MAX_BUILDERS elements")
    o = (Out * max(len(program.builders), 1))()
    for b, spec in enumerate(program.builders):
        t = outs[b]
        if spec["kind"] == "dictmerger":
            ksize = sum(np.dtype(TYPE_NP[k]).itemsize for k in spec["key_types"])
            vsize = sum(np.dtype(TYPE_NP[v]).itemsize for v in spec["val_types"])
            o[b].data, o[b].data2 = t[0].data_ptr(), t[1].data_ptr()
            o[b].capacity = min(t[0].numel() * t[0].element_size() // ksize, t[1].numel() * t[1].element_size() // vsize)
        else:
            o[b].data = t.data_ptr() if t.numel() else None
            o[b].capacity = t.numel()
    st = lib.weld_fused_for_static(C.byref(cs), n, C.byref(m.body), C.byref(m.builder), o, status.data_ptr())
    if st != OK:
        raise WeldError(st, lib.weld_last_error().decode())


def prepare(program, mode="fused", memory_limit=0, tune=None, inits=None):
    """The C description of a loop, built once: fused_for accepts it in place of the program, so a
    loop that runs many times is not marshalled again per call.  Later changes to the program
    are not seen; calls that share one prepared loop must not overlap on different host threads
    (the stream is written into it per call)."""
    return Marshalled(program, mode=mode, memory_limit=memory_limit, tune=tune, inits=inits)


def _col_array(tensors, types, what):
    cols = (Col * max(len(types), 1))()
    rows = None
    for k, ty in enumerate(types):
        cols[k].type = TYPE_ID[ty]
        if tensors is None:
            continue
        t = tensors[k]
        if not t.is_cuda or not t.is_contiguous():
            raise WeldError(ERR_INVALID_ARG, "%s vectors must be contiguous CUDA tensors" % what)
        if TORCH_TYPE.get(t.dtype) != ty:
            raise WeldError(ERR_TYPE, "%s vector %d: tensor dtype %s, declared %s" % (what, k, t.dtype, ty))
        cols[k].data = t.data_ptr()
        rows = t.numel() if rows is None else rows
    return cols, rows


class MarshalledNested:
    """C structs of a nested loop (workloads.ir.NestedProgram); tensors may be None (validation,
    ahead-of-time compilation)."""

    def __init__(self, nested, outer=None, inner=None, gather=None, stream=0, memory_limit=0, tune=None):
        self.mi = Marshalled(nested.inner)
        self.mo = Marshalled(nested.outer, stream=stream, memory_limit=memory_limit, tune=tune)
        self.ocols, n_outer = _col_array(outer, nested.outer.columns, "outer")
        self.icols, n_inner = _col_array(inner, nested.inner.columns, "inner")
        self.gcols, _ = _col_array(gather, nested.gather, "gather")
        if outer is not None and any(t.numel() != n_outer for t in outer):
            raise WeldError(ERR_INVALID_ARG, "outer vectors differ in length")
        if inner is not None and any(t.numel() != n_inner for t in inner):
            raise WeldError(ERR_INVALID_ARG, "inner vectors differ in length")
        ng = len(nested.gather)
        self.glen = (C.c_int64 * max(ng, 1))(*([t.numel() for t in gather] if gather is not None else [0] * ng))
        self.keep = (outer, inner, gather)
        s = self.struct = Nested()
        s.n_outer = n_outer or 0
        s.outer = Cols(len(nested.outer.columns), self.ocols)
        s.start_col, s.end_col = nested.start_col, nested.end_col
        s.n_inner = n_inner or 0
        s.inner = Cols(len(nested.inner.columns), self.icols)
        s.ngather = ng
        s.gather = self.gcols
        s.gather_len = self.glen
        s.inner_body = self.mi.body
        s.inner_type = TYPE_ID[nested.inner_type]
        s.inner_func = FUNC[nested.inner_func]
        s.outer_body = self.mo.body
        s.range_kind = 1 if getattr(nested, "ranges", "csr") == "any" else 0
        stride_col = getattr(nested, "stride_col", None)
        s.stride_col = -1 if stride_col is None else int(stride_col)


def nested_for(nested, outer, inner, gather, stream=None, memory_limit=0, tune=None):
    """weld_nested_for over torch CUDA tensors; returns a Result for the outer builders."""
    if stream is None:
        stream = torch.cuda.current_stream().cuda_stream
    m = MarshalledNested(nested, outer, inner, gather, stream=stream, memory_limit=memory_limit, tune=tune)
    out = C.c_void_p()
    st = lib.weld_nested_for(C.byref(m.struct), C.byref(m.mo.builder), C.byref(out))
    if st != OK:
        raise WeldError(st, lib.weld_last_error().decode())
    return Result(out, nested.outer, m)


def nested_validate(nested):
    m = MarshalledNested(nested)
    buf = C.create_string_buffer(512)
    st = lib.weld_nested_validate(C.byref(m.struct), C.byref(m.mo.builder), buf, 512)
    return st, buf.value.decode()


def nested_precompile(nested, tune=None):
    m = MarshalledNested(nested, tune=tune)
    st = lib.weld_nested_precompile(C.byref(m.struct), C.byref(m.mo.builder))
    if st != OK:
        raise WeldError(st, lib.weld_last_error().decode())


def validate(program, mode="fused"):
    m = Marshalled(program, mode=mode)
    buf = C.create_string_buffer(512)
    st = lib.weld_validate(m.col_types, m.ncols, C.byref(m.body), C.byref(m.builder), buf, 512)
    return st, buf.value.decode()


def precompile(program, tune=None):
    m = Marshalled(program, tune=tune)
    st = lib.weld_precompile(m.col_types, m.ncols, C.byref(m.body), C.byref(m.builder))
    if st != OK:
        raise WeldError(st, lib.weld_last_error().decode())


def generated_source(program, tune=None):
    m = Marshalled(program, tune=tune)
    need = lib.weld_generated_source(m.col_types, m.ncols, C.byref(m.body), C.byref(m.builder), None, 0)
    if need < 0:
        raise WeldError(ERR_INVALID_ARG, lib.weld_last_error().decode())
    buf = C.create_string_buffer(need)
    lib.weld_generated_source(m.col_types, m.ncols, C.byref(m.body), C.byref(m.builder), buf, need)
    return buf.value.decode()


def probe_read(tensor, stream=None):
    """Launch the streaming-read probe over a CUDA tensor; returns the checksum tensor."""
    if stream is None:
        stream = torch.cuda.current_stream().cuda_stream
    chk = torch.zeros(1, dtype=torch.int64, device="cuda")
    nbytes = tensor.numel() * tensor.element_size() // 16 * 16
    st = lib.weld_probe_read(tensor.data_ptr(), nbytes, chk.data_ptr(), stream)
    if st != OK:
        raise WeldError(st, "probe_read")
    return chk


def probe_copy(dst, src, stream=None):
    if stream is None:
        stream = torch.cuda.current_stream().cuda_stream
    nbytes = src.numel() * src.element_size() // 16 * 16
    st = lib.weld_probe_copy(dst.data_ptr(), src.data_ptr(), nbytes, stream)
    if st != OK:
        raise WeldError(st, "probe_copy")
