"""The lazy object API and its fusion pass, without a GPU: the fused loop is inspected
through weld_object_describe (the loop in the notation of the paper's listings)."""
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
LIB = os.path.join(ROOT, "paper_1709_06416_amd", "libweldhip.so")
pytestmark = pytest.mark.skipif(not os.path.exists(LIB), reason="libweldhip.so not built")


@pytest.fixture(scope="module")
def lz():
    from paper_1709_06416_amd import lazy
    return lazy


def _vec(lz, dtype, n=1000, addr=0x10000):
    return lz.Vec.from_pointer(addr, dtype, n)     # never dereferenced on the CPU


def test_pandas_numpy_example_fuses_into_the_printed_loop(lz):
    # Sec. 4.5: filtered = data[data > 500000]; sum = numpy.sum(filtered)
    # must become  for(v0, merger[+,0], (b, x) => if (x > 500000) merge(b, x) else b)
    pop = _vec(lz, "i64")
    total = pop[pop > 500000].sum()
    text = lz.describe(total)
    assert text.count("for(") == 1 and "zip" not in text
    assert "merger[i64,+]" in text
    assert "let t2 = x.0 > 500000;" in text
    assert "if (t2) merge(bs.0, x.0) else bs.0" in text


def test_vertical_and_horizontal_fusion_with_shared_subexpressions(lz):
    x, y = _vec(lz, "f64", addr=0x10000), _vec(lz, "f64", addr=0x20000)
    v = x * y + 1.0
    keep = x > 0.5
    text = lz.describe(v[keep].sum(), v[keep].count(), (x * y)[keep].max())
    assert text.count("for(") == 1 and "zip(v0, v1)" in text
    assert text.count("merge(") == 3
    assert len(re.findall(r"x\.0 \* x\.1", text)) == 1          # x*y is computed once for all three results
    assert len(re.findall(r"x\.0 > 0\.5", text)) == 1


def test_chained_filters_conjoin(lz):
    a = _vec(lz, "i32")
    b = a[a > 3]
    c = b[b < 10]
    text = lz.describe(c.sum())
    assert "&&" in text and text.count("for(") == 1


def test_what_cannot_be_fused_is_reported(lz):
    from paper_1709_06416_amd import binding as wb
    a, b = _vec(lz, "i64", n=1000), _vec(lz, "i64", n=999, addr=0x30000)
    with pytest.raises(wb.WeldError) as e:
        lz.describe((a + b).sum())                     # zip of vectors of different length
    assert "different length" in str(e.value)
    with pytest.raises(wb.WeldError):
        lz.describe((a[a > 1] + a).sum())              # one operand filtered, the other not
    with pytest.raises(wb.WeldError) as e:
        lz.describe(a.sum(), b.sum())                  # two iteration spaces in one evaluation
    assert "different lengths" in str(e.value)
    with pytest.raises(AssertionError):
        a + _vec(lz, "f64")                            # no implicit casts


def test_a_scalar_that_feeds_a_map_is_computed_by_an_earlier_loop(lz):
    # normalisation as a library writes it: the mean needs sum and count, the centred vector the mean
    x = _vec(lz, "f64")
    mean = x.sum() / x.count().cast("f64")
    d = x - mean
    text = lz.describe(d)
    assert text.count("for(") == 2
    first, second = text.split("\n\n")
    assert first.startswith("let {s0, s1} =") and "merger[f64,+], merger[i64,+]" in first
    assert "|v0: vec[f64], s0: f64, s1: i64|" in second and "for(v0," in second      # the scalars are not zipped
    assert "let t3 = f64(s1);" in second and "s0 / t3" in second and "x.0 - t4" in second
    # a third stage, a count written twice folded into one, a root that an earlier stage has computed
    ss = (d * d).sum()
    var = ss / x.count().cast("f64")
    z = d / var.sqrt()
    text = lz.describe(z, ss)
    assert text.count("for(") == 3 and text.count("merger[i64,+]") == 1
    assert "let {s2} =" in text and "sqrt(" in text
    last = text.split("\n\n")[-1]
    assert "vecbuilder[f64]" in last and "merger" not in last                      # the sum of squares is not computed twice


def test_scalar_operands_that_cannot_be_staged_are_reported(lz):
    from paper_1709_06416_amd import binding as wb
    a = _vec(lz, "i64")
    with pytest.raises(AssertionError):
        a - _vec(lz, "f64").sum()                      # no implicit casts, for scalars either
    s = a.sum()
    ops = (wb.Op * 2)()
    ops[0].opcode, ops[0].type, ops[0].a, ops[0].b, ops[0].c = wb.OPCODE["col"], wb.TYPE_ID["i64"], 0, -1, -1
    ops[1].opcode, ops[1].type, ops[1].a, ops[1].b, ops[1].c = wb.OPCODE["neg"], wb.TYPE_ID["i64"], 0, -1, -1
    import ctypes as C
    out = C.c_void_p()
    handles = (C.c_void_p * 1)(s._h)
    assert wb.lib.weld_object_new_map(handles, 1, ops, 2, C.byref(out)) == wb.OK     # a map over scalars alone is built ...
    roots = (C.c_void_p * 1)(out)
    assert wb.lib.weld_object_describe(roots, 1, None, 0) < 0                         # ... and turned down when fused
    assert "vector" in wb.lib.weld_last_error().decode()
    wb.lib.weld_object_free(out)


def test_groupby_becomes_a_dictmerger(lz):
    k1, k2 = _vec(lz, "i8", addr=0x1000), _vec(lz, "i8", addr=0x2000)
    q, p = _vec(lz, "f64", addr=0x3000), _vec(lz, "f64", addr=0x4000)
    d = lz.groupby([k1, k2], [q, p * (1.0 - q)], "add", 8)
    text = lz.describe(d)
    assert "dictmerger[{2 keys},{2 values},+]" in text and text.count("for(") == 1


def test_corrupted_maps_are_turned_down_at_construction_or_when_fused(lz):
    """weld_object_new_map with one field of its operator list overwritten (operands and dependency
    indices out of range or referring forward, unknown opcodes and types, counts that are not
    positive, a null dependency, operators that do not belong in a map, a result type that differs
    from its operands): an error at construction, or at the latest when the object is fused
    (weld_object_describe validates the fused loop like evaluation does).  Nothing is accepted."""
    import ctypes as C
    import numpy as np
    from paper_1709_06416_amd import binding as wb
    lazy, lib = lz, wb.lib
    for seed in range(300):
        rnd = np.random.RandomState(seed)
        t = str(rnd.choice(["i64", "f64", "i32"]))
        deps = [lazy.Vec.from_pointer(0x10000 * (k + 1), t, 1000) for k in range(int(rnd.randint(1, 4)))]
        nd = len(deps)
        ops = [("col", t, k, -1, -1, 0) for k in range(nd)] + [("const", t, -1, -1, -1, 3)]
        for _ in range(int(rnd.randint(1, 5))):
            a, b = int(rnd.randint(len(ops))), int(rnd.randint(len(ops)))
            ops.append((str(rnd.choice(["add", "mul", "sub", "min"])), t, a, b, -1, 0))
        arr = (wb.Op * len(ops))()
        for i, (code, ty, a, b, c, imm) in enumerate(ops):
            o = arr[i]; o.opcode, o.type, o.a, o.b, o.c = wb.OPCODE[code], wb.TYPE_ID[ty], a, b, c
            if code == "const": o.imm.i64 = 3
        handles = (C.c_void_p * nd)(*[d._h for d in deps])
        nops, ndeps = len(ops), nd
        kind = int(rnd.randint(0, 9)); label = None
        bad = int(rnd.choice([len(ops), 1 << 30, -2, -1000, 2**31 - 1]))
        if kind == 0: arr[len(ops) - 1].a = int(rnd.choice([len(ops) - 1, bad])); label = "operand"
        elif kind == 1: arr[int(rnd.randint(len(ops)))].opcode = int(rnd.choice([26, 77, -3, 2**31 - 1])); label = "opcode"
        elif kind == 2: arr[int(rnd.randint(len(ops)))].type = int(rnd.choice([5, -1, 99])); label = "type"
        elif kind == 3: arr[0].a = int(rnd.choice([nd, 64, -1, 1 << 30])); label = "dep index"
        elif kind == 4: nops = int(rnd.choice([0, -1, -2**31])); label = "nops"
        elif kind == 5: ndeps = int(rnd.choice([0, -1, -5])); label = "ndeps"
        elif kind == 6: handles[0] = None; label = "null dep"
        elif kind == 7: arr[len(ops) - 1].type = wb.TYPE_ID["f64" if t != "f64" else "i64"]; label = "result type differs from operands"
        elif kind == 8: arr[len(ops) - 1].opcode = wb.OPCODE["keyexists"]; label = "probe op in a map"
        out = C.c_void_p()
        st = lib.weld_object_new_map(handles, ndeps, arr, nops, C.byref(out))
        if st == wb.OK:
            need = lib.weld_object_describe((C.c_void_p * 1)(out), 1, None, 0)
            lib.weld_object_free(out)
            assert need < 0, (seed, label)
