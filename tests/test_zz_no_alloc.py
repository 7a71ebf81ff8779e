"""weld_fused_for_static (the entry point that allocates nothing) against weld_fused_for.

Both run the same kernels; the static one takes its workspace from the library's fixed device
buffer and writes into tensors allocated here.  Every case makes two static calls in a row, the
second on a smaller input, so that what the first call left in the shared buffer (descriptors,
tables, counters, partials) would show if it were not cleared.  Integer, order and key-set outputs
must be identical, f64 sums within 1e-9 relative.
"""
import numpy as np
import pytest
import torch

from tests import parity

from workloads import configs
from workloads.ir import Program

pytestmark = pytest.mark.gpu

NP = {"i8": np.int8, "i32": np.int32, "i64": np.int64, "f64": np.float64}
TT = {"i8": torch.int8, "i32": torch.int32, "i64": torch.int64, "f64": torch.float64}


@pytest.fixture(scope="module")
def wb():
    from paper_1709_06416_amd import binding
    return binding


def _alloc_outputs(prog, n):
    outs = []
    for spec in prog.builders:
        if spec["kind"] == "merger":
            outs.append(torch.full((1,), -77, dtype=torch.int64, device="cuda"))
        elif spec["kind"] == "vecbuilder":
            outs.append(torch.full((max(n, 1),), -77, dtype=TT[spec["type"]], device="cuda"))
        elif spec["kind"] == "vecmerger":
            outs.append(torch.full((spec["length"],), -77, dtype=TT[spec["type"]], device="cuda"))
        else:
            ks = sum(np.dtype(NP[t]).itemsize for t in spec["key_types"])
            vs = sum(np.dtype(NP[t]).itemsize for t in spec["val_types"])
            outs.append((torch.zeros(spec["capacity"] * ks, dtype=torch.uint8, device="cuda"),
                         torch.zeros(spec["capacity"] * vs, dtype=torch.uint8, device="cuda")))
    return outs


def _read_static(prog, outs, status):
    """The static call's results in the shapes binding.Result returns them in."""
    st = status.cpu().numpy()
    assert st[0] == 0, "error bits %d" % st[0]
    got = []
    for b, spec in enumerate(prog.builders):
        cnt = int(st[1 + b])
        if spec["kind"] == "merger":
            assert cnt == 1
            got.append(outs[b].cpu().numpy().view(np.uint8)[:np.dtype(NP[spec["type"]]).itemsize].view(NP[spec["type"]])[0])
        elif spec["kind"] in ("vecbuilder", "vecmerger"):
            got.append(outs[b][:cnt].cpu().numpy())
        else:
            kdt = np.dtype({"names": ["k%d" % i for i in range(len(spec["key_types"]))],
                            "formats": [NP[t] for t in spec["key_types"]]}, align=False)
            vdt = np.dtype({"names": ["v%d" % i for i in range(len(spec["val_types"]))],
                            "formats": [NP[t] for t in spec["val_types"]]}, align=False)
            keys = outs[b][0].cpu().numpy()[:cnt * kdt.itemsize].view(kdt)
            vals = outs[b][1].cpu().numpy()[:cnt * vdt.itemsize].view(vdt)
            kcols = [np.ascontiguousarray(keys[name]) for name in kdt.names]
            vcols = [np.ascontiguousarray(vals[name]) for name in vdt.names]
            order = np.lexsort(tuple(reversed(kcols)))
            got.append(([k[order] for k in kcols], [v[order] for v in vcols]))
    return got


def _read_ordinary(prog, res):
    res.check()
    got = []
    for b, spec in enumerate(prog.builders):
        if spec["kind"] == "merger":
            got.append(res.merger(b))
        elif spec["kind"] in ("vecbuilder", "vecmerger"):
            got.append(res.vec_host(b))
        else:
            got.append(parity.sorted_dict(res, b))
    return got


def _same(prog, a, b, label):
    for k, spec in enumerate(prog.builders):
        tag = "%s builder %d (%s)" % (label, k, spec["kind"])
        x, y = a[k], b[k]
        if spec["kind"] == "merger":
            if spec["type"] == "f64" and spec["func"] in ("add", "mul"):
                assert abs(float(x) - float(y)) <= 1e-9 * abs(float(y)), (tag, x, y)
            else:
                assert x == y, (tag, x, y)
        elif spec["kind"] in ("vecbuilder", "vecmerger"):
            assert len(x) == len(y), (tag, len(x), len(y))
            if spec["kind"] == "vecmerger" and spec["type"] == "f64":
                assert np.all(np.abs(x - y) <= 1e-9 * np.maximum(np.abs(y), np.max(np.abs(y)))), tag
            else:
                assert np.array_equal(x.view(np.uint8), y.view(np.uint8)), tag      # maps: same kernel, same bits
        else:
            assert len(x[0][0]) == len(y[0][0]), (tag, len(x[0][0]), len(y[0][0]))
            for g, w in zip(x[0], y[0]):
                assert np.array_equal(g, w), tag + " keys"
            for t, g, w in zip(spec["val_types"], x[1], y[1]):
                if t == "f64" and spec["func"] in ("add", "mul"):
                    assert np.all(np.abs(g - w) <= 1e-9 * np.abs(w)), tag + " values"
                else:
                    assert np.array_equal(g, w), tag + " values"


def _two_calls(wb, prog, cols, sizes, inits=None, tune=None, label=""):
    n_max = max(sizes)
    outs = _alloc_outputs(prog, n_max)
    status = torch.full((1 + wb.MAX_BUILDERS,), -5, dtype=torch.int64, device="cuda")
    for n in sizes:
        part = [c[:n] for c in cols]
        res = wb.fused_for(prog, part, inits=inits, tune=tune)          # also loads the loop's kernel
        want = _read_ordinary(prog, res)
        res.free()
        before = wb.lib.weld_pool_bytes()
        wb.fused_for_static(prog, part, outs, status, inits=inits, tune=tune)
        torch.cuda.synchronize()
        assert wb.lib.weld_pool_bytes() == before                        # nothing taken from the pool
        _same(prog, _read_static(prog, outs, status), want, "%s n=%d" % (label, n))


@pytest.mark.parametrize("name,sizes", [
    ("C1", (300_007, 70_001)),          # two mergers: partials of a larger grid left behind
    ("C2", (70_001, 4_097)),            # vectors written in place
    ("C3", (300_007, 1)),
    ("C4", (300_007, 70_001)),          # register dictionary, global table of 64 slots
    ("C5", (700_001, 70_001)),          # look-back descriptors, LDS dictionary, spill queues, extraction
])
def test_two_static_calls_match_the_ordinary_entry_point(wb, name, sizes):
    prog = configs.PROGRAMS[name]()
    cols = configs.make_columns(name, max(sizes), device="cuda")
    _two_calls(wb, prog, cols, sizes, label=name)


def test_static_call_with_global_dictionary_and_vecmerger(wb):
    # dictionary through device atomics only, and a vecmerger with an initial vector
    p = Program(["i64", "f64"])
    x, y = p.col(0), p.col(1)
    key = p.bin("mod", x, p.const("i64", 5000))
    pred = p.bin("gt", y, p.const("f64", 0.25))
    p.merge(p.dictmerger(["i64"], ["i64", "f64"], "add", 5000), [p.const("i64", 1), y], keys=[key], pred=pred)
    idx = p.bin("mod", x, p.const("i64", 1000))
    p.merge(p.vecmerger("i64", "add", 1000), [p.const("i64", 2)], keys=[idx], pred=None)
    n = 200_003
    g = torch.Generator(device="cpu").manual_seed(11)
    cols = [torch.randint(0, 10 ** 9, (n,), generator=g, dtype=torch.int64).cuda(),
            torch.rand(n, generator=g, dtype=torch.float64).cuda()]
    init = torch.arange(1000, dtype=torch.int64, device="cuda")
    _two_calls(wb, p, cols, (n, 30_011), inits={1: init}, tune={"dict_strategy": 3}, label="global dict")
    _two_calls(wb, p, cols, (n, 30_011), inits={1: init}, label="lds dict")


def test_static_call_with_a_vecmerger_queued_by_range(wb):
    # a vecmerger beyond one LDS copy: its queues lie in the fixed workspace (segments of the larger call's grid are
    # left behind for the smaller one), with a value column and with a constant
    n = 500_009
    g = torch.Generator(device="cpu").manual_seed(12)
    cols = [torch.randint(0, 60_000, (n,), generator=g, dtype=torch.int64).cuda(),
            torch.randint(-9, 9, (n,), generator=g, dtype=torch.int64).cuda()]
    init = torch.arange(60_000, dtype=torch.int64, device="cuda")
    p = Program(["i64", "i64"])
    p.merge(p.vecmerger("i64", "add", 60_000), [p.col(1)], keys=[p.col(0)], pred=p.bin("ne", p.col(1), p.const("i64", 3)))
    _two_calls(wb, p, cols, (n, 40_013), inits={0: init}, label="queued vecmerger, values")
    c = Program(["i64", "i64"])
    c.merge(c.vecmerger("i64", "max", 60_000), [c.const("i64", 7)], keys=[c.col(0)])
    _two_calls(wb, c, cols, (n, 40_013), inits={0: init}, label="queued vecmerger, constant")


def test_static_call_refuses_what_it_cannot_do(wb):
    status = torch.zeros(1 + wb.MAX_BUILDERS, dtype=torch.int64, device="cuda")
    # a loop that never ran through the ordinary entry point has no loaded kernel
    p = Program(["i64"])
    p.merge(p.merger("i64", "max"), p.bin("mul", p.col(0), p.const("i64", 12345)))
    col = torch.arange(1000, dtype=torch.int64, device="cuda")
    out = [torch.zeros(1, dtype=torch.int64, device="cuda")]
    with pytest.raises(wb.WeldError) as e:
        wb.fused_for_static(p, [col], out, status)
    assert e.value.status == wb.ERR_NOT_READY
    wb.fused_for(p, [col]).check().free()
    wb.fused_for_static(p, [col], out, status)
    torch.cuda.synchronize()
    assert int(out[0][0]) == 999 * 12345 and int(status[0]) == 0 and int(status[1]) == 1
    # an output with too little room
    q = Program(["i64"])
    q.merge(q.vecbuilder("i64"), q.col(0), pred=q.bin("gt", q.col(0), q.const("i64", 10)))
    with pytest.raises(wb.WeldError) as e:
        wb.fused_for_static(q, [col], [torch.zeros(999, dtype=torch.int64, device="cuda")], status)
    assert e.value.status == wb.ERR_INVALID_ARG
    # a dictionary whose table is larger than the fixed workspace
    d = Program(["i64"])
    d.merge(d.dictmerger(["i64"], ["i64"], "add", 4_000_000), [d.const("i64", 1)], keys=[d.col(0)])
    big = (torch.zeros(8 * 4_000_000, dtype=torch.uint8, device="cuda"), torch.zeros(8 * 4_000_000, dtype=torch.uint8, device="cuda"))
    wb.fused_for(d, [col]).check().free()
    with pytest.raises(wb.WeldError) as e:
        wb.fused_for_static(d, [col], [big], status)
    assert e.value.status == wb.ERR_OOM
    # groupbuilders are refused
    gp = Program(["i64"])
    gp.merge(gp.groupbuilder(["i64"], "i64", 100), [gp.col(0)], keys=[gp.bin("mod", gp.col(0), gp.const("i64", 100))])
    with pytest.raises(wb.WeldError) as e:
        wb.fused_for_static(gp, [col], [big[0]], status)
    assert e.value.status == wb.ERR_UNSUPPORTED
