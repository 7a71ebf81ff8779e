"""Host-side checks of the C ABI that need no GPU: the library loads, exports every
declared symbol, validates loop bodies (Sec. 3.2: typed IR, linear builders) and can
generate and compile kernels for gfx950 on a machine without the device."""
import ctypes
import os
import re

import pytest

from workloads import configs
from workloads.ir import Program

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
LIB = os.path.join(ROOT, "paper_1709_06416_amd", "libweldhip.so")

pytestmark = pytest.mark.skipif(not os.path.exists(LIB), reason="libweldhip.so not built (python -m paper_1709_06416_amd.build)")


@pytest.fixture(scope="module")
def wb():
    from paper_1709_06416_amd import binding
    return binding


def test_every_declared_symbol_is_exported(wb):
    names = set()
    inc = os.path.join(ROOT, "include")
    for fn in os.listdir(inc):
        text = open(os.path.join(inc, fn)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names |= set(re.findall(r"\b(weld_[a-z0-9_]+)\s*\(", text))
    assert "weld_fused_for" in names and len(names) >= 15
    lib = ctypes.CDLL(LIB)
    for n in sorted(names):
        assert hasattr(lib, n), n


@pytest.mark.parametrize("name", list(configs.PROGRAMS) + list(configs.EXAMPLES))
def test_standard_loops_validate(wb, name):
    make = configs.PROGRAMS.get(name) or configs.EXAMPLES[name]
    st, msg = wb.validate(make())
    assert st == wb.OK, msg


def test_linearity_violation_is_rejected(wb):
    p = Program(["i64"])
    m = p.merger("i64", "add")
    p.merge(m, p.col(0))
    p.merge(m, p.col(0))                      # the same builder consumed twice
    st, msg = wb.validate(p)
    assert st == wb.ERR_LINEARITY and "builder 0" in msg


def test_type_errors_are_rejected(wb):
    p = Program(["i32", "f64"])
    p.ops.append(("add", "f64", p.col(0), p.col(1)))          # i32 + f64 without a cast
    p.merge(p.merger("f64", "add"), len(p.ops) - 1)
    assert wb.validate(p)[0] == wb.ERR_TYPE

    p = Program(["f64"])
    p.merge(p.merger("i64", "add"), p.col(0))                  # f64 value into an i64 merger
    assert wb.validate(p)[0] == wb.ERR_TYPE

    p = Program(["f64"])
    p.merge(p.merger("f64", "add"), p.col(0), pred=p.col(0))   # predicate is not bool
    assert wb.validate(p)[0] == wb.ERR_TYPE

    p = Program(["i32"])
    p.ops.append(("lt", "bool", p.col(0), p.const("i64", 3)))  # compare i32 with i64
    p.merge(p.merger("i32", "add"), 0, pred=len(p.ops) - 1)
    assert wb.validate(p)[0] == wb.ERR_TYPE


def test_malformed_bodies_are_rejected(wb):
    p = Program(["i64"])
    p.ops.append(("col", "i64", 3))                            # undeclared column
    p.merge(p.merger("i64", "add"), 0)
    assert wb.validate(p)[0] == wb.ERR_INVALID_ARG

    p = Program(["i64"])
    p.ops.append(("add", "i64", 0, 1))                         # operand is not an earlier op
    p.merge(p.merger("i64", "add"), 0)
    assert wb.validate(p)[0] == wb.ERR_INVALID_ARG

    p = Program(["i64"])
    p.merge(p.merger("i64", "add"), p.bin("mod", p.col(0), p.const("i64", 0)))   # mod by constant 0
    assert wb.validate(p)[0] == wb.ERR_INVALID_ARG

    p = Program(["f64"])
    p.merge(p.dictmerger(["f64"], ["i64"], "add", 8), [p.const("i64", 1)], keys=[p.col(0)])  # f64 key
    assert wb.validate(p)[0] == wb.ERR_UNSUPPORTED

    p = Program(["i64"])
    p.merge(p.dictmerger(["i64", "i8"], ["i64"], "add", 8), [p.const("i64", 1)],
            keys=[p.col(0), p.un("cast", p.col(0), to="i8")])                    # 72-bit key struct
    assert wb.validate(p)[0] == wb.ERR_UNSUPPORTED


def test_merger_only_loops_finish_in_the_loop_kernel(wb):
    """The single-launch form: partials exchanged at device scope, one arrival per work-group, the last
    one folds; loops with any other builder, and the form switched off, keep the separate kernels."""
    src = wb.generated_source(configs.program_c1())
    assert "w_arrive_last(a.arrive)" in src and "w_publish_partial(a.b0_part" in src and "*a.b0_res = (double)r" in src
    assert "(int*)(a.arrive + 2)" in src
    off = wb.generated_source(configs.program_c1(), tune={"single_launch": -1})
    assert "w_arrive_last(a.arrive)" not in off and "w_store_partial(a.b0_part" in off and "(int*)(a.ctl + 2)" in off
    assert "w_arrive_last(a.arrive)" not in wb.generated_source(configs.program_c2())
    assert "w_arrive_last(a.arrive)" not in wb.generated_source(configs.program_c4())


def test_tables_choose_their_hash_by_size_and_slices_follow_the_table(wb):
    """Host logic read off the generated text: a dictionary of millions of keys queues its merges by slice of
    the global table, and the slice of a key comes from the TABLE's hash of it (which depends on the table's
    size), not from a hash of its own."""
    from workloads import joins
    src = wb.generated_source(joins.program_build(3_000_000))
    assert "#define W_SPILL_BY_SLOT 1" in src and "#define W_SPILL_SLICE_BITS 13" in src and "#define W_SPILL_PARTS 1024" in src
    assert "w_table_hash_slot(kbits, (u32)W_SPILL_PARTS << W_SPILL_SLICE_BITS) >> W_SPILL_SLICE_BITS" in src
    assert "if (slots >= (1u << 21))" in src
    small = wb.generated_source(configs.program_c5())
    assert "W_SPILL_BY_SLOT 1" not in small


def test_planner_chooses_the_vecmerger_strategy_by_length(wb):
    """Host logic read off the generated text: an LDS copy up to 8192 cells, LDS copies of ranges (every range
    scanning all rows) up to 16384 cells for a loop with no other builder, queues by range of cells beyond -
    at most 256 ranges up to 2^21 cells, ranges of 8192 cells above; a tile's entries sorted in LDS where they
    are 2 bytes or tiles are small -, device atomics on request and where the queues are ruled out."""
    def count(length, tune=None, second=False):
        p = Program(["i32"])
        p.merge(p.vecmerger("i64", "add", length), [p.const("i64", 1)], keys=[p.un("cast", p.col(0), to="i64")])
        if second:
            p.merge(p.merger("i64", "add"), p.un("cast", p.col(0), to="i64"))
        return wb.generated_source(p, tune=tune)
    assert "__shared__ i64 v0_l[8192]" in count(8192)
    assert "range_lo" in count(16384) and "v0_qn" not in count(16384)
    assert "v0_qn[128]" in count(32768) and "v0_qn[64]" in count(16384, second=True) and "range_lo" not in count(16384, second=True)
    src = count(1 << 20)
    assert "__shared__ u32 v0_qn[256]" in src and "(u64)ix >> 12" in src and "w_gstore_u16((unsigned short*)a.b0_log + at, (unsigned short)((u32)ix & 4095u))" in src
    # a full segment: combined in the work-group's LDS table, which goes to the result at the end
    assert "else w_vecm_overflow<0>(v0_ot, v0_ov, (u32)ix, (i64)(o).v0_0, a.b0_out)" in src
    assert "if (v0_ot[q] != W_VQ_NONE) w_atomic<0>(a.b0_out + v0_ot[q], v0_ov[q], 1);" in src
    assert "WELD_MERGE_TILE(o, vq_e[u * W_V + k], vq_v[u * W_V + k]);" in src and "__shared__ u32 v0_st[W_TILE];" in src and "u32 c[1], mine = 0;" in src
    unsorted = count(1 << 20, tune={"vecmerger_strategy": 6})
    assert "WELD_MERGE_TILE" not in unsorted and "w_gstore_u16((unsigned short*)a.b0_log + at" in unsorted and "sg" not in unsorted
    assert "v0_qn[132]" in count(65 * 1024 + 1024) and "(u64)ix >> 9" in count(65 * 1024 + 1024)
    big = count(1 << 24)
    assert "v0_qn[2048]" in big and "WELD_MERGE_TILE" in big and "u32 c[2], mine = 0;" in big
    assert "v0_qn[8192]" in count(1 << 26) and "WELD_MERGE_TILE" not in count(1 << 26)      # (four arrays of 8192 words and the staging: too much LDS)
    beside = Program(["i64"])            # (an LDS dictionary beside it leaves no room for the staging array)
    beside.merge(beside.vecmerger("i64", "add", 100_000), [beside.const("i64", 1)], keys=[beside.bin("mod", beside.col(0), beside.const("i64", 100_000))])
    beside.merge(beside.dictmerger(["i64"], ["i64"], "add", 100_000), [beside.const("i64", 1)], keys=[beside.col(0)])
    assert "v0_qn" in wb.generated_source(beside) and "WELD_MERGE_TILE" not in wb.generated_source(beside)
    for tune in ({"vecmerger_strategy": 3}, {"vecmerger_strategy": -1}, {"dict_spill": -1}):
        off = count(1 << 20, tune=tune)
        assert "v0_qn" not in off and "w_atomic<0>(a.b0_out + ix" in off
    valued = Program(["i64", "f64"])
    valued.merge(valued.vecmerger("f64", "max", 100_000), [valued.col(1)], keys=[valued.col(0)])
    vsrc = wb.generated_source(valued)          # (entries with a value: 8 + 2 bytes in two arrays per segment, sorted in tiles of 8192 rows)
    assert "w_gstore1((u64*)sg + pos, w_bits((double)(o).v0_0));" in vsrc
    assert "w_gstore_u16((unsigned short*)(sg + 8 * a.b0_qcap) + pos, (unsigned short)((u32)ix & 511u));" in vsrc
    assert "__shared__ u64 v0_sv[W_TILE];" in vsrc and "#define W_U 4" in vsrc and "#define W_V 2" in vsrc


def test_vecbuilders_under_one_predicate_share_the_look_back(wb):
    """Four compacting vecbuilders, three of them under the same predicate: two look-backs a tile, the first builder
    of a predicate writes the lengths of all, each builder stores at the prefix of its predicate's first."""
    p = Program(["i64", "f64", "i32"])
    pred = p.bin("gt", p.col(0), p.const("i64", 0))
    p.merge(p.vecbuilder("i64"), p.col(0), pred=pred)
    p.merge(p.vecbuilder("f64"), p.col(1), pred=pred)
    p.merge(p.vecbuilder("i32"), p.col(2), pred=p.bin("lt", p.col(2), p.const("i32", 5)))
    p.merge(p.vecbuilder("i32"), p.col(2), pred=pred)
    src = wb.generated_source(p)
    body = src[src.index('extern "C" __global__'):]
    assert body.count("w_lookback(") == 2 and "w_lookback(a.b0_desc" in body and "w_lookback(a.b2_desc" in body
    for b in (0, 1, 2, 3):
        assert body.count("*a.b%d_len = ex + tot;" % b) == 1
    assert body.count("i64 base = s_pfx[0];") == 3 and body.count("i64 base = s_pfx[2];") == 1


def test_planner_overlaps_tiles_only_where_the_registers_allow(wb):
    """Host logic only: which compacting loops load the next tile's columns ahead, read off the generated text."""
    c5 = wb.generated_source(configs.program_c5())
    assert "s_tile[2]" in c5 and "w_lookback_publish(" in c5 and "w_lookback_resolve(" in c5
    assert "s_tile[2]" not in wb.generated_source(configs.program_c5(), tune={"tile_pipeline": -1})
    grouped = wb.generated_source(configs.program_group_by_zip())      # key, wide value and first probes: too many registers
    assert "s_tile[2]" not in grouped and "w_lookback(" in grouped
    assert "s_tile[2]" in wb.generated_source(configs.program_group_by_zip(), tune={"tile_pipeline": 1})
    p = Program(["i64"])                                                # compaction alone: nothing to hide the loads behind
    p.merge(p.vecbuilder("i64"), p.col(0), pred=p.bin("gt", p.col(0), p.const("i64", 0)))
    assert "s_tile[2]" not in wb.generated_source(p)


def test_scalars_from_outside_the_loop_validate_and_reach_the_kernel_as_one_load(wb):
    p = Program(["f64", "f64", "i64"])
    x, s, c = p.col(0), p.scalar(1), p.scalar(2)
    p.merge(p.vecbuilder("f64"), p.bin("sub", x, p.bin("div", s, p.un("cast", c, "f64"))))
    st, msg = wb.validate(p)
    assert st == wb.OK, msg
    src = wb.generated_source(p)
    assert "const double sc1 = a.s1[0];" in src and "const i64 sc2 = a.s2[0];" in src      # read once per thread, not per row
    assert "a.c1" not in src and "a.c2" not in src                                       # and never streamed as vectors

    q = Program(["i64"])
    q.merge(q.merger("i64", "add"), q.bin("add", q.col(0), q.scalar(0)))                 # one entry, both ways
    st, msg = wb.validate(q)
    assert st == wb.ERR_INVALID_ARG and "column 0" in msg
    q = Program(["i64"])
    q.ops.append(("scalar", "f64", 0))                                                   # declared i64
    q.merge(q.merger("f64", "add"), 0)
    assert wb.validate(q)[0] == wb.ERR_TYPE
    q = Program(["i64"])
    q.ops.append(("scalar", "i64", 2))                                                   # not in the list
    q.merge(q.merger("i64", "add"), 0)
    assert wb.validate(q)[0] == wb.ERR_INVALID_ARG


def test_generated_source_has_one_statement_per_operator(wb):
    prog = configs.program_c3()
    src = wb.generated_source(prog)
    body = src[src.index("void weld_row("):src.index("#define WELD_MERGE")]
    assert len(re.findall(r"^\s+const \w[\w ]* t\d+ = ", body, flags=re.M)) == len(prog.ops)
    assert "weld_fused_" in src and "w_block_reduce" in src
    # constants are emitted bit-exactly
    assert "0x3fa999999999999a" in src            # 0.05


def test_planner_variants_of_a_compacting_loop_with_a_large_dictionary(wb):
    """Host logic only: which merge-phase form the generator picks, read off the generated text."""
    c5 = configs.program_c5()
    src = wb.generated_source(c5)
    # the first probes of a lane's rows are issued together and the hits settled in straight-line code;
    # the rest is queued per wavefront by one loop over the lane's rows
    assert "#define WELD_DRAIN()" in src and "WELD_MERGE_HIT(r, fs[j], fc[j], miss)" in src
    assert "WELD_MERGE_QUEUE(r, miss)" in src and '_Pragma("unroll 1")' in src
    # a count under a key that provably fits 32 bits (x mod 100000): compact cells, twice the slots, 8-byte queue entries
    assert "__shared__ u32 d1_ck[16384]" in src and "w_compact_entry(kb" in src
    general = wb.generated_source(c5, tune={"dict_compact": -1})
    assert "__shared__ u64 d1_lk[8192]" in general and "w_compact_entry(kb" not in general
    # the cleaned code fits 32 bits too: it is held and staged in one register and widened at the store
    assert "typedef int mt4_t" in src and "(i64)stg[e]" in src
    # the merged value is the constant 1: queue entries hold the key only (128 per wavefront)
    assert "dq_n + add > 128" in src
    # division by a constant: wavefront-wide shortcut in full tiles only
    assert "w_mod_const<100000ll, W_CONV>" in src
    assert "weld_row<true>(r0 + u * W_UNIT + k" in src and "if (i < a.n) { weld_row<false>(i" in src
    plain = wb.generated_source(c5, tune={"dict_defer": -1})
    assert "WELD_DRAIN" not in plain and "WELD_MERGE(o[u][k])" in plain
    rolled = wb.generated_source(c5, tune={"dict_defer": -1, "merge_loop": 1})
    assert "WELD_DRAIN" not in rolled and "WELD_MERGE_MEM(r)" in rolled
    # two merged values that are not constants: three words per entry, 42 < 64 entries fit the wavefront's
    # share of the staging buffer, so nothing is queued
    p = Program(["i64", "f64", "i64"])
    pred = p.bin("gt", p.col(1), p.const("f64", 0.0))
    p.merge(p.vecbuilder("f64"), p.col(1), pred=pred)
    p.merge(p.dictmerger(["i64"], ["f64", "i64"], "add", 50_000), [p.col(1), p.col(2)], keys=[p.col(0)], pred=pred)
    assert "WELD_DRAIN" not in wb.generated_source(p)
    # divisors that are not small positive constants keep the plain operator
    q = Program(["i64", "i64"])
    q.merge(p_b := q.vecbuilder("i64"), q.bin("div", q.col(0), q.col(1)))
    q.merge(q.vecbuilder("i64"), q.bin("mod", q.col(0), q.const("i64", 2**31)))
    q.merge(q.vecbuilder("i64"), q.bin("mod", q.col(0), q.const("i64", -7)))
    body = wb.generated_source(q)
    body = body[body.index("void weld_row("):body.index("#define WELD_MERGE")]
    assert "w_div_const<" not in body and "w_mod_const<" not in body
    assert p_b == 0


def test_kernels_compile_for_gfx950_without_a_gpu(wb, tmp_path):
    assert wb.lib.weld_set_cache_dir(str(tmp_path).encode()) == wb.OK
    try:
        p = Program(["i32", "f64"])
        pred = p.bin("lt", p.col(0), p.const("i32", 17))
        p.merge(p.vecbuilder("f64"), p.un("sqrt", p.col(1)), pred=pred)
        p.merge(p.merger("f64", "max"), p.col(1))
        wb.precompile(p)
        objs = [f for f in os.listdir(tmp_path) if f.endswith(".hsaco")]
        assert len(objs) == 2                      # aligned and scalar-load variants
        assert all(os.path.getsize(os.path.join(tmp_path, f)) > 1000 for f in objs)
    finally:
        wb.lib.weld_set_cache_dir(os.path.join(ROOT, "paper_1709_06416_amd", "kcache").encode())


def test_i8_products_go_through_the_opaque_helper(wb):
    """The remainder of an 8-bit product by 2: written as plain 8-bit arithmetic the compiler
    turned the product and the remainder's rounding term into one byte dot product with the wrong
    addend.  The generated code forms every 8-bit product behind a helper the optimiser cannot see
    through (checked here on the source); the GPU suite runs products, sums and differences of all
    pairs of i8 values through / and % against the oracle."""
    for consumer in ("mod", "div"):
        p = Program(["i8", "i8"])
        prod = p.bin("mul", p.col(0), p.col(1))
        key = p.bin(consumer, prod, p.const("i8", 2))
        p.merge(p.dictmerger(["i8"], ["i64"], "add", 130), [p.const("i64", 1)], keys=[key])
        p.merge(p.merger("i8", "mul"), p.col(0))
        body = wb.generated_source(p)
        row = body[body.index("void weld_row("):body.index("#define WELD_MERGE")]
        assert row.count("w_mul_i8(") == 1
        # no i8 product is written with the plain operator anywhere in the row function
        for line in row.splitlines():
            if "signed char" in line and " * " in line:
                raise AssertionError("plain 8-bit product: " + line)


# ----------------------------------------------------------------------
# corrupted descriptions
# ----------------------------------------------------------------------
def _corrupt(m, rnd):
    """One random corruption of the marshalled description; returns (label, must_reject)."""
    p = m.program
    nops, nm, nb = len(p.ops), len(p.merges), len(p.builders)
    kind = int(rnd.randint(0, 16))
    bad_index = int(rnd.choice([nops, nops + 7, 1 << 30, -2, -1000, 2**31 - 1, -2**31]))
    if kind == 0:      # operand refers forward / out of range
        cands = [i for i, o in enumerate(p.ops) if o[0] not in ("col", "const", "index")]
        if not cands: return None
        i = int(rnd.choice(cands)); which = str(rnd.choice(["a", "b", "c"]))
        if getattr(m.ops[i], which) < 0 and which != "a": which = "a"
        setattr(m.ops[i], which, int(rnd.choice([i, i + 1, bad_index])))
        return "operand %s of op %d" % (which, i), True
    if kind == 1:
        i = int(rnd.randint(nops)); m.ops[i].opcode = int(rnd.choice([26, 27, 28, 31, 77, -3, 1000, 2**31 - 1]))
        return "opcode of op %d" % i, True
    if kind == 2:
        i = int(rnd.randint(nops)); m.ops[i].type = int(rnd.choice([5, 6, -1, 99, 2**31 - 1]))
        return "type of op %d" % i, True
    if kind == 3:
        cands = [i for i, o in enumerate(p.ops) if o[0] == "col"]
        i = int(rnd.choice(cands)); m.ops[i].a = int(rnd.choice([len(p.columns), 64, -1, 1 << 30, -5]))
        return "column index of op %d" % i, True
    if kind == 4:
        i = int(rnd.randint(nm)); m.merges[i].builder = int(rnd.choice([nb, -1, 1 << 30, 8, -2**31]))
        return "builder of merge %d" % i, True
    if kind == 5:
        i = int(rnd.randint(nm)); m.merges[i].pred = int(rnd.choice([nops, 1 << 30, -2, -77]))
        return "pred of merge %d" % i, True
    if kind == 6:
        i = int(rnd.randint(nm)); m.merges[i].nvals = int(rnd.choice([9, -1, 100, 2**31 - 1, 0]))
        return "nvals of merge %d" % i, True
    if kind == 7:
        i = int(rnd.randint(nm)); m.merges[i].nkeys = int(rnd.choice([5, -1, 100, 2**31 - 1]))
        return "nkeys of merge %d" % i, True
    if kind == 8:
        i = int(rnd.randint(nm)); m.merges[i].val[0] = bad_index if bad_index != -1 else -2
        return "value of merge %d" % i, True
    if kind == 9:
        i = int(rnd.randint(nb)); m.specs[i].kind = int(rnd.choice([5, 6, -1, 99, 2**31 - 1]))
        return "kind of builder %d" % i, True
    if kind == 10:
        i = int(rnd.randint(nb)); m.specs[i].func = int(rnd.choice([4, -1, 99]))
        return "func of builder %d" % i, p.builders[i]["kind"] in ("merger", "dictmerger", "vecmerger")
    if kind == 11:
        cands = [i for i, b in enumerate(p.builders) if b["kind"] in ("dictmerger", "groupbuilder")]
        if not cands: return None
        i = int(rnd.choice(cands)); which = int(rnd.randint(3))
        if which == 0: m.specs[i].capacity = int(rnd.choice([0, -1, -2**62]))
        elif which == 1: m.specs[i].nkeys = int(rnd.choice([0, 5, -1, 2**31 - 1]))
        else: m.specs[i].key_type[0] = int(rnd.choice([4, 0, 7, -1]))      # f64 / bool / invalid key
        return "dictionary spec %d of builder %d" % (which, i), True
    if kind == 12:
        cands = [i for i, b in enumerate(p.builders) if b["kind"] == "vecmerger"]
        if not cands: return None
        i = int(rnd.choice(cands)); m.specs[i].length = int(rnd.choice([0, -1, -2**40]))
        return "vecmerger length of builder %d" % i, True
    if kind == 13:
        m.body.nops = int(rnd.choice([-1, 0, -2**31])); return "nops", True
    if kind == 14:
        m.builder.count = int(rnd.choice([0, -1, 9, 1000, 2**31 - 1])); return "builder count", True
    if kind == 15:
        if nm < 2: return None
        m.merges[1].builder = m.merges[0].builder; return "two merges into one builder", True
    return None


def test_validator_rejects_corrupted_descriptions(wb):
    """Random valid loop descriptions (workloads/random_programs.py) with one field of their C structs
    overwritten: operand, column, builder and merge indices out of range or referring forward,
    unknown opcodes / types / kinds / functions, field counts beyond the arrays, non-positive
    capacities and lengths, negative counts, two merges into one builder.  Every one of them is
    turned down with a status and a message by weld_validate and by the code generator's entry
    (which validates first); none is read out of bounds."""
    import numpy as np
    from workloads import random_programs
    tried = 0
    for seed in range(600):
        rnd = np.random.RandomState(seed)
        prog = random_programs.make(int(rnd.randint(1 << 30)))[0]
        m = wb.Marshalled(prog)
        c = _corrupt(m, rnd)
        if c is None:
            continue
        label, must_reject = c
        buf = ctypes.create_string_buffer(512)
        st = wb.lib.weld_validate(m.col_types, m.ncols, ctypes.byref(m.body), ctypes.byref(m.builder), buf, 512)
        need = wb.lib.weld_generated_source(m.col_types, m.ncols, ctypes.byref(m.body), ctypes.byref(m.builder), None, 0)
        if must_reject:
            assert st != wb.OK and buf.value and need < 0, (seed, label, st, buf.value)
            tried += 1
    assert tried > 400


def test_nested_validator_rejects_corrupted_descriptions(wb):
    """The same for nested loops: range columns, inner type and function, gather vectors, column
    counts, merge counts, and the operands of `lookup` / `outer` overwritten with values out of range."""
    import numpy as np
    from workloads import random_programs as rp
    C = ctypes
    tried = 0
    for seed in range(400):
        rnd = np.random.RandomState(seed)
        nested = rp.make_nested(int(rnd.randint(1 << 30)))[0]
        m = wb.MarshalledNested(nested)
        s = m.struct
        kind = int(rnd.randint(0, 12))
        label = None
        if kind == 0: s.start_col = int(rnd.choice([-1, len(nested.outer.columns), 99, 2**31 - 1])); label = "start_col"
        elif kind == 1: s.end_col = int(rnd.choice([-1, len(nested.outer.columns), 99, -2**31])); label = "end_col"
        elif kind == 2: s.inner_type = int(rnd.choice([0, 1, 2, 5, -1, 99])); label = "inner_type"
        elif kind == 3: s.inner_func = int(rnd.choice([4, -1, 99])); label = "inner_func"
        elif kind == 4: s.ngather = int(rnd.choice([-1, 9, 1000, 2**31 - 1])); label = "ngather"
        elif kind == 5:
            if not nested.gather: continue
            m.gcols[0].type = int(rnd.choice([0, 5, -1, 99])); label = "gather type"
        elif kind == 6:
            m.ocols[0].type = int(rnd.choice([0, 1, 4, 5, -1])); label = "offset column type"
        elif kind == 7:
            cands = [i for i, o in enumerate(nested.inner.ops) if o[0] == "lookup"]
            if not cands: continue
            i = int(rnd.choice(cands)); m.mi.ops[i].a = int(rnd.choice([len(nested.gather), -1, 64, 1 << 30])); label = "lookup vector"
        elif kind == 8:
            cands = [i for i, o in enumerate(nested.inner.ops) if o[0] == "outer"]
            if not cands: continue
            i = int(rnd.choice(cands)); m.mi.ops[i].a = int(rnd.choice([len(nested.outer.columns), -1, 64, 1 << 30])); label = "outer column"
        elif kind == 9:
            s.inner.ncols = int(rnd.choice([-1, 0, 65, 2**31 - 1])); label = "inner ncols"
        elif kind == 10:
            s.outer.ncols = int(rnd.choice([-1, 0, 1, 65, 2**31 - 1])); label = "outer ncols"
        elif kind == 11:
            s.inner_body.nmerges = int(rnd.choice([0, 2, -1, 100])); label = "inner merges"
        buf = C.create_string_buffer(512)
        st = wb.lib.weld_nested_validate(C.byref(s), C.byref(m.mo.builder), buf, 512)
        assert st != wb.OK and buf.value, (seed, label, st)
        tried += 1
    assert tried > 250
