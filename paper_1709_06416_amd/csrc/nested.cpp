// weld_nested_for: validation of a `for` nested in a `for` and its un-nesting into two flat
// loops (Sec. 3.2: loops nest; Sec. 5, "Partial GPU Backend": un-nesting turns a nested
// parallel program into a regular one).
//
//   inner loop  -> one flat loop over ALL inner elements with a segmented merger (one cell per
//                  outer element); lookup(v, i) and the current outer element are the two things
//                  its body may read besides its own vectors;
//   outer loop  -> the ordinary fused loop over the outer elements, in which the inner loop's
//                  result is one more zipped vector (the cells).
#include <cstring>

#include "weld_internal.h"

using namespace weld;

namespace {

Error fail(weld_status_t st, const std::string& text) {
    Error e;
    e.status = st;
    e.text = text;
    return e;
}

Error build(const weld_nested_t* in, const weld_builder_t* builders, bool need_data, NestedLoop* NL, NestedData* D) {
    if (!in || !builders) return fail(WELD_ERR_INVALID_ARG, "null argument");
    if (in->n_outer < 0 || in->n_inner < 0) return fail(WELD_ERR_INVALID_ARG, "negative element count");
    if (in->n_outer > 0x7ffffff0ll) return fail(WELD_ERR_UNSUPPORTED, "more than 2^31 outer elements");
    if (in->n_outer == 0 && in->n_inner != 0) return fail(WELD_ERR_INVALID_ARG, "inner elements without an outer element");
    const int no = in->outer.ncols, ni = in->inner.ncols, ng = in->ngather;
    if (no < 2 || no > WELD_MAX_COLS - 1 || !in->outer.col) return fail(WELD_ERR_INVALID_ARG, "outer vectors: 2..15 (start, end, ...)");
    if (ni < 0 || ni > WELD_MAX_COLS || (ni > 0 && !in->inner.col)) return fail(WELD_ERR_INVALID_ARG, "bad inner vector list");
    if (ng < 0 || ng > 8 || (ng > 0 && (!in->gather || !in->gather_len))) return fail(WELD_ERR_INVALID_ARG, "bad gather vector list");
    if (in->start_col < 0 || in->start_col >= no || in->end_col < 0 || in->end_col >= no)
        return fail(WELD_ERR_INVALID_ARG, "start / end column not among the outer vectors");
    const int ot = in->outer.col[in->start_col].type;
    if ((ot != WELD_I32 && ot != WELD_I64) || in->outer.col[in->end_col].type != ot)
        return fail(WELD_ERR_TYPE, "start and end vectors must both be i32 or both i64");
    if (in->inner_type != WELD_I64 && in->inner_type != WELD_F64)
        return fail(WELD_ERR_UNSUPPORTED, "inner merger of type " + std::to_string(in->inner_type) + " (i64 and f64 are implemented)");
    if (in->inner_func < WELD_FUNC_ADD || in->inner_func > WELD_FUNC_MAX) return fail(WELD_ERR_INVALID_ARG, "unknown inner merge function");
    NL->start_col = in->start_col;
    NL->end_col = in->end_col;
    NL->offset_type = ot;
    if (in->range_kind != WELD_RANGES_CSR && in->range_kind != WELD_RANGES_ANY) return fail(WELD_ERR_INVALID_ARG, "unknown range kind");
    NL->any_ranges = in->range_kind == WELD_RANGES_ANY;
    NL->stride_col = -1;
    if (NL->any_ranges && in->stride_col != -1) {
        if (in->stride_col < 0 || in->stride_col >= no) return fail(WELD_ERR_INVALID_ARG, "stride column not among the outer vectors");
        if (in->outer.col[in->stride_col].type != ot) return fail(WELD_ERR_TYPE, "the stride vector must have the type of start and end");
        NL->stride_col = in->stride_col;
    }

    // ---- inner body: one merger, may look vectors up and read the current outer element
    NestedContext nc;
    nc.ngather = ng;
    for (int g = 0; g < ng; ++g) {
        if (!type_is_num(in->gather[g].type)) return fail(WELD_ERR_TYPE, "gather vector " + std::to_string(g) + " has no numeric type");
        if (in->gather_len[g] < 0) return fail(WELD_ERR_INVALID_ARG, "negative gather vector length");
        nc.gather_type[g] = in->gather[g].type;
    }
    nc.nouter = no;
    for (int c = 0; c < no; ++c) nc.outer_type[c] = in->outer.col[c].type;
    int32_t itypes[WELD_MAX_COLS];
    for (int c = 0; c < ni; ++c) itypes[c] = in->inner.col[c].type;
    weld_builder_spec_t ms;
    memset(&ms, 0, sizeof ms);
    ms.kind = WELD_MERGER;
    ms.func = in->inner_func;
    ms.nvals = 1;
    ms.val_type[0] = in->inner_type;
    weld_builder_t ib;
    memset(&ib, 0, sizeof ib);
    ib.count = 1;
    ib.spec = &ms;
    Error e = validate(itypes, ni, &in->inner_body, &ib, &NL->inner, &nc);
    if (!e.ok()) { e.text = "inner body: " + e.text; return e; }
    if (in->inner_body.nmerges != 1) return fail(WELD_ERR_INVALID_ARG, "the inner body merges exactly once, into its merger");

    // ---- outer body: the inner loop's result becomes one more zipped vector
    if (in->outer_body.nops < 0 || in->outer_body.nops > 4096 || (in->outer_body.nops > 0 && !in->outer_body.ops))
        return fail(WELD_ERR_INVALID_ARG, "bad outer body");
    std::vector<weld_op_t> ops(in->outer_body.ops, in->outer_body.ops + in->outer_body.nops);
    for (size_t i = 0; i < ops.size(); ++i) {
        if (ops[i].opcode == WELD_OP_SCALAR) return fail(WELD_ERR_UNSUPPORTED, "outer body: scalars from outside the loop are not implemented in nested loops");
        if (ops[i].opcode != WELD_OP_INNER) continue;
        if (ops[i].type != in->inner_type)
            return fail(WELD_ERR_TYPE, "outer body op " + std::to_string(i) + ": the inner loop's result has type " + std::to_string(in->inner_type));
        ops[i].opcode = WELD_OP_COL;
        ops[i].a = no;
    }
    int32_t otypes[WELD_MAX_COLS];
    for (int c = 0; c < no; ++c) otypes[c] = in->outer.col[c].type;
    otypes[no] = in->inner_type;
    weld_body_t ob = in->outer_body;
    ob.ops = ops.data();
    e = validate(otypes, no + 1, &ob, builders, &NL->outer);
    if (!e.ok()) { e.text = "outer body: " + e.text; return e; }
    if (builders->conf.mode != WELD_MODE_FUSED) return fail(WELD_ERR_UNSUPPORTED, "nested loops run in fused mode only");

    if (!need_data) return Error();
    D->n_outer = in->n_outer;
    D->n_inner = in->n_inner;
    auto check = [&](const weld_col_t& c, int64_t n, bool used, const char* what) -> Error {
        if (n > 0 && used && !c.data) return fail(WELD_ERR_INVALID_ARG, std::string("null ") + what + " pointer");
        if ((uintptr_t)c.data % (uintptr_t)type_size(c.type)) return fail(WELD_ERR_INVALID_ARG, std::string(what) + " pointer not aligned to its element size");
        return Error();
    };
    for (int c = 0; c < no; ++c) {
        const bool used = NL->outer.col_used[c] || NL->inner.outer_used[c] || c == in->start_col || c == in->end_col || c == NL->stride_col;
        if (!(e = check(in->outer.col[c], in->n_outer, used, "outer vector")).ok()) return e;
        D->outer[c].data = in->outer.col[c].data;
        D->outer[c].type = in->outer.col[c].type;
    }
    for (int c = 0; c < ni; ++c) {
        if (!(e = check(in->inner.col[c], in->n_inner, NL->inner.col_used[c], "inner vector")).ok()) return e;
        D->inner[c].data = in->inner.col[c].data;
        D->inner[c].type = in->inner.col[c].type;
    }
    for (int g = 0; g < ng; ++g) {
        if (!(e = check(in->gather[g], in->gather_len[g], NL->inner.gather_used[g], "gather vector")).ok()) return e;
        D->gather[g].data = in->gather[g].data;
        D->gather[g].type = in->gather[g].type;
        D->gather_len[g] = in->gather_len[g];
    }
    return Error();
}

}  // namespace

extern "C" {

weld_status_t weld_nested_validate(const weld_nested_t* loop, const weld_builder_t* builders, char* err, size_t errlen) {
    NestedLoop NL;
    Error e = build(loop, builders, false, &NL, nullptr);
    if (err && errlen) {
        strncpy(err, e.text.c_str(), errlen - 1);
        err[errlen - 1] = 0;
    }
    if (!e.ok()) set_last_error(e.text);
    return e.status;
}

weld_status_t weld_nested_precompile(const weld_nested_t* loop, const weld_builder_t* builders) {
    NestedLoop NL;
    Error e = build(loop, builders, false, &NL, nullptr);
    if (!e.ok()) { set_last_error(e.text); return e.status; }
    for (int aligned = 1; aligned >= 0; --aligned) {
        Variant v1 = choose_segmented_variant(NL.inner, builders->conf.tune, aligned != 0);
        Generated g1 = generate_segmented(NL.inner, v1, NL.offset_type, NL.any_ranges ? (NL.stride_col >= 0 ? 2 : 1) : 0);
        Kernel* k = nullptr;
        e = jit_get(g1.source, g1.kernel_name, false, &k);
        if (!e.ok()) { set_last_error(e.text); return e.status; }
    }
    Variant v2 = choose_variant(NL.outer, builders->conf.tune, true);
    Generated g2 = generate(NL.outer, v2);
    Kernel* k = nullptr;
    e = jit_get(g2.source, g2.kernel_name, false, &k);
    if (!e.ok()) { set_last_error(e.text); return e.status; }
    return WELD_OK;
}

weld_status_t weld_nested_for(const weld_nested_t* loop, const weld_builder_t* builders, weld_result_t** out) {
    if (out) *out = nullptr;
    if (!out) { set_last_error("null argument"); return WELD_ERR_INVALID_ARG; }
    NestedLoop NL;
    NestedData D;
    Error e = build(loop, builders, true, &NL, &D);
    if (!e.ok()) { set_last_error(e.text); return e.status; }
    weld_result* r = new_result(builders->conf.stream);
    if (!r) {
        set_last_error("could not allocate pinned memory / events (no usable HIP device?)");
        return WELD_ERR_DEVICE;
    }
    e = run_nested(NL, D, builders->conf, r);
    if (!e.ok()) {
        set_last_error(e.text);
        destroy_result(r);
        return e.status;
    }
    *out = r;
    return WELD_OK;
}

}  // extern "C"
