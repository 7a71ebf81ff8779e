// Validation of a submitted loop: operand order, types, builder linearity.
//
// Sec. 3.2 of the paper: the body is an expression over the row index and the
// struct of zipped elements; each builder must be consumed exactly once per control
// path (builders are linear) and the function must return builders derived from its
// arguments.  In this ABI that becomes: every merge names a declared builder, no
// builder is named by two merges, and a builder that is never named is returned
// untouched.  The typed IR has no implicit conversions, so operand types must agree.
#include <cstdio>
#include <cstring>

#include "weld_internal.h"

namespace weld {

static Error fail(weld_status_t st, const char* fmt, int a = 0, int b = 0, int c = 0) {
    char buf[256];
    snprintf(buf, sizeof buf, fmt, a, b, c);
    Error e;
    e.status = st;
    e.text = buf;
    return e;
}

int key_bits(const weld_builder_spec_t& b) {
    int bits = 0;
    for (int k = 0; k < b.nkeys; ++k) bits += 8 * type_size(b.key_type[k]);
    return bits;
}

Error validate(const int32_t* col_types, int32_t ncols, const weld_body_t* body,
               const weld_builder_t* builder, Loop* out, const NestedContext* inner_of) {
    if (!body || !builder || !out) return fail(WELD_ERR_INVALID_ARG, "null argument");
    if (ncols < 0 || ncols > WELD_MAX_COLS) return fail(WELD_ERR_INVALID_ARG, "ncols %d out of range", ncols);
    if (ncols > 0 && !col_types) return fail(WELD_ERR_INVALID_ARG, "null column types");
    Loop& L = *out;
    L = Loop();
    L.ncols = ncols;
    if (inner_of) {
        L.ndicts = inner_of->ndicts;
        for (int d = 0; d < L.ndicts; ++d) L.dict_in[d] = inner_of->dict_in[d];
        L.ngather = inner_of->ngather;
        L.nouter = inner_of->nouter;
        for (int k = 0; k < L.ngather; ++k) L.gather_type[k] = inner_of->gather_type[k];
        for (int k = 0; k < L.nouter; ++k) L.outer_type[k] = inner_of->outer_type[k];
    }
    for (int k = 0; k < ncols; ++k) {
        if (!type_is_num(col_types[k])) return fail(WELD_ERR_TYPE, "column %d: type %d is not i8/i32/i64/f64", k, col_types[k]);
        L.col_type[k] = col_types[k];
    }
    if (body->nops < 0 || body->nops > 4096) return fail(WELD_ERR_INVALID_ARG, "nops %d out of range", body->nops);
    if (body->nops > 0 && !body->ops) return fail(WELD_ERR_INVALID_ARG, "null ops");
    if (builder->count < 1 || builder->count > WELD_MAX_BUILDERS)
        return fail(WELD_ERR_INVALID_ARG, "builder count %d out of range 1..%d", builder->count, WELD_MAX_BUILDERS);
    if (!builder->spec) return fail(WELD_ERR_INVALID_ARG, "null builder specs");
    if (body->nmerges < 0 || body->nmerges > 64) return fail(WELD_ERR_INVALID_ARG, "nmerges %d out of range", body->nmerges);
    if (body->nmerges > 0 && !body->merges) return fail(WELD_ERR_INVALID_ARG, "null merges");
    if (builder->conf.mode != WELD_MODE_FUSED && builder->conf.mode != WELD_MODE_UNFUSED)
        return fail(WELD_ERR_INVALID_ARG, "unknown mode %d", builder->conf.mode);
    if (builder->conf.memory_limit < 0) return fail(WELD_ERR_INVALID_ARG, "negative memory limit");

    // ---- expressions
    L.ops.assign(body->ops, body->ops + body->nops);
    for (int i = 0; i < body->nops; ++i) {
        const weld_op_t& o = L.ops[i];
        if (!type_valid(o.type)) return fail(WELD_ERR_TYPE, "op %d: bad result type %d", i, o.type);
        auto operand = [&](int x) { return x >= 0 && x < i; };
        auto ty = [&](int x) { return L.ops[x].type; };
        switch (o.opcode) {
            case WELD_OP_COL:
                if (o.a < 0 || o.a >= ncols) return fail(WELD_ERR_INVALID_ARG, "op %d: column %d not declared", i, o.a);
                if (o.type != L.col_type[o.a]) return fail(WELD_ERR_TYPE, "op %d: column %d has type %d", i, o.a, L.col_type[o.a]);
                if (L.col_scalar[o.a]) return fail(WELD_ERR_INVALID_ARG, "op %d: column %d is read as a scalar elsewhere in the body", i, o.a);
                L.col_used[o.a] = true;
                break;
            case WELD_OP_SCALAR:
                if (inner_of && inner_of->nouter > 0) return fail(WELD_ERR_UNSUPPORTED, "op %d: scalars from outside the loop are not implemented in nested bodies", i);
                if (o.a < 0 || o.a >= ncols) return fail(WELD_ERR_INVALID_ARG, "op %d: column %d not declared", i, o.a);
                if (o.type != L.col_type[o.a]) return fail(WELD_ERR_TYPE, "op %d: column %d has type %d", i, o.a, L.col_type[o.a]);
                if (L.col_used[o.a]) return fail(WELD_ERR_INVALID_ARG, "op %d: column %d is read as a vector elsewhere in the body", i, o.a);
                L.col_scalar[o.a] = true;
                break;
            case WELD_OP_CONST:
                if (o.type == WELD_BOOL && o.imm.i64 != 0 && o.imm.i64 != 1)
                    return fail(WELD_ERR_INVALID_ARG, "op %d: bool constant must be 0 or 1", i);
                if (o.type == WELD_I8 && (o.imm.i64 < -128 || o.imm.i64 > 127))
                    return fail(WELD_ERR_INVALID_ARG, "op %d: constant does not fit i8", i);
                if (o.type == WELD_I32 && (o.imm.i64 < INT32_MIN || o.imm.i64 > INT32_MAX))
                    return fail(WELD_ERR_INVALID_ARG, "op %d: constant does not fit i32", i);
                break;
            case WELD_OP_INDEX:
                if (o.type != WELD_I64) return fail(WELD_ERR_TYPE, "op %d: index has type i64", i);
                break;
            case WELD_OP_NEG:
                if (!operand(o.a)) return fail(WELD_ERR_INVALID_ARG, "op %d: operand %d is not an earlier op", i, o.a);
                if (!type_is_num(o.type) || ty(o.a) != o.type) return fail(WELD_ERR_TYPE, "op %d: neg needs a numeric operand of the result type", i);
                break;
            case WELD_OP_NOT:
                if (!operand(o.a)) return fail(WELD_ERR_INVALID_ARG, "op %d: operand %d is not an earlier op", i, o.a);
                if (o.type != WELD_BOOL || ty(o.a) != WELD_BOOL) return fail(WELD_ERR_TYPE, "op %d: not needs bool", i);
                break;
            case WELD_OP_CAST:
                if (!operand(o.a)) return fail(WELD_ERR_INVALID_ARG, "op %d: operand %d is not an earlier op", i, o.a);
                break;
            case WELD_OP_EXP: case WELD_OP_LOG: case WELD_OP_SQRT: case WELD_OP_ERF:
                if (!operand(o.a)) return fail(WELD_ERR_INVALID_ARG, "op %d: operand %d is not an earlier op", i, o.a);
                if (o.type != WELD_F64 || ty(o.a) != WELD_F64) return fail(WELD_ERR_TYPE, "op %d: math functions take f64", i);
                break;
            case WELD_OP_ADD: case WELD_OP_SUB: case WELD_OP_MUL: case WELD_OP_DIV: case WELD_OP_MOD:
            case WELD_OP_MIN: case WELD_OP_MAX:
                if (!operand(o.a) || !operand(o.b)) return fail(WELD_ERR_INVALID_ARG, "op %d: operands must be earlier ops", i);
                if (!type_is_num(o.type) || ty(o.a) != o.type || ty(o.b) != o.type)
                    return fail(WELD_ERR_TYPE, "op %d: arithmetic operands (types %d, %d) must equal the numeric result type", i, ty(o.a), ty(o.b));
                if ((o.opcode == WELD_OP_DIV || o.opcode == WELD_OP_MOD) && type_is_int(o.type) &&
                    L.ops[o.b].opcode == WELD_OP_CONST && L.ops[o.b].imm.i64 == 0)
                    return fail(WELD_ERR_INVALID_ARG, "op %d: integer division by constant zero", i);
                break;
            case WELD_OP_LT: case WELD_OP_LE: case WELD_OP_GT: case WELD_OP_GE: case WELD_OP_EQ: case WELD_OP_NE:
                if (!operand(o.a) || !operand(o.b)) return fail(WELD_ERR_INVALID_ARG, "op %d: operands must be earlier ops", i);
                if (o.type != WELD_BOOL) return fail(WELD_ERR_TYPE, "op %d: a comparison yields bool", i);
                if (ty(o.a) != ty(o.b) || !type_is_num(ty(o.a)))
                    return fail(WELD_ERR_TYPE, "op %d: comparison of types %d and %d", i, ty(o.a), ty(o.b));
                break;
            case WELD_OP_AND: case WELD_OP_OR:
                if (!operand(o.a) || !operand(o.b)) return fail(WELD_ERR_INVALID_ARG, "op %d: operands must be earlier ops", i);
                if (o.type != WELD_BOOL || ty(o.a) != WELD_BOOL || ty(o.b) != WELD_BOOL)
                    return fail(WELD_ERR_TYPE, "op %d: and/or need bool", i);
                break;
            case WELD_OP_SELECT:
                if (!operand(o.a) || !operand(o.b) || !operand(o.c)) return fail(WELD_ERR_INVALID_ARG, "op %d: operands must be earlier ops", i);
                if (ty(o.a) != WELD_BOOL || ty(o.b) != o.type || ty(o.c) != o.type)
                    return fail(WELD_ERR_TYPE, "op %d: select(bool, T, T) -> T", i);
                break;
            case WELD_OP_KEYEXISTS: case WELD_OP_DICTLOOKUP: {
                if (o.a < 0 || o.a >= L.ndicts) return fail(WELD_ERR_INVALID_ARG, "op %d: dictionary %d is not an input of this loop", i, o.a);
                const DictTable& t = L.dict_in[o.a];
                if (t.nkeys > 2) return fail(WELD_ERR_UNSUPPORTED, "op %d: probes of dictionaries with more than two key fields", i);
                if (!operand(o.b) || (t.nkeys == 2 && !operand(o.c)) || (t.nkeys == 1 && o.c != -1))
                    return fail(WELD_ERR_INVALID_ARG, "op %d: one earlier op per key field of the dictionary", i);
                if (ty(o.b) != t.key_type[0] || (t.nkeys == 2 && ty(o.c) != t.key_type[1]))
                    return fail(WELD_ERR_TYPE, "op %d: key operands do not have the dictionary's key types", i);
                if (o.opcode == WELD_OP_KEYEXISTS) {
                    if (o.type != WELD_BOOL) return fail(WELD_ERR_TYPE, "op %d: keyexists yields bool", i);
                } else {
                    if (o.reserved < 0 || o.reserved >= t.nvals) return fail(WELD_ERR_INVALID_ARG, "op %d: value field %d not in the dictionary", i, o.reserved);
                    if (o.type != t.val_type[o.reserved]) return fail(WELD_ERR_TYPE, "op %d: value field %d has type %d", i, o.reserved, t.val_type[o.reserved]);
                    L.dict_val_used[o.a][o.reserved] = true;
                }
                break;
            }
            case WELD_OP_LOOKUP:
                if (!inner_of || (inner_of->ngather == 0 && inner_of->nouter == 0)) return fail(WELD_ERR_UNSUPPORTED, "op %d: lookup is only implemented in the inner body of weld_nested_for", i);
                if (o.a < 0 || o.a >= L.ngather) return fail(WELD_ERR_INVALID_ARG, "op %d: gather vector %d not declared", i, o.a);
                if (!operand(o.b)) return fail(WELD_ERR_INVALID_ARG, "op %d: operand %d is not an earlier op", i, o.b);
                if (!type_is_int(ty(o.b))) return fail(WELD_ERR_TYPE, "op %d: lookup index must be an integer", i);
                if (o.type != L.gather_type[o.a]) return fail(WELD_ERR_TYPE, "op %d: gather vector %d has type %d", i, o.a, L.gather_type[o.a]);
                L.gather_used[o.a] = true;
                break;
            case WELD_OP_OUTER:
                if (!inner_of || inner_of->nouter == 0) return fail(WELD_ERR_INVALID_ARG, "op %d: outer-element access outside an inner body", i);
                if (o.a < 0 || o.a >= L.nouter) return fail(WELD_ERR_INVALID_ARG, "op %d: outer column %d not declared", i, o.a);
                if (o.type != L.outer_type[o.a]) return fail(WELD_ERR_TYPE, "op %d: outer column %d has type %d", i, o.a, L.outer_type[o.a]);
                L.outer_used[o.a] = true;
                break;
            case WELD_OP_INNER:
                return fail(WELD_ERR_INVALID_ARG, "op %d: inner-loop result outside the outer body of weld_nested_for", i);
            default:
                return fail(WELD_ERR_INVALID_ARG, "op %d: unknown opcode %d", i, o.opcode);
        }
    }

    // ---- builders
    L.builders.assign(builder->spec, builder->spec + builder->count);
    for (int b = 0; b < builder->count; ++b) {
        const weld_builder_spec_t& s = L.builders[b];
        switch (s.kind) {
            case WELD_MERGER:
                if (s.nvals != 1 || s.nkeys != 0) return fail(WELD_ERR_INVALID_ARG, "builder %d: merger takes one value", b);
                if (!type_is_num(s.val_type[0])) return fail(WELD_ERR_TYPE, "builder %d: merger of type %d", b, s.val_type[0]);
                if (s.func < WELD_FUNC_ADD || s.func > WELD_FUNC_MAX) return fail(WELD_ERR_INVALID_ARG, "builder %d: unknown func %d", b, s.func);
                break;
            case WELD_VECBUILDER:
                if (s.nvals != 1 || s.nkeys != 0) return fail(WELD_ERR_INVALID_ARG, "builder %d: vecbuilder takes one value", b);
                if (!type_is_num(s.val_type[0])) return fail(WELD_ERR_TYPE, "builder %d: vecbuilder of type %d", b, s.val_type[0]);
                break;
            case WELD_DICTMERGER:
                if (s.nkeys < 1 || s.nkeys > WELD_MAX_KEY_FIELDS || s.nvals < 1 || s.nvals > WELD_MAX_VAL_FIELDS)
                    return fail(WELD_ERR_INVALID_ARG, "builder %d: dictmerger needs 1..4 key fields and 1..8 value fields", b);
                for (int k = 0; k < s.nkeys; ++k)
                    if (!type_is_int(s.key_type[k])) return fail(WELD_ERR_UNSUPPORTED, "builder %d: key field %d must be an integer type", b, k);
                if (key_bits(s) > 64) return fail(WELD_ERR_UNSUPPORTED, "builder %d: key struct wider than 64 bits", b);
                for (int k = 0; k < s.nvals; ++k)
                    if (!type_is_num(s.val_type[k])) return fail(WELD_ERR_TYPE, "builder %d: value field %d has type %d", b, k, s.val_type[k]);
                if (s.func < WELD_FUNC_ADD || s.func > WELD_FUNC_MAX) return fail(WELD_ERR_INVALID_ARG, "builder %d: unknown func %d", b, s.func);
                if (s.capacity < 1 || s.capacity > (1ll << 30)) return fail(WELD_ERR_INVALID_ARG, "builder %d: capacity out of range", b);
                break;
            case WELD_GROUPBUILDER:
                if (s.nkeys < 1 || s.nkeys > WELD_MAX_KEY_FIELDS) return fail(WELD_ERR_INVALID_ARG, "builder %d: groupbuilder needs 1..4 key fields", b);
                if (s.nvals != 1) return fail(WELD_ERR_UNSUPPORTED, "builder %d: groupbuilder of a value struct (one scalar value is implemented)", b);
                for (int k = 0; k < s.nkeys; ++k)
                    if (!type_is_int(s.key_type[k])) return fail(WELD_ERR_UNSUPPORTED, "builder %d: key field %d must be an integer type", b, k);
                if (key_bits(s) > 64) return fail(WELD_ERR_UNSUPPORTED, "builder %d: key struct wider than 64 bits", b);
                if (!type_is_num(s.val_type[0])) return fail(WELD_ERR_TYPE, "builder %d: value has type %d", b, s.val_type[0]);
                if (s.capacity < 1 || s.capacity > (1ll << 30)) return fail(WELD_ERR_INVALID_ARG, "builder %d: capacity out of range", b);
                break;
            case WELD_VECMERGER:
                if (s.nvals != 1 || s.nkeys != 1) return fail(WELD_ERR_INVALID_ARG, "builder %d: vecmerger takes {index, value}", b);
                if (s.key_type[0] != WELD_I64) return fail(WELD_ERR_TYPE, "builder %d: vecmerger index must be i64", b);
                if (s.val_type[0] != WELD_I64 && s.val_type[0] != WELD_F64)
                    return fail(WELD_ERR_UNSUPPORTED, "builder %d: vecmerger of type %d (i64 and f64 are implemented)", b, s.val_type[0]);
                if (s.func < WELD_FUNC_ADD || s.func > WELD_FUNC_MAX) return fail(WELD_ERR_INVALID_ARG, "builder %d: unknown func %d", b, s.func);
                if (s.length < 1 || s.length > (1ll << 31)) return fail(WELD_ERR_INVALID_ARG, "builder %d: vecmerger length out of range", b);
                if (s.init && ((uintptr_t)s.init & 7)) return fail(WELD_ERR_INVALID_ARG, "builder %d: init vector not 8-byte aligned", b);
                break;
            default:
                return fail(WELD_ERR_INVALID_ARG, "builder %d: unknown kind %d", b, s.kind);
        }
    }

    // ---- merges
    L.merge_of.assign(builder->count, -1);
    L.merges.assign(body->merges, body->merges + body->nmerges);
    for (int m = 0; m < body->nmerges; ++m) {
        const weld_merge_t& g = L.merges[m];
        if (g.builder < 0 || g.builder >= builder->count) return fail(WELD_ERR_INVALID_ARG, "merge %d: builder %d not declared", m, g.builder);
        if (L.merge_of[g.builder] >= 0)
            return fail(WELD_ERR_LINEARITY, "merge %d: builder %d is already consumed by merge %d", m, g.builder, L.merge_of[g.builder]);
        L.merge_of[g.builder] = m;
        const weld_builder_spec_t& s = L.builders[g.builder];
        if (g.pred != -1) {
            if (g.pred < 0 || g.pred >= body->nops) return fail(WELD_ERR_INVALID_ARG, "merge %d: predicate %d is not an op", m, g.pred);
            if (L.ops[g.pred].type != WELD_BOOL) return fail(WELD_ERR_TYPE, "merge %d: predicate must be bool", m);
        }
        if (g.nvals != s.nvals || g.nkeys != s.nkeys)
            return fail(WELD_ERR_TYPE, "merge %d: builder %d takes %d value fields", m, g.builder, s.nvals);
        for (int k = 0; k < g.nvals; ++k) {
            if (g.val[k] < 0 || g.val[k] >= body->nops) return fail(WELD_ERR_INVALID_ARG, "merge %d: value %d is not an op", m, g.val[k]);
            if (L.ops[g.val[k]].type != s.val_type[k])
                return fail(WELD_ERR_TYPE, "merge %d: value field %d has type %d", m, k, L.ops[g.val[k]].type);
        }
        for (int k = 0; k < g.nkeys; ++k) {
            if (g.key[k] < 0 || g.key[k] >= body->nops) return fail(WELD_ERR_INVALID_ARG, "merge %d: key %d is not an op", m, g.key[k]);
            if (L.ops[g.key[k]].type != s.key_type[k])
                return fail(WELD_ERR_TYPE, "merge %d: key field %d has type %d", m, k, L.ops[g.key[k]].type);
        }
    }
    return Error();
}

}  // namespace weld
