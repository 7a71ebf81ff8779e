// HIP source generation for one fused loop.
//
// The paper's backends turn the optimised IR into one kernel per program (Sec. 5);
// this file does the same for gfx950.  What is generated is small: the row function
// (the loop body as straight-line SSA code, one C++ statement per IR operator, so
// shared sub-expressions are computed once), the merge statements, and a kernel
// skeleton that wires the hand-written building blocks of fused_prelude.hip.h
// (column loader, wavefront/work-group reductions, look-back scan, hash tables)
// together for the builders of this particular loop.
//
// Row ownership: a tile is W_WAVES consecutive runs of W_WAVE_ROWS rows, one run
// per wavefront; inside a run, load u of lane l covers rows
// run + (u*64 + l)*W_V .. +W_V-1.  Every wavefront-wide load is therefore one
// contiguous span, and index order inside a wavefront is (u, lane, k), which is
// what the order-preserving vecbuilder ranks rely on.
#include <cstdarg>
#include <cstdio>
#include <algorithm>
#include <cstring>

#include "weld_internal.h"

namespace weld {

extern const char* const kPreludeSource;  // fused_prelude.hip.h, embedded at build time

namespace {

struct Out {
    std::string s;
    void f(const char* fmt, ...) __attribute__((format(printf, 2, 3))) {
        char buf[2048];
        va_list ap;
        va_start(ap, fmt);
        vsnprintf(buf, sizeof buf, fmt, ap);
        va_end(ap);
        s += buf;
    }
};

const char* ctype(int t) {
    switch (t) {
        case WELD_BOOL: return "bool";
        case WELD_I8: return "signed char";
        case WELD_I32: return "int";
        case WELD_I64: return "i64";
        case WELD_F64: return "double";
    }
    return "void";
}
// type a value has in memory: predicates are stored as bytes holding 0 or 1
const char* stype(int t) { return t == WELD_BOOL ? "unsigned char" : ctype(t); }
// type a builder accumulates a value field in (integers widen to 64 bits: wrapping
// sums/products and min/max commute with the final truncation)
const char* acc_ctype(int t) { return t == WELD_F64 ? "double" : "i64"; }
const char* utype(int t) {
    switch (t) {
        case WELD_I8: return "unsigned char";
        case WELD_I32: return "u32";
        case WELD_I64: return "u64";
    }
    return "u64";
}

std::string ident_expr(int func, int t) {
    char buf[96];
    if (t == WELD_F64) snprintf(buf, sizeof buf, "w_identity_f64<%d>()", func);
    else snprintf(buf, sizeof buf, "w_identity_int<%d,%d>()", func, 8 * type_size(t));
    return buf;
}

std::string const_expr(const weld_op_t& o) {
    char buf[96];
    switch (o.type) {
        case WELD_BOOL: snprintf(buf, sizeof buf, "%s", o.imm.i64 ? "true" : "false"); break;
        case WELD_F64: {
            uint64_t bits;
            memcpy(&bits, &o.imm.f64, 8);
            snprintf(buf, sizeof buf, "__builtin_bit_cast(double, 0x%016llxull)", (unsigned long long)bits);
            break;
        }
        case WELD_I64:
            snprintf(buf, sizeof buf, "(i64)0x%016llxull", (unsigned long long)o.imm.i64);
            break;
        default:
            snprintf(buf, sizeof buf, "(%s)(%lld)", ctype(o.type), (long long)o.imm.i64);
    }
    return buf;
}

// wrapping integer arithmetic through the unsigned type
std::string wrap_bin(int t, const char* op, int a, int b) {
    char buf[160];
    if (t == WELD_I8 && op[0] == '*')
        snprintf(buf, sizeof buf, "w_mul_i8(t%d, t%d)", a, b);
    else if (t == WELD_I8)
        snprintf(buf, sizeof buf, "(signed char)(unsigned char)((u32)(unsigned char)t%d %s (u32)(unsigned char)t%d)", a, op, b);
    else
        snprintf(buf, sizeof buf, "(%s)((%s)t%d %s (%s)t%d)", ctype(t), utype(t), a, op, utype(t), b);
    return buf;
}

// `segmented`: the row function of a nested loop's inner body, which also gets the outer
// element it belongs to (`row`), the kernel arguments (gather and outer vectors) and the
// error word.
void emit_row_function(Out& o, const Loop& L, bool segmented = false) {
    // ---- RowOut
    o.f("struct RowOut {\n");
    for (size_t b = 0; b < L.builders.size(); ++b) {
        if (L.merge_of[b] < 0) continue;
        const weld_builder_spec_t& s = L.builders[b];
        o.f("  bool p%zu;", b);
        for (int k = 0; k < s.nkeys; ++k) o.f(" %s k%zu_%d;", ctype(s.key_type[k]), b, k);
        for (int k = 0; k < s.nvals; ++k) o.f(" %s v%zu_%d;", ctype(s.val_type[k]), b, k);
        o.f("\n");
    }
    o.f("  int unused_;\n};\n\n");
    // ---- invalid row (past the end of the input): merges nothing
    o.f("__device__ __forceinline__ void weld_row_none(RowOut& o) {\n");
    for (size_t b = 0; b < L.builders.size(); ++b) {
        if (L.merge_of[b] < 0) continue;
        const weld_builder_spec_t& s = L.builders[b];
        o.f("  o.p%zu = false;", b);
        for (int k = 0; k < s.nkeys; ++k) o.f(" o.k%zu_%d = 0;", b, k);
        for (int k = 0; k < s.nvals; ++k) o.f(" o.v%zu_%d = 0;", b, k);
        o.f("\n");
    }
    o.f("}\n\n");
    // ---- which predicate guards each value: an op that only feeds merges under one predicate
    // (computed before it) is only needed on rows where that predicate holds.  Used for the
    // operators that go to memory at a computed address (lookups, dictionary probes): they are
    // skipped on the other rows, which never read their result.
    const int kUnused = -1, kAlways = -2;
    std::vector<int> need(L.ops.size(), kUnused);
    auto mark = [&](int x, int g) {
        if (x < 0) return;
        if (need[x] == kUnused) need[x] = g;
        else if (need[x] != g) need[x] = kAlways;
    };
    for (const weld_merge_t& g : L.merges) {
        const int p = g.pred >= 0 ? g.pred : kAlways;
        for (int k = 0; k < g.nkeys; ++k) mark(g.key[k], p);
        for (int k = 0; k < g.nvals; ++k) mark(g.val[k], p);
        if (g.pred >= 0) mark(g.pred, kAlways);
    }
    for (int i = (int)L.ops.size() - 1; i >= 0; --i) {
        const weld_op_t& q = L.ops[i];
        if (need[i] == kUnused || q.opcode == WELD_OP_COL || q.opcode == WELD_OP_CONST || q.opcode == WELD_OP_INDEX ||
            q.opcode == WELD_OP_OUTER || q.opcode == WELD_OP_SCALAR)
            continue;
        const bool dict_op = q.opcode == WELD_OP_KEYEXISTS || q.opcode == WELD_OP_DICTLOOKUP;
        if (q.opcode != WELD_OP_LOOKUP && !dict_op) mark(q.a, need[i]);      // for those two, a is a vector / dictionary index
        mark(q.b, need[i]);
        mark(q.c, need[i]);
    }
    auto guarded = [&](size_t i) { return need[i] >= 0 && need[i] < (int)i; };

    // ---- the body, one statement per IR operator
    // W_CONV: every lane of the wavefront makes this call together (full tiles); only then may the
    // body take decisions for the whole wavefront
    o.f("template <bool W_CONV> __device__ __forceinline__ void weld_row(const i64 i");
    if (segmented) o.f(", const i64 row");
    if (segmented || L.ndicts > 0) o.f(", const KArgs& a, int* errp");
    for (int c = 0; c < L.ncols; ++c)
        if (L.col_used[c]) o.f(", const %s x%d", stype(L.col_type[c]), c);
    for (int c = 0; c < L.ncols; ++c)
        if (L.col_scalar[c]) o.f(", const %s sc%d", stype(L.col_type[c]), c);
    o.f(", RowOut& o) {\n");
    for (size_t i = 0; i < L.ops.size(); ++i) {
        const weld_op_t& q = L.ops[i];
        const int id = (int)i;
        const char* T = ctype(q.type);
        o.f("  const %s t%d = ", T, id);
        switch (q.opcode) {
            case WELD_OP_COL: o.f("x%d", q.a); break;
            case WELD_OP_SCALAR: o.f("sc%d", q.a); break;
            case WELD_OP_CONST: o.f("%s", const_expr(q).c_str()); break;
            case WELD_OP_INDEX: o.f("i"); break;
            case WELD_OP_NEG:
                if (q.type == WELD_F64) o.f("-t%d", q.a);
                else o.f("(%s)((%s)0 - (%s)t%d)", T, utype(q.type), utype(q.type), q.a);
                break;
            case WELD_OP_NOT: o.f("!t%d", q.a); break;
            case WELD_OP_CAST: {
                const int st = L.ops[q.a].type;
                if (q.type == WELD_BOOL) o.f("(t%d != 0)", q.a);
                else if (st == WELD_F64 && type_is_int(q.type)) o.f("(%s)w_f64_to_i64(t%d)", T, q.a);
                else o.f("(%s)t%d", T, q.a);
                break;
            }
            case WELD_OP_EXP: o.f("W_EXP(t%d)", q.a); break;
            case WELD_OP_LOG: o.f("W_LOG(t%d)", q.a); break;
            case WELD_OP_SQRT: o.f("sqrt(t%d)", q.a); break;
            case WELD_OP_ERF: o.f("w_erf(t%d)", q.a); break;
            case WELD_OP_ADD:
                if (q.type == WELD_F64) o.f("t%d + t%d", q.a, q.b);
                else o.f("%s", wrap_bin(q.type, "+", q.a, q.b).c_str());
                break;
            case WELD_OP_SUB:
                if (q.type == WELD_F64) o.f("t%d - t%d", q.a, q.b);
                else o.f("%s", wrap_bin(q.type, "-", q.a, q.b).c_str());
                break;
            case WELD_OP_MUL:
                if (q.type == WELD_F64) o.f("t%d * t%d", q.a, q.b);
                else o.f("%s", wrap_bin(q.type, "*", q.a, q.b).c_str());
                break;
            case WELD_OP_DIV: case WELD_OP_MOD: {
                const bool div = q.opcode == WELD_OP_DIV;
                const weld_op_t& d = L.ops[q.b];
                if (q.type == WELD_F64) {
                    if (div) o.f("t%d / t%d", q.a, q.b);
                    else o.f("fmod(t%d, t%d)", q.a, q.b);
                } else if (q.type == WELD_I64 && d.opcode == WELD_OP_CONST && d.imm.i64 >= 2 && d.imm.i64 < (1ll << 31)) {
                    // 64-bit operand, small constant divisor: 32-bit arithmetic when the wavefront's operands allow
                    o.f("w_%s_const<%lldll, W_CONV>(t%d, ", div ? "div" : "mod", (long long)d.imm.i64, q.a);
                    if (guarded(i)) o.f("t%d)", need[i]);
                    else o.f("true)");
                } else {
                    o.f("w_%s_int<%s>(t%d, t%d)", div ? "div" : "mod", T, q.a, q.b);
                }
                break;
            }
            case WELD_OP_MIN:
                if (q.type == WELD_F64) o.f("w_min_f64(t%d, t%d)", q.a, q.b);
                else o.f("(t%d < t%d ? t%d : t%d)", q.b, q.a, q.b, q.a);
                break;
            case WELD_OP_MAX:
                if (q.type == WELD_F64) o.f("w_max_f64(t%d, t%d)", q.a, q.b);
                else o.f("(t%d > t%d ? t%d : t%d)", q.b, q.a, q.b, q.a);
                break;
            case WELD_OP_LT: o.f("t%d < t%d", q.a, q.b); break;
            case WELD_OP_LE: o.f("t%d <= t%d", q.a, q.b); break;
            case WELD_OP_GT: o.f("t%d > t%d", q.a, q.b); break;
            case WELD_OP_GE: o.f("t%d >= t%d", q.a, q.b); break;
            case WELD_OP_EQ: o.f("t%d == t%d", q.a, q.b); break;
            case WELD_OP_NE: o.f("t%d != t%d", q.a, q.b); break;
            case WELD_OP_AND: o.f("(bool)((int)t%d & (int)t%d)", q.a, q.b); break;
            case WELD_OP_OR: o.f("(bool)((int)t%d | (int)t%d)", q.a, q.b); break;
            case WELD_OP_SELECT: o.f("t%d ? t%d : t%d", q.a, q.b, q.c); break;
            case WELD_OP_LOOKUP:
                if (guarded(i)) o.f("!t%d ? (%s)0 : ", need[i], T);
                o.f("w_lookup(a.g%d, a.g%d_len, (i64)t%d, errp)", q.a, q.a, q.b);
                break;
            case WELD_OP_OUTER: o.f("a.o%d[row]", q.a); break;
            case WELD_OP_KEYEXISTS: case WELD_OP_DICTLOOKUP: {
                const DictTable& t = L.dict_in[q.a];
                std::string key = std::string("((u64)(") + utype(t.key_type[0]) + ")t" + std::to_string(q.b) + ")";
                if (t.nkeys == 2)
                    key += std::string(" | ((u64)(") + utype(t.key_type[1]) + ")t" + std::to_string(q.c) + " << " +
                           std::to_string(8 * type_size(t.key_type[0])) + ")";
                // rows whose guarding predicate fails still issue the (cached) first load: see w_table_find
                const std::string live = guarded(i) ? "t" + std::to_string(need[i]) : std::string("true");
                if (q.opcode == WELD_OP_KEYEXISTS)
                    o.f("w_table_find(a.p%d_keys, a.p%d_hdr, a.p%d_slots, %s, %s) >= 0", q.a, q.a, q.a, key.c_str(), live.c_str());
                else
                    o.f("w_table_value<%s>(a.p%d_v%d, w_table_find(a.p%d_keys, a.p%d_hdr, a.p%d_slots, %s, %s))", T, q.a, q.reserved,
                        q.a, q.a, q.a, key.c_str(), live.c_str());
                break;
            }
        }
        o.f(";\n");
    }
    for (size_t b = 0; b < L.builders.size(); ++b) {
        const int m = L.merge_of[b];
        if (m < 0) continue;
        const weld_merge_t& g = L.merges[m];
        if (g.pred >= 0) o.f("  o.p%zu = t%d;", b, g.pred);
        else o.f("  o.p%zu = true;", b);
        for (int k = 0; k < g.nkeys; ++k) o.f(" o.k%zu_%d = t%d;", b, k, g.key[k]);
        for (int k = 0; k < g.nvals; ++k) o.f(" o.v%zu_%d = t%d;", b, k, g.val[k]);
        o.f("\n");
    }
    o.f("}\n\n");
}

// Static value ranges of the integer SSA values (interval arithmetic over the body): what a
// `mod` by a constant, a cast from a narrower type or a constant can be.  Used to hold 64-bit
// values that provably fit 32 bits in one register, and to give such keys compact cells.
struct IRange {
    __int128 lo, hi;
    bool fits32() const { return lo >= -((__int128)1 << 31) && hi <= ((__int128)1 << 31) - 1; }
};
IRange type_range(int t) {
    const int bits = t == WELD_BOOL ? 1 : 8 * type_size(t);
    if (t == WELD_BOOL) return IRange{0, 1};
    return IRange{-((__int128)1 << (bits - 1)), ((__int128)1 << (bits - 1)) - 1};
}
std::vector<IRange> static_ranges(const Loop& L) {
    std::vector<IRange> r(L.ops.size(), IRange{0, 0});
    for (size_t i = 0; i < L.ops.size(); ++i) {
        const weld_op_t& q = L.ops[i];
        if (q.type == WELD_F64) continue;
        const IRange full = type_range(q.type);
        IRange out = full;
        auto clamp = [&](__int128 lo, __int128 hi) {       // a result outside the type wraps: anything then
            if (lo >= full.lo && hi <= full.hi) out = IRange{lo, hi};
        };
        auto is_int = [&](int x) { return x >= 0 && L.ops[x].type != WELD_F64; };
        switch (q.opcode) {
            case WELD_OP_CONST: clamp(q.imm.i64, q.imm.i64); break;
            case WELD_OP_INDEX: out = IRange{0, full.hi}; break;
            case WELD_OP_CAST: if (is_int(q.a)) clamp(r[q.a].lo, r[q.a].hi); break;
            case WELD_OP_NEG: clamp(-r[q.a].hi, -r[q.a].lo); break;
            case WELD_OP_ADD: clamp(r[q.a].lo + r[q.b].lo, r[q.a].hi + r[q.b].hi); break;
            case WELD_OP_SUB: clamp(r[q.a].lo - r[q.b].hi, r[q.a].hi - r[q.b].lo); break;
            case WELD_OP_MUL: {
                const __int128 c[4] = {r[q.a].lo * r[q.b].lo, r[q.a].lo * r[q.b].hi, r[q.a].hi * r[q.b].lo, r[q.a].hi * r[q.b].hi};
                clamp(*std::min_element(c, c + 4), *std::max_element(c, c + 4));
                break;
            }
            case WELD_OP_MOD: case WELD_OP_DIV: {
                const weld_op_t& d = L.ops[q.b];
                if (d.opcode != WELD_OP_CONST || d.imm.i64 == 0 || d.imm.i64 == INT64_MIN) break;
                const __int128 m = d.imm.i64 < 0 ? -(__int128)d.imm.i64 : (__int128)d.imm.i64;
                if (q.opcode == WELD_OP_MOD) {      // truncating: the sign of the dividend, magnitude below |divisor|
                    clamp(r[q.a].lo >= 0 ? 0 : -(m - 1), r[q.a].hi <= 0 ? 0 : m - 1);
                } else if (d.imm.i64 > 0) {
                    clamp(r[q.a].lo / m, r[q.a].hi / m);
                }
                break;
            }
            case WELD_OP_MIN: clamp(std::min(r[q.a].lo, r[q.b].lo), std::min(r[q.a].hi, r[q.b].hi)); break;
            case WELD_OP_MAX: clamp(std::max(r[q.a].lo, r[q.b].lo), std::max(r[q.a].hi, r[q.b].hi)); break;
            case WELD_OP_SELECT: clamp(std::min(r[q.b].lo, r[q.c].lo), std::max(r[q.b].hi, r[q.c].hi)); break;
            default: break;     // columns, lookups, compares (bool: full range already)
        }
        r[i] = out;
    }
    return r;
}

// Whether dictmerger b (realised as an LDS table) can keep compact cells; *sext: the packed key is the
// sign extension of its low half; *guard: |constant| merged per row when the value is a 64-bit constant.
bool compact_eligible(const Loop& L, size_t b, bool* sext, long long* guard) {
    const weld_builder_spec_t& s = L.builders[b];
    const int m = L.merge_of[b];
    if (s.kind != WELD_DICTMERGER || m < 0 || s.nvals != 1 || s.func != WELD_FUNC_ADD || s.val_type[0] == WELD_F64) return false;
    const weld_merge_t& g = L.merges[m];
    const std::vector<IRange> r = static_ranges(L);
    int bytes = 0;
    for (int k = 0; k < s.nkeys; ++k) bytes += type_size(s.key_type[k]);
    *sext = false;
    if (bytes > 4) {
        if (s.nkeys != 1 || !r[g.key[0]].fits32()) return false;
        *sext = true;
    }
    *guard = 0;
    if (s.val_type[0] == WELD_I64) {      // a 32-bit partial sum must stay exact: constants only, with a flush before 2^31
        const weld_op_t& v = L.ops[g.val[0]];
        if (v.opcode != WELD_OP_CONST) return false;
        const long long c = v.imm.i64 < 0 ? -v.imm.i64 : v.imm.i64;
        if (c > (1 << 10)) return false;
        *guard = c > 0 ? c : 1;
    }
    return true;
}

bool body_uses(const Loop& L, int opcode) {
    for (const weld_op_t& q : L.ops)
        if (q.opcode == opcode) return true;
    return false;
}

// expression packing the key struct of builder b into 64 bits (field 0 lowest)
std::string pack_key(const weld_builder_spec_t& s, size_t b, const char* row) {
    std::string e;
    int shift = 0;
    for (int k = 0; k < s.nkeys; ++k) {
        char buf[128];
        snprintf(buf, sizeof buf, "%s((u64)(%s)%s.k%zu_%d << %d)", k ? " | " : "", utype(s.key_type[k]), row, b, k, shift);
        e += buf;
        shift += 8 * type_size(s.key_type[k]);
    }
    return e;
}

// builders whose merges go to memory at a computed address (as opposed to register accumulators)
bool merges_in_memory(int backend) {
    return backend == BK_DICT_LDS || backend == BK_DICT_GLOBAL || backend == BK_VECM_LDS || backend == BK_VECM_GLOBAL ||
           backend == BK_VECM_QUEUE;
}

}  // namespace

bool value_fits32(const Loop& L, int op) {
    if (op < 0 || (size_t)op >= L.ops.size() || L.ops[op].type == WELD_F64) return false;
    return static_ranges(L)[op].fits32();
}

Variant choose_variant(const Loop& L, const weld_tuning_t& tune, bool aligned) {
    Variant var;
    int widest = 1;
    bool any = false;
    for (int c = 0; c < L.ncols; ++c)
        if (L.col_used[c]) { any = true; if (type_size(L.col_type[c]) > widest) widest = type_size(L.col_type[c]); }
    var.backend.assign(L.builders.size(), BK_MERGER);
    for (size_t b = 0; b < L.builders.size(); ++b) {
        const weld_builder_spec_t& s = L.builders[b];
        const int m = L.merge_of[b];
        if (s.kind == WELD_MERGER) {
            var.backend[b] = BK_MERGER;
        } else if (s.kind == WELD_VECBUILDER) {
            const bool cond = m >= 0 && L.merges[m].pred >= 0;
            var.backend[b] = cond ? BK_VEC_COMPACT : BK_VEC_DIRECT;
            if (cond) var.ticketed = true;
            if (m >= 0 && type_size(s.val_type[0]) > widest) widest = type_size(s.val_type[0]);
        } else if (s.kind == WELD_VECMERGER) {
            // Sec. 7.7: thread-local copies, work-group copies with atomics, one global copy
            int strat = tune.vecmerger_strategy;
            const bool queues_allowed = strat >= 0;        // (-1: the library's choice among the strategies without workspace)
            if (strat < 0) strat = 0;
            if (strat == 1 && s.length > 8) strat = 0;
            if (strat == 2 && s.length > 16384) strat = 0;
            // measured with 1e8 uniform keys: LDS copy 0.09-0.12 ms up to 8192 cells; register copies
            // 0.24 ms at 8 cells (kept for f64, whose LDS atomics serialise on few addresses);
            // global copy 4.2 ms (23.7 G atomics/s) for large vectors, 13-390 ms below 1024 cells
            // A fourth strategy: the cells are split into 8192-cell ranges, each owned by a group of
            // work-groups that scans ALL rows and merges only its range in LDS.  Reading the keys R times
            // at 6+ TB/s (0.09 ms a pass) beats one pass of global atomics (4.2 ms) up to R ~ 40, but the
            // queues of the fifth strategy below only for two ranges (16384 cells: 0.24 ms against 0.44;
            // 32768 cells: 0.43 against 0.36).  Only for loops whose single builder is this vecmerger:
            // everything else would be repeated R times too.
            const bool alone = L.builders.size() == 1;
            if (strat == 4 && (!alone || s.length > 8192 * 64)) strat = 0;
            // Beyond that a fifth: every merge is appended to a queue by range of cells (segment [work-group][range],
            // 2 bytes an entry where the merged value is a constant, else 10), and a second kernel merges each
            // range in LDS and adds it to the result - two streaming passes instead of one device atomic per row.
            // One such vecmerger per loop; up to 8192 ranges of 8192 cells.
            const bool can_queue = queues_allowed && var.vq_builder < 0 && m >= 0 && s.length > 8192 && s.length <= (int64_t)8192 * 8192 && tune.dict_spill >= 0;
            bool unsorted = false;                 // (6: 5 without sorting a tile's entries in LDS)
            if (strat == 6) { strat = 5; unsorted = true; }
            if (strat == 5 && !can_queue) strat = 0;
            if (strat == 0) strat = (s.length <= 8 && s.val_type[0] == WELD_F64) ? 1
                                  : s.length <= 8192 ? 2 : (alone && s.length <= 8192 * 2) ? 4 : can_queue ? 5 : 3;
            var.backend[b] = strat == 1 ? BK_VECM_REG : (strat == 2 || strat == 4) ? BK_VECM_LDS : strat == 5 ? BK_VECM_QUEUE : BK_VECM_GLOBAL;
            if (strat == 4) var.ranges = (int)((s.length + 8191) / 8192);
            if (strat == 5) {
                var.vq_builder = (int)b;
                var.vq_shift = 8;
                // (1e8 uniform keys, 2^20 cells, one store per row (then of 4 bytes): 0.58 ms with 128 ranges, 0.62 with 256, 0.75 with 512,
                // 0.92 with 1024 - every range is one more line a work-group keeps open; with a tile's entries sorted in LDS
                // first 0.35 ms with 128 ranges and 0.32 with 256, which put the second kernel on every compute unit)
                while (var.vq_shift < 13 && ((s.length + ((int64_t)1 << var.vq_shift) - 1) >> var.vq_shift) > 256) ++var.vq_shift;
                var.vq_ranges = (int)((s.length + ((int64_t)1 << var.vq_shift) - 1) >> var.vq_shift);
                var.vq_const = L.ops[L.merges[m].val[0]].opcode == WELD_OP_CONST;
                var.vq_sorted = !unsorted;         // (if the rest of the loop allows: decided below)
            }
        } else {
            int strat = tune.dict_strategy;
            const bool few = s.capacity <= 8 && key_bits(s) < 64;
            const int blk = tune.block_threads > 0 ? tune.block_threads : 256;
            const bool lane_fits = few && (int64_t)s.capacity * s.nvals * 8 * blk <= 96 * 1024;
            if ((strat == 1 && !few) || (strat == 4 && !lane_fits)) strat = 0;
            if (strat == 0) strat = few ? 1 : 2;   // measured on C4: register slots 1.21 ms, LDS lane slots 1.20-1.52 ms
            var.backend[b] = strat == 1 ? BK_DICT_REG : strat == 4 ? BK_DICT_LANE
                           : strat == 2 ? BK_DICT_LDS : BK_DICT_GLOBAL;
        }
    }
    // a single LDS dictionary that counts, or sums 32-bit integers, under a key of 32 bits: compact cells
    {
        int ndl = 0, which = -1;
        for (size_t b = 0; b < L.builders.size(); ++b)
            if (var.backend[b] == BK_DICT_LDS) { ++ndl; which = (int)b; }
        bool sext = false;
        long long guard = 0;
        if (ndl == 1 && tune.dict_compact >= 0 && compact_eligible(L, (size_t)which, &sext, &guard)) {
            var.compact = which;
            var.compact_sext = sext;
            var.compact_guard = guard;
        }
    }
    // every LDS dictionary of the loop gets the same slot count; the LDS budget (64 KiB,
    // 128 KiB when some dictionary has more keys than 64 KiB hold) is shared among them
    bool big_dict = false;
    {
        int ndl = 0, per_slot = 0;
        int64_t max_cap = 0;
        for (size_t b = 0; b < L.builders.size(); ++b)
            if (var.backend[b] == BK_DICT_LDS) {
                ++ndl;
                per_slot += var.compact == (int)b ? 8 : 8 * (1 + L.builders[b].nvals);
                if (L.builders[b].capacity > max_cap) max_cap = L.builders[b].capacity;
            }
        if (ndl > 0) {
            int want = tune.lds_dict_slots;
            if (want <= 0) {
                want = 64;
                while (want * 2 * per_slot <= 64 * 1024 && want < 2 * max_cap) want *= 2;
                if (max_cap > want)
                    while (want * 2 * per_slot <= 128 * 1024) want *= 2;
            }
            int p2 = 64;
            while (p2 < want && p2 < (1 << 14)) p2 *= 2;
            var.lds_slots = p2;
            big_dict = (int64_t)p2 * per_slot > 64 * 1024;
            if (max_cap > p2 && ndl == 1) {
                // more keys than slots: an admission filter keeps the once-per-work-group keys
                // of a heavy tail out of the table, and the misses - the bulk of the kernel's
                // time when each is a device atomic (C5: 1.2e7 of them at 23.7 G/s) - are
                // queued for a second kernel instead
                if (tune.lds_filter_words >= 0) {
                    const int w = tune.lds_filter_words > 0 ? tune.lds_filter_words : 2048;   // 65536 bits
                    int p2w = 64;
                    while (p2w < w && p2w < 8192) p2w *= 2;
                    var.door_words = p2w;
                }
                // the second kernel aggregates one partition per LDS table, which needs a partition's share
                // of the keys to fit one; beyond that (below) the partitions become slices of the table
                int nv = 1;
                for (size_t b = 0; b < L.builders.size(); ++b)
                    if (var.backend[b] == BK_DICT_LDS) nv = L.builders[b].nvals;
                const int64_t part_slots = nv <= 1 ? 8192 : nv <= 3 ? 4096 : nv <= 7 ? 2048 : 1024;
                if (tune.dict_spill >= 0 && max_cap <= 256 * part_slots * 3 / 4) {
                    var.spill = true;
                } else if (tune.dict_spill >= 0 && dict_table_slots(max_cap) / part_slots <= 4096) {
                    // more keys than 256 LDS tables hold, but a global table of at most 4096 LDS tables:
                    // the queues are partitioned by slice of that table, which is then built slice by slice
                    var.spill = true;
                    var.spill_slices = true;
                    var.spill_parts = (int)(dict_table_slots(max_cap) / part_slots);
                }
            }
        }
    }
    if (var.spill_slices) var.compact = -1;      // the slice-building kernel reads full entries
    if (var.compact >= 0) var.door_words = 0;    // measured on the zip-code loop with 16384 compact slots: 11.7 % of the
                                                 // merges miss the table with the filter, 10.0 % without
    (void)any;
    var.v = widest >= 8 ? 2 : 4;
    // Look-back kernels pay one same-address device atomic (about 12 ns, serialised) and
    // three barriers per tile: they take large tiles (8192 rows).  Other kernels keep
    // 8 KiB (4 KiB for V=4) of loads in flight per wavefront and column.
    if (big_dict || var.vq_builder >= 0) {
        var.u = tune.units_per_thread > 0 ? tune.units_per_thread : 16 / var.v;
        var.block = tune.block_threads > 0 ? tune.block_threads : 1024;
    } else if (var.ticketed) {
        // (measured on the zip-code compaction, 1e8 rows: 0.42 ms with 256 threads, 0.36 with 512, 0.32 with 1024:
        // the per-tile costs - ticket, look-back, three barriers - are paid once per 16384 rows)
        var.u = tune.units_per_thread > 0 ? tune.units_per_thread : 16 / var.v;
        var.block = tune.block_threads > 0 ? tune.block_threads : 1024;
    } else {
        // register-slot dictionaries hold capacity x fields accumulators per lane: fewer loads in
        // flight leave room for a third wavefront per SIMD (C4: 1.22 -> 1.17 ms)
        bool reg_dict = false;
        for (size_t b = 0; b < L.builders.size(); ++b)
            if (var.backend[b] == BK_DICT_REG && L.builders[b].capacity * L.builders[b].nvals >= 24) reg_dict = true;
        var.u = tune.units_per_thread > 0 ? tune.units_per_thread : (var.v == 2 ? (reg_dict ? 2 : 4) : 2);
        // rows that look a key up in a dictionary wait for two dependent reads of random lines: more wavefronts with
        // fewer rows each hide that better than more loads per lane (the join's probe loop, 6e7 rows: 0.21 -> 0.19 ms when the
        // table's lines are still in the memory-side cache from the probe before; right after the build 0.26 ms either way)
        if (tune.units_per_thread <= 0 && (body_uses(L, WELD_OP_DICTLOOKUP) || body_uses(L, WELD_OP_KEYEXISTS))) var.u = 1;
        // ... and 2048-row tiles in 512-thread work-groups, one per compute unit, are 2 % faster for them than
        // 1024-row tiles in two 256-thread work-groups (C4: 1.14 -> 1.11 ms; the same eight wavefronts per unit)
        var.block = tune.block_threads > 0 ? tune.block_threads : (reg_dict ? 512 : 256);
    }
    if (var.u > 16) var.u = 16;
    // (the sorted form of the queued vecmerger stages a tile's indices in LDS, 4 bytes each: static tiles of at most 16384 rows)
    // (... and entries with a value, 12 bytes a row in the staging arrays: tiles of 8192 rows, at most 2048 ranges)
    var.vq_sorted = var.vq_sorted && var.vq_builder >= 0 && var.vq_ranges <= (var.vq_const ? 4096 : 2048) && !var.ticketed && var.ranges == 1;
    // (LDS at the limits: staging 64 or 96 KiB, four arrays of 4 bytes a range, 12 KiB for merges that find their segment full)
    if (var.vq_sorted && !var.vq_const && tune.units_per_thread <= 0)
        while (var.u > 1 && (int64_t)var.block * var.v * var.u > 8192) var.u /= 2;
    var.vq_sorted = var.vq_sorted && (int64_t)var.block * var.v * var.u <= (var.vq_const ? 16384 : 8192);
    for (size_t b = 0; b < L.builders.size(); ++b)      // (the staging array takes 64 KiB: not beside another builder's LDS state)
        if (var.backend[b] == BK_DICT_LDS || var.backend[b] == BK_DICT_LANE || var.backend[b] == BK_VECM_LDS) var.vq_sorted = false;
    if (var.block < 64) var.block = 64;
    if (var.block > 1024) var.block = 1024;
    var.block = (var.block / 64) * 64;
    var.aligned = aligned ? 1 : 0;
    var.own_math = tune.device_math >= 0;
    // the LDS dictionary shares the 160 KiB with the compaction's staging buffer, the admission
    // filter, the spill counters and the erf table: halve it until everything fits
    if (var.lds_slots > 0) {
        int per_slot = 0;
        for (size_t b = 0; b < L.builders.size(); ++b)
            if (var.backend[b] == BK_DICT_LDS) per_slot += var.compact == (int)b ? 8 : 8 * (1 + L.builders[b].nvals);
        int other = (var.ticketed ? 8 * var.block * var.v : 0) + 4 * var.door_words + (var.spill ? 4 * var.spill_parts : 0) +
                    (body_uses(L, WELD_OP_ERF) ? 7680 : 0) + (body_uses(L, WELD_OP_LOG) ? 2184 : 0) + (body_uses(L, WELD_OP_EXP) ? 1024 : 0) + 2048 +
                    (var.vq_builder >= 0 ? 4 * var.vq_ranges + 12 * 1024 : 0);
        for (size_t b = 0; b < L.builders.size(); ++b) {
            if (var.backend[b] == BK_VECM_LDS) other += 8 * (var.ranges > 1 ? 8192 : (int)L.builders[b].length);
            if (var.backend[b] == BK_DICT_REG || var.backend[b] == BK_DICT_LANE) other += 8 * (int)L.builders[b].capacity;
            if (var.backend[b] == BK_DICT_LANE) other += 8 * (int)L.builders[b].capacity * L.builders[b].nvals * var.block;
        }
        while (var.lds_slots > 64 && var.lds_slots * per_slot + other > 160 * 1024) var.lds_slots /= 2;
    }
    // Merges into hash tables and vecmergers are divergent code (probe, claim, overflow paths).
    // Unrolled over the rows a lane holds per tile they multiply the kernel text and leave the
    // compiler short of scalar registers for the execution masks; one loop over the rows, which
    // indexes the lane's values with the loop counter, keeps that code once.
    {
        bool in_memory = false;
        for (size_t b = 0; b < L.builders.size(); ++b)
            if (L.merge_of[b] >= 0 && merges_in_memory(var.backend[b])) in_memory = true;
        const int rows = var.u * var.v;
        // one LDS dictionary in a compacting loop: its merges beyond the first probe are queued per
        // wavefront (in the wavefront's part of the staging buffer, free while the tile merges)
        int nlds = 0, which = -1;
        for (size_t b = 0; b < L.builders.size(); ++b)
            if (var.backend[b] == BK_DICT_LDS && L.merge_of[b] >= 0) { ++nlds; which = (int)b; }
        if (tune.dict_defer >= 0 && nlds == 1 && var.ticketed && rows >= 4 && rows <= 16) {
            const weld_merge_t& g = L.merges[L.merge_of[which]];
            int words = 1;
            for (int k = 0; k < g.nvals; ++k)
                if (L.ops[g.val[k]].opcode != WELD_OP_CONST) ++words;
            const int cap = 64 * var.v / words;
            if (cap >= 64) { var.defer_builder = which; var.defer_cap = cap; }
        }
        var.merge_loop = (tune.merge_loop > 0 || var.defer_builder >= 0) && var.ticketed && in_memory && rows >= 4 && rows <= 16;
    }
    // Compacting loops that also merge into memory: the next tile's columns are loaded while this tile
    // is merged and stored (C5, 1e8 rows: loop kernel 0.50 -> 0.46 ms).  Those columns then occupy
    // registers through the merge phase, next to the tile's gathered values and the slots and keys of
    // the first probes; where the three together pass about 80 registers a lane the kernel spills and
    // loses more than it gains (the same column grouped by key: 0.73 -> 0.90 ms), and a loop that only
    // compacts has no merge phase to hide the loads behind (0.32 -> 0.34 ms): both keep the plain form.
    if (var.ticketed && var.merge_loop && tune.tile_pipeline >= 0) {
        const int rows = var.u * var.v;
        int regs = 0;
        for (int c = 0; c < L.ncols; ++c)
            if (L.col_used[c]) regs += (type_size(L.col_type[c]) * rows + 3) / 4;
        const std::vector<IRange> rg = static_ranges(L);
        std::vector<int> held;
        for (size_t b = 0; b < L.builders.size(); ++b) {
            const int m = L.merge_of[b];
            if (m < 0 || (!merges_in_memory(var.backend[b]) && var.backend[b] != BK_VEC_COMPACT)) continue;
            const weld_merge_t& g = L.merges[m];
            for (int f = 0; f < g.nkeys + g.nvals; ++f) {
                const int op = f < g.nkeys ? g.key[f] : g.val[f - g.nkeys];
                if (L.ops[op].opcode == WELD_OP_CONST || std::find(held.begin(), held.end(), op) != held.end()) continue;
                held.push_back(op);
                const int t = L.ops[op].type;
                regs += ((t == WELD_F64 || (t == WELD_I64 && !rg[op].fits32())) ? 2 : 1) * rows;
            }
        }
        if (var.defer_builder >= 0) regs += (var.compact == var.defer_builder ? 2 : 3) * rows;
        if (tune.tile_pipeline > 0 || regs <= 80) var.pipeline = 1;
    }
    // Mergers only: the kernel can finish the call by itself.  Every work-group publishes its partials, then
    // counts itself in; the one that arrives last combines all partials in index order and writes the
    // results and the status words, so the call is one launch instead of three (at 1e6 rows the loop kernel
    // takes 8 us and the two small kernels around it, with the gaps between dependent launches, twice that).
    // No cache maintenance is involved: partials and counter are device-scope atomics, which are performed
    // where every XCD sees them, and a wavefront counts itself in only after its own have been acknowledged.
    if (tune.single_launch >= 0 && !var.ticketed && !L.builders.empty()) {
        var.single = true;
        for (int bk : var.backend)
            if (bk != BK_MERGER) var.single = false;
    }
    return var;
}

// Stores of one spill-queue entry at word offset `ei` of builder b's log: 16 bytes at a time
// when the entry has an even number of words (entries are then 16-byte aligned).
static void emit_log_stores(Out& o, size_t b, const std::vector<std::string>& words, const char* eol) {
    const size_t n = words.size();
    if (n % 2 == 0) {
        for (size_t q = 0; q < n; q += 2)
            o.f("        w_gstore2(a.b%zu_log + ei + %zu, %s, %s);%s\n", b, q, words[q].c_str(), words[q + 1].c_str(), eol);
    } else {
        for (size_t q = 0; q < n; ++q)
            o.f("        w_gstore1(a.b%zu_log + ei + %zu, %s);%s\n", b, q, words[q].c_str(), eol);
    }
}

Generated generate(const Loop& L, const Variant& var) {
    Generated G;
    Out o;
    const size_t NB = L.builders.size();
    const std::vector<IRange> ranges = static_ranges(L);
    o.f("// generated: fused for-loop kernel, %d columns, %zu builders\n", L.ncols, NB);
    o.f("#define W_BLOCK %d\n#define W_V %d\n#define W_U %d\n#define W_ALIGNED %d\n", var.block, var.v, var.u, var.aligned);
    if (var.spill_slices) {
        int nv = 1;
        for (size_t b = 0; b < NB; ++b)
            if (var.backend[b] == BK_DICT_LDS) nv = L.builders[b].nvals;
        const int slice_bits = nv <= 1 ? 13 : nv <= 3 ? 12 : nv <= 7 ? 11 : 10;       // slots of a slice: what the LDS holds of this entry size
        o.f("#define W_SPILL_PARTS %d\n#define W_SPILL_SLICE_BITS %d\n#define W_SPILL_BY_SLOT 1\n", var.spill_parts, slice_bits);
    }
    const bool uses_erf = body_uses(L, WELD_OP_ERF);
    if (uses_erf) o.f("#define W_USE_ERF 1\n");
    const bool uses_log = var.own_math && body_uses(L, WELD_OP_LOG), uses_exp = var.own_math && body_uses(L, WELD_OP_EXP);
    if (uses_log) o.f("#define W_USE_LOG 1\n#define W_LOG w_log\n");
    else o.f("#define W_LOG log\n");
    if (uses_exp) o.f("#define W_USE_EXP 1\n#define W_EXP w_exp\n");
    else o.f("#define W_EXP exp\n");
    o.s += kPreludeSource;
    o.f("\n");

    // ------------------------------------------------------------ kernel arguments
    auto slot = [&](SlotKind k, int builder, int field, const std::string& name, const std::string& ct) {
        Slot s{k, builder, field, name, ct};
        G.slots.push_back(s);
    };
    slot(SLOT_N, -1, 0, "n", "i64");
    slot(SLOT_SPIN, -1, 0, "spin_limit", "i64");
    for (int c = 0; c < L.ncols; ++c)
        if (L.col_used[c]) slot(SLOT_COL, c, 0, "c" + std::to_string(c), std::string("const ") + stype(L.col_type[c]) + "* __restrict__");
    for (int c = 0; c < L.ncols; ++c)   // scalars from outside the loop: one element each
        if (L.col_scalar[c]) slot(SLOT_COL, c, 0, "s" + std::to_string(c), std::string("const ") + stype(L.col_type[c]) + "* __restrict__");
    slot(SLOT_CTL, -1, 0, "ctl", "u32*");
    if (var.single) slot(SLOT_ARRIVE, -1, 0, "arrive", "u32*");
    for (int d = 0; d < L.ndicts; ++d) {
        const std::string P = "p" + std::to_string(d);
        slot(SLOT_PKEYS, d, 0, P + "_keys", "const u64* __restrict__");
        slot(SLOT_PHDR, d, 0, P + "_hdr", "const u32* __restrict__");
        slot(SLOT_PSLOTS, d, 0, P + "_slots", "i64");
        for (int k = 0; k < L.dict_in[d].nvals; ++k)
            if (L.dict_val_used[d][k])
                slot(SLOT_PVAL, d, k, P + "_v" + std::to_string(k), std::string("const ") + acc_ctype(L.dict_in[d].val_type[k]) + "* __restrict__");
    }
    int ncompact = 0;
    for (size_t b = 0; b < NB; ++b) {
        const weld_builder_spec_t& s = L.builders[b];
        const std::string B = "b" + std::to_string(b);
        switch (var.backend[b]) {
            case BK_MERGER:
                slot(SLOT_PARTIAL, (int)b, 0, B + "_part", "u64*");
                if (var.single) slot(SLOT_RES, (int)b, 0, B + "_res", std::string(stype(s.val_type[0])) + "*");
                break;
            case BK_VEC_DIRECT:
                slot(SLOT_OUT, (int)b, 0, B + "_out", std::string(stype(s.val_type[0])) + "* __restrict__");
                break;
            case BK_VEC_COMPACT:
                slot(SLOT_OUT, (int)b, 0, B + "_out", std::string(stype(s.val_type[0])) + "* __restrict__");
                slot(SLOT_DESC, (int)b, 0, B + "_desc", "u64*");
                slot(SLOT_LEN, (int)b, 0, B + "_len", "i64*");
                ++ncompact;
                break;
            case BK_VECM_REG: case BK_VECM_LDS: case BK_VECM_GLOBAL:
                slot(SLOT_OUT, (int)b, 0, B + "_out", std::string(acc_ctype(s.val_type[0])) + "*");
                break;
            case BK_VECM_QUEUE:
                slot(SLOT_OUT, (int)b, 0, B + "_out", std::string(acc_ctype(s.val_type[0])) + "*");
                slot(SLOT_DLOG, (int)b, 0, B + "_log", "u64*");
                slot(SLOT_DQCNT, (int)b, 0, B + "_qcnt", "u32*");
                slot(SLOT_DQCAP, (int)b, 0, B + "_qcap", "i64");
                break;
            default:
                slot(SLOT_DKEYS, (int)b, 0, B + "_keys", "u64*");
                slot(SLOT_DHDR, (int)b, 0, B + "_hdr", "u32*");
                slot(SLOT_DSLOTS, (int)b, 0, B + "_slots", "i64");
                for (int k = 0; k < s.nvals; ++k)
                    slot(SLOT_DVAL, (int)b, k, B + "_v" + std::to_string(k), std::string(acc_ctype(s.val_type[k])) + "*");
                if (var.backend[b] == BK_DICT_LDS && var.spill) {
                    slot(SLOT_DLOG, (int)b, 0, B + "_log", "u64*");
                    slot(SLOT_DQCNT, (int)b, 0, B + "_qcnt", "u32*");
                    slot(SLOT_DQCAP, (int)b, 0, B + "_qcap", "i64");
                }
        }
    }
    o.f("struct KArgs {\n");
    for (const Slot& s : G.slots) o.f("  %s %s;\n", s.ctype.c_str(), s.name.c_str());
    o.f("};\n\n");

    emit_row_function(o, L);

    // ------------------------------------------------------------ merge statements
    // (everything except vecbuilders, which the tile code handles)
    // The whole merge of one (key, values) into dictionary b, given `kb` and the value
    // expressions: LDS table (up to three probes, admission filter), then spill queue, then
    // the global table.  Lines of a macro body.
    auto emit_dict_slow = [&](Out& o, size_t b, const std::vector<std::string>& vals) {
        const weld_builder_spec_t& s = L.builders[b];
        const int F = s.func;
        const bool compact = var.compact == (int)b;
        if (compact) {
            o.f("    const int sl = w_lds_slot32(d%zu_ck, %d, kb, 3); \\\n", b, var.lds_slots);
            o.f("    if (sl >= 0) { \\\n      w_lds_add32(d%zu_cv, sl, (i64)%s); \\\n    } else { \\\n", b, vals[0].c_str());
        } else if (var.backend[b] == BK_DICT_LDS) {
            if (var.door_words > 0)
                o.f("    const int sl = w_lds_slot_filtered(d%zu_lk, %d, kb, 3, d%zu_door, %d); \\\n", b, var.lds_slots, b, var.door_words);
            else
                o.f("    const int sl = w_lds_slot(d%zu_lk, %d, kb, 3); \\\n", b, var.lds_slots);
            o.f("    if (sl >= 0) { \\\n");
            for (int k = 0; k < s.nvals; ++k)
                o.f("      w_atomic<%d>(d%zu_lv%d + sl, %s, 0); \\\n", F, b, k, vals[k].c_str());
            o.f("    } else { \\\n");
        } else {
            o.f("    { \\\n");
        }
        const bool spill = var.backend[b] == BK_DICT_LDS && var.spill;
        if (spill) {
            o.f("      const i64 ei = w_spill_index(d%zu_qn, a.b%zu_qcap, %d, kb); \\\n", b, b, compact ? 1 : 1 + s.nvals);
            o.f("      if (ei >= 0) { \\\n");
            std::vector<std::string> words;
            if (compact) {
                words.push_back("w_compact_entry(kb, (i64)" + vals[0] + ")");
            } else {
                words.push_back("kb");
                for (int k = 0; k < s.nvals; ++k) words.push_back("w_bits(" + vals[k] + ")");
            }
            emit_log_stores(o, b, words, " \\");
            o.f("      } else { \\\n");
            // (tells the kernel that builds the table slice by slice that the table is no longer empty)
            if (var.spill_slices) o.f("      __hip_atomic_store(a.b%zu_hdr, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); \\\n", b);
        }
        o.f("      const i64 g = w_table_slot(a.b%zu_keys, a.b%zu_hdr, a.b%zu_slots, kb, errp); \\\n", b, b, b);
        o.f("      if (g >= 0) { \\\n");
        for (int k = 0; k < s.nvals; ++k)
            o.f("        w_atomic<%d>(a.b%zu_v%d + g, %s, 1); \\\n", F, b, k, vals[k].c_str());
        if (spill) o.f("      } \\\n");
        o.f("      } \\\n    } \\\n");
    };
    if (var.defer_builder >= 0) {
        // the queued merges of one wavefront, 64 at a time: entry e is key word dq[e] and value
        // words dq[cap * w + e]; merged values that are constants are not stored
        const size_t b = (size_t)var.defer_builder;
        const weld_builder_spec_t& s = L.builders[b];
        const weld_merge_t& g = L.merges[L.merge_of[b]];
        o.f("#define WELD_DRAIN() do { \\\n  __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, \"wavefront\"); \\\n");
        o.f("  for (int qb = 0; qb < dq_n; qb += 64) { \\\n    const int e = qb + lane; \\\n    if (e < dq_n) { \\\n    const u64 kb = dq[e]; \\\n");
        std::vector<std::string> vals;
        int w = 1;
        for (int k = 0; k < s.nvals; ++k) {
            char buf[160];
            const char* A = acc_ctype(s.val_type[k]);
            if (L.ops[g.val[k]].opcode == WELD_OP_CONST) {
                snprintf(buf, sizeof buf, "(%s)(%s)%s", A, ctype(s.val_type[k]), const_expr(L.ops[g.val[k]]).c_str());
            } else {
                snprintf(buf, sizeof buf, "w_from_bits<%s>(dq[%d + e])", A, var.defer_cap * w);
                ++w;
            }
            vals.push_back(buf);
        }
        emit_dict_slow(o, b, vals);
        o.f("    } \\\n  } \\\n  __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, \"wavefront\"); \\\n  dq_n = 0; \\\n} while (0)\n\n");
    }

    // which: 0 = every builder, 1 = those held in registers, 2 = those held in memory; tile: the merge of the
    // vecmerger whose tile entries are sorted in LDS only notes its index in `e` (0xffffffff: nothing to merge)
    auto emit_merge_macro = [&](const char* name, int which, bool tile = false) {
    o.f(tile ? "#define %s(o, e, vb) do { \\\n" : "#define %s(o) do { \\\n", name);
    for (size_t b = 0; b < NB; ++b) {
        if (L.merge_of[b] < 0) continue;
        if (which == 1 && merges_in_memory(var.backend[b])) continue;
        if (which == 2 && !merges_in_memory(var.backend[b])) continue;
        const weld_builder_spec_t& s = L.builders[b];
        if (tile && (int)b == var.vq_builder) {
            o.f("  (e) = 0xffffffffu; \\\n  if ((o).p%zu) { \\\n    const i64 ix = (o).k%zu_0; \\\n", b, b);
            if (var.vq_const)
                o.f("    if ((u64)ix < (u64)%lldll) (e) = (u32)ix; else atomicOr(errp, 4); \\\n  } \\\n", (long long)s.length);
            else
                o.f("    if ((u64)ix < (u64)%lldll) { (e) = (u32)ix; (vb) = w_bits((%s)(o).v%zu_0); } else atomicOr(errp, 4); \\\n  } \\\n",
                    (long long)s.length, acc_ctype(s.val_type[0]), b);
            continue;
        }
        const int F = s.func;
        if (var.backend[b] == BK_MERGER) {
            o.f("  if ((o).p%zu) m%zu = w_combine<%d>(m%zu, (%s)(o).v%zu_0); \\\n", b, b, F, b, acc_ctype(s.val_type[0]), b);
        } else if (var.backend[b] == BK_DICT_REG || var.backend[b] == BK_DICT_LANE) {
            const int S = (int)s.capacity;
            o.f("  if ((o).p%zu) { \\\n", b);
            o.f("    const u64 kb = %s; \\\n", pack_key(s, b, "(o)").c_str());
            o.f("    int sl = -1; \\\n");
            o.f("    _Pragma(\"unroll\") for (int q = 0; q < %d; ++q) if (kb == d%zu_kreg[q]) sl = q; \\\n", S, b);
            o.f("    if (sl < 0) { \\\n");
            o.f("      sl = w_slot_list_insert<%d>(d%zu_lk, kb, errp); \\\n", S, b);
            o.f("      _Pragma(\"unroll\") for (int q = 0; q < %d; ++q) d%zu_kreg[q] = __hip_atomic_load(d%zu_lk + q, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP); \\\n", S, b, b);
            o.f("    } \\\n");
            if (var.backend[b] == BK_DICT_REG) {
                o.f("    _Pragma(\"unroll\") for (int q = 0; q < %d; ++q) if (sl == q) { \\\n", S);
                for (int k = 0; k < s.nvals; ++k)
                    o.f("      d%zu_a%d[q] = w_combine<%d>(d%zu_a%d[q], (%s)(o).v%zu_%d); \\\n", b, k, F, b, k, acc_ctype(s.val_type[k]), b, k);
                o.f("    } \\\n");
            } else {
                // this lane's own cell of group sl: [slot][lane] layout, so the 64 lanes of a
                // wavefront touch 64 consecutive 8-byte cells (no bank conflict, no atomic)
                o.f("    if (sl >= 0) { \\\n      const int cell = sl * W_BLOCK + (int)threadIdx.x; \\\n");
                for (int k = 0; k < s.nvals; ++k)
                    o.f("      d%zu_l%d[cell] = w_combine<%d>(d%zu_l%d[cell], (%s)(o).v%zu_%d); \\\n", b, k, F, b, k, acc_ctype(s.val_type[k]), b, k);
                o.f("    } \\\n");
            }
            o.f("  } \\\n");
        } else if (var.backend[b] == BK_VECM_QUEUE) {
            // a full segment (skewed indices, or a memory limit that left the queues short) sends the merge to the
            // result with a device atomic, as the global strategy does with every merge
            const char* A = acc_ctype(s.val_type[0]);
            o.f("  if ((o).p%zu) { \\\n    const i64 ix = (o).k%zu_0; \\\n", b, b);
            o.f("    if ((u64)ix < (u64)%lldll) { \\\n", (long long)s.length);
            o.f("      const u32 part = (u32)((u64)ix >> %d); \\\n", var.vq_shift);
            o.f("      const u32 pos = __hip_atomic_fetch_add(v%zu_qn + part, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP); \\\n", b);
            o.f("      if ((i64)pos < a.b%zu_qcap) { \\\n", b);
            o.f("        const u64 at = ((u64)blockIdx.x * %du + part) * (u64)a.b%zu_qcap + pos; \\\n", var.vq_ranges, b);
            if (var.vq_const) {
                o.f("        w_gstore_u16((unsigned short*)a.b%zu_log + at, (unsigned short)((u32)ix & %du)); \\\n", b, (1u << var.vq_shift) - 1);
            } else {
                // (a segment of entries with values: its values, 8 bytes each, then its cells within the range, 2 bytes each)
                o.f("        char* const sg = (char*)a.b%zu_log + (at - pos) * 10; \\\n", b);
                o.f("        w_gstore1((u64*)sg + pos, w_bits((%s)(o).v%zu_0)); \\\n", A, b);
                o.f("        w_gstore_u16((unsigned short*)(sg + 8 * a.b%zu_qcap) + pos, (unsigned short)((u32)ix & %du)); \\\n", b, (1u << var.vq_shift) - 1);
            }
            o.f("      } else w_vecm_overflow<%d>(v%zu_ot, v%zu_ov, (u32)ix, (%s)(o).v%zu_0, a.b%zu_out); \\\n", F, b, b, A, b, b);
            o.f("    } else atomicOr(errp, 4); \\\n  } \\\n");
        } else if (var.backend[b] == BK_VECM_REG || var.backend[b] == BK_VECM_LDS || var.backend[b] == BK_VECM_GLOBAL) {
            const char* A = acc_ctype(s.val_type[0]);
            o.f("  if ((o).p%zu) { \\\n    const i64 ix = (o).k%zu_0; \\\n", b, b);
            o.f("    if ((u64)ix < (u64)%lldll) { \\\n", (long long)s.length);
            if (var.backend[b] == BK_VECM_REG)
                o.f("      _Pragma(\"unroll\") for (int q = 0; q < %d; ++q) if (ix == q) v%zu_a[q] = w_combine<%d>(v%zu_a[q], (%s)(o).v%zu_0); \\\n", (int)s.length, b, F, b, A, b);
            else if (var.backend[b] == BK_VECM_LDS && var.ranges > 1)
                o.f("      const i64 rx = ix - range_lo; \\\n      if ((u64)rx < 8192ull) w_atomic<%d>(v%zu_l + rx, (%s)(o).v%zu_0, 0); \\\n", F, b, A, b);
            else if (var.backend[b] == BK_VECM_LDS)
                o.f("      w_atomic<%d>(v%zu_l + ix, (%s)(o).v%zu_0, 0); \\\n", F, b, A, b);
            else
                o.f("      w_atomic<%d>(a.b%zu_out + ix, (%s)(o).v%zu_0, 1); \\\n", F, b, A, b);
            o.f("    } else atomicOr(errp, 4); \\\n  } \\\n");
        } else if (var.backend[b] == BK_DICT_LDS || var.backend[b] == BK_DICT_GLOBAL) {
            std::vector<std::string> vals;
            for (int k = 0; k < s.nvals; ++k) {
                char buf[96];
                snprintf(buf, sizeof buf, "(%s)(o).v%zu_%d", acc_ctype(s.val_type[k]), b, k);
                vals.push_back(buf);
            }
            if (var.defer_builder != (int)b) {
                o.f("  if ((o).p%zu) { \\\n", b);
                o.f("    const u64 kb = %s; \\\n", pack_key(s, b, "(o)").c_str());
                emit_dict_slow(o, b, vals);
                o.f("  } \\\n");
            } else {
                // first probe only; whatever it does not settle is queued for the wavefront to
                // handle 64 at a time (WELD_DRAIN), instead of every lane walking the long path
                // of probes, admission filter, claim and overflow whenever one lane has to
                const weld_merge_t& g = L.merges[L.merge_of[b]];
                o.f("  { \\\n    const u64 kb = %s; \\\n    bool miss = false; \\\n", pack_key(s, b, "(o)").c_str());
                o.f("    if ((o).p%zu) { \\\n      miss = true; \\\n      if (kb != W_EMPTY_KEY) { \\\n", b);
                if (var.compact == (int)b) {
                    o.f("        const int s0 = (int)w_hash_slot32((u32)kb, %du); \\\n", var.lds_slots);
                    o.f("        if ((u32)kb != W_EMPTY_KEY32 && __hip_atomic_load(d%zu_ck + s0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP) == (u32)kb) { \\\n          miss = false; \\\n", b);
                    o.f("          w_lds_add32(d%zu_cv, s0, (i64)%s); \\\n", b, vals[0].c_str());
                } else {
                o.f("        const int s0 = (int)w_hash_slot(kb, %du); \\\n", var.lds_slots);
                o.f("        if (__hip_atomic_load(d%zu_lk + s0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP) == kb) { \\\n          miss = false; \\\n", b);
                for (int k = 0; k < s.nvals; ++k)
                    o.f("          w_atomic<%d>(d%zu_lv%d + s0, %s, 0); \\\n", F, b, k, vals[k].c_str());
                }
                o.f("        } \\\n      } \\\n    } \\\n");
                o.f("    const u64 mb = w_ballot(miss); \\\n    if (mb) { \\\n      const int add = __popcll(mb); \\\n");
                o.f("      if (dq_n + add > %d) WELD_DRAIN(); \\\n", var.defer_cap);
                o.f("      if (miss) { \\\n        const int e = dq_n + w_rank_below(mb); \\\n        dq[e] = kb; \\\n");
                int w = 1;
                for (int k = 0; k < s.nvals; ++k) {
                    if (L.ops[g.val[k]].opcode == WELD_OP_CONST) continue;
                    o.f("        dq[%d + e] = w_bits(%s); \\\n", var.defer_cap * w, vals[k].c_str());
                    ++w;
                }
                o.f("      } \\\n      dq_n += add; \\\n    } \\\n  } \\\n");
            }
        }
    }
    o.f("} while (0)\n\n");
    };
    emit_merge_macro("WELD_MERGE", 0);
    if (var.vq_sorted) emit_merge_macro("WELD_MERGE_TILE", 0, true);
    // The deferred dictionary as the loop's only builder in memory: the first probes of all rows a lane
    // holds are issued together (one LDS latency per tile instead of one per row), then a loop settles
    // the hits and queues the rest.
    bool probe_ahead = false;
    if (var.merge_loop && var.defer_builder >= 0) {
        int in_mem = 0;
        for (size_t b = 0; b < NB; ++b)
            if (L.merge_of[b] >= 0 && merges_in_memory(var.backend[b])) ++in_mem;
        probe_ahead = in_mem == 1;
    }
    if (var.merge_loop) {
        emit_merge_macro("WELD_MERGE_REG", 1);
        emit_merge_macro("WELD_MERGE_MEM", 2);
    }
    if (probe_ahead) {
        const size_t b = (size_t)var.defer_builder;
        const weld_builder_spec_t& sb = L.builders[b];
        const weld_merge_t& g = L.merges[L.merge_of[b]];
        // WELD_MERGE_HIT: settles row `o` if the key word `cur` read at slot `s0` is its key; sets `miss` otherwise
        o.f("#define WELD_MERGE_HIT(o, s0, cur, miss) do { \\\n  const u64 kb = %s; \\\n  (miss) = (o).p%zu; \\\n", pack_key(sb, b, "(o)").c_str(), b);
        if (var.compact == (int)b) {
            o.f("  if ((o).p%zu && (u32)kb != W_EMPTY_KEY32 && (cur) == (u32)kb) { \\\n    (miss) = false; \\\n", b);
            o.f("    w_lds_add32(d%zu_cv, (s0), (i64)(o).v%zu_0); \\\n  } \\\n} while (0)\n\n", b, b);
        } else {
            o.f("  if ((o).p%zu && kb != W_EMPTY_KEY && (cur) == kb) { \\\n    (miss) = false; \\\n", b);
            for (int k = 0; k < sb.nvals; ++k)
                o.f("    w_atomic<%d>(d%zu_lv%d + (s0), (%s)(o).v%zu_%d, 0); \\\n", sb.func, b, k, acc_ctype(sb.val_type[k]), b, k);
            o.f("  } \\\n} while (0)\n\n");
        }
        // WELD_MERGE_QUEUE: appends the rows of the wavefront with `miss` set to its queue (drained when full)
        o.f("#define WELD_MERGE_QUEUE(o, miss) do { \\\n  const u64 mb = w_ballot(miss); \\\n  if (mb) { \\\n    const int add = __popcll(mb); \\\n");
        o.f("    if (dq_n + add > %d) WELD_DRAIN(); \\\n", var.defer_cap);
        o.f("    if (miss) { \\\n      const int e = dq_n + w_rank_below(mb); \\\n      dq[e] = %s; \\\n", pack_key(sb, b, "(o)").c_str());
        int w = 1;
        for (int k = 0; k < sb.nvals; ++k) {
            if (L.ops[g.val[k]].opcode == WELD_OP_CONST) continue;
            o.f("      dq[%d + e] = w_bits((%s)(o).v%zu_%d); \\\n", var.defer_cap * w, acc_ctype(sb.val_type[k]), b, k);
            ++w;
        }
        o.f("    } \\\n    dq_n += add; \\\n  } \\\n} while (0)\n\n");
    }

    // ------------------------------------------------------------ kernel
    o.f("extern \"C\" __global__ void __launch_bounds__(W_BLOCK) weld_kernel(const KArgs a) {\n");
    o.f("  __shared__ u64 s_red[W_WAVES];\n");
    // (single-launch form: the status words are written once, at the end; until then the error bits
    // collect beside the arrival counter, in words that are zero between calls)
    o.f("  int* const errp = (int*)(%s + 2);\n", var.single ? "a.arrive" : "a.ctl");
    for (int c = 0; c < L.ncols; ++c)
        if (L.col_scalar[c]) o.f("  const %s sc%d = a.s%d[0];\n", stype(L.col_type[c]), c, c);
    o.f("  const int lane = threadIdx.x & 63;\n  const int wave = threadIdx.x >> 6;\n");
    o.f("  (void)lane; (void)wave; (void)errp;\n");
    int lds = 8 * (var.block / 64) + 4;
    if (uses_erf) {
        o.f("  w_erf_init();\n");
        lds += 8 * 960;
    }
    if (uses_log) {
        o.f("  w_log_init();\n");
        lds += 8 * 273;
    }
    if (uses_exp) {
        o.f("  w_exp_init();\n");
        lds += 8 * 128;
    }
    if (var.ticketed) {
        if (var.pipeline)   // two tiles overlap: the next tile's number and this tile's counts live side by side
            o.f("  __shared__ i64 s_tile[2];\n  __shared__ i64 s_cnt[%d][2][W_WAVES];\n  __shared__ i64 s_pfx[%d];\n", ncompact, ncompact);
        else
            o.f("  __shared__ i64 s_tile;\n  __shared__ i64 s_cnt[%d][W_WAVES];\n  __shared__ i64 s_pfx[%d];\n", ncompact, ncompact);
        o.f("  __shared__ u64 s_stage[W_WAVES * W_UNIT];\n");
        if (var.defer_builder >= 0)   // the wavefront's queue of unsettled merges lives in its part of the staging buffer
            o.f("  u64* const dq = s_stage + wave * W_UNIT;\n  int dq_n = 0;\n");
        lds += 8 + 8 * ncompact * (var.block / 64) + 8 * ncompact + 8 * (var.block / 64) * 64 * var.v;
    }
    // builder state
    bool need_sync = false;
    for (size_t b = 0; b < NB; ++b) {
        const weld_builder_spec_t& s = L.builders[b];
        if (var.backend[b] == BK_MERGER) {
            o.f("  %s m%zu = %s;\n", acc_ctype(s.val_type[0]), b, ident_expr(s.func, s.val_type[0]).c_str());
        } else if (var.backend[b] == BK_VECM_REG) {
            o.f("  %s v%zu_a[%d];\n", acc_ctype(s.val_type[0]), b, (int)s.length);
            o.f("  _Pragma(\"unroll\") for (int q = 0; q < %d; ++q) v%zu_a[q] = %s;\n", (int)s.length, b, ident_expr(s.func, s.val_type[0]).c_str());
        } else if (var.backend[b] == BK_VECM_QUEUE) {
            o.f("  __shared__ u32 v%zu_qn[%d];\n", b, var.vq_ranges);
            lds += 4 * var.vq_ranges;
            o.f("  for (int q = threadIdx.x; q < %d; q += W_BLOCK) v%zu_qn[q] = 0;\n", var.vq_ranges, b);
            // merges that find their segment full are combined here before they go to the result (w_vecm_overflow)
            o.f("  __shared__ u32 v%zu_ot[W_VQ_OVERFLOW];\n  __shared__ %s v%zu_ov[W_VQ_OVERFLOW];\n", b, acc_ctype(s.val_type[0]), b);
            o.f("  for (int q = threadIdx.x; q < W_VQ_OVERFLOW; q += W_BLOCK) { v%zu_ot[q] = W_VQ_NONE; v%zu_ov[q] = %s; }\n", b, b, ident_expr(s.func, s.val_type[0]).c_str());
            lds += 12 * 1024;
            if (var.vq_sorted) {
                // a tile's entries per range, where each range's run begins in the staging array (and the tile's total),
                // where it goes in the range's segment, and the entries sorted by range
                o.f("  __shared__ u32 v%zu_tc[%d];\n  __shared__ u32 v%zu_to[%d];\n  __shared__ u32 v%zu_tb[%d];\n  __shared__ u32 v%zu_st[W_TILE];\n",
                    b, var.vq_ranges, b, var.vq_ranges + 1, b, var.vq_ranges, b);
                lds += 12 * var.vq_ranges + 4 + 4 * var.block * var.v * var.u;
                if (!var.vq_const) {
                    o.f("  __shared__ u64 v%zu_sv[W_TILE];\n", b);
                    lds += 8 * var.block * var.v * var.u;
                }
                o.f("  for (int q = threadIdx.x; q < %d; q += W_BLOCK) v%zu_tc[q] = 0;\n", var.vq_ranges, b);
            }
            need_sync = true;
        } else if (var.backend[b] == BK_VECM_LDS) {
            const int cells = var.ranges > 1 ? 8192 : (int)s.length;
            o.f("  __shared__ %s v%zu_l[%d];\n", acc_ctype(s.val_type[0]), b, cells);
            lds += 8 * cells;
            o.f("  for (int q = threadIdx.x; q < %d; q += W_BLOCK) v%zu_l[q] = %s;\n", cells, b, ident_expr(s.func, s.val_type[0]).c_str());
            need_sync = true;
        } else if (var.backend[b] == BK_DICT_REG || var.backend[b] == BK_DICT_LANE) {
            const int S = (int)s.capacity;
            o.f("  __shared__ u64 d%zu_lk[%d];\n", b, S);
            lds += 8 * S;
            o.f("  if (threadIdx.x < %d) d%zu_lk[threadIdx.x] = W_EMPTY_KEY;\n", S, b);
            o.f("  u64 d%zu_kreg[%d];\n", b, S);
            o.f("  _Pragma(\"unroll\") for (int q = 0; q < %d; ++q) d%zu_kreg[q] = W_EMPTY_KEY;\n", S, b);
            for (int k = 0; k < s.nvals; ++k) {
                if (var.backend[b] == BK_DICT_REG) {
                    o.f("  %s d%zu_a%d[%d];\n", acc_ctype(s.val_type[k]), b, k, S);
                    o.f("  _Pragma(\"unroll\") for (int q = 0; q < %d; ++q) d%zu_a%d[q] = %s;\n", S, b, k, ident_expr(s.func, s.val_type[k]).c_str());
                } else {
                    o.f("  __shared__ %s d%zu_l%d[%d * W_BLOCK];\n", acc_ctype(s.val_type[k]), b, k, S);
                    o.f("  _Pragma(\"unroll\") for (int q = 0; q < %d; ++q) d%zu_l%d[q * W_BLOCK + threadIdx.x] = %s;\n", S, b, k, ident_expr(s.func, s.val_type[k]).c_str());
                    lds += 8 * S * var.block;
                }
            }
            need_sync = true;
        } else if (var.backend[b] == BK_DICT_LDS) {
            const bool compact = var.compact == (int)b;
            if (compact) {
                o.f("  __shared__ u32 d%zu_ck[%d];\n  __shared__ u32 d%zu_cv[%d];\n", b, var.lds_slots, b, var.lds_slots);
                lds += 8 * var.lds_slots;
            } else {
                o.f("  __shared__ u64 d%zu_lk[%d];\n", b, var.lds_slots);
                lds += 8 * var.lds_slots * (1 + s.nvals);
                for (int k = 0; k < s.nvals; ++k) o.f("  __shared__ %s d%zu_lv%d[%d];\n", acc_ctype(s.val_type[k]), b, k, var.lds_slots);
            }
            if (var.door_words > 0) {
                o.f("  __shared__ u32 d%zu_door[%d];\n  for (int q = threadIdx.x; q < %d; q += W_BLOCK) d%zu_door[q] = 0;\n", b, var.door_words, var.door_words, b);
                lds += 4 * var.door_words;
            }
            if (var.spill) {
                o.f("  __shared__ u32 d%zu_qn[W_SPILL_PARTS];\n  for (int q = threadIdx.x; q < W_SPILL_PARTS; q += W_BLOCK) d%zu_qn[q] = 0;\n", b, b);
                lds += 4 * var.spill_parts;
            }
            if (compact) {
                o.f("  for (int q = threadIdx.x; q < %d; q += W_BLOCK) {\n    d%zu_ck[q] = W_EMPTY_KEY32;\n    d%zu_cv[q] = 0;\n  }\n", var.lds_slots, b, b);
            } else {
            o.f("  for (int q = threadIdx.x; q < %d; q += W_BLOCK) {\n    d%zu_lk[q] = W_EMPTY_KEY;\n", var.lds_slots, b);
            for (int k = 0; k < s.nvals; ++k) o.f("    d%zu_lv%d[q] = %s;\n", b, k, ident_expr(s.func, s.val_type[k]).c_str());
            o.f("  }\n");
            }
            need_sync = true;
        }
    }
    if (need_sync) o.f("  __syncthreads();\n");
    if (var.compact >= 0) {
        // The compact table's contents leave through the same road as its misses (queue entry, else the
        // global table).  Called by the whole work-group: at the end, and - when the merged value is a
        // 64-bit constant - before a 32-bit partial sum could pass 2^31 (the keys stay, the sums restart).
        const size_t b = (size_t)var.compact;
        o.f("  i64 wg_rows = 0;\n  (void)wg_rows;\n");
        o.f("  auto flush_d%zu = [&]() {\n    __syncthreads();\n", b);
        o.f("    for (int q = threadIdx.x; q < %d; q += W_BLOCK) {\n      const u32 k32 = d%zu_ck[q];\n      if (k32 == W_EMPTY_KEY32) continue;\n", var.lds_slots, b);
        o.f("      const u64 kb = %s;\n", var.compact_sext ? "(u64)(i64)(int)k32" : "(u64)k32");
        o.f("      const i64 val = (i64)(int)d%zu_cv[q];\n      d%zu_cv[q] = 0;\n", b, b);
        if (var.spill) {
            o.f("      const i64 ei = w_spill_index(d%zu_qn, a.b%zu_qcap, 1, kb);\n", b, b);
            o.f("      if (ei >= 0) {\n        w_gstore1(a.b%zu_log + ei, w_compact_entry(kb, val));\n        continue;\n      }\n", b);
            if (var.spill_slices) o.f("      __hip_atomic_store(a.b%zu_hdr, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);\n", b);
        }
        o.f("      const i64 g = w_table_slot(a.b%zu_keys, a.b%zu_hdr, a.b%zu_slots, kb, errp);\n", b, b, b);
        o.f("      if (g >= 0) w_atomic<0>(a.b%zu_v0 + g, val, 1);\n    }\n    __syncthreads();\n  };\n", b);
    }
    // after each tile: flush the compact table before a partial sum could overflow
    std::string guard_text;
    if (var.compact >= 0 && var.compact_guard > 0) {
        char buf[256];
        snprintf(buf, sizeof buf, "    wg_rows += W_TILE;\n    if ((wg_rows + W_TILE) * %lldll >= (1ll << 31)) { flush_d%d(); wg_rows = 0; }\n",
                 var.compact_guard, var.compact);
        guard_text = buf;
    }

    // row evaluation call text
    auto row_call = [&](const char* idx, const char* fmt_col, const char* dst, bool together) {
        // fmt_col is a printf format taking the column number
        std::string c = together ? "weld_row<true>(" : "weld_row<false>(";
        c += idx;
        if (L.ndicts > 0) c += ", a, errp";
        for (int k = 0; k < L.ncols; ++k)
            if (L.col_used[k]) {
                char buf[96];
                snprintf(buf, sizeof buf, fmt_col, k);
                c += ", ";
                c += buf;
            }
        for (int k = 0; k < L.ncols; ++k)
            if (L.col_scalar[k]) c += ", sc" + std::to_string(k);
        c += ", ";
        c += dst;
        c += ");";
        return c;
    };

    if (!var.ticketed) {
        // ---------------- static tile order: no barriers inside the main loop
        o.f("  const i64 nfull = a.n / W_TILE;\n");
        if (var.ranges > 1) {
            // work-group g belongs to range g % R and is member g / R of that range's group
            o.f("  const i64 range_lo = (i64)(blockIdx.x %% %d) * 8192;\n", var.ranges);
            o.f("  const u32 member = blockIdx.x / %d, members = gridDim.x / %d;\n", var.ranges, var.ranges);
            o.f("  for (i64 t = member; t < nfull; t += members) {\n");
        } else {
            o.f("  for (i64 t = blockIdx.x; t < nfull; t += gridDim.x) {\n");
        }
        o.f("    const i64 r0 = t * W_TILE + (i64)wave * W_WAVE_ROWS + lane * W_V;\n");
        for (int c = 0; c < L.ncols; ++c)
            if (L.col_used[c]) o.f("    wvec<%s, W_V> x%d[W_U];\n", stype(L.col_type[c]), c);
        o.f("    _Pragma(\"unroll\") for (int u = 0; u < W_U; ++u) {\n");
        for (int c = 0; c < L.ncols; ++c)
            if (L.col_used[c]) o.f("      x%d[u] = w_load<%s, W_V>(a.c%d + r0 + u * W_UNIT);\n", c, stype(L.col_type[c]), c);
        o.f("    }\n");
        if (var.vq_sorted) o.f("    u32 vq_e[W_U * W_V];\n    u64 vq_v[W_U * W_V];\n    (void)vq_v;\n");
        o.f("    _Pragma(\"unroll\") for (int u = 0; u < W_U; ++u) {\n");
        for (size_t b = 0; b < NB; ++b)
            if (var.backend[b] == BK_VEC_DIRECT && L.merge_of[b] >= 0) o.f("      wvec<%s, W_V> y%zu;\n", stype(L.builders[b].val_type[0]), b);
        o.f("      _Pragma(\"unroll\") for (int k = 0; k < W_V; ++k) {\n");
        o.f("        RowOut o;\n        %s\n", row_call("r0 + u * W_UNIT + k", "x%d[u].e[k]", "o", true).c_str());
        o.f(var.vq_sorted ? "        WELD_MERGE_TILE(o, vq_e[u * W_V + k], vq_v[u * W_V + k]);\n" : "        WELD_MERGE(o);\n");
        for (size_t b = 0; b < NB; ++b)
            if (var.backend[b] == BK_VEC_DIRECT && L.merge_of[b] >= 0) o.f("        y%zu.e[k] = o.v%zu_0;\n", b, b);
        o.f("      }\n");
        for (size_t b = 0; b < NB; ++b)
            if (var.backend[b] == BK_VEC_DIRECT && L.merge_of[b] >= 0)
                o.f("      w_store<%s, W_V>(a.b%zu_out + r0 + u * W_UNIT, y%zu);\n", stype(L.builders[b].val_type[0]), b, b);
        o.f("    }\n");
        if (var.vq_sorted) {
            // The tile's entries, sorted by range in LDS, leave as runs: a range's entries of one tile go to neighbouring
            // addresses of its segment from neighbouring threads - a few stores of whole lines per (tile, range) instead
            // of one small store per row to a line of its own (the loop was bound by the number of stores, not by bytes).
            // Rank within (tile, range) from an LDS counter; a scan across the work-group turns the counts into where each
            // range's run begins in the staging array and in the segment; four barriers a tile.
            const size_t b = (size_t)var.vq_builder;
            const weld_builder_spec_t& s = L.builders[b];
            const int R = var.vq_ranges;
            const std::string cv = !var.vq_const ? std::string() :
                std::string("(") + acc_ctype(s.val_type[0]) + ")(" + ctype(s.val_type[0]) + ")" + const_expr(L.ops[L.merges[L.merge_of[b]].val[0]]);
            o.f("    {\n      u32 rk[W_U * W_V];\n      _Pragma(\"unroll\") for (int j = 0; j < W_U * W_V; ++j) {\n        rk[j] = 0;\n");
            o.f("        if (vq_e[j] != 0xffffffffu) rk[j] = __hip_atomic_fetch_add(v%zu_tc + (vq_e[j] >> %d), 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);\n      }\n", b, var.vq_shift);
            const int K = (R + var.block - 1) / var.block;          // ranges per thread in the scan of the counts
            o.f("      __syncthreads();\n      {\n        u32 c[%d], mine = 0;\n", K);
            o.f("        _Pragma(\"unroll\") for (int k = 0; k < %d; ++k) { const int q = (int)threadIdx.x * %d + k; c[k] = q < %d ? v%zu_tc[q] : 0u; mine += c[k]; }\n", K, K, R, b);
            o.f("        u32 incl = mine;\n        for (int d = 1; d < 64; d <<= 1) { const u32 up = __shfl_up(incl, d, 64); if (lane >= d) incl += up; }\n");
            o.f("        if (lane == 63) s_red[wave] = incl;\n        __syncthreads();\n        u32 run = incl - mine;\n");
            o.f("        for (int w = 0; w < wave; ++w) run += (u32)s_red[w];\n");
            o.f("        _Pragma(\"unroll\") for (int k = 0; k < %d; ++k) {\n          const int q = (int)threadIdx.x * %d + k;\n", K, K);
            o.f("          if (q < %d) { v%zu_to[q] = run; v%zu_tb[q] = v%zu_qn[q]; v%zu_qn[q] += c[k]; v%zu_tc[q] = 0; }\n          run += c[k];\n        }\n", R, b, b, b, b, b);
            o.f("        if (threadIdx.x == W_BLOCK - 1) v%zu_to[%d] = run;\n      }\n      __syncthreads();\n", b, R);
            if (var.vq_const)
                o.f("      _Pragma(\"unroll\") for (int j = 0; j < W_U * W_V; ++j)\n        if (vq_e[j] != 0xffffffffu) v%zu_st[v%zu_to[vq_e[j] >> %d] + rk[j]] = vq_e[j];\n      __syncthreads();\n", b, b, var.vq_shift);
            else
                o.f("      _Pragma(\"unroll\") for (int j = 0; j < W_U * W_V; ++j)\n        if (vq_e[j] != 0xffffffffu) {\n          const u32 at = v%zu_to[vq_e[j] >> %d] + rk[j];\n          v%zu_st[at] = vq_e[j];\n          v%zu_sv[at] = vq_v[j];\n        }\n      __syncthreads();\n", b, var.vq_shift, b, b);
            o.f("      const u32 staged = v%zu_to[%d];\n      for (u32 i = threadIdx.x; i < staged; i += W_BLOCK) {\n        const u32 e = v%zu_st[i];\n        const u32 part = e >> %d;\n", b, R, b, var.vq_shift);
            o.f("        const u64 pos = (u64)v%zu_tb[part] + (i - v%zu_to[part]);\n", b, b);
            if (var.vq_const) {
                o.f("        if ((i64)pos < a.b%zu_qcap) w_gstore_u16((unsigned short*)a.b%zu_log + ((u64)blockIdx.x * %du + part) * (u64)a.b%zu_qcap + pos, (unsigned short)(e & %du));\n", b, b, R, b, (1u << var.vq_shift) - 1);
                o.f("        else w_vecm_overflow<%d>(v%zu_ot, v%zu_ov, e, %s, a.b%zu_out);\n      }\n    }\n", s.func, b, b, cv.c_str(), b);
            } else {
                o.f("        if ((i64)pos < a.b%zu_qcap) {\n          char* const sg = (char*)a.b%zu_log + ((u64)blockIdx.x * %du + part) * (u64)a.b%zu_qcap * 10;\n", b, b, R, b);
                o.f("          w_gstore1((u64*)sg + pos, v%zu_sv[i]);\n          w_gstore_u16((unsigned short*)(sg + 8 * a.b%zu_qcap) + pos, (unsigned short)(e & %du));\n        }\n", b, b, (1u << var.vq_shift) - 1);
                o.f("        else w_vecm_overflow<%d>(v%zu_ot, v%zu_ov, e, w_from_bits<%s>(v%zu_sv[i]), a.b%zu_out);\n      }\n    }\n", s.func, b, b, acc_ctype(s.val_type[0]), b, b);
            }
        }
        o.f("%s  }\n", guard_text.c_str());
        // tail rows, one per thread
        if (var.ranges > 1)
            o.f("  for (i64 i = nfull * W_TILE + (i64)member * W_BLOCK + threadIdx.x; i < a.n; i += (i64)members * W_BLOCK) {\n");
        else
            o.f("  for (i64 i = nfull * W_TILE + (i64)blockIdx.x * W_BLOCK + threadIdx.x; i < a.n; i += (i64)gridDim.x * W_BLOCK) {\n");
        o.f("    RowOut o;\n    %s\n    WELD_MERGE(o);\n", row_call("i", "a.c%d[i]", "o", false).c_str());
        for (size_t b = 0; b < NB; ++b)
            if (var.backend[b] == BK_VEC_DIRECT && L.merge_of[b] >= 0) o.f("    a.b%zu_out[i] = o.v%zu_0;\n", b, b);
        o.f("  }\n");
    } else {
        // ---------------- ticketed tile order (needed by the look-back scan)
        // Plain form: a tile's ticket is drawn when the tile starts, its columns are loaded, its counts are
        // published and the sum of its predecessors is collected at once (the look-back), the other
        // wavefronts merge meanwhile, and after a barrier the selected values are stored.
        // Pipelined form (var.pipeline): the columns of the NEXT tile are loaded into registers while
        // this tile is still being merged and stored, so the loads' latency is hidden and the memory
        // pipe does not idle between a tile's stores and the next tile's loads.  The next tile's ticket
        // is therefore drawn at the top of the current tile.  A ticket drawn ahead delays the tile's
        // counts, and the tiles behind it wait for them in their look-back (with the look-back in one
        // piece, drawing tickets a tile ahead cost C5 20 %); so the look-back is split: a tile publishes
        // its own counts as soon as they are known and collects the sum of its predecessors after its
        // merges, when the tiles in front have had time to publish theirs (7 % over collecting at once).
        // Measured and dropped: loads issued only after the merges (no gain over the plain form), the
        // wavefront that finishes its merges first collecting the sum (2 % slower), the tile's stores
        // moved into the next tile so that one barrier per tile is left (2 % slower, more registers),
        // the descriptors of the look-back requested before the queued merges are drained (3 % slower),
        // first probes issued in two halves to free registers, and a 24-bit multiplication in the table
        // hash (both within the noise: the kernel is bound by how little the phases of its one
        // work-group per compute unit overlap, not by the instructions it issues; two work-groups of
        // 512 threads with tables of half the size: 0.52 ms against 0.46).  Clock reads around a tile's
        // phases put a working wavefront's two barrier waits at 2.0 and 4.3 of the tile's 16.4 us (the ticket's
        // round trip; the first wavefront's look-back, 2.7 us at 0.1 polls per tile), and three forms without
        // them were built and measured: the ticket drawn behind the second barrier (no change), a first
        // wavefront that holds no rows and only draws tickets, publishes and looks back (0.468 against 0.438 ms),
        // the next tile's counts published a tile early from its prefetched columns (0.454).  A wavefront at a
        // barrier leaves its issue slots and LDS time to the others: the waits are slack, and what the
        // work-group lacks is memory operations in flight while it merges (a plain copy in this launch shape
        // moves 6.0 TB/s, this loop 4.4).
        const std::string cb = var.pipeline ? "[it & 1]" : "";
        // (drawn ahead, the ticket is a wrapping increment rather than an addition: the compiler turns an
        // addition by some lanes into one by the wavefront's first lane and waits for the result on the
        // spot, and that wait - with the tile's stores still in flight - would stop the first wavefront)
        const char* ticket = var.pipeline ? "(i64)__builtin_amdgcn_atomic_inc32(a.ctl, 0xffffffffu, __ATOMIC_RELAXED, \"agent\")"
                                          : "(i64)__hip_atomic_fetch_add(a.ctl, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)";
        Out prefetch;
        if (var.pipeline) {
            prefetch.f("    const i64 tn = s_tile[(it + 1) & 1];\n");
            prefetch.f("    if ((tn + 1) * W_TILE <= a.n) {\n      const i64 rn = tn * W_TILE + (i64)wave * W_WAVE_ROWS + lane * W_V;\n");
            prefetch.f("      _Pragma(\"unroll\") for (int u = 0; u < W_U; ++u) {\n");
            for (int c = 0; c < L.ncols; ++c)
                if (L.col_used[c]) prefetch.f("        x%d[u] = w_load<%s, W_V>(a.c%d + rn + u * W_UNIT);\n", c, stype(L.col_type[c]), c);
            prefetch.f("      }\n    }\n");
        }
        // The loads issued ahead are waited for where nothing else is in flight (before the tile's stores
        // are issued, by naming their registers in an empty asm statement): the one counter of vector
        // memory operations cannot tell loads from stores, so a wait for these loads placed where the
        // next tile first uses them would also wait for this tile's stores to complete.
        Out landed;
        if (var.pipeline) {
            landed.f("    _Pragma(\"unroll\") for (int u = 0; u < W_U; ++u)\n      _Pragma(\"unroll\") for (int k = 0; k < W_V; ++k) {\n");
            for (int c = 0; c < L.ncols; ++c)
                if (L.col_used[c])
                    landed.f("        asm volatile(\"\" :: \"v\"(%sx%d[u].e[k]));\n", type_size(L.col_type[c]) < 4 ? "(int)" : "", c);
            landed.f("      }\n");
        }
        o.f("  const i64 ntiles = (a.n + W_TILE - 1) / W_TILE;\n");
        if (var.pipeline) {
            o.f("  if (threadIdx.x == 0) s_tile[0] = %s;\n  __syncthreads();\n  i64 t = s_tile[0];\n", ticket);
            for (int c = 0; c < L.ncols; ++c)
                if (L.col_used[c]) o.f("  wvec<%s, W_V> x%d[W_U];\n", stype(L.col_type[c]), c);
            o.f("  if ((t + 1) * W_TILE <= a.n) {\n    const i64 rn = t * W_TILE + (i64)wave * W_WAVE_ROWS + lane * W_V;\n");
            o.f("    _Pragma(\"unroll\") for (int u = 0; u < W_U; ++u) {\n");
            for (int c = 0; c < L.ncols; ++c)
                if (L.col_used[c]) o.f("      x%d[u] = w_load<%s, W_V>(a.c%d + rn + u * W_UNIT);\n", c, stype(L.col_type[c]), c);
            o.f("    }\n  }\n");
            o.s += landed.s;
            o.f("  int it = 0;\n  for (; t < ntiles; ++it) {\n");
            if (var.pipeline) o.f("    u32 tk = 0;\n    if (threadIdx.x == 0) tk = (u32)%s;\n", ticket);
        } else {
            o.f("  for (;;) {\n");
            o.f("    if (threadIdx.x == 0) s_tile = %s;\n", ticket);
            o.f("    __syncthreads();\n    const i64 t = s_tile;\n    if (t >= ntiles) break;\n");
        }
        o.f("    const i64 r0 = t * W_TILE + (i64)wave * W_WAVE_ROWS + lane * W_V;\n");
        o.f("    const bool full = (t + 1) * W_TILE <= a.n;\n");
        o.f("    RowOut o[W_U][W_V];\n");
        o.f("    if (full) {\n");
        if (!var.pipeline) {
            for (int c = 0; c < L.ncols; ++c)
                if (L.col_used[c]) o.f("      wvec<%s, W_V> x%d[W_U];\n", stype(L.col_type[c]), c);
            o.f("      _Pragma(\"unroll\") for (int u = 0; u < W_U; ++u) {\n");
            for (int c = 0; c < L.ncols; ++c)
                if (L.col_used[c]) o.f("        x%d[u] = w_load<%s, W_V>(a.c%d + r0 + u * W_UNIT);\n", c, stype(L.col_type[c]), c);
            o.f("      }\n");
        }
        o.f("      _Pragma(\"unroll\") for (int u = 0; u < W_U; ++u)\n        _Pragma(\"unroll\") for (int k = 0; k < W_V; ++k) {\n");
        o.f("          %s\n        }\n", row_call("r0 + u * W_UNIT + k", "x%d[u].e[k]", "o[u][k]", true).c_str());
        o.f("    } else {\n");
        o.f("      _Pragma(\"unroll\") for (int u = 0; u < W_U; ++u)\n        _Pragma(\"unroll\") for (int k = 0; k < W_V; ++k) {\n");
        o.f("          const i64 i = r0 + u * W_UNIT + k;\n");
        o.f("          if (i < a.n) { %s } else weld_row_none(o[u][k]);\n        }\n", row_call("i", "a.c%d[i]", "o[u][k]", false).c_str());
        o.f("    }\n");
        Out mm;      // merges that go to memory, when they come after the tile's counts are published
        Out gather_text;
        bool gathered = false;
        std::vector<int> seen_op, seen_pred;
        // how the later phases name "row (u, k) is selected for builder b" and its value
        auto sel_expr = [&](size_t b) {
            char buf[96];
            if (gathered) snprintf(buf, sizeof buf, "((mp%d >> (u * W_V + k)) & 1u)", L.merges[L.merge_of[b]].pred + 1);
            else snprintf(buf, sizeof buf, "o[u][k].p%zu", b);
            return std::string(buf);
        };
        auto val_expr = [&](size_t b) {
            char buf[96];
            if (gathered) snprintf(buf, sizeof buf, "mt%d[u * W_V + k]", L.merges[L.merge_of[b]].val[0]);
            else snprintf(buf, sizeof buf, "o[u][k].v%zu_0", b);
            return std::string(buf);
        };
        if (!var.merge_loop) {
            o.f("    _Pragma(\"unroll\") for (int u = 0; u < W_U; ++u)\n      _Pragma(\"unroll\") for (int k = 0; k < W_V; ++k) WELD_MERGE(o[u][k]);\n");
        } else {
            // register accumulators unrolled as ever; the merges that go to memory in one loop over
            // the lane's rows: their operands are gathered into vectors indexed by the loop counter
            // (the compiler turns that into relative register addressing), constants stay literals
            o.f("    _Pragma(\"unroll\") for (int u = 0; u < W_U; ++u)\n      _Pragma(\"unroll\") for (int k = 0; k < W_V; ++k) WELD_MERGE_REG(o[u][k]);\n");
            // What the rows of the tile leave behind for the later phases - the operands of the
            // merges that go to memory and the values and predicates of the compacting vecbuilders -
            // is gathered into vectors (one per IR value) and bit masks (one per predicate) of
            // tile scope; the row structs die here, and a value used twice is held once.
            std::vector<std::string> gather, scatter;     // statements filling the vectors / the row of one iteration
            // (a 64-bit integer that provably fits 32 bits is held in one register)
            auto vec_elem = [&](int op) {
                const int t = L.ops[op].type;
                return t == WELD_F64 ? "double" : (t == WELD_I64 && !ranges[op].fits32()) ? "i64" : "int";
            };
            char buf[256];
            Out decl;
            for (size_t b = 0; b < NB; ++b) {
                const int m = L.merge_of[b];
                const bool mem = m >= 0 && merges_in_memory(var.backend[b]);
                if (m < 0 || (!mem && var.backend[b] != BK_VEC_COMPACT)) continue;
                const weld_merge_t& g = L.merges[m];
                if (std::find(seen_pred.begin(), seen_pred.end(), g.pred) == seen_pred.end()) {
                    seen_pred.push_back(g.pred);
                    decl.f("    u32 mp%d = 0;\n", g.pred + 1);
                    snprintf(buf, sizeof buf, "mp%d |= (o[u][k].p%zu ? 1u : 0u) << (u * W_V + k);", g.pred + 1, b);
                    gather.push_back(buf);
                }
                if (mem) {
                    snprintf(buf, sizeof buf, "r.p%zu = (mp%d >> j) & 1u;", b, g.pred + 1);
                    scatter.push_back(buf);
                }
                for (int f = 0; f < g.nkeys + g.nvals; ++f) {
                    const bool is_key = f < g.nkeys;
                    const int fi = is_key ? f : f - g.nkeys;
                    const int op = is_key ? g.key[fi] : g.val[fi];
                    const int ft = is_key ? L.builders[b].key_type[fi] : L.builders[b].val_type[fi];
                    const char* fn = is_key ? "k" : "v";
                    if (mem && L.ops[op].opcode == WELD_OP_CONST) {
                        snprintf(buf, sizeof buf, "r.%s%zu_%d = (%s)%s;", fn, b, fi, ctype(ft), const_expr(L.ops[op]).c_str());
                        scatter.push_back(buf);
                        continue;
                    }
                    if (std::find(seen_op.begin(), seen_op.end(), op) == seen_op.end()) {
                        seen_op.push_back(op);
                        decl.f("    typedef %s mt%d_t __attribute__((ext_vector_type(W_U * W_V)));\n    mt%d_t mt%d;\n", vec_elem(op), op, op, op);
                        snprintf(buf, sizeof buf, "mt%d[u * W_V + k] = (%s)o[u][k].%s%zu_%d;", op, vec_elem(op), fn, b, fi);
                        gather.push_back(buf);
                    }
                    if (mem) {
                        snprintf(buf, sizeof buf, "r.%s%zu_%d = (%s)mt%d[j];", fn, b, fi, ctype(ft), op);
                        scatter.push_back(buf);
                    }
                }
            }
            gathered = true;
            // the gather itself comes after the direct vecbuilders below, the last readers of the row structs
            gather_text.f("%s", decl.s.c_str());
            gather_text.f("    _Pragma(\"unroll\") for (int u = 0; u < W_U; ++u)\n      _Pragma(\"unroll\") for (int k = 0; k < W_V; ++k) {\n");
            for (const std::string& g : gather) gather_text.f("        %s\n", g.c_str());
            gather_text.f("      }\n");
            if (probe_ahead) {
                const size_t db = (size_t)var.defer_builder;
                const bool compact = var.compact == (int)db;
                mm.f("    typedef int fs_t __attribute__((ext_vector_type(W_U * W_V)));\n    fs_t fs;\n");
                mm.f("    typedef %s fc_t __attribute__((ext_vector_type(W_U * W_V)));\n    fc_t fc;\n", compact ? "u32" : "u64");
                mm.f("    _Pragma(\"unroll\") for (int j = 0; j < W_U * W_V; ++j) {\n      RowOut r;\n");
                for (const std::string& g : scatter) mm.f("      %s\n", g.c_str());
                mm.f("      const u64 kb = %s;\n", pack_key(L.builders[db], db, "r").c_str());
                if (compact)
                    mm.f("      fs[j] = (int)w_hash_slot32((u32)kb, %du);\n      fc[j] = __hip_atomic_load(d%zu_ck + fs[j], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);\n    }\n", var.lds_slots, db);
                else
                    mm.f("      fs[j] = (int)w_hash_slot(kb, %du);\n      fc[j] = __hip_atomic_load(d%zu_lk + fs[j], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);\n    }\n", var.lds_slots, db);
                // hits settle here, straight-line; what is left is a bit per row
                mm.f("    u32 miss_bits = 0;\n");
                mm.f("    _Pragma(\"unroll\") for (int j = 0; j < W_U * W_V; ++j) {\n      RowOut r;\n");
                for (const std::string& g : scatter) mm.f("      %s\n", g.c_str());
                mm.f("      bool miss;\n      WELD_MERGE_HIT(r, fs[j], fc[j], miss);\n      miss_bits |= (miss ? 1u : 0u) << j;\n    }\n");
                mm.f("    _Pragma(\"unroll 1\") for (int j = 0; j < W_U * W_V; ++j) {\n      RowOut r;\n");
                for (const std::string& g : scatter) mm.f("      %s\n", g.c_str());
                mm.f("      const bool miss = (miss_bits >> j) & 1u;\n      WELD_MERGE_QUEUE(r, miss);\n    }\n");
            } else {
                mm.f("    _Pragma(\"unroll 1\") for (int j = 0; j < W_U * W_V; ++j) {\n      RowOut r;\n");
                for (const std::string& g : scatter) mm.f("      %s\n", g.c_str());
                mm.f("      WELD_MERGE_MEM(r);\n    }\n");
            }
            if (var.defer_builder >= 0) mm.f("    WELD_DRAIN();\n");
        }
        // direct vecbuilders inside a ticketed kernel
        for (size_t b = 0; b < NB; ++b)
            if (var.backend[b] == BK_VEC_DIRECT && L.merge_of[b] >= 0) {
                o.f("    _Pragma(\"unroll\") for (int u = 0; u < W_U; ++u)\n      _Pragma(\"unroll\") for (int k = 0; k < W_V; ++k) {\n");
                o.f("        const i64 i = r0 + u * W_UNIT + k;\n        if (i < a.n) a.b%zu_out[i] = o[u][k].v%zu_0;\n      }\n", b, b);
            }
        o.s += gather_text.s;
        // Compacting builders under the same predicate select the same rows (the columns of a filtered table, the
        // keys and values of a groupbuilder): the first of them counts, publishes and looks back for all, the others
        // take its counts and its prefix.  cj[b]: the slot of s_cnt / s_pfx builder b reads.
        std::vector<int> cj(NB, -1);
        std::vector<bool> leads(NB, false);
        {
            int slot_no = 0;
            for (size_t b = 0; b < NB; ++b) {
                if (var.backend[b] != BK_VEC_COMPACT) continue;
                for (size_t q = 0; q < b; ++q)
                    if (var.backend[q] == BK_VEC_COMPACT && leads[q] && L.merges[L.merge_of[q]].pred == L.merges[L.merge_of[b]].pred) { cj[b] = cj[q]; break; }
                if (cj[b] < 0) { cj[b] = slot_no; leads[b] = true; }
                ++slot_no;
            }
        }
        auto followers_len = [&](Out& d, size_t b, const char* indent, const char* cond) {
            for (size_t q = b + 1; q < NB; ++q)
                if (var.backend[q] == BK_VEC_COMPACT && !leads[q] && cj[q] == cj[b]) d.f("%s  if (%s) *a.b%zu_len = ex + tot;\n", indent, cond, q);
        };
        // ranks of the selected rows inside this wavefront's run, per compacting builder
        int j = 0;
        for (size_t b = 0; b < NB; ++b) {
            if (var.backend[b] != BK_VEC_COMPACT) continue;
            if (!leads[b]) { ++j; continue; }
            // per load unit: how many rows the wavefront selected and where its run starts; the rank
            // of a row inside the run is recomputed when the values are staged (a few instructions,
            // cheaper than holding sixteen ranks per lane through the merge phase)
            if (gathered) {
                // the lane's selected rows are the bits of its mask: one population count and a sum over the wavefront
                o.f("    {\n      const int wtot = w_wave_sum(__popc(mp%d));\n", L.merges[L.merge_of[b]].pred + 1);
            } else {
                o.f("    {\n      int wtot = 0;\n");
                o.f("      _Pragma(\"unroll\") for (int u = 0; u < W_U; ++u)\n");
                o.f("        _Pragma(\"unroll\") for (int k = 0; k < W_V; ++k) wtot += __popcll(w_ballot(%s));\n", sel_expr(b).c_str());
            }
            o.f("      if (lane == 0) s_cnt[%d]%s[wave] = wtot;\n    }\n", j, cb.c_str());
            ++j;
        }
        if (var.pipeline) o.f("    if (threadIdx.x == 0) s_tile[(it + 1) & 1] = (i64)tk;\n");
        o.f("    __syncthreads();\n");
        if (var.pipeline) o.s += prefetch.s;
        o.f("    if (wave == 0) {\n");
        j = 0;
        for (size_t b = 0; b < NB; ++b) {
            if (var.backend[b] != BK_VEC_COMPACT) continue;
            if (!leads[b]) { ++j; continue; }
            o.f("      {\n        i64 tot = 0;\n        _Pragma(\"unroll\") for (int w = 0; w < W_WAVES; ++w) tot += s_cnt[%d]%s[w];\n", j, cb.c_str());
            if (var.pipeline) {
                o.f("        w_lookback_publish(a.b%zu_desc, t, tot);\n      }\n", b);
            } else {
                o.f("        const i64 ex = w_lookback(a.b%zu_desc, t, tot, a.spin_limit, errp);\n", b);
                o.f("        if (lane == 0) {\n          s_pfx[%d] = ex;\n          if (t == ntiles - 1) *a.b%zu_len = ex + tot;\n", j, b);
                followers_len(o, b, "        ", "t == ntiles - 1");
                o.f("        }\n      }\n");
            }
            ++j;
        }
        o.f("    }\n");
        // second half of the split look-back for tile `tile`, whose counts are in slot `cslot`
        auto resolve_text = [&](const char* tile, const std::string& cslot, const std::string& pslot) {
            Out d;
            d.f("    if (wave == 0) {\n");
            int jj = 0;
            for (size_t b = 0; b < NB; ++b) {
                if (var.backend[b] != BK_VEC_COMPACT) continue;
                if (!leads[b]) { ++jj; continue; }
                d.f("      {\n        i64 tot = 0;\n        _Pragma(\"unroll\") for (int w = 0; w < W_WAVES; ++w) tot += s_cnt[%d]%s[w];\n", jj, cslot.c_str());
                d.f("        const i64 ex = w_lookback_resolve(a.b%zu_desc, %s, tot, a.spin_limit, errp);\n", b, tile);
                d.f("        if (lane == 0) {\n          s_pfx[%d]%s = ex;\n          if (%s == ntiles - 1) *a.b%zu_len = ex + tot;\n", jj, pslot.c_str(), tile, b);
                const std::string last = std::string(tile) + " == ntiles - 1";
                followers_len(d, b, "        ", last.c_str());
                d.f("        }\n      }\n");
                ++jj;
            }
            d.f("    }\n");
            return d.s;
        };
        // the selected values of a tile go to their places in the output vectors
        auto staging_text = [&](const std::string& cslot, const std::string& pslot) {
            Out d;
            int jj = 0;
            for (size_t b = 0; b < NB; ++b) {
                if (var.backend[b] != BK_VEC_COMPACT) continue;
                d.f("    {\n      i64 base = s_pfx[%d]%s;\n      for (int w = 0; w < wave; ++w) base += s_cnt[%d]%s[w];\n", cj[b], pslot.c_str(), cj[b], cslot.c_str());
                // The selected values of one load unit are packed in LDS at their ranks and written
                // out as one dense run per instruction (lane l writes elements l, l+64, ...), so HBM
                // sees full lines instead of scattered 8-byte pieces.
                const char* ST = stype(L.builders[b].val_type[0]);
                // (a 64-bit value that provably fits 32 bits is staged in 4 bytes and widened at the store)
                const int vop = L.merges[L.merge_of[b]].val[0];
                const char* SG = (gathered && L.builders[b].val_type[0] == WELD_I64 && ranges[vop].fits32()) ? "int" : ST;
                d.f("      %s* const stg = (%s*)(s_stage + wave * W_UNIT);\n", SG, SG);
                // (how many rows of each load unit are selected is counted again here: a few scalar
                // instructions, cheaper than holding the counts of every unit through the merge phase)
                d.f("      int run = 0;\n");
                d.f("      _Pragma(\"unroll\") for (int u = 0; u < W_U; ++u) {\n");
                d.f("        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, \"wavefront\");\n");
                d.f("        int rank = 0, ucnt = 0;\n        _Pragma(\"unroll\") for (int k = 0; k < W_V; ++k) {\n          const u64 bal = w_ballot(%s);\n          rank += w_rank_below(bal);\n          ucnt += __popcll(bal);\n        }\n", sel_expr(b).c_str());
                d.f("        _Pragma(\"unroll\") for (int k = 0; k < W_V; ++k)\n          if (%s) stg[rank++] = (%s)%s;\n", sel_expr(b).c_str(), SG, val_expr(b).c_str());
                d.f("        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, \"wavefront\");\n");
                d.f("        _Pragma(\"unroll\") for (int q = 0; q < W_V; ++q) {\n          const int e = q * 64 + lane;\n");
                d.f("          if (e < ucnt) __builtin_nontemporal_store((%s)stg[e], a.b%zu_out + base + run + e);\n        }\n        run += ucnt;\n      }\n    }\n", ST, b);
                ++jj;
            }
            return d.s;
        };
        // The predicate masks are redefined opaquely at the phase boundaries: otherwise the compiler
        // extracts every row's bit once, up front, and carries sixteen registers of single bits
        // through all phases (spilling them where the merge code needs the room).
        std::string opaque;
        for (int pr : seen_pred) opaque += "    asm volatile(\"\" : \"+v\"(mp" + std::to_string(pr + 1) + "));\n";
        o.s += opaque;
        // while the first wavefront waits for the tiles before this one, the others merge
        o.s += mm.s;
        o.s += opaque;
        if (var.pipeline) o.s += resolve_text("t", cb, "");
        o.f("    __syncthreads();\n");
        o.s += landed.s;
        o.s += staging_text(cb, "");
        o.s += guard_text;
        if (var.pipeline) o.f("    t = tn;\n");
        o.f("  }\n");
    }

    // ------------------------------------------------------------ builder results
    for (size_t b = 0; b < NB; ++b) {
        const weld_builder_spec_t& s = L.builders[b];
        if (var.backend[b] == BK_MERGER) {
            const char* A = acc_ctype(s.val_type[0]);
            o.f("  {\n    const %s tot = w_block_reduce<%d>(m%zu, (%s*)s_red, %s);\n", A, s.func, b, A, ident_expr(s.func, s.val_type[0]).c_str());
            o.f("    if (threadIdx.x == 0) %s(a.b%zu_part, tot);\n  }\n", var.single ? "w_publish_partial" : "w_store_partial", b);
        } else if (var.backend[b] == BK_VECM_REG) {
            const char* A = acc_ctype(s.val_type[0]);
            o.f("  _Pragma(\"unroll\") for (int q = 0; q < %d; ++q) {\n", (int)s.length);
            o.f("    const %s r = w_block_reduce<%d>(v%zu_a[q], (%s*)s_red, %s);\n", A, s.func, b, A, ident_expr(s.func, s.val_type[0]).c_str());
            o.f("    if (threadIdx.x == 0) w_atomic<%d>(a.b%zu_out + q, r, 1);\n  }\n", s.func, b);
        } else if (var.backend[b] == BK_VECM_QUEUE) {
            o.f("  __syncthreads();\n  for (int q = threadIdx.x; q < %d; q += W_BLOCK)\n", var.vq_ranges);
            o.f("    a.b%zu_qcnt[(u64)blockIdx.x * %du + q] = (i64)v%zu_qn[q] < a.b%zu_qcap ? v%zu_qn[q] : (u32)a.b%zu_qcap;\n", b, var.vq_ranges, b, b, b, b);
            o.f("  for (int q = threadIdx.x; q < W_VQ_OVERFLOW; q += W_BLOCK)\n    if (v%zu_ot[q] != W_VQ_NONE) w_atomic<%d>(a.b%zu_out + v%zu_ot[q], v%zu_ov[q], 1);\n", b, s.func, b, b, b);
        } else if (var.backend[b] == BK_VECM_LDS) {
            // cells this work-group never touched still hold the identity: nothing to send
            const char* A = acc_ctype(s.val_type[0]);
            const int cells = var.ranges > 1 ? 8192 : (int)s.length;
            o.f("  __syncthreads();\n  for (int q = threadIdx.x; q < %d; q += W_BLOCK) {\n    const %s x = v%zu_l[q];\n", cells, A, b);
            o.f("    const %s id = %s;\n    u64 xb, ib;\n    __builtin_memcpy(&xb, &x, 8);\n    __builtin_memcpy(&ib, &id, 8);\n", A, ident_expr(s.func, s.val_type[0]).c_str());
            if (var.ranges > 1)
                o.f("    if (xb != ib && range_lo + q < %lldll) w_atomic<%d>(a.b%zu_out + range_lo + q, x, 1);\n  }\n", (long long)s.length, s.func, b);
            else
                o.f("    if (xb != ib) w_atomic<%d>(a.b%zu_out + q, x, 1);\n  }\n", s.func, b);
        } else if (var.backend[b] == BK_DICT_REG || var.backend[b] == BK_DICT_LANE) {
            const int S = (int)s.capacity;
            const bool lanes = var.backend[b] == BK_DICT_LANE;
            o.f("  __syncthreads();\n");
            o.f("  _Pragma(\"unroll\") for (int q = 0; q < %d; ++q) {\n    const u64 kb = d%zu_lk[q];\n    if (kb != W_EMPTY_KEY) {\n", S, b);
            for (int k = 0; k < s.nvals; ++k) {
                const char* A = acc_ctype(s.val_type[k]);
                if (lanes)
                    o.f("      const %s r%d = w_block_reduce<%d>(d%zu_l%d[q * W_BLOCK + threadIdx.x], (%s*)s_red, %s);\n", A, k, s.func, b, k, A, ident_expr(s.func, s.val_type[k]).c_str());
                else
                    o.f("      const %s r%d = w_block_reduce<%d>(d%zu_a%d[q], (%s*)s_red, %s);\n", A, k, s.func, b, k, A, ident_expr(s.func, s.val_type[k]).c_str());
            }
            o.f("      if (threadIdx.x == 0) {\n        const i64 g = w_table_slot(a.b%zu_keys, a.b%zu_hdr, a.b%zu_slots, kb, errp);\n        if (g >= 0) {\n", b, b, b);
            for (int k = 0; k < s.nvals; ++k) o.f("          w_atomic<%d>(a.b%zu_v%d + g, r%d, 1);\n", s.func, b, k, k);
            o.f("        }\n      }\n    }\n  }\n");
        } else if (var.backend[b] == BK_DICT_LDS && var.compact == (int)b) {
            o.f("  flush_d%zu();\n", b);
            if (var.spill) {
                o.f("  for (int q = threadIdx.x; q < W_SPILL_PARTS; q += W_BLOCK)\n");
                o.f("    a.b%zu_qcnt[(u64)blockIdx.x * W_SPILL_PARTS + q] = d%zu_qn[q] < (u64)a.b%zu_qcap ? d%zu_qn[q] : (u32)a.b%zu_qcap;\n", b, b, b, b, b);
            }
        } else if (var.backend[b] == BK_DICT_LDS) {
            o.f("  __syncthreads();\n");
            o.f("  for (int q = threadIdx.x; q < %d; q += W_BLOCK) {\n    const u64 kb = d%zu_lk[q];\n    if (kb != W_EMPTY_KEY) {\n", var.lds_slots, b);
            if (var.spill) {
                // the table's own contents take the same road as the misses
                o.f("      const i64 ei = w_spill_index(d%zu_qn, a.b%zu_qcap, %d, kb);\n", b, b, 1 + s.nvals);
                o.f("      if (ei >= 0) {\n");
                {
                    std::vector<std::string> words;
                    words.push_back("kb");
                    for (int k = 0; k < s.nvals; ++k) {
                        char buf[96];
                        snprintf(buf, sizeof buf, "w_bits(d%zu_lv%d[q])", b, k);
                        words.push_back(buf);
                    }
                    emit_log_stores(o, b, words, "");
                }
                o.f("        continue;\n      }\n");
                if (var.spill_slices) o.f("      __hip_atomic_store(a.b%zu_hdr, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);\n", b);
            }
            o.f("      const i64 g = w_table_slot(a.b%zu_keys, a.b%zu_hdr, a.b%zu_slots, kb, errp);\n      if (g >= 0) {\n", b, b, b);
            for (int k = 0; k < s.nvals; ++k) o.f("        w_atomic<%d>(a.b%zu_v%d + g, d%zu_lv%d[q], 1);\n", s.func, b, k, b, k);
            o.f("      }\n    }\n  }\n");
            if (var.spill) {
                o.f("  __syncthreads();\n  for (int q = threadIdx.x; q < W_SPILL_PARTS; q += W_BLOCK)\n");
                o.f("    a.b%zu_qcnt[(u64)blockIdx.x * W_SPILL_PARTS + q] = d%zu_qn[q] < (u64)a.b%zu_qcap ? d%zu_qn[q] : (u32)a.b%zu_qcap;\n", b, b, b, b, b);
            }
        }
    }
    if (var.single) {
        o.f("  if (w_arrive_last(a.arrive)) {\n");
        for (size_t b = 0; b < NB; ++b) {
            const weld_builder_spec_t& s = L.builders[b];
            const char* A = acc_ctype(s.val_type[0]);
            o.f("    {\n      const %s r = w_fold_partials<%d>(a.b%zu_part, gridDim.x, (%s*)s_red, %s);\n", A, s.func, b, A, ident_expr(s.func, s.val_type[0]).c_str());
            o.f("      if (threadIdx.x == 0) *a.b%zu_res = (%s)r;\n    }\n", b, stype(s.val_type[0]));
        }
        o.f("    w_finish_status(a.ctl, a.arrive);\n  }\n");
    }
    o.f("}\n");
    // the kernel is named after its own text, so that profiles tell loops apart
    uint64_t hsh = 0xcbf29ce484222325ull;
    for (unsigned char c : o.s) { hsh ^= c; hsh *= 0x100000001b3ull; }
    char name[48];
    snprintf(name, sizeof name, "weld_fused_%016llx", (unsigned long long)hsh);
    const std::string placeholder = "weld_kernel";
    const size_t at = o.s.find(placeholder + "(const KArgs a)");
    if (at != std::string::npos) o.s.replace(at, placeholder.size(), name);
    G.kernel_name = name;
    G.source = o.s;
    G.lds_bytes = lds;
    return G;
}

// ---------------------------------------------------------------------------------------
// Flattened inner loop of a nested `for` (un-nesting, Sec. 5 "Partial GPU Backend").
//
// The inner loops of all outer elements become ONE loop over the inner elements, tiled like
// every other loop here, so the work is balanced by inner elements whatever the lengths of the
// ranges.  The merger of the inner loop becomes a segmented merger with one cell per outer
// element: a tile stages the range boundaries that fall into it in LDS (relative to the tile
// start), every lane finds the outer element of its first inner element by binary search and
// walks from there, runs of equal outer element are combined in registers, each run ends in
// one LDS atomic on that outer element's cell, and at the end of the tile the cells go to
// memory: outer elements that lie entirely inside the tile with a plain store, the (at most
// two) that continue in a neighbouring tile with a device atomic.  The first outer element of
// every tile comes from a small kernel run before this one.
Variant choose_segmented_variant(const Loop& L, const weld_tuning_t& tune, bool aligned) {
    Variant var;
    int widest = 4;
    for (int c = 0; c < L.ncols; ++c)
        if (L.col_used[c] && type_size(L.col_type[c]) > widest) widest = type_size(L.col_type[c]);
    var.v = widest >= 8 ? 2 : 4;
    var.u = tune.units_per_thread > 0 ? tune.units_per_thread : 4;
    if (var.u > 16) var.u = 16;
    var.block = tune.block_threads > 0 ? tune.block_threads : 256;
    if (var.block < 64) var.block = 64;
    if (var.block > 1024) var.block = 1024;
    var.block = (var.block / 64) * 64;
    // range boundaries staged per tile: tiles with more fall back to device memory
    var.lds_slots = tune.lds_dict_slots > 0 ? tune.lds_dict_slots : 2048;
    if (var.lds_slots < 64) var.lds_slots = 64;
    if (var.lds_slots > 8192) var.lds_slots = 8192;
    var.aligned = aligned ? 1 : 0;
    var.own_math = tune.device_math >= 0;
    var.backend.assign(1, BK_MERGER);
    return var;
}

Generated generate_segmented(const Loop& L, const Variant& var, int offset_type, int mapped) {
    Generated G;
    Out o;
    const weld_builder_spec_t& s = L.builders[0];
    const char* A = acc_ctype(s.val_type[0]);
    const std::string ID = ident_expr(s.func, s.val_type[0]);
    const int F = s.func;
    o.f("// generated: flattened inner loop of a nested for, %d inner columns\n", L.ncols);
    o.f("#define W_BLOCK %d\n#define W_V %d\n#define W_U %d\n#define W_ALIGNED %d\n#define W_SEG_CAP %d\n", var.block, var.v, var.u, var.aligned, var.lds_slots);
    const bool uses_erf = body_uses(L, WELD_OP_ERF);
    if (uses_erf) o.f("#define W_USE_ERF 1\n");
    const bool uses_log = var.own_math && body_uses(L, WELD_OP_LOG), uses_exp = var.own_math && body_uses(L, WELD_OP_EXP);
    if (uses_log) o.f("#define W_USE_LOG 1\n#define W_LOG w_log\n");
    else o.f("#define W_LOG log\n");
    if (uses_exp) o.f("#define W_USE_EXP 1\n#define W_EXP w_exp\n");
    else o.f("#define W_EXP exp\n");
    o.s += kPreludeSource;
    o.f("\n");
    auto slot = [&](SlotKind k, int idx, const std::string& name, const std::string& ct) {
        Slot sl{k, idx, 0, name, ct};
        G.slots.push_back(sl);
    };
    slot(SLOT_N, -1, "n", "i64");
    slot(SLOT_N_OUTER, -1, "n_outer", "i64");
    for (int c = 0; c < L.ncols; ++c)
        if (L.col_used[c]) slot(SLOT_COL, c, "c" + std::to_string(c), std::string("const ") + stype(L.col_type[c]) + "* __restrict__");
    for (int g = 0; g < L.ngather; ++g)
        if (L.gather_used[g]) {
            slot(SLOT_GATHER, g, "g" + std::to_string(g), std::string("const ") + stype(L.gather_type[g]) + "* __restrict__");
            slot(SLOT_GATHER_LEN, g, "g" + std::to_string(g) + "_len", "i64");
        }
    for (int c = 0; c < L.nouter; ++c)
        if (L.outer_used[c]) slot(SLOT_OUTER_COL, c, "o" + std::to_string(c), std::string("const ") + stype(L.outer_type[c]) + "* __restrict__");
    slot(SLOT_SEG_START, -1, "seg_start", std::string("const ") + (mapped ? "i64" : ctype(offset_type)) + "* __restrict__");
    if (mapped) slot(SLOT_MAP_START, -1, "map_start", std::string("const ") + ctype(offset_type) + "* __restrict__");
    if (mapped == 2) slot(SLOT_MAP_STRIDE, -1, "map_stride", std::string("const ") + ctype(offset_type) + "* __restrict__");
    slot(SLOT_TILE_ROW, -1, "tile_row", "const int* __restrict__");
    slot(SLOT_SUMS, -1, "sums", std::string(A) + "*");
    slot(SLOT_CTL, -1, "ctl", "u32*");
    o.f("struct KArgs {\n");
    for (const Slot& sl : G.slots) o.f("  %s %s;\n", sl.ctype.c_str(), sl.name.c_str());
    o.f("};\n\n");
    emit_row_function(o, L, true);

    std::string call_args;      // the column values of element (u, k)
    for (int c = 0; c < L.ncols; ++c)
        if (L.col_used[c]) call_args += ", x" + std::to_string(c) + "[u].e[k]";

    o.f("extern \"C\" __global__ void __launch_bounds__(W_BLOCK) weld_kernel(const KArgs a) {\n");
    o.f("  __shared__ int s_b[W_SEG_CAP + 2];\n  __shared__ %s s_acc[W_SEG_CAP + 1];\n", A);
    o.f("  int* const errp = (int*)(a.ctl + 2);\n");
    o.f("  const int lane = threadIdx.x & 63;\n  const int wave = threadIdx.x >> 6;\n");
    if (uses_erf) o.f("  w_erf_init();\n");
    if (uses_log) o.f("  w_log_init();\n");
    if (uses_exp) o.f("  w_exp_init();\n");
    o.f("  const i64 ntiles = (a.n + W_TILE - 1) / W_TILE;\n");
    o.f("  for (i64 t = blockIdx.x; t < ntiles; t += gridDim.x) {\n");
    o.f("    const i64 e0 = t * W_TILE;\n    const i64 e1 = e0 + W_TILE < a.n ? e0 + W_TILE : a.n;\n");
    o.f("    const i64 r0 = a.tile_row[t], r1 = a.tile_row[t + 1];\n");
    o.f("    const i64 nrows = r1 - r0 + 1;\n");
    o.f("    if (nrows < 1) continue;                 // only with boundaries that are not sorted (reported elsewhere)\n");
    o.f("    const bool staged = nrows <= W_SEG_CAP;\n");
    // boundary of outer element r: its start; one past the last outer element: n
    o.f("    if (staged) {\n");
    o.f("      for (int k = threadIdx.x; k <= (int)nrows; k += W_BLOCK) {\n");
    o.f("        const i64 r = r0 + k;\n        const i64 bnd = r < a.n_outer ? (i64)a.seg_start[r] : a.n;\n");
    o.f("        i64 rel = bnd - e0;\n        rel = rel < -1 ? -1 : (rel > W_TILE + 1 ? W_TILE + 1 : rel);\n");
    o.f("        s_b[k] = (int)rel;\n        if (k < (int)nrows) s_acc[k] = %s;\n      }\n", ID.c_str());
    o.f("      __syncthreads();\n    }\n");
    o.f("    const i64 base = e0 + (i64)wave * W_WAVE_ROWS + lane * W_V;\n");
    // ---- loads (streamed form; the mapped form gathers them once it knows every position's outer element)
    for (int c = 0; c < L.ncols; ++c)
        if (L.col_used[c]) o.f("    wvec<%s, W_V> x%d[W_U];\n", stype(L.col_type[c]), c);
    if (!mapped) o.f("    if (e0 + W_TILE <= a.n) {\n      _Pragma(\"unroll\") for (int u = 0; u < W_U; ++u) {\n");
    if (!mapped) {
    for (int c = 0; c < L.ncols; ++c)
        if (L.col_used[c]) o.f("        x%d[u] = w_load<%s, W_V>(a.c%d + base + u * W_UNIT);\n", c, stype(L.col_type[c]), c);
    o.f("      }\n    } else {\n      _Pragma(\"unroll\") for (int u = 0; u < W_U; ++u)\n        _Pragma(\"unroll\") for (int k = 0; k < W_V; ++k) {\n");
    o.f("          const i64 e = base + u * W_UNIT + k;\n");
    for (int c = 0; c < L.ncols; ++c)
        if (L.col_used[c]) o.f("          x%d[u].e[k] = e < a.n ? a.c%d[e] : (%s)0;\n", c, c, stype(L.col_type[c]));
    o.f("        }\n    }\n");
    }
    // ---- outer element of every inner element of this lane (relative to r0)
    o.f("    int rowid[W_U][W_V];\n");
    o.f("    _Pragma(\"unroll\") for (int u = 0; u < W_U; ++u) {\n");
    o.f("      const i64 e = base + u * W_UNIT;\n      int rl = 0;\n");
    o.f("      if (e < e1) {\n");
    o.f("        if (staged) {\n          const int rel = (int)(e - e0);\n          int lo = 0, hi = (int)nrows;       // s_b[lo] <= rel < s_b[hi]\n");
    o.f("          while (hi - lo > 1) { const int mid = (lo + hi) >> 1; if (s_b[mid] <= rel) lo = mid; else hi = mid; }\n          rl = lo;\n");
    o.f("        } else {\n          i64 lo = r0, hi = r1 + 1;\n");
    o.f("          while (hi - lo > 1) { const i64 mid = (lo + hi) >> 1; if ((i64)a.seg_start[mid] <= e) lo = mid; else hi = mid; }\n          rl = (int)(lo - r0);\n        }\n");
    o.f("      }\n");
    o.f("      _Pragma(\"unroll\") for (int k = 0; k < W_V; ++k) {\n");
    o.f("        if (e + k < e1) {\n");
    o.f("          if (staged) { const int rel = (int)(e + k - e0); while (rl < (int)nrows - 1 && rel >= s_b[rl + 1]) ++rl; }\n");
    o.f("          else { while (rl < (int)nrows - 1 && e + k >= (i64)a.seg_start[r0 + rl + 1]) ++rl; }\n");
    o.f("        }\n        rowid[u][k] = rl;\n      }\n    }\n");
    // ---- values (all gathers of the lane are independent of each other: issued together)
    o.f("    RowOut o[W_U][W_V];\n");
    o.f("    _Pragma(\"unroll\") for (int u = 0; u < W_U; ++u)\n      _Pragma(\"unroll\") for (int k = 0; k < W_V; ++k) {\n");
    o.f("        const i64 e = base + u * W_UNIT + k;\n");
    if (mapped) {
        // position e of outer element `row` is inner element start[row] + (e - boundary[row]) * stride[row]; the
        // host has checked the ranges (every visited element lies inside the inner vectors) before this kernel runs
        o.f("        i64 ie = 0;\n        if (e < e1) {\n          const i64 row = r0 + rowid[u][k];\n");
        o.f("          ie = (i64)a.map_start[row] + (e - a.seg_start[row])%s;\n        }\n", mapped == 2 ? " * (i64)a.map_stride[row]" : "");
        for (int c = 0; c < L.ncols; ++c)
            if (L.col_used[c]) o.f("        x%d[u].e[k] = e < e1 ? a.c%d[ie] : (%s)0;\n", c, c, stype(L.col_type[c]));
        o.f("        if (e < e1) weld_row<false>(ie, r0 + rowid[u][k], a, errp%s, o[u][k]); else weld_row_none(o[u][k]);\n      }\n", call_args.c_str());
    } else {
    o.f("        if (e < e1) weld_row<false>(e, r0 + rowid[u][k], a, errp%s, o[u][k]); else weld_row_none(o[u][k]);\n      }\n", call_args.c_str());
    }
    // ---- segmented combine: runs of equal outer element in registers, one atomic per run
    o.f("    _Pragma(\"unroll\") for (int u = 0; u < W_U; ++u) {\n");
    o.f("      %s acc = %s;\n      bool any = false;\n      int cur = rowid[u][0];\n", A, ID.c_str());
    o.f("      _Pragma(\"unroll\") for (int k = 0; k < W_V; ++k) {\n");
    o.f("        if (rowid[u][k] != cur) {\n");
    o.f("          if (any) { if (staged) w_atomic<%d>(s_acc + cur, acc, 0); else w_atomic<%d>(a.sums + r0 + cur, acc, 1); }\n", F, F);
    o.f("          acc = %s; any = false; cur = rowid[u][k];\n        }\n", ID.c_str());
    o.f("        if (o[u][k].p0) { acc = w_combine<%d>(acc, (%s)o[u][k].v0_0); any = true; }\n      }\n", F, A);
    o.f("      if (any) { if (staged) w_atomic<%d>(s_acc + cur, acc, 0); else w_atomic<%d>(a.sums + r0 + cur, acc, 1); }\n    }\n", F, F);
    // ---- cells to memory
    o.f("    if (staged) {\n      __syncthreads();\n");
    o.f("      for (int k = threadIdx.x; k < (int)nrows; k += W_BLOCK) {\n");
    o.f("        const %s x = s_acc[k];\n        const %s id = %s;\n        u64 xb, ib;\n", A, A, ID.c_str());
    o.f("        __builtin_memcpy(&xb, &x, 8);\n        __builtin_memcpy(&ib, &id, 8);\n        if (xb == ib) continue;\n");
    o.f("        const bool inside = s_b[k] >= 0 && s_b[k + 1] <= (int)(e1 - e0);\n");
    o.f("        if (inside) a.sums[r0 + k] = x; else w_atomic<%d>(a.sums + r0 + k, x, 1);\n      }\n", F);
    o.f("      __syncthreads();\n    }\n");
    o.f("  }\n}\n");
    uint64_t hsh = 0xcbf29ce484222325ull;
    for (unsigned char c : o.s) { hsh ^= c; hsh *= 0x100000001b3ull; }
    char name[48];
    snprintf(name, sizeof name, "weld_inner_%016llx", (unsigned long long)hsh);
    const std::string placeholder = "weld_kernel";
    const size_t at = o.s.find(placeholder + "(const KArgs a)");
    if (at != std::string::npos) o.s.replace(at, placeholder.size(), name);
    G.kernel_name = name;
    G.source = o.s;
    G.lds_bytes = 4 * (var.lds_slots + 2) + 8 * (var.lds_slots + 1);
    return G;
}

}  // namespace weld
