// Lazy objects and the loop-fusion pass (paper Sec. 4.1, Table 2; Sec. 5, Table 3).
//
// Every object is either external data or one macro applied to other objects (Sec. 3.3:
// map, filter, reduce; group-by as a dictmerger).  Evaluation lowers the DAG below the
// requested roots into ONE loop over the leaf vectors:
//   * a vector object is represented by (value expression, predicate expression) over the
//     elements of the leaves: map composes value expressions (vertical fusion of a
//     producer into its consumer), filter conjoins predicates (a filter becomes the
//     predicate of the final merge; predication of Table 3);
//   * every root becomes one builder of the same loop (horizontal fusion);
//   * expressions are hash-consed while lowering, so a sub-computation shared by several
//     objects - even objects built by different callers - is evaluated once (CSE of Table 3).
// The fused loop is then submitted through weld_fused_for, fused or operator at a time.
//
// A scalar (the result of a reduce) may be an operand of a map (Sec. 4.1: an object depends on
// other objects; the Pandas / NumPy pipelines of Sec. 4.5 and Sec. 7 normalise by a mean, divide
// by a sum).  A loop cannot read a value that the same loop is still reducing, so evaluation
// then runs in STAGES: every scalar that some map reads is computed by an earlier fused loop
// (all scalars of one stage that iterate over vectors of one length share a loop), and the
// loops that use it read it from device memory with WELD_OP_SCALAR, in stream order: there is
// no host wait and no host copy between the stages.
#include <cstdio>
#include <algorithm>
#include <cstring>
#include <map>
#include <set>
#include <string>
#include <tuple>
#include <vector>

#include "weld_internal.h"
#include "weld_object.h"

enum ObjOp { OBJ_DATA = 0, OBJ_MAP = 1, OBJ_FILTER = 2, OBJ_REDUCE = 3, OBJ_GROUPBY = 4 };

struct weld_object {
    int op = OBJ_DATA;
    int refs = 1;
    std::vector<weld_object*> deps;
    std::vector<weld_op_t> ops;   // OBJ_MAP: the mapped function
    const void* data = nullptr;   // OBJ_DATA
    int64_t len = 0;
    int type = -1;                // element type (vectors), scalar type (reduce)
    int func = 0;
    int64_t capacity = 0;
    int nkeys = 0;                // OBJ_GROUPBY: deps = keys then values
};

namespace {

using weld::Error;

Error bad(weld_status_t st, const std::string& s) {
    Error e;
    e.status = st;
    e.text = s;
    return e;
}

void retain(weld_object* o) { ++o->refs; }
void release(weld_object* o) {
    if (!o) return;
    if (--o->refs > 0) return;
    for (weld_object* d : o->deps) release(d);
    delete o;
}

bool is_vec(const weld_object* o) { return o && (o->op == OBJ_DATA || o->op == OBJ_MAP || o->op == OBJ_FILTER); }

// A vector as the fuser sees it: element value and filter predicate, both ids of ops of the
// fused body; n = length of the underlying leaves.
struct Virt {
    int value = -1;
    int pred = -1;
    int64_t n = 0;
    bool scalar = false;   // a reduce result read by a map: the same value for every element
};

// One input of the fused loop: a caller's vector, or the scalar that an earlier stage computed.
struct Leaf {
    const void* data = nullptr;
    int type = -1;
    int64_t len = 0;
    const weld_object* scalar_of = nullptr;
};

// Scalars that earlier stages have computed (device address) and the name each has in listings.
struct Scalars {
    std::map<const weld_object*, const void*> where;
    std::map<const weld_object*, int> name;
    std::map<const weld_object*, const weld_object*> same_as;   // a scalar that repeats another one's computation
    const weld_object* canon(const weld_object* o) const {
        auto it = same_as.find(o);
        return it == same_as.end() ? o : it->second;
    }
    int id_of(const weld_object* o) {
        o = canon(o);
        auto it = name.find(o);
        if (it != name.end()) return it->second;
        const int id = (int)name.size();
        return name[o] = id;
    }
};

struct Fuser {
    std::vector<weld_op_t> ops;                 // the fused body, in dependency order
    std::map<std::tuple<int, int, int, int, int, int64_t>, int> cse;
    std::vector<Leaf> leaves;                   // column k of the fused loop
    std::map<const weld_object*, Virt> memo;
    Scalars* scalars = nullptr;                 // results of earlier stages

    int add(weld_op_t o) {
        o.reserved = 0;
        if (o.opcode != WELD_OP_CONST) o.imm.i64 = 0;
        auto key = std::make_tuple(o.opcode, o.type, o.a, o.b, o.c, o.imm.i64);
        auto it = cse.find(key);
        if (it != cse.end()) return it->second;
        ops.push_back(o);
        return cse[key] = (int)ops.size() - 1;
    }
    int leaf_column(const weld_object* o) {
        for (size_t k = 0; k < leaves.size(); ++k)
            if (!leaves[k].scalar_of && leaves[k].data == o->data && leaves[k].type == o->type && leaves[k].len == o->len)
                return (int)k;
        Leaf l;
        l.data = o->data;
        l.type = o->type;
        l.len = o->len;
        leaves.push_back(l);
        return (int)leaves.size() - 1;
    }
    int scalar_column(const weld_object* o) {
        if (scalars) o = scalars->canon(o);
        for (size_t k = 0; k < leaves.size(); ++k)
            if (leaves[k].scalar_of == o) return (int)k;
        Leaf l;
        l.type = o->type;
        l.len = 1;
        l.scalar_of = o;
        if (scalars) {
            auto it = scalars->where.find(o);
            if (it != scalars->where.end()) l.data = it->second;
        }
        leaves.push_back(l);
        return (int)leaves.size() - 1;
    }

    Error lower(const weld_object* o, Virt* out) {
        auto it = memo.find(o);
        if (it != memo.end()) { *out = it->second; return Error(); }
        Virt v;
        if (o->op == OBJ_DATA) {
            const int column = leaf_column(o);
            if (column >= WELD_MAX_COLS) return bad(WELD_ERR_UNSUPPORTED, "more than 16 leaf vectors in one fused loop");
            weld_op_t c;
            memset(&c, 0, sizeof c);
            c.opcode = WELD_OP_COL;
            c.type = o->type;
            c.a = column;
            c.b = c.c = -1;
            v.value = add(c);
            v.n = o->len;
        } else if (o->op == OBJ_MAP) {
            std::vector<Virt> in(o->deps.size());
            int first = -1;                              // the first dependency that is a vector
            for (size_t k = 0; k < o->deps.size(); ++k) {
                Error e = lower(o->deps[k], &in[k]);
                if (!e.ok()) return e;
                if (in[k].scalar) continue;
                if (first < 0) first = (int)k;
                else if (in[k].n != in[first].n || in[k].pred != in[first].pred)
                    return bad(WELD_ERR_INVALID_ARG, "map over vectors of different length or with different filters");
            }
            if (first < 0 && !in.empty()) return bad(WELD_ERR_INVALID_ARG, "map: at least one dependency must be a vector");
            v.n = first < 0 ? 0 : in[first].n;
            v.pred = first < 0 ? -1 : in[first].pred;
            std::vector<int> id(o->ops.size(), -1);
            for (size_t i = 0; i < o->ops.size(); ++i) {
                weld_op_t q = o->ops[i];
                if (q.opcode < WELD_OP_COL || q.opcode > WELD_OP_SELECT)
                    return bad(WELD_ERR_INVALID_ARG, "map: operator " + std::to_string(q.opcode) + " does not belong in a map");
                if (q.opcode == WELD_OP_COL) {
                    if (q.a < 0 || q.a >= (int)in.size()) return bad(WELD_ERR_INVALID_ARG, "map refers to a dependency it does not have");
                    if (ops[in[q.a].value].type != q.type) return bad(WELD_ERR_TYPE, "map: dependency has a different element type");
                    id[i] = in[q.a].value;
                    continue;
                }
                if (q.opcode == WELD_OP_INDEX && v.pred >= 0)
                    return bad(WELD_ERR_UNSUPPORTED, "position inside a filtered vector needs the vector materialised first");
                auto remap = [&](int x) { return (x >= 0 && x < (int)i) ? id[x] : -1; };
                if (q.opcode != WELD_OP_CONST && q.opcode != WELD_OP_INDEX) {
                    const int ar = q.opcode == WELD_OP_SELECT ? 3 : (q.opcode >= WELD_OP_ADD ? 2 : 1);
                    const int opnd[3] = {q.a, q.b, q.c};
                    for (int k = 0; k < ar; ++k)
                        if (opnd[k] < 0 || opnd[k] >= (int)i) return bad(WELD_ERR_INVALID_ARG, "map: operand is not an earlier op");
                    q.a = remap(q.a);
                    q.b = ar > 1 ? remap(q.b) : -1;
                    q.c = ar > 2 ? remap(q.c) : -1;
                } else {
                    q.a = q.b = q.c = -1;
                }
                id[i] = add(q);
            }
            if (id.empty()) return bad(WELD_ERR_INVALID_ARG, "empty map");
            v.value = id.back();
        } else if (o->op == OBJ_FILTER) {
            Virt vec, mask;
            Error e = lower(o->deps[0], &vec);
            if (!e.ok()) return e;
            e = lower(o->deps[1], &mask);
            if (!e.ok()) return e;
            if (vec.n != mask.n || vec.pred != mask.pred)
                return bad(WELD_ERR_INVALID_ARG, "filter: mask and vector differ in length or filters");
            if (ops[mask.value].type != WELD_BOOL) return bad(WELD_ERR_TYPE, "filter: mask is not a bool vector");
            v.n = vec.n;
            v.value = vec.value;
            if (vec.pred < 0) {
                v.pred = mask.value;
            } else {
                weld_op_t a;
                memset(&a, 0, sizeof a);
                a.opcode = WELD_OP_AND;
                a.type = WELD_BOOL;
                a.a = vec.pred;
                a.b = mask.value;
                a.c = -1;
                v.pred = add(a);
            }
        } else if (o->op == OBJ_REDUCE) {
            // a scalar that an earlier stage leaves in device memory: one more input of this loop
            const int column = scalar_column(o);
            if (column >= WELD_MAX_COLS) return bad(WELD_ERR_UNSUPPORTED, "more than 16 inputs in one fused loop");
            weld_op_t c;
            memset(&c, 0, sizeof c);
            c.opcode = WELD_OP_SCALAR;
            c.type = o->type;
            c.a = column;
            c.b = c.c = -1;
            v.value = add(c);
            v.n = -1;
            v.scalar = true;
        } else {
            return bad(WELD_ERR_UNSUPPORTED, "a dictionary cannot feed another operator without being evaluated first");
        }
        memo[o] = v;
        *out = v;
        return Error();
    }
};

// The fused program in C-ABI form.
struct Fused {
    Fuser f;
    std::vector<weld_builder_spec_t> specs;
    std::vector<weld_merge_t> merges;
    int64_t n = -1;
};

Error fuse(const weld_object* const* roots, int nroots, Scalars* scalars, Fused* F, bool any_count = false) {
    if (!roots || nroots < 1 || (nroots > WELD_MAX_BUILDERS && !any_count)) return bad(WELD_ERR_INVALID_ARG, "1..8 roots");
    F->f.scalars = scalars;
    for (int r = 0; r < nroots; ++r) {
        const weld_object* o = roots[r];
        if (!o) return bad(WELD_ERR_INVALID_ARG, "null root");
        weld_builder_spec_t s;
        memset(&s, 0, sizeof s);
        weld_merge_t m;
        memset(&m, 0, sizeof m);
        m.builder = r;
        std::vector<Virt> in;
        auto take = [&](const weld_object* d) -> Error {
            Virt v;
            Error e = F->f.lower(d, &v);
            if (!e.ok()) return e;
            if (F->n >= 0 && v.n != F->n) return bad(WELD_ERR_UNSUPPORTED, "roots iterate over vectors of different lengths");
            F->n = v.n;
            if (!in.empty() && v.pred != in[0].pred) return bad(WELD_ERR_INVALID_ARG, "operands went through different filters");
            in.push_back(v);
            return Error();
        };
        if (is_vec(o)) {
            Error e = take(o);
            if (!e.ok()) return e;
            s.kind = WELD_VECBUILDER;
            s.nvals = 1;
            s.val_type[0] = F->f.ops[in[0].value].type;
            m.nvals = 1;
            m.val[0] = in[0].value;
        } else if (o->op == OBJ_REDUCE) {
            Error e = take(o->deps[0]);
            if (!e.ok()) return e;
            s.kind = WELD_MERGER;
            s.func = o->func;
            s.nvals = 1;
            s.val_type[0] = F->f.ops[in[0].value].type;
            m.nvals = 1;
            m.val[0] = in[0].value;
        } else {
            s.kind = WELD_DICTMERGER;
            s.func = o->func;
            s.capacity = o->capacity;
            s.nkeys = o->nkeys;
            s.nvals = (int)o->deps.size() - o->nkeys;
            for (size_t k = 0; k < o->deps.size(); ++k) {
                Error e = take(o->deps[k]);
                if (!e.ok()) return e;
                const int t = F->f.ops[in[k].value].type;
                if ((int)k < o->nkeys) { s.key_type[k] = t; m.key[k] = in[k].value; }
                else { s.val_type[k - o->nkeys] = t; m.val[k - o->nkeys] = in[k].value; }
            }
            m.nkeys = s.nkeys;
            m.nvals = s.nvals;
        }
        m.pred = in[0].pred;
        F->specs.push_back(s);
        F->merges.push_back(m);
    }
    return Error();
}

const char* tname(int t) {
    static const char* n[] = {"bool", "i8", "i32", "i64", "f64"};
    return t >= 0 && t <= 4 ? n[t] : "?";
}
const char* fname(int f) {
    static const char* n[] = {"+", "*", "min", "max"};
    return f >= 0 && f <= 3 ? n[f] : "?";
}

std::string describe(const Fused& F, Scalars* scalars) {
    const std::vector<weld_op_t>& ops = F.f.ops;
    std::string s = "|";
    char b[256];
    std::vector<size_t> vecs;                 // the zipped vectors; scalars of earlier stages are parameters only
    std::vector<int> zip_pos(F.f.leaves.size(), -1);
    for (size_t k = 0; k < F.f.leaves.size(); ++k) {
        const Leaf& l = F.f.leaves[k];
        if (l.scalar_of) snprintf(b, sizeof b, "%ss%d: %s", k ? ", " : "", scalars ? scalars->id_of(l.scalar_of) : (int)k, tname(l.type));
        else { snprintf(b, sizeof b, "%sv%zu: vec[%s]", k ? ", " : "", k, tname(l.type)); zip_pos[k] = (int)vecs.size(); vecs.push_back(k); }
        s += b;
    }
    s += "|\nresult(for(";
    if (vecs.size() != 1) s += "zip(";
    for (size_t k = 0; k < vecs.size(); ++k) { snprintf(b, sizeof b, "%sv%zu", k ? ", " : "", vecs[k]); s += b; }
    if (vecs.size() != 1) s += ")";
    s += ", {";
    for (size_t r = 0; r < F.specs.size(); ++r) {
        const weld_builder_spec_t& sp = F.specs[r];
        if (r) s += ", ";
        if (sp.kind == WELD_VECBUILDER) snprintf(b, sizeof b, "vecbuilder[%s]", tname(sp.val_type[0]));
        else if (sp.kind == WELD_MERGER) snprintf(b, sizeof b, "merger[%s,%s]", tname(sp.val_type[0]), fname(sp.func));
        else snprintf(b, sizeof b, "dictmerger[{%d keys},{%d values},%s]", sp.nkeys, sp.nvals, fname(sp.func));
        s += b;
    }
    s += "}, |bs, i, x|\n";
    static const char* sym[] = {"", "", "", "-", "!", "cast", "exp", "log", "sqrt", "erf", "+", "-", "*", "/", "%",
                                "min", "max", "<", "<=", ">", ">=", "==", "!=", "&&", "||", "select"};
    auto ref = [&](int id) {
        const weld_op_t& q = ops[id];
        char t[64];
        if (q.opcode == WELD_OP_COL) snprintf(t, sizeof t, "x.%d", zip_pos[q.a]);
        else if (q.opcode == WELD_OP_SCALAR) snprintf(t, sizeof t, "s%d", scalars ? scalars->id_of(F.f.leaves[q.a].scalar_of) : q.a);
        else if (q.opcode == WELD_OP_INDEX) snprintf(t, sizeof t, "i");
        else if (q.opcode == WELD_OP_CONST) {
            if (q.type == WELD_F64) snprintf(t, sizeof t, "%.17g", q.imm.f64);
            else snprintf(t, sizeof t, "%lld", (long long)q.imm.i64);
        } else snprintf(t, sizeof t, "t%d", id);
        return std::string(t);
    };
    for (size_t i = 0; i < ops.size(); ++i) {
        const weld_op_t& q = ops[i];
        if (q.opcode <= WELD_OP_INDEX || q.opcode == WELD_OP_SCALAR) continue;
        std::string e;
        if (q.opcode == WELD_OP_SELECT) e = "select(" + ref(q.a) + ", " + ref(q.b) + ", " + ref(q.c) + ")";
        else if (q.opcode >= WELD_OP_ADD && q.opcode != WELD_OP_MIN && q.opcode != WELD_OP_MAX) e = ref(q.a) + " " + sym[q.opcode] + " " + ref(q.b);
        else if (q.opcode == WELD_OP_MIN || q.opcode == WELD_OP_MAX) e = std::string(sym[q.opcode]) + "(" + ref(q.a) + ", " + ref(q.b) + ")";
        else if (q.opcode == WELD_OP_CAST) e = std::string(tname(q.type)) + "(" + ref(q.a) + ")";
        else if (q.opcode == WELD_OP_NEG || q.opcode == WELD_OP_NOT) e = std::string(sym[q.opcode]) + ref(q.a);
        else e = std::string(sym[q.opcode]) + "(" + ref(q.a) + ")";
        snprintf(b, sizeof b, "  let t%zu = ", i);
        s += b + e + ";\n";
    }
    s += "  {";
    for (size_t r = 0; r < F.merges.size(); ++r) {
        const weld_merge_t& m = F.merges[r];
        std::string v;
        if (m.nkeys) {
            v = "{";
            for (int k = 0; k < m.nkeys; ++k) v += (k ? ", " : "") + ref(m.key[k]);
            for (int k = 0; k < m.nvals; ++k) v += ", " + ref(m.val[k]);
            v += "}";
        } else v = ref(m.val[0]);
        if (r) s += ",\n   ";
        if (m.pred >= 0) snprintf(b, sizeof b, "if (%s) merge(bs.%zu, %s) else bs.%zu", ref(m.pred).c_str(), r, v.c_str(), r);
        else snprintf(b, sizeof b, "merge(bs.%zu, %s)", r, v.c_str());
        s += b;
    }
    s += "}))\n";
    return s;
}

// ---- staged evaluation -----------------------------------------------------------------------

// The scalars that the vectors below `o` read directly (not those behind another scalar).
void scalars_below(const weld_object* o, std::set<const weld_object*>* visited, std::vector<const weld_object*>* found) {
    if (!visited->insert(o).second || o->op == OBJ_DATA) return;
    for (const weld_object* d : o->deps) {
        if (d->op == OBJ_REDUCE) {
            bool known = false;
            for (const weld_object* f : *found) known = known || f == d;
            if (!known) found->push_back(d);
        } else {
            scalars_below(d, visited, found);
        }
    }
}

// Below a root: a scalar or dictionary root is an operator over vectors, a vector root is its own tree.
void scalars_of_root(const weld_object* o, std::set<const weld_object*>* visited, std::vector<const weld_object*>* found) {
    if (is_vec(o)) { scalars_below(o, visited, found); return; }
    for (const weld_object* d : o->deps) scalars_below(d, visited, found);
}

// Stage in which scalar s can be computed: one more than the latest scalar its operand reads.
int stage_of(const weld_object* s, std::map<const weld_object*, int>* memo) {
    auto it = memo->find(s);
    if (it != memo->end()) return it->second;
    std::set<const weld_object*> visited;
    std::vector<const weld_object*> need;
    scalars_of_root(s, &visited, &need);
    int latest = 0;
    for (const weld_object* t : need) latest = std::max(latest, stage_of(t, memo));
    return (*memo)[s] = latest + 1;
}

int64_t length_of(const weld_object* o) {
    if (o->op == OBJ_DATA) return o->len;
    if (o->op == OBJ_FILTER || o->op == OBJ_REDUCE) return length_of(o->deps[0]);
    for (const weld_object* d : o->deps)
        if (is_vec(d)) return length_of(d);
    return 0;
}

Error submit(Fused& F, const weld_conf_t* conf, weld_result_t** out) {
    std::vector<weld_col_t> cols(F.f.leaves.size());
    for (size_t k = 0; k < cols.size(); ++k) {
        cols[k].data = F.f.leaves[k].data;
        cols[k].type = F.f.leaves[k].type;
        if (F.f.leaves[k].scalar_of && !cols[k].data) return bad(WELD_ERR_INVALID_ARG, "internal: a scalar was not computed before the loop that reads it");
    }
    weld_cols_t cs;
    cs.ncols = (int32_t)cols.size();
    cs.col = cols.data();
    weld_body_t body;
    body.nops = (int32_t)F.f.ops.size();
    body.ops = F.f.ops.data();
    body.nmerges = (int32_t)F.merges.size();
    body.merges = F.merges.data();
    weld_builder_t b;
    memset(&b, 0, sizeof b);
    b.count = (int32_t)F.specs.size();
    b.spec = F.specs.data();
    if (conf) b.conf = *conf;
    weld_status_t st = weld_fused_for(&cs, F.n < 0 ? 0 : F.n, &body, &b, out);
    if (st != WELD_OK) return bad(st, weld_last_error());
    return Error();
}

// What evaluation would turn down is turned down by a listing as well (maps are checked when fused).
Error check(Fused& F) {
    std::vector<int32_t> types(F.f.leaves.size());
    for (size_t k = 0; k < types.size(); ++k) types[k] = F.f.leaves[k].type;
    weld_body_t body;
    body.nops = (int32_t)F.f.ops.size();
    body.ops = F.f.ops.data();
    body.nmerges = (int32_t)F.merges.size();
    body.merges = F.merges.data();
    weld_builder_t b;
    memset(&b, 0, sizeof b);
    b.count = (int32_t)F.specs.size();
    b.spec = F.specs.data();
    weld::Loop checked;
    return weld::validate(types.data(), (int32_t)types.size(), &body, &b, &checked);
}

// Evaluates (conf, out) or lists (text) the roots: the stages that compute the scalars some map
// reads, then the loop of the roots themselves.
Error run_stages(weld_object* const* roots, int nroots, const weld_conf_t* conf, weld_result_t** out, std::string* text) {
    if (!roots || nroots < 1 || nroots > WELD_MAX_BUILDERS) return bad(WELD_ERR_INVALID_ARG, "1..8 roots");
    for (int r = 0; r < nroots; ++r)
        if (!roots[r]) return bad(WELD_ERR_INVALID_ARG, "null root");

    // every scalar that has to exist before the roots' loop, with its stage
    std::vector<const weld_object*> wanted;
    {
        std::set<const weld_object*> visited;
        for (int r = 0; r < nroots; ++r) scalars_of_root(roots[r], &visited, &wanted);
        for (size_t k = 0; k < wanted.size(); ++k) {     // and what those read in turn
            std::set<const weld_object*> v2;
            scalars_of_root(wanted[k], &v2, &wanted);
        }
    }
    std::map<const weld_object*, int> stage;
    int last_stage = 0;
    for (const weld_object* s : wanted) last_stage = std::max(last_stage, stage_of(s, &stage));

    Scalars scalars;
    std::vector<weld_result_t*> earlier;                 // results of the stages: they own the scalars
    auto fail = [&](Error e) {
        for (weld_result_t* r : earlier) weld_result_free(r);
        return e;
    };
    for (int st = 1; st <= last_stage; ++st) {
        std::map<int64_t, std::vector<const weld_object*>> by_length;
        for (const weld_object* s : wanted)
            if (stage[s] == st) by_length[length_of(s)].push_back(s);
        for (auto& group : by_length) {
            // two scalars that reduce the same expression under the same filter with the same function
            // (x.count() written twice) are one computation: the fuser's expression ids tell
            std::vector<const weld_object*> todo;
            {
                Fused all;
                Error e = fuse(group.second.data(), (int)group.second.size(), &scalars, &all, true);
                if (!e.ok()) return fail(e);
                std::map<std::tuple<int, int, int>, const weld_object*> first;
                for (size_t k = 0; k < group.second.size(); ++k) {
                    const auto key = std::make_tuple(all.specs[k].func, all.merges[k].val[0], all.merges[k].pred);
                    auto it = first.find(key);
                    if (it == first.end()) { first[key] = group.second[k]; todo.push_back(group.second[k]); }
                    else scalars.same_as[group.second[k]] = it->second;
                }
            }
            for (size_t at = 0; at < todo.size(); at += WELD_MAX_BUILDERS) {
                const size_t cnt = std::min<size_t>(WELD_MAX_BUILDERS, todo.size() - at);
                Fused F;
                Error e = fuse(todo.data() + at, (int)cnt, &scalars, &F);
                if (!e.ok()) return fail(e);
                if (text) {
                    if (!(e = check(F)).ok()) return fail(e);
                    *text += "let {";
                    for (size_t k = 0; k < cnt; ++k) *text += (k ? ", s" : "s") + std::to_string(scalars.id_of(todo[at + k]));
                    *text += "} =\n" + describe(F, &scalars) + "\n";
                    continue;
                }
                weld_result_t* r = nullptr;
                if (!(e = submit(F, conf, &r)).ok()) return fail(e);
                earlier.push_back(r);
                for (size_t k = 0; k < cnt; ++k) scalars.where[todo[at + k]] = weld_result_scalar(r, (int32_t)k);
            }
        }
    }

    // the roots' own loop; a root that an earlier stage has computed is not computed again
    std::vector<const weld_object*> rest;
    std::vector<int> slot(nroots, -1);
    for (int r = 0; r < nroots; ++r) {
        if (stage.count(roots[r])) continue;
        slot[r] = (int)rest.size();
        rest.push_back(roots[r]);
    }
    Fused F;
    Error e = fuse(rest.data(), (int)rest.size(), &scalars, &F);
    if (!e.ok()) return fail(e);
    if (text) {
        if (!(e = check(F)).ok()) return fail(e);
        *text += describe(F, &scalars);
        return Error();
    }
    weld_result_t* r = nullptr;
    if (!(e = submit(F, conf, &r)).ok()) return fail(e);
    if (!earlier.empty()) {
        std::vector<BuilderResult> res(nroots);
        for (int k = 0; k < nroots; ++k) {
            if (slot[k] >= 0) {
                res[k] = r->res[slot[k]];
                if (res[k].ctl_index < 0) res[k].ctl_index = slot[k];   // its length word keeps its place
            } else {
                res[k].kind = WELD_MERGER;
                res[k].scalar = const_cast<void*>(scalars.where[scalars.canon(roots[k])]);
                res[k].elem_size = weld::type_size(roots[k]->type);
            }
        }
        r->res.swap(res);
        r->earlier = earlier;
    }
    *out = r;
    return Error();
}

weld_status_t make(int op, weld_object** out, weld_object** created) {
    if (!out) return WELD_ERR_INVALID_ARG;
    *out = nullptr;
    weld_object* o = new weld_object();
    o->op = op;
    *created = o;
    return WELD_OK;
}

int last_type(const std::vector<weld_op_t>& ops) { return ops.empty() ? -1 : ops.back().type; }

}  // namespace

extern "C" {

weld_status_t weld_object_new_data(const void* data, int32_t type, int64_t len, weld_object_t** out) {
    if (!out) return WELD_ERR_INVALID_ARG;
    *out = nullptr;
    if (len < 0 || !weld::type_is_num(type)) { weld::set_last_error("data object: bad type or length"); return WELD_ERR_INVALID_ARG; }
    if (len > 0 && !data) { weld::set_last_error("data object: null pointer"); return WELD_ERR_INVALID_ARG; }
    weld_object* o;
    make(OBJ_DATA, out, &o);
    o->data = data;
    o->type = type;
    o->len = len;
    *out = o;
    return WELD_OK;
}

weld_status_t weld_object_new_map(weld_object_t* const* deps, int32_t ndeps, const weld_op_t* ops, int32_t nops,
                                  weld_object_t** out) {
    if (!out) return WELD_ERR_INVALID_ARG;
    *out = nullptr;
    if (ndeps < 0 || ndeps > WELD_MAX_COLS || nops < 1 || nops > 4096 || !ops || (ndeps > 0 && !deps)) {
        weld::set_last_error("map: bad arguments");
        return WELD_ERR_INVALID_ARG;
    }
    for (int k = 0; k < ndeps; ++k)
        if (!is_vec(deps[k]) && !(deps[k] && deps[k]->op == OBJ_REDUCE)) {
            weld::set_last_error("map: dependencies must be vectors or scalars");
            return WELD_ERR_TYPE;
        }
    weld_object* o;
    make(OBJ_MAP, out, &o);
    o->ops.assign(ops, ops + nops);
    o->type = last_type(o->ops);
    for (int k = 0; k < ndeps; ++k) { retain(deps[k]); o->deps.push_back(deps[k]); }
    *out = o;
    return WELD_OK;
}

weld_status_t weld_object_new_filter(weld_object_t* vec, weld_object_t* mask, weld_object_t** out) {
    if (!out) return WELD_ERR_INVALID_ARG;
    *out = nullptr;
    if (!is_vec(vec) || !is_vec(mask)) { weld::set_last_error("filter: operands must be vectors"); return WELD_ERR_TYPE; }
    if (mask->type != WELD_BOOL) { weld::set_last_error("filter: mask is not a bool vector"); return WELD_ERR_TYPE; }
    weld_object* o;
    make(OBJ_FILTER, out, &o);
    o->type = vec->type;
    retain(vec);
    retain(mask);
    o->deps = {vec, mask};
    *out = o;
    return WELD_OK;
}

weld_status_t weld_object_new_reduce(weld_object_t* vec, int32_t func, weld_object_t** out) {
    if (!out) return WELD_ERR_INVALID_ARG;
    *out = nullptr;
    if (!is_vec(vec)) { weld::set_last_error("reduce: operand must be a vector"); return WELD_ERR_TYPE; }
    if (func < WELD_FUNC_ADD || func > WELD_FUNC_MAX || !weld::type_is_num(vec->type)) {
        weld::set_last_error("reduce: bad function or element type");
        return WELD_ERR_INVALID_ARG;
    }
    weld_object* o;
    make(OBJ_REDUCE, out, &o);
    o->func = func;
    o->type = vec->type;
    retain(vec);
    o->deps = {vec};
    *out = o;
    return WELD_OK;
}

weld_status_t weld_object_new_groupby(weld_object_t* const* keys, int32_t nkeys, weld_object_t* const* vals,
                                      int32_t nvals, int32_t func, int64_t capacity, weld_object_t** out) {
    if (!out) return WELD_ERR_INVALID_ARG;
    *out = nullptr;
    if (!keys || !vals || nkeys < 1 || nkeys > WELD_MAX_KEY_FIELDS || nvals < 1 || nvals > WELD_MAX_VAL_FIELDS ||
        func < WELD_FUNC_ADD || func > WELD_FUNC_MAX || capacity < 1) {
        weld::set_last_error("groupby: bad arguments");
        return WELD_ERR_INVALID_ARG;
    }
    for (int k = 0; k < nkeys; ++k)
        if (!is_vec(keys[k])) { weld::set_last_error("groupby: keys must be vectors"); return WELD_ERR_TYPE; }
    for (int k = 0; k < nvals; ++k)
        if (!is_vec(vals[k])) { weld::set_last_error("groupby: values must be vectors"); return WELD_ERR_TYPE; }
    weld_object* o;
    make(OBJ_GROUPBY, out, &o);
    o->func = func;
    o->capacity = capacity;
    o->nkeys = nkeys;
    o->type = -1;
    for (int k = 0; k < nkeys; ++k) { retain(keys[k]); o->deps.push_back(keys[k]); }
    for (int k = 0; k < nvals; ++k) { retain(vals[k]); o->deps.push_back(vals[k]); }
    *out = o;
    return WELD_OK;
}

int32_t weld_object_kind(const weld_object_t* o) {
    if (!o) return -1;
    return is_vec(o) ? WELD_OBJ_VEC : (o->op == OBJ_REDUCE ? WELD_OBJ_SCALAR : WELD_OBJ_DICT);
}

int32_t weld_object_elem_type(const weld_object_t* o) { return o ? o->type : -1; }

weld_status_t weld_object_evaluate(weld_object_t* const* roots, int32_t nroots, const weld_conf_t* conf,
                                   weld_result_t** out) {
    if (out) *out = nullptr;
    if (!out) return WELD_ERR_INVALID_ARG;
    Error e = run_stages(roots, nroots, conf, out, nullptr);
    if (!e.ok()) { weld::set_last_error(e.text); return e.status; }
    return WELD_OK;
}

int64_t weld_object_describe(weld_object_t* const* roots, int32_t nroots, char* buf, int64_t buflen) {
    std::string s;
    Error e = run_stages(roots, nroots, nullptr, nullptr, &s);
    if (!e.ok()) { weld::set_last_error(e.text); return -1; }
    if (buf && buflen > 0) snprintf(buf, (size_t)buflen, "%s", s.c_str());
    return (int64_t)s.size() + 1;
}

void weld_object_free(weld_object_t* o) { release(o); }

}  // extern "C"
