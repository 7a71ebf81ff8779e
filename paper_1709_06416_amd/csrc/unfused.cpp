// Operator-at-a-time execution of a submitted loop: the comparison arm.
//
// This is the program BEFORE loop fusion (Sec. 4.5 of the paper, the per-operator
// fragments that the libraries hand over; Sec. 3.3, map / filter / reduce as loops
// over builders): every expression operator becomes its own loop
//     for(operands, vecbuilder[T], x => merge(b, op(x)))
// whose output is a full column in HBM; a predicated merge becomes a filter loop per
// surviving column (Pandas-style `col[mask]`) followed by a loop that only feeds the
// builder.  Each of these loops runs through the same kernel generator and the same
// builder back-ends as the fused mode, so the two modes differ in fusion only: the
// unfused kernels are as bandwidth-efficient as the fused one, there are just many
// more of them and every intermediate makes a round trip through memory.
// Scalar constants stay scalars (as in `x > 0.5` on a NumPy array) unless they are
// merged directly, in which case they are materialised like `np.full(n, c)`.
#include <cstring>
#include <map>

#include "weld_internal.h"

namespace weld {
namespace {

struct Val {
    bool is_const = false;
    bool is_index = false;
    bool is_scalar = false;        // one element in device memory, defined outside the loop: stays a scalar operand
    weld_op_t cst;
    ColRef col;
    weld_result* owner = nullptr;  // sub-result whose block holds `col` (nullptr: caller's column)
    int last_use = -1;             // index of the last operator that reads it; 1<<30 if merged
};

// Builds the Loop of one operator.
struct SubLoop {
    Loop L;
    std::vector<ColRef> cols;
    std::map<const void*, int> col_op;  // column pointer -> op id of its COL op

    int add_col(const ColRef& c) {
        auto it = c.data ? col_op.find(c.data) : col_op.end();
        if (it != col_op.end()) return it->second;
        const int k = L.ncols++;
        L.col_type[k] = c.type;
        L.col_used[k] = true;
        cols.push_back(c);
        weld_op_t o;
        memset(&o, 0, sizeof o);
        o.opcode = WELD_OP_COL;
        o.type = c.type;
        o.a = k;
        o.b = o.c = -1;
        L.ops.push_back(o);
        const int id = (int)L.ops.size() - 1;
        if (c.data) col_op[c.data] = id;
        return id;
    }
    int add_scalar(const ColRef& c) {
        const int k = L.ncols++;
        L.col_type[k] = c.type;
        L.col_scalar[k] = true;
        cols.push_back(c);
        weld_op_t o;
        memset(&o, 0, sizeof o);
        o.opcode = WELD_OP_SCALAR;
        o.type = c.type;
        o.a = k;
        o.b = o.c = -1;
        L.ops.push_back(o);
        return (int)L.ops.size() - 1;
    }
    int add_raw(const weld_op_t& o) {
        L.ops.push_back(o);
        return (int)L.ops.size() - 1;
    }
    int operand(const Val& v) {
        if (v.is_const) return add_raw(v.cst);
        if (v.is_index) {
            weld_op_t o;
            memset(&o, 0, sizeof o);
            o.opcode = WELD_OP_INDEX;
            o.type = WELD_I64;
            o.a = o.b = o.c = -1;
            return add_raw(o);
        }
        if (v.is_scalar) return add_scalar(v.col);
        return add_col(v.col);
    }
    void set_builder(const weld_builder_spec_t& spec, int pred, const std::vector<int>& keys, const std::vector<int>& vals) {
        L.builders.push_back(spec);
        weld_merge_t m;
        memset(&m, 0, sizeof m);
        m.builder = 0;
        m.pred = pred;
        m.nkeys = (int)keys.size();
        m.nvals = (int)vals.size();
        for (size_t k = 0; k < keys.size(); ++k) m.key[k] = keys[k];
        for (size_t k = 0; k < vals.size(); ++k) m.val[k] = vals[k];
        L.merges.push_back(m);
        L.merge_of.assign(1, 0);
    }
};

weld_builder_spec_t vec_spec(int type) {
    weld_builder_spec_t s;
    memset(&s, 0, sizeof s);
    s.kind = WELD_VECBUILDER;
    s.nvals = 1;
    s.val_type[0] = type;
    return s;
}

struct Runner {
    const weld_conf_t& conf;
    weld_result* top;
    std::vector<weld_result*> subs;  // every sub-result still alive
    std::vector<std::pair<hipEvent_t, hipEvent_t>> timers;   // around each finished sub-loop's work, read at the end

    Error run(SubLoop& s, int64_t n, weld_result** out) {
        weld_result* r = new_result(conf.stream);
        if (!r) {
            Error e;
            e.status = WELD_ERR_DEVICE;
            e.text = "could not allocate pinned memory / events";
            return e;
        }
        weld_conf_t c = conf;
        c.mode = WELD_MODE_FUSED;
        Error e = run_fused(s.L, s.cols.data(), n, c, r);
        if (!e.ok()) {
            destroy_result(r);
            return e;
        }
        top->kernel_count += r->kernel_count;
        subs.push_back(r);
        *out = r;
        return Error();
    }
    // give a sub-result's memory back; later work on the same stream may reuse it
    void release(weld_result* r) {
        if (!r) return;
        for (size_t i = 0; i < subs.size(); ++i)
            if (subs[i] == r) { subs.erase(subs.begin() + i); break; }
        r->synced = true;  // stream order protects the memory: no host wait needed
        if (r->recorded) {
            timers.push_back({r->ev0, r->ev1});   // the events outlive the sub-result: its GPU time is summed at the end
            r->ev0 = r->ev1 = nullptr;
        }
        destroy_result(r);
    }
    // move a sub-result's memory into the caller-visible result
    void adopt(weld_result* r) {
        for (void* p : r->blocks) top->blocks.push_back(p);
        r->blocks.clear();
    }
    void release_all() {
        while (!subs.empty()) release(subs.back());
    }
    ~Runner() {
        for (auto& t : timers) { recycle_event(t.first); recycle_event(t.second); }
    }
};

int arity(int opcode) {
    if (opcode == WELD_OP_SELECT) return 3;
    if (opcode >= WELD_OP_ADD && opcode <= WELD_OP_OR) return 2;
    if (opcode >= WELD_OP_NEG && opcode <= WELD_OP_ERF) return 1;
    return 0;
}

}  // namespace

Error run_unfused(const Loop& L, const ColRef* cols, int64_t n, const weld_conf_t& conf, weld_result* top) {
    hipStream_t stream = (hipStream_t)conf.stream;
    Runner R{conf, top, {}};
    const int nops = (int)L.ops.size();
    const size_t NB = L.builders.size();
    std::vector<Val> val(nops);
    hipError_t h;
    auto fail = [&](Error e) { R.release_all(); return e; };
    auto hipfail = [&](const char* what, hipError_t he) {
        Error e;
        e.status = WELD_ERR_DEVICE;
        e.text = std::string(what) + ": " + hipGetErrorString(he);
        R.release_all();
        return e;
    };

    // ---- liveness of every SSA value
    for (int i = 0; i < nops; ++i) {
        const weld_op_t& o = L.ops[i];
        const int ar = arity(o.opcode);
        const int opnd[3] = {o.a, o.b, o.c};
        for (int k = 0; k < ar; ++k) val[opnd[k]].last_use = i;
    }
    for (const weld_merge_t& m : L.merges) {
        if (m.pred >= 0) val[m.pred].last_use = 1 << 30;
        for (int k = 0; k < m.nkeys; ++k) val[m.key[k]].last_use = 1 << 30;
        for (int k = 0; k < m.nvals; ++k) val[m.val[k]].last_use = 1 << 30;
    }

    if ((h = hipEventRecord(top->ev0, stream)) != hipSuccess) return hipfail("hipEventRecord", h);

    // ---- one loop per expression operator, in program order
    for (int i = 0; i < nops; ++i) {
        const weld_op_t& o = L.ops[i];
        Val& v = val[i];
        if (o.opcode == WELD_OP_COL) {
            v.col = cols[o.a];
            continue;
        }
        if (o.opcode == WELD_OP_CONST) {
            v.is_const = true;
            v.cst = o;
            continue;
        }
        if (o.opcode == WELD_OP_INDEX) {
            v.is_index = true;
            continue;
        }
        if (o.opcode == WELD_OP_SCALAR) {
            v.is_scalar = true;
            v.col = cols[o.a];
            continue;
        }
        if (v.last_use < 0) continue;  // dead code: never read
        SubLoop s;
        const int ar = arity(o.opcode);
        const int opnd[3] = {o.a, o.b, o.c};
        weld_op_t q = o;
        int mapped[3] = {-1, -1, -1};
        for (int k = 0; k < ar; ++k) mapped[k] = s.operand(val[opnd[k]]);
        q.a = mapped[0];
        q.b = mapped[1];
        q.c = mapped[2];
        const int id = s.add_raw(q);
        s.set_builder(vec_spec(o.type), -1, {}, {id});
        weld_result* r = nullptr;
        Error e = R.run(s, n, &r);
        if (!e.ok()) return fail(e);
        v.col.data = r->res[0].vec.ptr;
        v.col.type = o.type;
        v.owner = r;
        // operands read for the last time by this operator go back to the pool
        for (int k = 0; k < ar; ++k) {
            Val& u = val[opnd[k]];
            if (u.owner && u.last_use == i) {
                R.release(u.owner);
                u.owner = nullptr;
            }
        }
    }

    // a column for a value that is merged directly: scalars and the row index are
    // materialised first (np.full / np.arange)
    auto as_column = [&](int id, Val* out) -> Error {
        Val& v = val[id];
        if (!v.is_const && !v.is_index && !v.is_scalar) {   // a column already (also: materialised for an earlier merge)
            *out = v;
            return Error();
        }
        SubLoop s;
        const int op = s.operand(v);
        s.set_builder(vec_spec(L.ops[id].type), -1, {}, {op});
        weld_result* r = nullptr;
        Error e = R.run(s, n, &r);
        if (!e.ok()) return e;
        v.col.data = r->res[0].vec.ptr;
        v.col.type = L.ops[id].type;
        v.owner = r;
        v.is_const = v.is_index = v.is_scalar = false;   // every expression operator has run: from here on it is a column
        *out = v;
        return Error();
    };

    // ---- one filter loop per surviving column, then one loop per builder
    top->res.assign(NB, BuilderResult());
    std::vector<weld_result*> final_sub(NB, nullptr);
    std::vector<int64_t> known_len(NB, -1);
    for (size_t b = 0; b < NB; ++b) {
        const weld_builder_spec_t& spec = L.builders[b];
        const int mi = L.merge_of[b];
        std::vector<Val> keycols, valcols;
        int64_t rows = n;
        if (mi >= 0) {
            const weld_merge_t& m = L.merges[mi];
            for (int k = 0; k < m.nkeys; ++k) {
                Val c;
                Error e = as_column(m.key[k], &c);
                if (!e.ok()) return fail(e);
                keycols.push_back(c);
            }
            for (int k = 0; k < m.nvals; ++k) {
                Val c;
                Error e = as_column(m.val[k], &c);
                if (!e.ok()) return fail(e);
                valcols.push_back(c);
            }
            if (m.pred >= 0) {
                Val mask;
                Error e = as_column(m.pred, &mask);
                if (!e.ok()) return fail(e);
                std::map<const void*, Val> filtered;  // same column merged twice is filtered once
                bool have_len = false;
                auto filter = [&](Val& c) -> Error {
                    auto it = filtered.find(c.col.data);
                    if (it != filtered.end()) { c = it->second; return Error(); }
                    SubLoop s;
                    const int pm = s.add_col(mask.col);
                    const int pc = s.add_col(c.col);
                    s.set_builder(vec_spec(c.col.type), pm, {}, {pc});
                    weld_result* r = nullptr;
                    Error e2 = R.run(s, n, &r);
                    if (!e2.ok()) return e2;
                    if (!have_len) {
                        // the length of a filtered column is data dependent: like any
                        // operator-at-a-time library, wait for it before going on
                        weld_status_t st = weld_result_status(r);
                        if (st != WELD_OK) {
                            Error e3;
                            e3.status = st;
                            e3.text = r->error;
                            return e3;
                        }
                        rows = r->res[0].vec.len;
                        have_len = true;
                    }
                    Val f;
                    f.col.data = r->res[0].vec.ptr;
                    f.col.type = c.col.type;
                    f.owner = r;
                    filtered[c.col.data] = f;
                    c = f;
                    return Error();
                };
                for (Val& c : keycols) { e = filter(c); if (!e.ok()) return fail(e); }
                for (Val& c : valcols) { e = filter(c); if (!e.ok()) return fail(e); }
            }
        } else {
            rows = 0;  // a builder that is never merged returns its empty result
        }

        if (spec.kind == WELD_VECBUILDER && mi >= 0 && valcols[0].owner) {
            // the (filtered or mapped) column is the result vector itself
            weld_result* own = valcols[0].owner;
            bool shared = false;          // the same column may feed another builder too
            for (size_t b2 = 0; b2 < b; ++b2)
                if (final_sub[b2] == own) shared = true;
            if (!shared) {
                final_sub[b] = own;
                known_len[b] = rows;
                top->res[b].kind = WELD_VECBUILDER;
                top->res[b].elem_size = type_size(spec.val_type[0]);
                top->res[b].vec.ptr = const_cast<void*>(valcols[0].col.data);
                continue;
            }
        }
        SubLoop s;
        std::vector<int> kops, vops;
        for (Val& c : keycols) kops.push_back(s.add_col(c.col));
        for (Val& c : valcols) vops.push_back(s.add_col(c.col));
        if (mi >= 0) {
            s.set_builder(spec, -1, kops, vops);
        } else {
            s.L.builders.push_back(spec);
            s.L.merge_of.assign(1, -1);
        }
        weld_result* r = nullptr;
        Error e = R.run(s, rows, &r);
        if (!e.ok()) return fail(e);
        final_sub[b] = r;
        top->res[b] = r->res[0];
    }

    if ((h = hipEventRecord(top->ev1, stream)) != hipSuccess) return hipfail("hipEventRecord", h);
    if ((h = hipStreamSynchronize(stream)) != hipSuccess) return hipfail("hipStreamSynchronize", h);
    (void)hipEventElapsedTime(&top->ms, top->ev0, top->ev1);
    auto sum_timers = [&]() {
        for (auto& t : R.timers) {
            float ms = 0.f;
            if (hipEventElapsedTime(&ms, t.first, t.second) == hipSuccess) top->busy_ms = (top->busy_ms < 0.f ? 0.f : top->busy_ms) + ms;
            recycle_event(t.first);
            recycle_event(t.second);
        }
        R.timers.clear();
        (void)hipGetLastError();
    };

    // ---- collect lengths and error flags, keep the result memory, drop the rest
    for (size_t b = 0; b < NB; ++b) {
        weld_result* r = final_sub[b];
        weld_status_t st = weld_result_status(r);
        if (st != WELD_OK && top->status == WELD_OK) {
            top->status = st;
            top->error = r->error;
        }
        if (known_len[b] >= 0) {
            top->res[b].vec.len = known_len[b];
        } else {
            top->res[b] = r->res[0];
        }
    }
    for (weld_result* s : R.subs) {
        if (s->host_ctl[2] != 0 && top->status == WELD_OK) {
            top->status = (s->host_ctl[2] & 4) ? WELD_ERR_INVALID_ARG : (s->host_ctl[2] & 2) ? WELD_ERR_DEVICE : WELD_ERR_CAPACITY;
            top->error = "an operator kernel reported an error";
        }
    }
    for (size_t b = 0; b < NB; ++b) {
        bool seen = false;
        for (size_t b2 = 0; b2 < b; ++b2)
            if (final_sub[b2] == final_sub[b]) seen = true;
        if (!seen) R.adopt(final_sub[b]);
    }
    R.release_all();
    sum_timers();
    top->synced = true;
    return Error();
}

}  // namespace weld
