// The C ABI: planning, workspace layout, launches and result handles.
//
// weld_fused_for is the evaluation entry of Sec. 4.1 of the paper restricted to one
// already-fused loop: it validates the submitted body, plans how each builder is
// realised on the GPU, takes one block from the device pool that holds results and
// workspace together, and enqueues the kernels on the caller's stream.  The handle it
// returns is the paper's WeldResult: checked for failure, queried for pointers, freed
// by the caller (Sec. 4.1, 4.3).
#include <hip/hip_runtime_api.h>

#include <cstdio>
#include <cmath>
#include <cstring>
#include <map>
#include <memory>
#include <mutex>

#include "aot_kernels.h"
#include "weld_internal.h"

namespace weld {

static thread_local std::string g_last_error;
void set_last_error(const std::string& s) { g_last_error = s; }

}  // namespace weld

using namespace weld;

namespace {

const int kCtlBytes = 256;
// control words (u32 index): 0 tile ticket, 2 error bits (1 capacity, 2 bounded wait gave up,
// 4 index / lookup out of range, 8 nested ranges not consecutive),
// byte 16 + 8*b: length / entry count of builder b, byte 96 + 8*b: dictionary header
inline size_t ctl_count_off(int b) { return 16 + 8 * (size_t)b; }
inline size_t ctl_hdr_off(int b) { return 96 + 8 * (size_t)b; }

std::mutex g_cache_mu;
std::vector<uint32_t*> g_pinned;
std::vector<hipEvent_t> g_events;

uint32_t* get_pinned() {
    std::lock_guard<std::mutex> lk(g_cache_mu);
    if (!g_pinned.empty()) { uint32_t* p = g_pinned.back(); g_pinned.pop_back(); return p; }
    void* p = nullptr;
    if (hipHostMalloc(&p, kCtlBytes, hipHostMallocDefault) != hipSuccess) return nullptr;
    return (uint32_t*)p;
}
hipEvent_t get_event() {
    std::lock_guard<std::mutex> lk(g_cache_mu);
    if (!g_events.empty()) { hipEvent_t e = g_events.back(); g_events.pop_back(); return e; }
    hipEvent_t e = nullptr;
    if (hipEventCreate(&e) != hipSuccess) return nullptr;
    return e;
}
void put_back(weld_result* r) {
    std::lock_guard<std::mutex> lk(g_cache_mu);
    if (r->host_ctl) g_pinned.push_back(r->host_ctl);
    if (r->ev0) g_events.push_back(r->ev0);
    if (r->ev1) g_events.push_back(r->ev1);
    if (r->ev2) g_events.push_back(r->ev2);
    if (r->ev3) g_events.push_back(r->ev3);
    r->host_ctl = nullptr;
    r->ev0 = r->ev1 = r->ev2 = r->ev3 = nullptr;
}

// Single-launch loop kernels count their work-groups in, and collect their error bits, in a cell of
// kArriveBytes (a root line and 32 leaf lines) that is zero whenever no such kernel runs (the kernel's last work-group clears it).  Calls on
// one stream run one after the other and share a cell; kernels on different streams may overlap, so
// every (device, stream) gets its own.  Cells are never given back: 4 KiB per stream ever used.
std::mutex g_arrive_mu;
std::map<std::pair<int, void*>, uint32_t*> g_arrive;
char* g_arrive_chunk = nullptr;
int g_arrive_chunk_dev = -1;
size_t g_arrive_used = 0;
const size_t kArriveBytes = 64 * 33;
const size_t kArriveChunk = 65536;

hipError_t arrive_cell(hipStream_t stream, uint32_t** out) {
    int dev = 0;
    hipError_t h = hipGetDevice(&dev);
    if (h != hipSuccess) return h;
    std::lock_guard<std::mutex> lk(g_arrive_mu);
    const auto key = std::make_pair(dev, (void*)stream);
    auto it = g_arrive.find(key);
    if (it != g_arrive.end()) { *out = it->second; return hipSuccess; }
    if (!g_arrive_chunk || g_arrive_chunk_dev != dev || g_arrive_used + kArriveBytes > kArriveChunk) {
        void* p = nullptr;
        if ((h = hipMalloc(&p, kArriveChunk)) != hipSuccess) return h;
        if ((h = hipMemset(p, 0, kArriveChunk)) != hipSuccess) return h;
        if ((h = hipDeviceSynchronize()) != hipSuccess) return h;
        g_arrive_chunk = (char*)p;
        g_arrive_chunk_dev = dev;
        g_arrive_used = 0;
    }
    *out = (uint32_t*)(g_arrive_chunk + g_arrive_used);
    g_arrive_used += kArriveBytes;
    g_arrive[key] = *out;
    return hipSuccess;
}

Error mk(weld_status_t st, const std::string& s) {
    Error e;
    e.status = st;
    e.text = s;
    return e;
}
Error hip_err(const char* what, hipError_t h) {
    return mk(WELD_ERR_DEVICE, std::string(what) + ": " + hipGetErrorString(h));
}

struct DeviceInfo {
    bool ok = false;
    int cus = 256;
};
DeviceInfo& device_info() {
    static DeviceInfo d;
    if (!d.ok) {
        int dev = 0;
        hipDeviceProp_t p;
        if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&p, dev) == hipSuccess) {
            d.cus = p.multiProcessorCount > 0 ? p.multiProcessorCount : 256;
            d.ok = true;
        }
    }
    return d;
}

uint64_t ident_bits(int func, int type) {
    if (type == WELD_F64) {
        double v = func == WELD_FUNC_ADD ? 0.0 : func == WELD_FUNC_MUL ? 1.0
                 : func == WELD_FUNC_MIN ? __builtin_huge_val() : -__builtin_huge_val();
        uint64_t b;
        memcpy(&b, &v, 8);
        return b;
    }
    const int bits = 8 * type_size(type);
    int64_t v = func == WELD_FUNC_ADD ? 0 : func == WELD_FUNC_MUL ? 1
              : func == WELD_FUNC_MIN ? (int64_t)((1ull << (bits - 1)) - 1) : -(int64_t)(1ull << (bits - 1));
    return (uint64_t)v;
}

struct Layout {
    size_t total = 0;
    size_t take(size_t bytes) {
        const size_t off = total;
        total += (bytes + 255) / 256 * 256;
        return off;
    }
};

}  // namespace

namespace weld {

// ---------------------------------------------------------------------------------------
// Plans.  Generating a kernel's text (about 150 KB with the prelude) and looking it up in the
// code-object cache costs the host more than 100 us a call, which shows as idle GPU time
// whenever the previous kernel is short.  A loop that was planned before - same body, builders,
// tuning and alignment - takes its variant, argument slots, loaded kernel and occupancy from here.
namespace {

struct Plan {
    Variant var;
    std::vector<Slot> slots;
    std::string kernel_name;
    Kernel* kern = nullptr;
    int per_cu = 0;
};
std::mutex g_plan_mu;
std::map<std::string, std::shared_ptr<Plan>> g_plans;

template <class T> void key_add(std::string& k, const T& v) { k.append(reinterpret_cast<const char*>(&v), sizeof v); }

std::string plan_key(const Loop& L, const weld_tuning_t& tune, bool aligned, int kind, int extra) {
    std::string k;
    k.reserve(256 + 32 * L.ops.size());
    key_add(k, kind);
    key_add(k, extra);
    key_add(k, aligned);
    key_add(k, tune);
    key_add(k, L.ncols);
    for (int c = 0; c < L.ncols; ++c) { key_add(k, L.col_type[c]); key_add(k, L.col_used[c]); key_add(k, L.col_scalar[c]); }
    for (const weld_op_t& o : L.ops) {
        key_add(k, o.opcode); key_add(k, o.type); key_add(k, o.a); key_add(k, o.b); key_add(k, o.c);
        key_add(k, o.reserved); key_add(k, o.imm.i64);
    }
    for (weld_builder_spec_t b : L.builders) {
        b.init = nullptr;                       // data, not shape
        key_add(k, b.kind); key_add(k, b.func); key_add(k, b.nkeys); key_add(k, b.key_type); key_add(k, b.nvals);
        key_add(k, b.val_type); key_add(k, b.capacity); key_add(k, b.length);
    }
    for (const weld_merge_t& m : L.merges) {
        key_add(k, m.builder); key_add(k, m.pred); key_add(k, m.nkeys); key_add(k, m.key); key_add(k, m.nvals); key_add(k, m.val);
    }
    key_add(k, L.ngather);
    for (int g = 0; g < L.ngather; ++g) { key_add(k, L.gather_type[g]); key_add(k, L.gather_used[g]); }
    key_add(k, L.nouter);
    for (int c = 0; c < L.nouter; ++c) { key_add(k, L.outer_type[c]); key_add(k, L.outer_used[c]); }
    key_add(k, L.ndicts);
    for (int d = 0; d < L.ndicts; ++d) {
        const DictTable& t = L.dict_in[d];
        key_add(k, t.nkeys); key_add(k, t.key_type); key_add(k, t.nvals); key_add(k, t.val_type); key_add(k, L.dict_val_used[d]);
    }
    return k;
}

// kind 0: fused loop; kind 1: flattened inner loop of a nested for (extra = offset type + 16 * how positions map to inner elements)
// create == false: only a plan that an earlier call made is returned (compiling and loading a kernel
// allocates device memory, which some callers must not do)
Error get_plan(const Loop& L, const weld_tuning_t& tune, bool aligned, int kind, int extra, std::shared_ptr<Plan>* out,
               bool create = true) {
    const std::string key = plan_key(L, tune, aligned, kind, extra);
    {
        std::lock_guard<std::mutex> lk(g_plan_mu);
        auto it = g_plans.find(key);
        if (it != g_plans.end()) { *out = it->second; return Error(); }
    }
    if (!create)
        return mk(WELD_ERR_NOT_READY, "this loop has no loaded kernel yet: run it once through weld_fused_for (same body, builders, "
                                      "tuning and 16-byte alignment of the columns) before the call that must not allocate");
    auto p = std::make_shared<Plan>();
    p->var = kind == 0 ? choose_variant(L, tune, aligned) : choose_segmented_variant(L, tune, aligned);
    Generated G = kind == 0 ? generate(L, p->var) : generate_segmented(L, p->var, extra & 15, extra >> 4);
    Error e = jit_get(G.source, G.kernel_name, true, &p->kern);
    if (!e.ok()) return e;
    p->slots = G.slots;
    p->kernel_name = G.kernel_name;
    p->per_cu = jit_blocks_per_cu(p->kern, p->var.block);
    if (p->per_cu <= 0 || p->per_cu > 8) p->per_cu = 8;
    std::lock_guard<std::mutex> lk(g_plan_mu);
    if (g_plans.size() >= 4096) g_plans.clear();      // a program generator gone wild: start over (plans in use stay alive)
    g_plans[key] = p;
    *out = p;
    return Error();
}

}  // namespace

Loop expand_groups(const Loop& in, std::vector<GroupLink>* links) {
    links->clear();
    bool any = false;
    for (const weld_builder_spec_t& s : in.builders)
        if (s.kind == WELD_GROUPBUILDER) any = true;
    if (!any) return in;
    Loop L = in;
    const size_t NB = in.builders.size();
    for (size_t b = 0; b < NB; ++b) {
        if (in.builders[b].kind != WELD_GROUPBUILDER) continue;
        const weld_builder_spec_t g = in.builders[b];
        GroupLink link;
        link.dict = (int)b;
        // the counting dictionary: dictmerger[K, i64, +] of the constant 1
        weld_builder_spec_t d = g;
        d.kind = WELD_DICTMERGER;
        d.func = WELD_FUNC_ADD;
        d.nvals = 1;
        d.val_type[0] = WELD_I64;
        L.builders[b] = d;
        const int m = in.merge_of[b];
        int one = -1;
        if (m >= 0) {
            weld_op_t c;
            memset(&c, 0, sizeof c);
            c.opcode = WELD_OP_CONST;
            c.type = WELD_I64;
            c.a = c.b = c.c = -1;
            c.imm.i64 = 1;
            L.ops.push_back(c);
            one = (int)L.ops.size() - 1;
            L.merges[m].nvals = 1;
            L.merges[m].val[0] = one;
        }
        auto add_vec = [&](int type, int value_op) {
            weld_builder_spec_t v;
            memset(&v, 0, sizeof v);
            v.kind = WELD_VECBUILDER;
            v.nvals = 1;
            v.val_type[0] = type;
            L.builders.push_back(v);
            L.merge_of.push_back(-1);
            const int nb = (int)L.builders.size() - 1;
            if (m >= 0) {
                weld_merge_t mg;
                memset(&mg, 0, sizeof mg);
                mg.builder = nb;
                mg.pred = in.merges[m].pred;
                mg.nvals = 1;
                mg.val[0] = value_op;
                L.merges.push_back(mg);
                L.merge_of[nb] = (int)L.merges.size() - 1;
            }
            return nb;
        };
        // A 64-bit key that provably fits 32 bits (say a remainder by a constant) is written as its low half: the
        // pairs' keys are scratch that is written once and read once, the result's keys come from the dictionary.
        if (g.nkeys == 1 && g.key_type[0] == WELD_I64 && m >= 0 && value_fits32(in, in.merges[m].key[0])) {
            weld_op_t c;
            memset(&c, 0, sizeof c);
            c.opcode = WELD_OP_CAST;
            c.type = WELD_I32;
            c.a = in.merges[m].key[0];
            c.b = c.c = -1;
            L.ops.push_back(c);
            link.key_low_half = true;
            link.key_vec[0] = add_vec(WELD_I32, (int)L.ops.size() - 1);
        } else
        for (int k = 0; k < g.nkeys; ++k) link.key_vec[k] = add_vec(g.key_type[k], m >= 0 ? in.merges[m].key[k] : -1);
        link.val_vec = add_vec(g.val_type[0], m >= 0 ? in.merges[m].val[0] : -1);
        links->push_back(link);
    }
    return L;
}

static Error run_fused_plain(const Loop& L, const std::vector<GroupLink>& links, size_t user_builders, const ColRef* cols,
                             int64_t n, const weld_conf_t& conf, weld_result* r, const void* prior_ctl, const DictTable* tables,
                             const StaticTarget* st = nullptr);

Error run_fused(const Loop& L, const ColRef* cols, int64_t n, const weld_conf_t& conf, weld_result* r,
                const void* prior_ctl, const DictTable* tables) {
    std::vector<GroupLink> links;
    const Loop X = expand_groups(L, &links);
    if (X.builders.size() > 10) return mk(WELD_ERR_UNSUPPORTED, "too many builders once the groupbuilders are expanded (10 at most)");
    if (L.ndicts > 0 && !tables) return mk(WELD_ERR_INVALID_ARG, "the loop probes dictionaries but none were passed");
    return run_fused_plain(X, links, L.builders.size(), cols, n, conf, r, prior_ctl, tables);
}

Error run_fused_static(const Loop& L, const ColRef* cols, int64_t n, const weld_conf_t& conf, const StaticTarget& st) {
    for (const weld_builder_spec_t& s : L.builders)
        if (s.kind == WELD_GROUPBUILDER) return mk(WELD_ERR_UNSUPPORTED, "groupbuilders need workspace in proportion to the rows: not in the call that allocates nothing");
    if (L.ndicts > 0) return mk(WELD_ERR_UNSUPPORTED, "loops that probe dictionaries run through weld_fused_for_probe only");
    weld_result r;                       // never handed out: no events, no pinned words, no pool block
    r.stream = conf.stream;
    const std::vector<GroupLink> none;
    return run_fused_plain(L, none, L.builders.size(), cols, n, conf, &r, nullptr, nullptr, &st);
}

// Loops with static tiles whose builders all live in registers (mergers, vectors written in place,
// dictionaries of a few keys) and that make no trip to memory at a computed address: their grid
// follows from what the body does between its loads.  0: not such a loop; 1: light arithmetic only;
// 2: operators with long dependent chains (division, roots, transcendentals), whose latency other
// wavefronts have to hide.
static int streaming_class(const Loop& L, const Variant& var) {
    if (var.ticketed || var.spill || var.ranges > 1 || L.ndicts > 0 || L.ngather > 0) return 0;
    for (size_t b = 0; b < L.builders.size(); ++b)
        if (var.backend[b] != BK_MERGER && var.backend[b] != BK_VEC_DIRECT && var.backend[b] != BK_DICT_REG) return 0;
    for (const weld_op_t& o : L.ops) {
        switch (o.opcode) {
            case WELD_OP_EXP: case WELD_OP_LOG: case WELD_OP_SQRT: case WELD_OP_ERF: case WELD_OP_DIV: case WELD_OP_MOD:
                return 2;
            default: break;
        }
    }
    return 1;
}

// how a dictmerger's entries lie in the packed result arrays (C struct layout without padding, Sec. 4.2)
static DictLayout packed_layout(const weld_builder_spec_t& s) {
    DictLayout dl;
    memset(&dl, 0, sizeof dl);
    dl.nkeys = s.nkeys;
    int shift = 0;
    for (int k = 0; k < s.nkeys; ++k) {
        dl.key_size[k] = type_size(s.key_type[k]);
        dl.key_shift[k] = shift;
        shift += 8 * dl.key_size[k];
        dl.key_stride += dl.key_size[k];
    }
    dl.nvals = s.nvals;
    for (int k = 0; k < s.nvals; ++k) {
        dl.val_size[k] = type_size(s.val_type[k]);
        dl.val_stride += dl.val_size[k];
    }
    return dl;
}

// entries the slice-building kernel may hand on to the global insert (those that probe past the end of their slice)
static const size_t kOverflowEntries = 1 << 16;

static Error run_fused_plain(const Loop& L, const std::vector<GroupLink>& links, size_t user_builders, const ColRef* cols,
                             int64_t n, const weld_conf_t& conf, weld_result* r, const void* prior_ctl, const DictTable* tables,
                             const StaticTarget* st) {
    hipStream_t stream = (hipStream_t)conf.stream;
    bool aligned = true;
    for (int c = 0; c < L.ncols; ++c)
        if (L.col_used[c] && ((uintptr_t)cols[c].data & 15)) aligned = false;
    std::shared_ptr<Plan> plan;
    // the single-launch form writes the status words whole (it cannot add to an earlier step's), and its
    // arrival cell belongs to one stream: the per-thread default stream is a different stream in every thread
    weld_tuning_t tune = conf.tune;
    if (prior_ctl || stream == hipStreamPerThread) tune.single_launch = -1;
    Error e = get_plan(L, tune, aligned, 0, 0, &plan, st == nullptr);
    if (!e.ok()) return e;
    const Variant& var = plan->var;
    Kernel* kern = plan->kern;
    if (!prior_ctl) r->kernel_name = plan->kernel_name;

    const size_t NB = L.builders.size();
    const int64_t tile = (int64_t)var.block * var.v * var.u;
    const int64_t ntiles = (n + tile - 1) / tile;
    // persistent grid: as many work-groups as are resident at once (registers and LDS
    // of this kernel decide), at most 8 per CU
    int per_cu = plan->per_cu;
    const int sclass = streaming_class(L, var);
    if (sclass == 1) {
        // A loop that only streams its columns through light arithmetic into registers runs best with
        // about 56 KB of loads in flight per compute unit (measured: 28 B/row, 2048-row tiles: one
        // work-group per unit is 3-7 % faster than the eight that fit; seven columns and a register
        // dictionary, 1024-row tiles: two per unit, 4 % slower with three, 20 % with four; one is too few).
        int64_t row_bytes = 0;
        for (int c = 0; c < L.ncols; ++c)
            if (L.col_used[c]) row_bytes += type_size(L.col_type[c]);
        const int64_t tile_bytes = tile * (row_bytes > 0 ? row_bytes : 1);
        const int64_t want = (57344 + tile_bytes - 1) / tile_bytes;
        if (want < per_cu) per_cu = (int)(want < 1 ? 1 : want);
    } else if (sclass == 2) {
        // A loop that computes about as long as it loads: many more work-groups than are resident at once
        // (four fit for the Black-Scholes loop), so that they drift apart and one group's arithmetic
        // overlaps another's loads; a resident grid marches in step.  Measured on that loop, 5e7 rows:
        // 0.465 ms with the 4 per unit that fit, 0.451 with 8, 0.439 with 16, 0.428 with 32, 0.407 with 48,
        // 0.41 with 64 and with one work-group per tile.
        per_cu = 48;
    }
    int64_t grid = conf.tune.grid_blocks > 0 ? conf.tune.grid_blocks : (int64_t)device_info().cus * per_cu;
    if (grid > ntiles) grid = ntiles;
    if (grid < 1) grid = 1;
    if (var.spill && grid > 1024) grid = 1024;   // the queue aggregation scans one segment per work-group and thread
    if (var.vq_builder >= 0 && grid > 2 * (int64_t)device_info().cus) grid = 2 * (int64_t)device_info().cus;   // (segments: grid x ranges)
    if (var.ranges > 1) {   // range-partitioned vecmerger: the same number of work-groups for every range
        grid = grid / var.ranges * var.ranges;
        if (grid < var.ranges) grid = var.ranges;
    }

    // ---- one block: control words, per-builder workspace, results
    Layout lay;
    const size_t off_ctl = lay.take(kCtlBytes);
    // with a StaticTarget the results go to the caller's buffers and only the workspace is laid out
    // (in the library's fixed buffer, whose size then plays the part of the memory limit)
    const int64_t mem_limit = st ? (int64_t)st->scratch_bytes : conf.memory_limit;
    auto take_out = [&](size_t bytes) -> size_t { return st ? 0 : lay.take(bytes); };
    struct Off { size_t part = 0, res = 0, out = 0, desc = 0, keys = 0, vals[8] = {0}, okeys = 0, ovals = 0, log = 0, qcnt = 0,
                        slot_pos = 0, kp32 = 0, kwide = 0, goffsets = 0, gcursor = 0, gdesc = 0, gvalues = 0, gbcursor = 0, gtmp_group = 0, gtmp_value = 0,
                        ovf = 0, ovf_count = 0, packed = 0;
                        int64_t slots = 0, qcap = 0; int glog = -1; };
    auto link_of = [&](size_t b) -> const GroupLink* {
        for (const GroupLink& g : links)
            if ((size_t)g.dict == b) return &g;
        return nullptr;
    };
    std::vector<Off> off(NB);
    for (size_t b = 0; b < NB; ++b) {
        const weld_builder_spec_t& s = L.builders[b];
        switch (var.backend[b]) {
            case BK_MERGER:
                off[b].part = lay.take(8 * (size_t)grid);
                off[b].res = take_out(8);
                break;
            case BK_VEC_DIRECT:
                off[b].out = take_out((size_t)n * type_size(s.val_type[0]));
                break;
            case BK_VEC_COMPACT:
                off[b].out = take_out((size_t)n * type_size(s.val_type[0]));
                off[b].desc = lay.take(8 * (size_t)ntiles);
                break;
            case BK_VECM_REG: case BK_VECM_LDS: case BK_VECM_GLOBAL: case BK_VECM_QUEUE:
                off[b].out = take_out(8 * (size_t)s.length);
                break;
            default: {
                const int64_t slots = dict_table_slots(s.capacity);
                off[b].slots = slots;
                off[b].keys = lay.take(8 * (size_t)(slots + 1));
                for (int k = 0; k < s.nvals; ++k) off[b].vals[k] = lay.take(8 * (size_t)(slots + 1));
                int ks = 0, vs = 0;
                for (int k = 0; k < s.nkeys; ++k) ks += type_size(s.key_type[k]);
                for (int k = 0; k < s.nvals; ++k) vs += type_size(s.val_type[k]);
                off[b].okeys = take_out((size_t)s.capacity * ks);
                off[b].ovals = take_out((size_t)s.capacity * vs);
                if (const GroupLink* g = link_of(b)) {      // second half of a groupbuilder
                    off[b].slot_pos = lay.take(4 * (size_t)(slots + 1));
                    off[b].kwide = lay.take(8);
                    off[b].goffsets = lay.take(8 * (size_t)(s.capacity + 1));
                    off[b].gcursor = lay.take(8 * (size_t)s.capacity);
                    off[b].gdesc = lay.take(8 * (size_t)((s.capacity + 8191) / 8192));
                    off[b].gvalues = lay.take((size_t)n * type_size(L.builders[g->val_vec].val_type[0]));
                }
            }
        }
    }
    // groupbuilders of many groups: the pairs are partitioned by ranges of 2^glog groups first (at
    // most 256 ranges of at most 4096 groups), which takes 10 bytes of scratch per row - unless
    // the memory limit has no room for that next to everything else the loop needs
    {
        size_t still_to_come = 0;
        for (size_t b = 0; b < NB; ++b)
            if (var.backend[b] == BK_DICT_LDS && var.spill) still_to_come += 4 * (size_t)grid * var.spill_parts + 512;
        for (size_t b = 0; b < NB; ++b) {
            const weld_builder_spec_t& s = L.builders[b];
            if (!link_of(b) || s.capacity <= 1024 || s.capacity > 256 * 4096) continue;
            int lg = 10;     // (1e5 groups: 98 ranges of 1024 give the partition longer runs to write than 196 of 512: 2.42 -> 2.34 ms)
            while (((int64_t)256 << lg) < s.capacity) ++lg;
            // (and 8 bytes per table slot for the words the partition step looks keys up in)
            const size_t need = 10 * (size_t)n + 8 * (size_t)(off[b].slots + 1) + 256 * 8 + 1024;
            if (mem_limit > 0 && (int64_t)(lay.total + need + still_to_come) > mem_limit) continue;
            off[b].glog = lg;
            off[b].kp32 = lay.take(8 * (size_t)(off[b].slots + 1));
            off[b].gbcursor = lay.take(256 * 8);
            off[b].gtmp_group = lay.take(2 * (size_t)n);
            off[b].gtmp_value = lay.take(8 * (size_t)n);
        }
    }
    // spill queues of a large LDS dictionary come last, so that they can shrink to what
    // the memory limit leaves: a full segment only sends its merges to the global table
    for (size_t b = 0; b < NB; ++b) {
        if (var.backend[b] != BK_DICT_LDS || !var.spill) continue;
        const weld_builder_spec_t& s = L.builders[b];
        const size_t entry = var.compact == (int)b ? 8 : 8 * (size_t)(1 + s.nvals);
        off[b].qcnt = lay.take(4 * (size_t)grid * var.spill_parts);
        if (var.spill_slices) {
            off[b].ovf_count = lay.take(8);
            off[b].packed = lay.take(8);
            off[b].ovf = lay.take(kOverflowEntries * entry);
        }
        int64_t cap = conf.tune.dict_spill;
        if (cap <= 0) {
            // every row of a work-group may miss: its share of the rows (tickets hand tiles out
            // unevenly: a quarter more), spread over the partitions by a hash (six standard
            // deviations more), plus what the table itself holds when it is flushed
            const double rows = (double)((ntiles + grid - 1) / grid) * (double)tile * (var.ticketed ? 1.25 : 1.0);
            const double mean = (rows + var.lds_slots) / var.spill_parts;
            cap = (int64_t)(mean + 6.0 * std::sqrt(mean) + 16.0);
        }
        if (cap > (1 << 23) - 1) cap = (1 << 23) - 1;   // the kernel indexes a work-group's segments with 32 bits
        const size_t seg = (size_t)grid * var.spill_parts * entry;
        if (mem_limit > 0) {
            const int64_t room = mem_limit - (int64_t)lay.total;
            const int64_t fit = room > 0 ? (room - 256) / (int64_t)seg : 0;
            if (cap > fit) cap = fit > 0 ? fit : 0;
        }
        off[b].qcap = cap;
        off[b].log = lay.take(seg * (size_t)cap);
    }
    // queues of a vecmerger whose merges are queued by range of cells: every row of a work-group may merge, spread
    // over the ranges by its indices (uniform ones: six standard deviations above the mean); a full segment only
    // sends its merges to the result with device atomics, so a memory limit may shrink them too
    if (var.vq_builder >= 0) {
        const size_t b = (size_t)var.vq_builder;
        const size_t entry = var.vq_const ? 2 : 10;
        off[b].qcnt = lay.take(4 * (size_t)grid * var.vq_ranges);
        const double rows = (double)((ntiles + grid - 1) / grid) * (double)tile;
        const double mean = rows / var.vq_ranges;
        int64_t cap = (int64_t)(mean + 6.0 * std::sqrt(mean) + 16.0);
        cap = (cap + 7) / 8 * 8;                        // (segments of 2-byte entries begin at 16-byte addresses)
        const size_t seg = (size_t)grid * var.vq_ranges * entry;
        if (mem_limit > 0) {
            const int64_t room = mem_limit - (int64_t)lay.total;
            const int64_t fit = room > 0 ? (room - 256) / (int64_t)seg / 8 * 8 : 0;
            if (cap > fit) cap = fit > 0 ? fit : 0;
        }
        off[b].qcap = cap;
        off[b].log = lay.take(seg * (size_t)cap);
    }
    if (mem_limit > 0 && (int64_t)lay.total > mem_limit)
        return mk(WELD_ERR_OOM, "the loop needs " + std::to_string(lay.total) + " bytes of device memory, " +
                                    (st ? "the fixed workspace of the call that allocates nothing holds " : "limit is ") +
                                    std::to_string(mem_limit));
    void* block = nullptr;
    if (st) {
        block = st->scratch;
    } else {
        e = pool_alloc(lay.total, &block);
        if (!e.ok()) return e;
        r->blocks.push_back(block);
    }
    char* base = (char*)block;
    // where the results go: pieces of the block, or the caller's buffers
    struct OutPtr { char *res = nullptr, *out = nullptr, *okeys = nullptr, *ovals = nullptr; };
    std::vector<OutPtr> op(NB);
    for (size_t b = 0; b < NB; ++b) {
        if (st) {
            op[b].res = op[b].out = op[b].okeys = (char*)st->outs[b].data;
            op[b].ovals = (char*)st->outs[b].data2;
        } else {
            op[b].res = base + off[b].res;
            op[b].out = base + off[b].out;
            op[b].okeys = base + off[b].okeys;
            op[b].ovals = base + off[b].ovals;
        }
    }

    // ---- results
    r->res.assign(NB, BuilderResult());
    for (size_t b = 0; b < NB; ++b) {
        const weld_builder_spec_t& s = L.builders[b];
        BuilderResult& br = r->res[b];
        br.kind = s.kind;
        br.elem_size = type_size(s.val_type[0]);
        if (s.kind == WELD_MERGER) {
            br.scalar = op[b].res;
        } else if (s.kind == WELD_VECMERGER) {
            br.kind = WELD_VECBUILDER;   // read back like any vector
            br.vec.ptr = op[b].out;
            br.known_len = s.length;
        } else if (s.kind == WELD_VECBUILDER) {
            br.vec.ptr = op[b].out;
            br.known_len = (var.backend[b] == BK_VEC_DIRECT) ? (L.merge_of[b] >= 0 ? n : 0) : -1;
        } else {
            for (int k = 0; k < s.nkeys; ++k) br.key_stride += type_size(s.key_type[k]);
            for (int k = 0; k < s.nvals; ++k) br.val_stride += type_size(s.val_type[k]);
            br.dict.keys.ptr = op[b].okeys;
            br.dict.values.ptr = op[b].ovals;
            br.table.keys = base + off[b].keys;
            br.table.hdr = base + off_ctl + ctl_hdr_off((int)b);
            br.table.slots = off[b].slots;
            br.table.nkeys = s.nkeys;
            br.table.nvals = s.nvals;
            for (int k = 0; k < s.nkeys; ++k) br.table.key_type[k] = s.key_type[k];
            for (int k = 0; k < s.nvals; ++k) {
                br.table.val_type[k] = s.val_type[k];
                br.table.vals[k] = base + off[b].vals[k];
            }
        }
    }

    uint32_t* arrive = nullptr;
    if (var.single) {
        if (st) {
            arrive = st->arrive;
        } else {
            const hipError_t ha = arrive_cell(stream, &arrive);
            if (ha != hipSuccess) return hip_err("arrival cell", ha);
        }
    }

    // ---- kernel arguments, in the order the generated struct declares them
    std::vector<uint64_t> args;
    for (const Slot& s : plan->slots) {
        uint64_t v = 0;
        const int b = s.builder;
        switch (s.kind) {
            case SLOT_N: v = (uint64_t)n; break;
            case SLOT_SPIN: v = conf.tune.spin_limit > 0 ? (uint64_t)conf.tune.spin_limit : (uint64_t)1 << 22; break;
            case SLOT_COL: v = (uint64_t)(uintptr_t)cols[b].data; break;
            // (a single-launch kernel only writes the status words, once: straight into the pinned copy)
            case SLOT_CTL: v = (uint64_t)(uintptr_t)(var.single && !st ? (char*)r->host_ctl : base + off_ctl); break;
            case SLOT_PARTIAL: v = (uint64_t)(uintptr_t)(base + off[b].part); break;
            case SLOT_ARRIVE: v = (uint64_t)(uintptr_t)arrive; break;
            case SLOT_RES: v = (uint64_t)(uintptr_t)op[b].res; break;
            case SLOT_OUT: v = (uint64_t)(uintptr_t)op[b].out; break;
            case SLOT_DESC: v = (uint64_t)(uintptr_t)(base + off[b].desc); break;
            case SLOT_LEN: v = (uint64_t)(uintptr_t)(base + off_ctl + ctl_count_off(b)); break;
            case SLOT_DKEYS: v = (uint64_t)(uintptr_t)(base + off[b].keys); break;
            case SLOT_DHDR: v = (uint64_t)(uintptr_t)(base + off_ctl + ctl_hdr_off(b)); break;
            case SLOT_DSLOTS: v = (uint64_t)off[b].slots; break;
            case SLOT_DVAL: v = (uint64_t)(uintptr_t)(base + off[b].vals[s.field]); break;
            case SLOT_DLOG: v = (uint64_t)(uintptr_t)(base + off[b].log); break;
            case SLOT_DQCNT: v = (uint64_t)(uintptr_t)(base + off[b].qcnt); break;
            case SLOT_DQCAP: v = (uint64_t)off[b].qcap; break;
            case SLOT_PKEYS: v = (uint64_t)(uintptr_t)tables[b].keys; break;
            case SLOT_PHDR: v = (uint64_t)(uintptr_t)tables[b].hdr; break;
            case SLOT_PSLOTS: v = (uint64_t)tables[b].slots; break;
            case SLOT_PVAL: v = (uint64_t)(uintptr_t)tables[b].vals[s.field]; break;
            default: break;
        }
        args.push_back(v);
    }

    // ---- enqueue
    hipError_t h;
    const bool timed = !prior_ctl && !st;
    // Timing events ride on the dispatches they bracket wherever they can (they take the dispatch's own start
    // or end time): an event recorded by itself is a barrier packet, about 4.5 us during which the queue
    // starts nothing, and four of them cost a short call more than its kernels.  The call's start is the
    // start of its first fill kernel, the loop kernel's events are its own (the end is the end of the last
    // queue aggregation where there is one), and only the event the host waits for, behind the copy of the
    // control words, is recorded as before.  A single-launch kernel is all its call enqueues: it carries
    // the call's two events and there are no others.
    const bool lone = timed && var.single;
    bool copies_first = false;              // a vecmerger's initial vector is copied before the first fill kernel runs
    size_t spill_left = 0;
    for (size_t b = 0; b < NB; ++b) {
        if (L.builders[b].kind == WELD_VECMERGER && L.builders[b].init) copies_first = true;
        if (var.backend[b] == BK_DICT_LDS && var.spill) ++spill_left;
    }
    if (var.vq_builder >= 0) ++spill_left;        // (the kernel that merges the vecmerger's queues: the last of them is timed)
    hipEvent_t start_pending = timed && !lone && !copies_first ? r->ev0 : nullptr;
    if (timed && !lone && copies_first && (h = hipEventRecord(r->ev0, stream)) != hipSuccess) return hip_err("hipEventRecord", h);
    // the workspace of the call is cleared by ONE kernel (a dictionary alone has a key column
    // and up to eight value columns; a launch each left the GPU idle for microseconds apiece)
    FillList fills;
    auto fill = [&](void* p, int64_t count, uint64_t value) -> hipError_t {
        if (fills.add(p, count, value)) return hipSuccess;
        const hipError_t he = launch_fill_list(fills, stream, start_pending);
        start_pending = nullptr;
        r->kernel_count++;
        fills = FillList();
        fills.add(p, count, value);
        return he;
    };
    // (a single-launch kernel writes the control words itself, at its end)
    if (!var.single && (h = fill(base + off_ctl, kCtlBytes / 8, 0)) != hipSuccess) return hip_err("fill", h);
    for (size_t b = 0; b < NB; ++b) {
        const weld_builder_spec_t& s = L.builders[b];
        if (var.backend[b] == BK_VEC_COMPACT && ntiles > 0) {
            if ((h = fill(base + off[b].desc, ntiles, 0)) != hipSuccess) return hip_err("fill", h);
        } else if (s.kind == WELD_VECMERGER) {
            // the result starts as a copy of the caller's vector (or as identities)
            if (s.init) {
                h = hipMemcpyAsync(op[b].out, s.init, 8 * (size_t)s.length, hipMemcpyDeviceToDevice, stream);
                r->kernel_count++;
            } else {
                h = fill(op[b].out, s.length, ident_bits(s.func, s.val_type[0]));
            }
            if (h != hipSuccess) return hip_err("vecmerger init", h);
        } else if (s.kind == WELD_DICTMERGER) {
            if ((h = fill(base + off[b].keys, off[b].slots + 1, 0x8000000000000000ull)) != hipSuccess) return hip_err("fill", h);
            for (int k = 0; k < s.nvals; ++k)
                if ((h = fill(base + off[b].vals[k], off[b].slots + 1, ident_bits(s.func, s.val_type[k]))) != hipSuccess)
                    return hip_err("fill", h);
            if (off[b].glog >= 0 && (h = fill(base + off[b].gbcursor, 256, 0)) != hipSuccess) return hip_err("fill", h);
            if (link_of(b) && (h = fill(base + off[b].gdesc, (s.capacity + 8191) / 8192, 0)) != hipSuccess) return hip_err("fill", h);
            if (link_of(b) && (h = fill(base + off[b].kwide, 1, 0)) != hipSuccess) return hip_err("fill", h);
            if (var.spill_slices && var.backend[b] == BK_DICT_LDS && (h = fill(base + off[b].ovf_count, 1, 0)) != hipSuccess) return hip_err("fill", h);
            if (var.spill_slices && var.backend[b] == BK_DICT_LDS && (h = fill(base + off[b].packed, 1, 0)) != hipSuccess) return hip_err("fill", h);
        }
    }
    if (fills.n > 0) {
        if ((h = launch_fill_list(fills, stream, start_pending)) != hipSuccess) return hip_err("fill", h);
        start_pending = nullptr;
        r->kernel_count++;
    }
    for (const GroupLink& g : links) {
        // pairs of a groupbuilder merged without a predicate: their number is n, known now
        // (after the control words have been cleared)
        if (var.backend[g.val_vec] != BK_VEC_DIRECT || L.merge_of[g.val_vec] < 0) continue;
        if ((h = launch_fill64(base + off_ctl + ctl_count_off(g.val_vec), 1, (uint64_t)n, stream)) != hipSuccess) return hip_err("fill", h);
        r->kernel_count++;
    }
    r->lone_kernel = lone;
    e = jit_launch(kern, (unsigned)grid, (unsigned)var.block, args.data(), args.size() * 8, stream,
                   lone ? r->ev0 : timed ? r->ev2 : nullptr, lone ? r->ev1 : timed && spill_left == 0 ? r->ev3 : nullptr);
    if (!e.ok()) return e;
    r->kernel_count++;
    if (!prior_ctl) r->grid = grid;
    // queued dictionary merges: aggregated per key partition, then added to the global table
    // (timed with the loop kernel: it is the second half of that kernel's work)
    for (size_t b = 0; b < NB; ++b) {
        if (var.backend[b] != BK_DICT_LDS || !var.spill) continue;
        const weld_builder_spec_t& s = L.builders[b];
        SpillMerge sm;
        memset(&sm, 0, sizeof sm);
        sm.log = (const unsigned long long*)(base + off[b].log);
        sm.qcnt = (const unsigned int*)(base + off[b].qcnt);
        sm.groups = (int)grid;
        sm.cap = off[b].qcap;
        sm.func = s.func;
        for (int k = 0; k < s.nvals; ++k) {
            sm.is_f64[k] = s.val_type[k] == WELD_F64;
            sm.ident[k] = ident_bits(s.func, s.val_type[k]);
            sm.vals[k] = (unsigned long long*)(base + off[b].vals[k]);
        }
        sm.keys = (unsigned long long*)(base + off[b].keys);
        sm.hdr = (unsigned int*)(base + off_ctl + ctl_hdr_off((int)b));
        sm.slots = off[b].slots;
        sm.err = (int*)(base + off_ctl + 8);
        sm.compact = var.compact == (int)b ? (var.compact_sext ? 2 : 1) : 0;
        sm.capacity = s.capacity;
        if (var.spill_slices) {
            sm.parts = var.spill_parts;
            sm.overflow = (unsigned long long*)(base + off[b].ovf);
            sm.overflow_count = (unsigned int*)(base + off[b].ovf_count);
            sm.overflow_cap = kOverflowEntries;
            if (!link_of(b)) {      // (a groupbuilder's dictionary also needs every slot's position: the extraction kernel's work)
                sm.pack = 1;
                sm.lay = packed_layout(s);
                sm.out_keys = (unsigned char*)op[b].okeys;
                sm.out_vals = (unsigned char*)op[b].ovals;
                sm.out_count = (unsigned long long*)(base + off_ctl + ctl_count_off((int)b));
                sm.packed = (unsigned int*)(base + off[b].packed);
            }
            h = launch_dict_slice_build(sm, s.nvals, stream, timed && spill_left == 1 ? r->ev3 : nullptr);
            r->kernel_count += sm.pack ? 2 : 1;
        } else {
            h = launch_dict_spill_merge(sm, s.nvals, stream, timed && spill_left == 1 ? r->ev3 : nullptr);
        }
        --spill_left;
        if (h != hipSuccess) return hip_err("dict spill merge", h);
        r->kernel_count++;
    }
    if (var.vq_builder >= 0) {
        const size_t b = (size_t)var.vq_builder;
        const weld_builder_spec_t& s = L.builders[b];
        VecmRanges vr;
        memset(&vr, 0, sizeof vr);
        vr.log = base + off[b].log;
        vr.qcnt = (const unsigned int*)(base + off[b].qcnt);
        vr.groups = (int)grid;
        vr.ranges = var.vq_ranges;
        vr.shift = var.vq_shift;
        vr.cap = off[b].qcap;
        vr.length = s.length;
        vr.func = s.func;
        vr.is_f64 = s.val_type[0] == WELD_F64;
        vr.ident = ident_bits(s.func, s.val_type[0]);
        vr.entry_bytes = var.vq_const ? 2 : 10;
        vr.long_segments = (double)n / ((double)grid * var.vq_ranges) >= 1024.0 ? 1 : 0;
        if (var.vq_const) {
            const weld_op_t& c = L.ops[L.merges[L.merge_of[b]].val[0]];
            if (s.val_type[0] == WELD_F64) memcpy(&vr.const_bits, &c.imm.f64, 8);
            else vr.const_bits = (unsigned long long)c.imm.i64;
        }
        vr.out = (unsigned long long*)op[b].out;
        if ((h = launch_vecm_ranges(vr, stream, timed && spill_left == 1 ? r->ev3 : nullptr)) != hipSuccess) return hip_err("vecmerger ranges", h);
        --spill_left;
        r->kernel_count++;
    }
    MergerFinish mf;
    memset(&mf, 0, sizeof mf);
    for (size_t b = 0; b < NB; ++b) {
        const weld_builder_spec_t& s = L.builders[b];
        if (s.kind != WELD_MERGER) continue;
        const int k = mf.n++;
        mf.partial[k] = (const unsigned long long*)(base + off[b].part);
        mf.result[k] = op[b].res;
        mf.func[k] = s.func;
        mf.is_f64[k] = s.val_type[0] == WELD_F64;
        mf.elem_size[k] = type_size(s.val_type[0]);
        mf.bits[k] = 8 * type_size(s.val_type[0]);
    }
    if (mf.n > 0 && !var.single) {
        if ((h = launch_merger_finish(mf, (int)grid, stream)) != hipSuccess) return hip_err("merger finish", h);
        r->kernel_count++;
    }
    for (size_t b = 0; b < NB; ++b) {
        const weld_builder_spec_t& s = L.builders[b];
        if (s.kind != WELD_DICTMERGER) continue;
        const DictLayout dl = packed_layout(s);
        DictValues dv;
        memset(&dv, 0, sizeof dv);
        for (int k = 0; k < s.nvals; ++k) dv.p[k] = (const unsigned long long*)(base + off[b].vals[k]);
        const GroupLink* g = link_of(b);
        h = launch_dict_extract(base + off[b].keys, base + off_ctl + ctl_hdr_off((int)b), off[b].slots, dv, dl, s.capacity,
                                op[b].okeys, op[b].ovals, base + off_ctl + ctl_count_off((int)b),
                                base + off_ctl + 8, g ? (int*)(base + off[b].slot_pos) : nullptr,
                                g && off[b].glog >= 0 ? (unsigned long long*)(base + off[b].kp32) : nullptr,
                                g ? (unsigned int*)(base + off[b].kwide) : nullptr,
                                var.spill_slices && var.backend[b] == BK_DICT_LDS && !g ? (const unsigned int*)(base + off[b].packed) : nullptr, stream);
        if (h != hipSuccess) return hip_err("dict extract", h);
        r->kernel_count++;
        if (!g) continue;
        // groupbuilder: group sizes -> offsets, then every compacted pair to its group's vector
        h = launch_group_offsets(op[b].ovals, base + off_ctl + ctl_count_off((int)b), s.capacity,
                                 base + off[b].goffsets, base + off[b].gcursor, base + off[b].gdesc, base + off_ctl + 8,
                                 device_info().cus, stream);
        if (h != hipSuccess) return hip_err("group offsets", h);
        GroupScatter gs;
        memset(&gs, 0, sizeof gs);
        gs.npairs = (const unsigned long long*)(base + off_ctl + ctl_count_off(g->val_vec));
        gs.nkeys = s.nkeys;
        for (int k = 0; k < s.nkeys; ++k) {
            gs.key[k] = op[g->key_vec[k]].out;
            gs.key_size[k] = dl.key_size[k];
            gs.key_shift[k] = dl.key_shift[k];
        }
        if (g->key_low_half) {
            gs.key_size[0] = 4;
            gs.key_sext32 = 1;
        }
        gs.value = op[g->val_vec].out;
        gs.value_size = type_size(L.builders[g->val_vec].val_type[0]);
        gs.table_keys = (const unsigned long long*)(base + off[b].keys);
        gs.hdr = (const unsigned int*)(base + off_ctl + ctl_hdr_off((int)b));
        gs.slots = off[b].slots;
        gs.slot_pos = (const int*)(base + off[b].slot_pos);
        gs.kp32 = off[b].glog >= 0 ? (const unsigned long long*)(base + off[b].kp32) : nullptr;
        gs.kwide = (const unsigned int*)(base + off[b].kwide);
        gs.capacity = s.capacity;
        gs.offsets = (const long long*)(base + off[b].goffsets);
        gs.cursor = (unsigned long long*)(base + off[b].gcursor);
        gs.values_out = base + off[b].gvalues;
        int64_t gblocks = (n + 4095) / 4096;
        if (gblocks > 2 * device_info().cus) gblocks = 2 * device_info().cus;     // two work-groups fit a CU (64 KiB of LDS each)
        if (gblocks > 0 && off[b].glog >= 0) {
            gs.ngroups = (const unsigned long long*)(base + off_ctl + ctl_count_off((int)b));
            gs.log_bucket = off[b].glog;
            gs.nbuckets = (int)((s.capacity + ((int64_t)1 << off[b].glog) - 1) >> off[b].glog);
            gs.bcursor = (unsigned long long*)(base + off[b].gbcursor);
            gs.tmp_group = (unsigned short*)(base + off[b].gtmp_group);
            gs.tmp_value = (unsigned long long*)(base + off[b].gtmp_value);
            if ((h = launch_group_partition(gs, (int)gblocks, stream)) != hipSuccess) return hip_err("group partition", h);
            if ((h = launch_group_place(gs, 2 * device_info().cus, stream)) != hipSuccess) return hip_err("group place", h);
            r->kernel_count += 2;
        } else if (gblocks > 0) {
            if ((h = launch_group_scatter(gs, (int)gblocks, stream)) != hipSuccess) return hip_err("group scatter", h);
            r->kernel_count++;
        }
        r->kernel_count++;
        BuilderResult& br = r->res[b];
        br.kind = WELD_GROUPBUILDER;
        br.groups.keys.ptr = op[b].okeys;
        br.groups.offsets.ptr = base + off[b].goffsets;
        br.groups.values.ptr = base + off[b].gvalues;
        br.elem_size = gs.value_size;
        br.ctl_index = (int)b;
        br.ctl_index2 = g->val_vec;
    }
    r->res.resize(user_builders);            // the vecbuilders of expanded groupbuilders are internal
    if (prior_ctl) {
        if ((h = launch_or_error(base + off_ctl, prior_ctl, stream)) != hipSuccess) return hip_err("error word", h);
        r->kernel_count++;
    }
    if (st) {
        // no handle, no pinned copy: the error bits and the builders' lengths go to the caller's
        // device array, written by a kernel behind everything else of the call
        StaticLengths sl;
        memset(&sl, 0, sizeof sl);
        sl.count = (int)user_builders;
        for (size_t b = 0; b < user_builders; ++b) {
            const BuilderResult& br = r->res[b];
            sl.known[b] = br.kind == WELD_MERGER ? 1 : br.kind == WELD_VECBUILDER ? br.known_len : -1;
        }
        if ((h = launch_static_status(base + off_ctl, sl, st->status_dev, stream)) != hipSuccess) return hip_err("status", h);
        return Error();
    }
    // The call's last operation: a small kernel that writes the control words to the handle's pinned copy and
    // carries the event the evaluation point waits for (for the event, not for the stream, so work enqueued
    // after this call keeps the GPU busy while the host looks at the result).  A single-launch kernel has
    // written the words itself: if it is all the call enqueued it carries the event too.
    if (!var.single) {
        if ((h = launch_ctl_to_host(base + off_ctl, r->host_ctl, stream, r->ev1)) != hipSuccess) return hip_err("control words", h);
    } else if (!lone && (h = hipEventRecord(r->ev1, stream)) != hipSuccess) {
        return hip_err("hipEventRecord", h);
    }
    r->recorded = true;
    return Error();
}

// ---------------------------------------------------------------------------------------
// Nested loop = flattened inner loop (segmented merger, one cell per outer element) followed
// by the ordinary fused loop over the outer elements with the cells as one more column.
Error run_nested(const NestedLoop& NL, const NestedData& D, const weld_conf_t& conf, weld_result* r) {
    hipStream_t stream = (hipStream_t)conf.stream;
    const Loop& L = NL.inner;
    bool aligned = true;
    for (int c = 0; c < L.ncols; ++c)
        if (L.col_used[c] && ((uintptr_t)D.inner[c].data & 15)) aligned = false;
    const int mapped = NL.any_ranges ? (NL.stride_col >= 0 ? 2 : 1) : 0;
    std::shared_ptr<Plan> plan;
    Error e = get_plan(L, conf.tune, aligned, 1, NL.offset_type + 16 * mapped, &plan);
    if (!e.ok()) return e;
    const Variant& var = plan->var;
    Kernel* kern = plan->kern;
    r->kernel_name = plan->kernel_name;
    const int64_t tile = (int64_t)var.block * var.v * var.u;
    const int is64 = NL.offset_type == WELD_I64;
    const weld_builder_spec_t& ms = L.builders[0];
    hipError_t h;

    // Ranges with strides, overlaps or gaps: the flattened loop runs over the positions 0 .. total-1, total =
    // the sum of the ranges' element counts, which a small kernel computes together with their prefix sums
    // (the boundaries of the outer elements among the positions).  The rest of the call is sized by that
    // total, so the host waits for it here - and learns whether the ranges are valid before anything
    // reads through them.
    int64_t n_flat = D.n_inner;
    char* pre = nullptr;              // control words of this step, then the prefix sums
    size_t pre_bytes = 0;
    if (mapped) {
        Layout lp;
        const size_t o_ctl = lp.take(kCtlBytes);
        const size_t o_off = lp.take(8 * (size_t)(D.n_outer + 1));
        pre_bytes = lp.total;
        if (conf.memory_limit > 0 && (int64_t)pre_bytes > conf.memory_limit)
            return mk(WELD_ERR_OOM, "the ranges' prefix sums need " + std::to_string(pre_bytes) + " bytes of device memory, limit is " +
                                        std::to_string(conf.memory_limit));
        void* block = nullptr;
        e = pool_alloc(pre_bytes, &block);
        if (!e.ok()) return e;
        r->blocks.push_back(block);
        pre = (char*)block;
        if ((h = hipEventRecord(r->ev0, stream)) != hipSuccess) return hip_err("hipEventRecord", h);
        FillList fl;
        fl.add(pre + o_ctl, kCtlBytes / 8, 0);
        if ((h = launch_fill_list(fl, stream)) != hipSuccess) return hip_err("fill", h);
        h = launch_ranges_offsets(D.outer[NL.start_col].data, D.outer[NL.end_col].data,
                                  NL.stride_col >= 0 ? D.outer[NL.stride_col].data : nullptr, is64, D.n_outer, D.n_inner,
                                  pre + o_off, pre + o_ctl + 192, pre + o_ctl + 8, stream);
        if (h != hipSuccess) return hip_err("ranges offsets", h);
        r->kernel_count += 2;
        if ((h = hipMemcpyAsync(r->host_ctl, pre + o_ctl, kCtlBytes, hipMemcpyDeviceToHost, stream)) != hipSuccess) return hip_err("hipMemcpyAsync", h);
        if ((h = hipStreamSynchronize(stream)) != hipSuccess) return hip_err("hipStreamSynchronize", h);
        if (r->host_ctl[2] & 8)
            return mk(WELD_ERR_INVALID_ARG, "a range of the nested loop is invalid (start < 0, end < start, end > n_inner or stride < 1)");
        memcpy(&n_flat, (const char*)r->host_ctl + 192, 8);
        memset(r->host_ctl, 0, kCtlBytes);
        pre += o_off;                 // from here on: the prefix sums
    }
    const int64_t ntiles = (n_flat + tile - 1) / tile;
    const int per_cu = plan->per_cu;
    int64_t grid = conf.tune.grid_blocks > 0 ? conf.tune.grid_blocks : (int64_t)device_info().cus * per_cu;
    if (grid > ntiles) grid = ntiles;
    if (grid < 1) grid = 1;

    Layout lay;
    const size_t off_ctl = lay.take(kCtlBytes);
    const size_t off_tiles = lay.take(4 * (size_t)(ntiles + 1));
    const size_t off_sums = lay.take(8 * (size_t)(D.n_outer > 0 ? D.n_outer : 1));
    if (conf.memory_limit > 0 && (int64_t)(lay.total + pre_bytes) > conf.memory_limit)
        return mk(WELD_ERR_OOM, "the inner loop needs " + std::to_string(lay.total + pre_bytes) + " bytes of device memory, limit is " +
                                    std::to_string(conf.memory_limit));
    void* block = nullptr;
    e = pool_alloc(lay.total, &block);
    if (!e.ok()) return e;
    r->blocks.push_back(block);
    char* base = (char*)block;
    const void* boundaries = mapped ? (const void*)pre : D.outer[NL.start_col].data;

    std::vector<uint64_t> args;
    for (const Slot& s : plan->slots) {
        uint64_t v = 0;
        switch (s.kind) {
            case SLOT_N: v = (uint64_t)n_flat; break;
            case SLOT_N_OUTER: v = (uint64_t)D.n_outer; break;
            case SLOT_COL: v = (uint64_t)(uintptr_t)D.inner[s.builder].data; break;
            case SLOT_GATHER: v = (uint64_t)(uintptr_t)D.gather[s.builder].data; break;
            case SLOT_GATHER_LEN: v = (uint64_t)D.gather_len[s.builder]; break;
            case SLOT_OUTER_COL: v = (uint64_t)(uintptr_t)D.outer[s.builder].data; break;
            case SLOT_SEG_START: v = (uint64_t)(uintptr_t)boundaries; break;
            case SLOT_MAP_START: v = (uint64_t)(uintptr_t)D.outer[NL.start_col].data; break;
            case SLOT_MAP_STRIDE: v = (uint64_t)(uintptr_t)D.outer[NL.stride_col].data; break;
            case SLOT_TILE_ROW: v = (uint64_t)(uintptr_t)(base + off_tiles); break;
            case SLOT_SUMS: v = (uint64_t)(uintptr_t)(base + off_sums); break;
            case SLOT_CTL: v = (uint64_t)(uintptr_t)(base + off_ctl); break;
            default: break;
        }
        args.push_back(v);
    }
    if (!mapped && (h = hipEventRecord(r->ev0, stream)) != hipSuccess) return hip_err("hipEventRecord", h);
    FillList fills;
    fills.add(base + off_ctl, kCtlBytes / 8, 0);
    fills.add(base + off_sums, D.n_outer, ident_bits(ms.func, ms.val_type[0]));
    if ((h = launch_fill_list(fills, stream)) != hipSuccess) return hip_err("fill", h);
    r->kernel_count++;
    if (!mapped) {
        if ((h = launch_segments_check(D.outer[NL.start_col].data, D.outer[NL.end_col].data, is64, D.n_outer, D.n_inner,
                                       base + off_ctl + 8, stream)) != hipSuccess) return hip_err("segments check", h);
        r->kernel_count++;
    }
    if ((h = launch_tile_rows(boundaries, mapped ? 1 : is64, D.n_outer, tile, ntiles, base + off_tiles, stream)) != hipSuccess)
        return hip_err("tile rows", h);
    r->kernel_count++;
    if (ntiles > 0 && D.n_outer > 0) {
        // (the kernel's events are the dispatch's own start and end: no packets of their own in the queue)
        e = jit_launch(kern, (unsigned)grid, (unsigned)var.block, args.data(), args.size() * 8, stream, r->ev2, r->ev3);
        if (!e.ok()) return e;
        r->kernel_count++;
    } else {
        if ((h = hipEventRecord(r->ev2, stream)) != hipSuccess) return hip_err("hipEventRecord", h);
        if ((h = hipEventRecord(r->ev3, stream)) != hipSuccess) return hip_err("hipEventRecord", h);
    }

    // the outer loop: the cells are its last column
    ColRef cols[WELD_MAX_COLS];
    for (int c = 0; c + 1 < NL.outer.ncols; ++c) cols[c] = D.outer[c];
    cols[NL.outer.ncols - 1].data = base + off_sums;
    cols[NL.outer.ncols - 1].type = ms.val_type[0];
    weld_conf_t conf2 = conf;
    if (conf.memory_limit > 0) {
        conf2.memory_limit = conf.memory_limit - (int64_t)(lay.total + pre_bytes);
        if (conf2.memory_limit <= 0) return mk(WELD_ERR_OOM, "no device memory left for the outer loop under the limit");
    }
    return run_fused(NL.outer, cols, D.n_outer, conf2, r, base + off_ctl);
}

void destroy_result(weld_result* r) {
    if (!r) return;
    if (!r->synced && !r->blocks.empty()) (void)hipStreamSynchronize((hipStream_t)r->stream);
    for (weld_result* c : r->earlier) destroy_result(c);
    for (void* p : r->blocks) pool_free(p);
    put_back(r);
    delete r;
}

void recycle_event(hipEvent_t e) {
    if (!e) return;
    std::lock_guard<std::mutex> lk(g_cache_mu);
    g_events.push_back(e);
}

weld_result* new_result(void* stream) {
    weld_result* r = new weld_result();
    r->stream = stream;
    r->host_ctl = get_pinned();
    r->ev0 = get_event();
    r->ev1 = get_event();
    r->ev2 = get_event();
    r->ev3 = get_event();
    if (!r->host_ctl || !r->ev0 || !r->ev1 || !r->ev2 || !r->ev3) {
        destroy_result(r);
        return nullptr;
    }
    memset(r->host_ctl, 0, kCtlBytes);
    return r;
}

}  // namespace weld

extern "C" {

weld_status_t weld_fused_for(const weld_cols_t* cols, int64_t n, const weld_body_t* body,
                             const weld_builder_t* builder, weld_result_t** out) {
    if (out) *out = nullptr;
    if (!cols || !body || !builder || !out) { set_last_error("null argument"); return WELD_ERR_INVALID_ARG; }
    if (n < 0) { set_last_error("negative row count"); return WELD_ERR_INVALID_ARG; }
    if (cols->ncols < 0 || cols->ncols > WELD_MAX_COLS || (cols->ncols > 0 && !cols->col)) {
        set_last_error("bad column list");
        return WELD_ERR_INVALID_ARG;
    }
    int32_t types[WELD_MAX_COLS];
    for (int c = 0; c < cols->ncols; ++c) types[c] = cols->col[c].type;
    Loop L;
    Error e = validate(types, cols->ncols, body, builder, &L);
    if (!e.ok()) { set_last_error(e.text); return e.status; }
    for (int c = 0; c < cols->ncols; ++c) {
        if (((n > 0 && L.col_used[c]) || L.col_scalar[c]) && !cols->col[c].data) { set_last_error("null column pointer"); return WELD_ERR_INVALID_ARG; }
        if ((uintptr_t)cols->col[c].data % (uintptr_t)type_size(L.col_type[c])) {
            set_last_error("column pointer not aligned to its element size");
            return WELD_ERR_INVALID_ARG;
        }
    }
    weld_result* r = new_result(builder->conf.stream);
    if (!r) {
        set_last_error("could not allocate pinned memory / events (no usable HIP device?)");
        return WELD_ERR_DEVICE;
    }
    ColRef refs[WELD_MAX_COLS];
    for (int c = 0; c < cols->ncols; ++c) { refs[c].data = cols->col[c].data; refs[c].type = cols->col[c].type; }
    e = builder->conf.mode == WELD_MODE_FUSED ? run_fused(L, refs, n, builder->conf, r)
                                              : run_unfused(L, refs, n, builder->conf, r);
    if (!e.ok()) {
        set_last_error(e.text);
        destroy_result(r);
        return e.status;
    }
    *out = r;
    return WELD_OK;
}

weld_status_t weld_fused_for_probe(const weld_cols_t* cols, int64_t n, const weld_dict_ref_t* dicts, int32_t ndicts,
                                   const weld_body_t* body, const weld_builder_t* builder, weld_result_t** out) {
    if (out) *out = nullptr;
    if (!cols || !body || !builder || !out) { set_last_error("null argument"); return WELD_ERR_INVALID_ARG; }
    if (n < 0) { set_last_error("negative row count"); return WELD_ERR_INVALID_ARG; }
    if (ndicts < 0 || ndicts > WELD_MAX_DICT_INPUTS || (ndicts > 0 && !dicts)) { set_last_error("bad dictionary list"); return WELD_ERR_INVALID_ARG; }
    if (cols->ncols < 0 || cols->ncols > WELD_MAX_COLS || (cols->ncols > 0 && !cols->col)) {
        set_last_error("bad column list");
        return WELD_ERR_INVALID_ARG;
    }
    DictTable tables[WELD_MAX_DICT_INPUTS];
    for (int d = 0; d < ndicts; ++d) {
        const weld_result* src = dicts[d].result;
        if (!src || dicts[d].builder < 0 || dicts[d].builder >= (int)src->res.size() ||
            src->res[dicts[d].builder].kind != WELD_DICTMERGER || !src->res[dicts[d].builder].table.keys) {
            set_last_error("dictionary input " + std::to_string(d) + " is not the dictmerger result of an earlier call");
            return WELD_ERR_INVALID_ARG;
        }
        tables[d] = src->res[dicts[d].builder].table;
    }
    if (builder->conf.mode != WELD_MODE_FUSED) { set_last_error("loops that probe dictionaries run in fused mode only"); return WELD_ERR_UNSUPPORTED; }
    NestedContext ctx;
    ctx.ndicts = ndicts;
    ctx.dict_in = tables;
    int32_t types[WELD_MAX_COLS];
    for (int c = 0; c < cols->ncols; ++c) types[c] = cols->col[c].type;
    Loop L;
    Error e = validate(types, cols->ncols, body, builder, &L, &ctx);
    if (!e.ok()) { set_last_error(e.text); return e.status; }
    for (int c = 0; c < cols->ncols; ++c) {
        if (((n > 0 && L.col_used[c]) || L.col_scalar[c]) && !cols->col[c].data) { set_last_error("null column pointer"); return WELD_ERR_INVALID_ARG; }
        if ((uintptr_t)cols->col[c].data % (uintptr_t)type_size(L.col_type[c])) {
            set_last_error("column pointer not aligned to its element size");
            return WELD_ERR_INVALID_ARG;
        }
    }
    weld_result* r = new_result(builder->conf.stream);
    if (!r) {
        set_last_error("could not allocate pinned memory / events (no usable HIP device?)");
        return WELD_ERR_DEVICE;
    }
    ColRef refs[WELD_MAX_COLS];
    for (int c = 0; c < cols->ncols; ++c) { refs[c].data = cols->col[c].data; refs[c].type = cols->col[c].type; }
    e = run_fused(L, refs, n, builder->conf, r, nullptr, tables);
    if (!e.ok()) {
        set_last_error(e.text);
        destroy_result(r);
        return e.status;
    }
    *out = r;
    return WELD_OK;
}

weld_status_t weld_result_status(weld_result_t* r) {
    if (!r) return WELD_ERR_INVALID_ARG;
    if (r->synced) return r->status;
    hipError_t h = r->recorded ? hipEventSynchronize(r->ev1) : hipStreamSynchronize((hipStream_t)r->stream);
    r->synced = true;
    if (h != hipSuccess) {
        r->status = WELD_ERR_DEVICE;
        r->error = std::string("waiting for the call's work: ") + hipGetErrorString(h);
        return r->status;
    }
    (void)hipEventElapsedTime(&r->ms, r->ev0, r->ev1);
    if (r->lone_kernel) r->kernel_ms = r->ms;
    else if (hipEventQuery(r->ev3) == hipSuccess) (void)hipEventElapsedTime(&r->kernel_ms, r->ev2, r->ev3);
    (void)hipGetLastError();
    for (weld_result* c : r->earlier) {   // a staged evaluation fails if one of its stages did; its time is theirs and its own
        const weld_status_t cs = weld_result_status(c);
        if (cs != WELD_OK && r->status == WELD_OK) { r->status = cs; r->error = c->error; }
        if (c->ms > 0.f) r->ms += c->ms;
        r->kernel_count += c->kernel_count;
    }
    const uint32_t err = r->host_ctl[2];
    if (err & 8) {
        r->status = WELD_ERR_INVALID_ARG;
        r->error = "the inner ranges of the nested loop are not consecutive (start[0] == 0, end[i] == start[i+1], end[last] == n_inner)";
    } else if (err & 4) {
        r->status = WELD_ERR_INVALID_ARG;
        r->error = "a vecmerger index or a lookup position was outside its vector";
    } else if (err & 2) {
        r->status = WELD_ERR_DEVICE;
        r->error = "a tile gave up waiting for the prefix of its predecessors (spin limit reached)";
    } else if (err & 1) {
        r->status = WELD_ERR_CAPACITY;
        r->error = "dictmerger met more distinct keys than its declared capacity";
    }
    for (size_t b = 0; b < r->res.size(); ++b) {
        BuilderResult& br = r->res[b];
        int64_t cnt;
        memcpy(&cnt, (const char*)r->host_ctl + ctl_count_off(br.ctl_index >= 0 ? br.ctl_index : (int)b), 8);
        if (br.kind == WELD_GROUPBUILDER) {
            int64_t pairs;
            memcpy(&pairs, (const char*)r->host_ctl + ctl_count_off(br.ctl_index2), 8);
            br.groups.keys.len = cnt;
            br.groups.offsets.len = cnt + 1;
            br.groups.values.len = pairs;
        } else if (br.kind == WELD_VECBUILDER) {
            br.vec.len = br.known_len >= 0 ? br.known_len : cnt;
        } else if (br.kind == WELD_DICTMERGER) {
            br.dict.keys.len = cnt;
            br.dict.values.len = cnt;
        }
    }
    return r->status;
}

const char* weld_result_error(const weld_result_t* r) { return r ? r->error.c_str() : ""; }

const void* weld_result_data(weld_result_t* r, int32_t idx) {
    if (!r || idx < 0 || idx >= (int32_t)r->res.size()) return nullptr;
    if (weld_result_status(r) != WELD_OK) return nullptr;
    BuilderResult& br = r->res[idx];
    if (br.kind == WELD_MERGER) return br.scalar;
    if (br.kind == WELD_VECBUILDER) return &br.vec;
    if (br.kind == WELD_GROUPBUILDER) return &br.groups;
    return &br.dict;
}

const void* weld_result_scalar(const weld_result_t* r, int32_t idx) {
    if (!r || idx < 0 || idx >= (int32_t)r->res.size() || r->res[idx].kind != WELD_MERGER) return nullptr;
    return r->res[idx].scalar;
}

weld_status_t weld_result_fetch(weld_result_t* r, int32_t idx, int32_t part, void* dst, int64_t offset,
                                int64_t bytes, int32_t dst_is_device) {
    if (!r || idx < 0 || idx >= (int32_t)r->res.size() || !dst || offset < 0 || bytes < 0) return WELD_ERR_INVALID_ARG;
    weld_status_t st = weld_result_status(r);
    if (st != WELD_OK) return st;
    BuilderResult& br = r->res[idx];
    const char* src = nullptr;
    int64_t avail = 0;
    if (br.kind == WELD_MERGER) { src = (const char*)br.scalar; avail = br.elem_size; }
    else if (br.kind == WELD_VECBUILDER) { src = (const char*)br.vec.ptr; avail = br.vec.len * br.elem_size; }
    else if (br.kind == WELD_GROUPBUILDER) {
        if (part == 0) { src = (const char*)br.groups.keys.ptr; avail = br.groups.keys.len * br.key_stride; }
        else if (part == 1) { src = (const char*)br.groups.offsets.ptr; avail = br.groups.offsets.len * 8; }
        else { src = (const char*)br.groups.values.ptr; avail = br.groups.values.len * br.elem_size; }
    }
    else if (part == 0) { src = (const char*)br.dict.keys.ptr; avail = br.dict.keys.len * br.key_stride; }
    else { src = (const char*)br.dict.values.ptr; avail = br.dict.values.len * br.val_stride; }
    if (offset + bytes > avail) return WELD_ERR_INVALID_ARG;
    if (bytes == 0) return WELD_OK;
    hipError_t h = hipMemcpy(dst, src + offset, (size_t)bytes, dst_is_device ? hipMemcpyDeviceToDevice : hipMemcpyDeviceToHost);
    if (h != hipSuccess) { r->error = std::string("hipMemcpy: ") + hipGetErrorString(h); return WELD_ERR_DEVICE; }
    return WELD_OK;
}

weld_status_t weld_result_elapsed_ms(weld_result_t* r, float* ms) {
    if (!r || !ms) return WELD_ERR_INVALID_ARG;
    weld_status_t st = weld_result_status(r);
    *ms = r->ms;
    return st;
}

weld_status_t weld_result_busy_ms(weld_result_t* r, float* ms) {
    if (!r || !ms) return WELD_ERR_INVALID_ARG;
    weld_status_t st = weld_result_status(r);
    *ms = r->busy_ms >= 0.f ? r->busy_ms : r->ms;
    return st;
}

weld_status_t weld_result_kernel_ms(weld_result_t* r, float* ms) {
    if (!r || !ms) return WELD_ERR_INVALID_ARG;
    weld_status_t st = weld_result_status(r);
    *ms = r->kernel_ms;
    return st;
}

const char* weld_result_kernel_name(const weld_result_t* r) { return r ? r->kernel_name.c_str() : ""; }

int32_t weld_result_kernel_count(const weld_result_t* r) { return r ? r->kernel_count : 0; }

int64_t weld_result_grid(const weld_result_t* r) { return r ? r->grid : 0; }

void weld_result_free(weld_result_t* r) { destroy_result(r); }

weld_status_t weld_validate(const int32_t* col_types, int32_t ncols, const weld_body_t* body,
                            const weld_builder_t* builder, char* err, size_t errlen) {
    Loop L;
    Error e = validate(col_types, ncols, body, builder, &L);
    if (err && errlen) snprintf(err, errlen, "%s", e.text.c_str());
    if (!e.ok()) set_last_error(e.text);
    return e.status;
}

int64_t weld_generated_source(const int32_t* col_types, int32_t ncols, const weld_body_t* body,
                              const weld_builder_t* builder, char* buf, int64_t buflen) {
    Loop L;
    Error e = validate(col_types, ncols, body, builder, &L);
    if (!e.ok()) { set_last_error(e.text); return -1; }
    std::vector<GroupLink> links;
    const Loop X = expand_groups(L, &links);
    Variant var = choose_variant(X, builder->conf.tune, true);
    Generated G = generate(X, var);
    if (buf && buflen > 0) snprintf(buf, (size_t)buflen, "%s", G.source.c_str());
    return (int64_t)G.source.size() + 1;
}

weld_status_t weld_precompile(const int32_t* col_types, int32_t ncols, const weld_body_t* body,
                              const weld_builder_t* builder) {
    Loop L;
    Error e = validate(col_types, ncols, body, builder, &L);
    if (!e.ok()) { set_last_error(e.text); return e.status; }
    if (builder->conf.mode != WELD_MODE_FUSED) return WELD_OK;  // unfused kernels are compiled ahead of time
    std::vector<GroupLink> links;
    const Loop X = expand_groups(L, &links);
    for (int aligned = 1; aligned >= 0; --aligned) {
        Variant var = choose_variant(X, builder->conf.tune, aligned != 0);
        Generated G = generate(X, var);
        Kernel* k = nullptr;
        e = jit_get(G.source, G.kernel_name, false, &k);
        if (!e.ok()) { set_last_error(e.text); return e.status; }
    }
    return WELD_OK;
}

weld_status_t weld_set_cache_dir(const char* path) { return set_cache_dir(path).status; }

void weld_pool_trim(void) { pool_trim(); }
int64_t weld_pool_bytes(void) { return pool_bytes(); }
const char* weld_last_error(void) { return g_last_error.c_str(); }

weld_status_t weld_probe_read(const void* data, int64_t bytes, void* checksum_dev, void* stream) {
    if (!data || !checksum_dev || bytes < 0 || ((uintptr_t)data & 15)) return WELD_ERR_INVALID_ARG;
    hipError_t h = launch_probe_read(data, bytes, checksum_dev, device_info().cus, (hipStream_t)stream);
    return h == hipSuccess ? WELD_OK : WELD_ERR_DEVICE;
}

weld_status_t weld_probe_copy(void* dst, const void* src, int64_t bytes, void* stream) {
    if (!dst || !src || bytes < 0 || ((uintptr_t)dst & 15) || ((uintptr_t)src & 15)) return WELD_ERR_INVALID_ARG;
    hipError_t h = launch_probe_copy(dst, src, bytes, (hipStream_t)stream);
    return h == hipSuccess ? WELD_OK : WELD_ERR_DEVICE;
}

const char* weld_version(void) { return "weld-hip 0.1 (gfx950)"; }

}  // extern "C"
