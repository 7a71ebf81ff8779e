// Internal declarations shared by the host-side translation units of libweldhip.
#pragma once

#include <cstdint>
#include <string>
#include <vector>

#include "weld_hip.h"
#include "weld_nested.h"

#include <hip/hip_runtime_api.h>

// The open-addressing table a dictmerger leaves behind (device pointers into the result's
// block), kept so that a later loop can probe it.
struct DictTable {
    const void* keys = nullptr;
    const void* vals[WELD_MAX_VAL_FIELDS] = {nullptr};
    const void* hdr = nullptr;
    int64_t slots = 0;
    int nkeys = 0, nvals = 0;
    int key_type[WELD_MAX_KEY_FIELDS] = {0};
    int val_type[WELD_MAX_VAL_FIELDS] = {0};
};

struct BuilderResult {
    int kind = 0;
    void* scalar = nullptr;   // merger: device pointer to the scalar
    weld_vec_t vec = {0, nullptr};
    weld_dict_t dict = {{0, nullptr}, {0, nullptr}};
    int elem_size = 0;        // vecbuilder element / merger scalar size
    int key_stride = 0, val_stride = 0;
    int64_t known_len = -1;   // vecbuilder without predicate: n
    weld_groups_t groups = {{0, nullptr}, {0, nullptr}, {0, nullptr}};   // groupbuilder
    int ctl_index = -1;       // which length word of the control block belongs to this result (-1: its own index)
    int ctl_index2 = -1;      // groupbuilder: the word holding the number of grouped values
    DictTable table;          // dictmerger
};

struct weld_result {
    std::vector<BuilderResult> res;
    std::vector<void*> blocks;   // pool blocks owned by this result
    void* stream = nullptr;
    hipEvent_t ev0 = nullptr, ev1 = nullptr;   // around everything the call enqueues
    hipEvent_t ev2 = nullptr, ev3 = nullptr;   // around the main loop kernel alone
    uint32_t* host_ctl = nullptr;  // pinned copy of the control words
    bool synced = false;
    bool recorded = false;         // ev1 stands after the call's last operation on the stream
    bool lone_kernel = false;      // the call enqueued one kernel and nothing else: ev2 / ev3 not recorded, kernel_ms = ms
    int64_t grid = 0;              // work-groups of the main loop kernel
    weld_status_t status = WELD_OK;
    std::string error;
    int kernel_count = 0;
    float ms = -1.f;
    float kernel_ms = -1.f;
    float busy_ms = -1.f;          // unfused mode: sum of the operator loops' own GPU time (no host waits between them)
    std::string kernel_name;
    std::vector<weld_result*> earlier;   // staged evaluation: the loops that ran before this one; freed with it
};

namespace weld {

inline int type_size(int t) {
    switch (t) {
        case WELD_BOOL: return 1;
        case WELD_I8: return 1;
        case WELD_I32: return 4;
        case WELD_I64: return 8;
        case WELD_F64: return 8;
    }
    return 0;
}
inline bool type_is_int(int t) { return t == WELD_I8 || t == WELD_I32 || t == WELD_I64; }
inline bool type_is_num(int t) { return type_is_int(t) || t == WELD_F64; }
inline bool type_valid(int t) { return t >= WELD_BOOL && t <= WELD_F64; }

// A validated copy of one submitted loop.
struct Loop {
    int ncols = 0;
    int col_type[WELD_MAX_COLS] = {0};
    bool col_used[WELD_MAX_COLS] = {false};
    bool col_scalar[WELD_MAX_COLS] = {false};   // read by WELD_OP_SCALAR: one element, the same for every row
    std::vector<weld_op_t> ops;
    std::vector<weld_builder_spec_t> builders;
    std::vector<int> merge_of;           // per builder: index into merges, or -1
    std::vector<weld_merge_t> merges;
    // inner loop of a nested `for` only: vectors WELD_OP_LOOKUP may read, and the outer
    // vectors WELD_OP_OUTER reads at the current outer element
    int ngather = 0;
    int gather_type[8] = {0};
    bool gather_used[8] = {false};
    int nouter = 0;
    int outer_type[WELD_MAX_COLS] = {0};
    bool outer_used[WELD_MAX_COLS] = {false};
    // dictionaries of earlier calls that WELD_OP_KEYEXISTS / WELD_OP_DICTLOOKUP probe (types only)
    int ndicts = 0;
    DictTable dict_in[WELD_MAX_DICT_INPUTS];
    bool dict_val_used[WELD_MAX_DICT_INPUTS][WELD_MAX_VAL_FIELDS] = {{false}};
};

// groupbuilder b of a loop, rewritten into builders the kernels know: a dictmerger that counts
// the pairs of every key (it takes b's place), and, appended to the builder list, one
// vecbuilder per key field and one for the value, all under b's predicate.
struct GroupLink {
    int dict = 0;                  // index of the counting dictmerger (= the groupbuilder's index)
    int key_vec[WELD_MAX_KEY_FIELDS] = {0};
    int val_vec = 0;
    bool key_low_half = false;     // the one 64-bit key provably fits 32 bits: its vecbuilder holds the low halves
};
// Whether integer value `op` of the body provably lies in the 32-bit range (interval arithmetic over the body:
// a remainder by a constant, a cast from a narrower type, a constant).
bool value_fits32(const Loop& loop, int op);
// Returns `loop` with every groupbuilder rewritten that way (links in builder order); a loop
// without groupbuilders comes back unchanged.
Loop expand_groups(const Loop& loop, std::vector<GroupLink>* links);

// What the body of an inner loop may refer to besides its own zipped vectors.
struct NestedContext {
    int ndicts = 0;                       // (also used alone, for a loop that probes dictionaries)
    const DictTable* dict_in = nullptr;
    int ngather = 0;
    int gather_type[8] = {0};
    int nouter = 0;
    int outer_type[WELD_MAX_COLS] = {0};
};

struct Error {
    weld_status_t status = WELD_OK;
    std::string text;
    bool ok() const { return status == WELD_OK; }
};

void set_last_error(const std::string& s);

// validate.cpp
Error validate(const int32_t* col_types, int32_t ncols, const weld_body_t* body,
               const weld_builder_t* builder, Loop* out, const NestedContext* inner_of = nullptr);

// How each builder is realised inside the fused kernel.
enum Backend {
    BK_MERGER = 0,      // register accumulator, work-group partials, last-arriver combine
    BK_VEC_DIRECT = 1,  // no predicate: out[i] = v, length known in advance (size analysis)
    BK_VEC_COMPACT = 2, // ballot/popcount ranks + decoupled look-back over tile descriptors
    BK_DICT_REG = 3,    // <= 8 groups: key list in LDS, per-lane register accumulators
    BK_DICT_LDS = 4,    // work-group hash table in LDS in front of the global table
    BK_DICT_GLOBAL = 5, // global open-addressing table only
    BK_DICT_LANE = 6,   // <= 8 groups: key list in LDS, per-lane accumulators in LDS ([slot][lane])
    BK_VECM_REG = 7,    // vecmerger, <= 8 cells: per-lane register copies ("local")
    BK_VECM_LDS = 8,    // vecmerger: work-group copy in LDS, LDS atomics ("shared")
    BK_VECM_GLOBAL = 9, // vecmerger: one global copy, device atomics ("global")
    BK_VECM_QUEUE = 10  // vecmerger: merges appended to queues by range of cells, a second kernel merges a range in LDS
};

// Compile-time shape of one fused kernel.  Two loops with equal Variant and equal
// body text share one compiled code object.
// slots of a dictmerger's global table: the power of two >= twice the declared capacity
inline int64_t dict_table_slots(int64_t capacity) {
    int64_t slots = 64;
    while (slots < 2 * capacity) slots *= 2;
    return slots;
}
// slots of the LDS table that aggregates one partition of the spill queues (128 KiB for keys and values)
inline int spill_table_slots(int nvals) { return nvals <= 1 ? 8192 : nvals <= 3 ? 4096 : nvals <= 7 ? 2048 : 1024; }

struct Variant {
    int block = 256;      // W_BLOCK
    int v = 2;            // W_V rows per lane per load
    int u = 4;            // W_U loads in flight per lane and column
    int aligned = 1;      // 16-byte accesses legal for every pointer
    bool ticketed = false;// tile order taken from an atomic ticket (needed by look-back)
    int lds_slots = 0;    // slots of the LDS dictionary (BK_DICT_LDS)
    int ranges = 1;       // > 1: vecmerger cells split into this many 8192-cell ranges, one per group of
                          // work-groups; every group scans all rows and merges only its own range
    int door_words = 0;   // > 0: admission filter of that many 32-bit words in front of the LDS table
    bool spill = false;   // merges that miss the LDS dictionary are appended to key-partitioned queues
                          // which a second kernel aggregates, instead of device atomics on the global table
    int spill_parts = 256;      // partitions of the spill queues
    bool spill_slices = false;  // the partitions are slices of the global table (a partition = the keys whose home
                                // slot lies in one slice) that a second kernel builds in LDS, slice by slice
    bool merge_loop = false;    // merges into builders that live in memory run in one loop over the rows a
                                // lane holds (their code exists once per kernel instead of once per row)
    int defer_builder = -1;     // LDS dictionary whose merges beyond the first probe are queued per wavefront
    int defer_cap = 0;          // and handled 64 at a time; entries the queue holds
    int compact = -1;           // LDS dictionary with 8-byte cells (32-bit key, 32-bit partial sum) and 8-byte queue
                                // entries: a dictmerger[K,V,+] whose key provably fits 32 bits and whose one value is a
                                // constant or a 32-bit integer
    bool compact_sext = false;  // the 64-bit key is the sign extension (else the zero extension) of its low half
    long long compact_guard = 0;// > 0: |constant merged|; a work-group flushes its table before a cell could pass 2^31
    bool own_math = true;       // exp and log evaluated by the library's own code (else the device math library's)
    int pipeline = 0;          // ticketed loops: 1 = the next tile's columns are loaded while this tile is merged and stored
    bool single = false;        // mergers only: the last work-group to finish combines the partials and writes results and
                                // status (no fill kernel before the loop kernel, no combining kernel behind it)
    int vq_builder = -1;        // vecmerger whose merges are queued by range of 2^vq_shift cells (vq_ranges ranges): segment
    int vq_shift = 13;          // [work-group][range] of a log in global memory, entries of 2 bytes (the cell within its
    int vq_ranges = 0;          // range; vq_const: the merged value is a constant the second kernel is told) or 10 bytes
    bool vq_const = false;      // (a segment's values, 8 bytes each, then its cells within the range, 2 bytes each)
    bool vq_sorted = false;     // a tile's entries are sorted by range in LDS and leave as runs
    std::vector<int> backend;   // per builder
};

// One 8-byte kernel argument.  The generated `struct KArgs` lists them in this order.
enum SlotKind {
    SLOT_N = 0, SLOT_SPIN, SLOT_COL, SLOT_CTL,
    SLOT_PARTIAL,                       // merger
    SLOT_ARRIVE, SLOT_RES,              // single-launch form: arrival counter and error bits; a merger's result
    SLOT_OUT, SLOT_DESC, SLOT_LEN,      // vecbuilder
    SLOT_DKEYS, SLOT_DHDR, SLOT_DSLOTS, SLOT_DVAL,  // dictmerger
    SLOT_DLOG, SLOT_DQCNT, SLOT_DQCAP,              // dictmerger spill queues
    // flattened inner loop of a nested for
    SLOT_N_OUTER, SLOT_GATHER, SLOT_GATHER_LEN, SLOT_OUTER_COL, SLOT_SEG_START, SLOT_TILE_ROW, SLOT_SUMS,
    SLOT_MAP_START, SLOT_MAP_STRIDE,    // ranges with strides: the caller's start and stride vectors
    // dictionaries probed by the body
    SLOT_PKEYS, SLOT_PHDR, SLOT_PSLOTS, SLOT_PVAL
};
struct Slot {
    SlotKind kind;
    int builder;  // or column index
    int field;    // value field for SLOT_DVAL
    std::string name;
    std::string ctype;
};

struct Generated {
    std::string source;
    std::string kernel_name;
    std::vector<Slot> slots;
    int lds_bytes = 0;
};

// codegen.cpp
Variant choose_variant(const Loop& loop, const weld_tuning_t& tune, bool aligned);
Generated generate(const Loop& loop, const Variant& var);
// The flattened inner loop of a nested for: `loop` is the inner body with one merger;
// offset_type is the type of the outer start/end vectors.  Uses var.block / v / u / aligned and
// var.lds_slots (range boundaries a tile stages in LDS).
Variant choose_segmented_variant(const Loop& loop, const weld_tuning_t& tune, bool aligned);
// mapped: 0 = consecutive ranges (position p of the flattened loop IS inner element p, the inner vectors are
// streamed); 1 / 2 = ranges with gaps, overlaps and (2) a stride vector: the boundaries are the prefix sums of
// the ranges' element counts (64-bit), position p of outer element r is inner element
// start[r] + (p - boundary[r]) * stride[r], and the inner vectors are gathered.
Generated generate_segmented(const Loop& loop, const Variant& var, int offset_type, int mapped = 0);
int key_bits(const weld_builder_spec_t& b);

// jit.cpp
struct Kernel;  // compiled + loaded
Error jit_get(const std::string& source, const std::string& kernel_name, bool load_on_device, Kernel** out);
int jit_blocks_per_cu(Kernel* k, int block);  // resident work-groups per CU, 0 if unknown
// start_event / stop_event (hipEvent_t or null): take the dispatch's own start and end times
Error jit_launch(Kernel* k, unsigned grid, unsigned block, void* args, size_t args_bytes, void* stream, void* start_event = nullptr,
                 void* stop_event = nullptr);
Error set_cache_dir(const char* path);

// pool.cpp
Error pool_alloc(size_t bytes, void** out);
void pool_free(void* p);
void pool_trim();
int64_t pool_bytes();

// A device column handed to a loop.
struct ColRef {
    const void* data = nullptr;
    int type = 0;
};

// runtime.cpp: enqueue one fused loop (validated `loop`) on conf.stream into `r`
// prior_ctl: control block (device) of work already enqueued for the same result handle (the
// flattened inner loop of a nested for).  When given, the handle's start and kernel events are
// left to the caller and that block's error word is folded into this loop's.
// tables: the loop.ndicts dictionaries the body probes.
Error run_fused(const Loop& loop, const ColRef* cols, int64_t n, const weld_conf_t& conf, weld_result* r,
                const void* prior_ctl = nullptr, const DictTable* tables = nullptr);
// A validated nested loop: `inner` holds the inner body with its merger as builder 0, `outer`
// the outer body in which the inner loop's result is column `outer.ncols - 1`.
struct NestedLoop {
    Loop inner, outer;
    int start_col = 0, end_col = 0;
    int offset_type = WELD_I64;
    bool any_ranges = false;    // ranges with strides, overlaps and gaps: positions mapped to inner elements
    int stride_col = -1;        // any_ranges: outer column with the strides, -1 = all 1
};
struct NestedData {
    int64_t n_outer = 0, n_inner = 0;
    ColRef outer[WELD_MAX_COLS];
    ColRef inner[WELD_MAX_COLS];
    ColRef gather[8];
    int64_t gather_len[8] = {0};
};
// Where a loop's results and workspace go when the caller supplies the outputs and the workspace is
// the library's fixed device buffer (weld_fused_for_static): no pool block, no events, no pinned copy.
struct StaticTarget {
    char* scratch = nullptr;            // device; the call's control words and workspace
    uint32_t* arrive = nullptr;         // device; 33 * 64 bytes that are zero between calls (single-launch kernels count in here)
    size_t scratch_bytes = 0;
    const weld_out_t* outs = nullptr;   // one per builder, checked by the caller of run_fused_static
    int64_t* status_dev = nullptr;      // device; 1 + WELD_MAX_BUILDERS words
};
// runtime.cpp: the fused loop with such a target.  Uses only a plan (compiled, loaded kernel) that an
// earlier weld_fused_for call made; WELD_ERR_NOT_READY otherwise.
Error run_fused_static(const Loop& loop, const ColRef* cols, int64_t n, const weld_conf_t& conf, const StaticTarget& st);
Error run_nested(const NestedLoop& loop, const NestedData& data, const weld_conf_t& conf, weld_result* r);
weld_result* new_result(void* stream);   // with pinned control words and events; nullptr on failure
void recycle_event(hipEvent_t e);        // back to the cache new_result takes its events from
void destroy_result(weld_result* r);

// unfused.cpp: the same loop as one kernel per operator, every intermediate in HBM
Error run_unfused(const Loop& loop, const ColRef* cols, int64_t n, const weld_conf_t& conf, weld_result* r);

}  // namespace weld
