/*
 * weld_hip.h -- C ABI of the fused data-parallel `for` loop on one MI355X.
 *
 * One call submits what the paper's runtime hands to a backend after loop
 * fusion (Sec. 4.5, the loop "after loop fusion"; Sec. 3.2, parallel `for` and
 * builders; Table 1, builder types): a set of zipped input vectors, a loop
 * body that maps one row to at most one merge per builder, and the builders.
 * The library runs it as ONE pass over the columns in HBM (fused mode) or as
 * one kernel per operator with every intermediate materialised in HBM
 * (unfused mode, the function-call interface the paper argues against,
 * Sec. 1 / Sec. 2.1).
 *
 * Conventions (Sec. 4.2, 4.3 of the paper):
 *   - scalars and structs use C packed layout; a vector is {int64 len, T* ptr};
 *   - input columns are DEVICE pointers owned by the caller; the library never
 *     writes to them and never frees them;
 *   - everything the library allocates, results included, is owned by the
 *     library until weld_result_free(); temporaries go back to its pool when
 *     the result is freed;
 *   - a call only enqueues work on the caller's HIP stream and returns; the
 *     accessors below are the evaluation point and wait for that call's work
 *     (for an event recorded after its last operation, not for what was
 *     enqueued on the stream later: calls can be pipelined);
 *   - every function returns a status; nothing throws across this boundary;
 *     on error from weld_fused_for, *out is NULL.
 *   - all pointers inside the argument structs are HOST pointers to host
 *     arrays, except weld_col_t.data (device) and weld_conf_t.stream (a
 *     hipStream_t, may be NULL for the default stream).
 */
#ifndef WELD_HIP_H
#define WELD_HIP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    WELD_OK = 0,
    WELD_ERR_INVALID_ARG = 1, /* null pointer, negative size, bad index, malformed body    */
    WELD_ERR_TYPE = 2,        /* operand / builder types do not match (no implicit casts)  */
    WELD_ERR_LINEARITY = 3,   /* a builder is merged more than once on a control path      */
    WELD_ERR_UNSUPPORTED = 4, /* legal IR outside the implemented subset                   */
    WELD_ERR_OOM = 5,         /* needs more device memory than conf.memory_limit / device  */
    WELD_ERR_CAPACITY = 6,    /* dictmerger saw more distinct keys than its capacity       */
    WELD_ERR_DEVICE = 7,      /* HIP runtime / runtime-compiler failure, kernel-side abort */
    WELD_ERR_NOT_READY = 8
} weld_status_t;

/* Scalar types of the data model (Sec. 3.1); WELD_BOOL is the type of predicates. */
typedef enum { WELD_BOOL = 0, WELD_I8 = 1, WELD_I32 = 2, WELD_I64 = 3, WELD_F64 = 4 } weld_type_t;

/* Expression operators of the loop body (Sec. 3.2: arithmetic, comparisons, select;
 * exp/log/sqrt/erf are the math operators the Black-Scholes workload of Sec. 7.1 needs;
 * exp, log and erf are evaluated by the library itself - tables and polynomials, within about
 * one unit in the last place (1e-15 relative) of the correctly rounded value - unless
 * weld_tuning_t.device_math asks for the device math library's exp and log).
 * Integers wrap modulo 2^w; integer DIV and MOD truncate toward zero; f64 is IEEE
 * round-to-nearest with one rounding per operator (no contraction).
 * Where the paper is silent the library fixes one behaviour (its tests pin it): an integer x / 0 is 0
 * and x % 0 is 0; the most negative value over -1 wraps to itself (remainder 0); MIN / MAX of anything
 * with a NaN is NaN, as operators and as merge functions; a CAST of f64 to an integer truncates toward
 * zero, NaN gives 0 and values beyond the 64-bit range its nearest end (narrower types then wrap). */
typedef enum {
    WELD_OP_COL = 0,   /* a = column index: the i-th element of that zipped vector        */
    WELD_OP_CONST = 1, /* imm: i64 bits for integer/bool types, f64 for WELD_F64          */
    WELD_OP_INDEX = 2, /* the row index i, type WELD_I64                                  */
    WELD_OP_NEG = 3, WELD_OP_NOT = 4, WELD_OP_CAST = 5,
    WELD_OP_EXP = 6, WELD_OP_LOG = 7, WELD_OP_SQRT = 8, WELD_OP_ERF = 9,
    WELD_OP_ADD = 10, WELD_OP_SUB = 11, WELD_OP_MUL = 12, WELD_OP_DIV = 13, WELD_OP_MOD = 14,
    WELD_OP_MIN = 15, WELD_OP_MAX = 16,
    WELD_OP_LT = 17, WELD_OP_LE = 18, WELD_OP_GT = 19, WELD_OP_GE = 20, WELD_OP_EQ = 21,
    WELD_OP_NE = 22, WELD_OP_AND = 23, WELD_OP_OR = 24,
    WELD_OP_SELECT = 25 /* a = bool condition, b = value if true, c = value if false      */
} weld_opcode_t;

/* One SSA value of the body.  Operands a, b, c are indices of EARLIER entries of
 * weld_body_t.ops (or a column index for WELD_OP_COL); unused operands are -1.
 * Giving every sub-result a name once is the `:=` binding of Sec. 3.2 and makes
 * common sub-expressions shared by construction. */
typedef struct {
    int32_t opcode; /* weld_opcode_t */
    int32_t type;   /* weld_type_t of the result */
    int32_t a, b, c;
    int32_t reserved;
    union { int64_t i64; double f64; } imm;
} weld_op_t;

#define WELD_MAX_KEY_FIELDS 4
#define WELD_MAX_VAL_FIELDS 8
#define WELD_MAX_BUILDERS 8
#define WELD_MAX_COLS 16

/* `if (pred) merge(builders[builder], {keys.., vals..}) else builders[builder]`
 * (Sec. 3.2, third builder example; Sec. 5, predication).  pred = -1 merges on
 * every row.  merger and vecbuilder take nvals == 1, nkeys == 0; dictmerger takes
 * the key struct fields in key[] and the value struct fields in val[]. */
typedef struct {
    int32_t builder;
    int32_t pred;
    int32_t nkeys;
    int32_t key[WELD_MAX_KEY_FIELDS];
    int32_t nvals;
    int32_t val[WELD_MAX_VAL_FIELDS];
} weld_merge_t;

typedef struct {
    int32_t nops;
    const weld_op_t* ops;       /* host */
    int32_t nmerges;
    const weld_merge_t* merges; /* host; at most one merge per builder */
} weld_body_t;

typedef struct {
    const void* data; /* DEVICE pointer to n contiguous elements; never written */
    int32_t type;     /* weld_type_t (not WELD_BOOL) */
} weld_col_t;

typedef struct {
    int32_t ncols;
    const weld_col_t* col; /* host array */
} weld_cols_t;

typedef enum { WELD_MERGER = 0, WELD_VECBUILDER = 1, WELD_DICTMERGER = 2, WELD_VECMERGER = 3, WELD_GROUPBUILDER = 4 } weld_builder_kind_t;
typedef enum { WELD_FUNC_ADD = 0, WELD_FUNC_MUL = 1, WELD_FUNC_MIN = 2, WELD_FUNC_MAX = 3 } weld_func_t;

/* One builder of Table 1.
 *   merger[T,func,id]     : val_type[0] = T; id is func's identity (0, 1, +max, -max).
 *   vecbuilder[T]         : val_type[0] = T; output keeps index order.
 *   dictmerger[K,V,func]  : K = struct of key_type[0..nkeys), V = struct of
 *                           val_type[0..nvals); func is applied field by field; the first
 *                           merge of a key stores its value.  capacity = upper bound on the
 *                           number of distinct keys (exceeding it -> WELD_ERR_CAPACITY).
 *   vecmerger[T,func]     : merges {index, T} pairs into the cells of a vector of `length`
 *                           elements that starts as a copy of `init` (a DEVICE pointer to
 *                           `length` elements of T owned by the caller, never written; NULL =
 *                           every cell starts at func's identity).  key_type[0] = WELD_I64 (the
 *                           index), val_type[0] = T (WELD_I64 or WELD_F64).  An index outside
 *                           0..length-1 makes the call fail with WELD_ERR_INVALID_ARG.
 *   groupbuilder[K,V]     : groups the merged {K, V} pairs by key: the result maps every key
 *                           to the vector of its values (dict[K, vec[V]]).  K as for
 *                           dictmerger, V one scalar: val_type[0]; capacity = upper bound on
 *                           the number of distinct keys.  The order of the values inside a
 *                           group is unspecified (merges may run in any order). */
typedef struct {
    int32_t kind; /* weld_builder_kind_t */
    int32_t func; /* weld_func_t (ignored by vecbuilder) */
    int32_t nkeys;
    int32_t key_type[WELD_MAX_KEY_FIELDS];
    int32_t nvals;
    int32_t val_type[WELD_MAX_VAL_FIELDS];
    int64_t capacity;
    int64_t length;   /* vecmerger only */
    const void* init; /* vecmerger only */
} weld_builder_spec_t;

typedef enum { WELD_MODE_FUSED = 0, WELD_MODE_UNFUSED = 1 } weld_mode_t;

/* Tuning knobs; 0 always means "library default".  They select among kernel
 * variants that all return the same result. */
typedef struct {
    int32_t block_threads;   /* work-group size: 64..1024, multiple of 64            */
    int32_t units_per_thread;/* 128-bit load groups in flight per lane and column    */
    int32_t grid_blocks;     /* work-groups of the loop kernel; 0: as many as are resident at
                                once, fewer for loops that only stream columns through light
                                arithmetic (about 56 KB of loads in flight per compute unit),
                                48 per unit for register-only loops with division, roots or
                                transcendentals; weld_tune_launch measures it instead */
    int32_t dict_strategy;   /* 0 auto, 1 register slots, 2 LDS hash table, 3 global only,
                                4 per-lane LDS slots                                */
    int32_t lds_dict_slots;  /* slots of the per-block LDS hash table (power of two) */
    int32_t spin_limit;      /* polls a tile waits for its predecessors before the call
                                fails with WELD_ERR_DEVICE (the wait is always bounded)  */
    int32_t vecmerger_strategy; /* 0 auto, 1 per-lane register copies (length <= 8), 2 work-group
                                   copy in LDS updated with LDS atomics, 3 global atomics only,
                                   4 LDS copies of 8192-cell ranges, each range scanning all rows,
                                   5 merges queued by range of cells in device memory (workspace: 2 bytes
                                   per row where the merged value is a constant, else 10) and merged range by
                                   range in LDS by a second kernel (lengths from 8193 to 2^26; one vecmerger
                                   per loop, the others then use 3; a segment that is full sends its merges
                                   to the result with device atomics; up to 2^25 cells (2^24 where entries
                                   carry a value) a tile's entries are sorted by range in LDS and stored as
                                   runs),
                                   6 = 5 without that sort, -1 = auto without 5 */
    int32_t lds_filter_words;   /* admission filter in front of an LDS hash table that is smaller than
                                   the key set: 32-bit words of its bitmap (power of two); -1 = none */
    int32_t dict_spill;         /* merges that miss such an LDS table: -1 = device atomics on the global
                                   table; otherwise they are appended to key-partitioned queues that a
                                   second kernel aggregates in LDS (> 0: entries per queue segment,
                                   0 = sized for the case that every row misses; a full segment
                                   sends its merges to the global table)                            */
    int32_t merge_loop;         /* merges into builders that live in memory (LDS / global hash tables,
                                   vecmergers) of the rows a lane holds per tile: 1 = one loop over the
                                   rows (the merge code exists once), -1 = unrolled per row, 0 = library's
                                   choice                                                            */
    int32_t dict_defer;         /* LDS hash table in a loop that also compacts: 0 = merges that the first
                                   probe does not settle are queued per wavefront and handled 64 at a
                                   time, -1 = every merge walks the whole path where it stands      */
    int32_t dict_compact;       /* LDS hash table of a dictmerger[K,V,+] whose key provably fits 32 bits and
                                   whose one value is a constant or a 32-bit integer: 0 = 8-byte cells (32-bit
                                   key, 32-bit partial sum: twice the slots) and 8-byte queue entries,
                                   -1 = the general 64-bit cells                                    */
    int32_t device_math;        /* exp and log of the body: 0 = the library's own (tables and polynomials, about a
                                   third of the instructions), -1 = the device math library's          */
    int32_t tile_pipeline;      /* loops that compact (a vecbuilder under a predicate) and merge into memory:
                                   1 = the next tile's columns are loaded into registers while this tile is
                                   merged and stored, -1 = one tile at a time, 0 = library's choice (on when
                                   those columns, the tile's gathered values and the first probes take a
                                   lane at most about 80 registers)                                  */
    int32_t single_launch;      /* loops whose builders are all mergers: 0 = one launch per call (the work-group
                                   that finishes last combines the work-groups' partial results in index order
                                   and writes the results and the status words itself), -1 = a fill kernel
                                   before and a combining kernel behind the loop kernel                */
} weld_tuning_t;

typedef struct {
    void* stream;         /* hipStream_t the work is enqueued on (NULL = default stream)      */
    int32_t mode;         /* weld_mode_t                                                      */
    int32_t flags;        /* reserved, 0                                                      */
    int64_t memory_limit; /* bytes the call may hold in device memory (results + workspace);
                             0 = unlimited.  Sec. 4.3: Evaluate takes a memory limit.         */
    weld_tuning_t tune;
} weld_conf_t;

typedef struct {
    int32_t count;
    const weld_builder_spec_t* spec; /* host array, result order = this order */
    weld_conf_t conf;
} weld_builder_t;

/* paper layout of vec[T] (Sec. 4.2): ptr is a DEVICE pointer owned by the library */
typedef struct { int64_t len; void* ptr; } weld_vec_t;
/* a dictionary result: entry i is (keys[i], values[i]); packed structs; unordered */
typedef struct { weld_vec_t keys; weld_vec_t values; } weld_dict_t;

/* a groupbuilder result, dict[K, vec[V]] in compressed form: group g has key keys[g] (packed
 * struct) and the values values[offsets[g] .. offsets[g+1]); offsets holds keys.len + 1 int64;
 * groups are unordered */
typedef struct { weld_vec_t keys; weld_vec_t offsets; weld_vec_t values; } weld_groups_t;

typedef struct weld_result weld_result_t; /* opaque (the paper's WeldResult handle, Sec. 4.1) */

/*
 * weld_fused_for -- run `result(for(cols, builders, body))` over rows 0..n-1.
 * Sec. 3.2 (for + builders), Sec. 4.1 (Evaluate returns a handle that can be checked
 * for failure or queried for a pointer to the data), Sec. 4.3 (ownership, memory limit).
 *
 *  cols    : host struct; each column a device pointer to n elements of its type
 *  n       : number of rows, >= 0 (0 is legal: every builder returns its empty result)
 *  body    : host struct; validated (types, operand order, linearity) before any launch
 *  builder : host struct; builders + configuration
 *  out     : receives a new handle on WELD_OK, NULL otherwise
 * Returns WELD_OK after the kernels are ENQUEUED on conf.stream; they may still be
 * running.  The input columns must stay alive and unmodified until
 * weld_result_status() has returned.  Thread-compatible, not thread-safe.
 */
weld_status_t weld_fused_for(const weld_cols_t* cols, int64_t n, const weld_body_t* body,
                             const weld_builder_t* builder, weld_result_t** out);

/*
 * Launch-shape tuning (beyond the paper: its CPU backend sizes its task grain itself, Sec. 5).
 * Runs the loop over the given columns a few times for each of several persistent-grid sizes
 * (the library's own choice first, then 1..64 work-groups per compute unit), times the loop
 * kernel with HIP events, and returns builder->conf.tune with grid_blocks set to the fastest
 * in *best (unchanged fields are kept; another grid replaces the library's choice only if it is
 * more than 2.5 % faster: below that, runs of one grid differ as much).  best_ms / default_ms (may be NULL): loop-kernel milliseconds of the
 * winner and of the library's choice.  The results of the runs are discarded.  Synchronous;
 * fused mode only; arguments as for weld_fused_for.  How many work-groups a streaming loop wants
 * in flight depends on its mix of loads and arithmetic, which the kernel's resource use does not
 * tell; a host program that runs a loop many times asks once and passes the record on.
 */
weld_status_t weld_tune_launch(const weld_cols_t* cols, int64_t n, const weld_body_t* body,
                               const weld_builder_t* builder, weld_tuning_t* best, float* best_ms,
                               float* default_ms);

/*
 * Dictionaries built by earlier calls as inputs of a loop: the probe side of a hash join
 * (Sec. 3.1: dictionaries are the data type joins are implemented with).  The body may use
 *   WELD_OP_KEYEXISTS : a = index into `dicts`, b (and c) = the key struct's fields; bool
 *   WELD_OP_DICTLOOKUP: same operands, reserved = index of a value field; the field of that
 *                       key's value struct, 0 if the key is absent
 * on dictionaries of one or two key fields.  Each dictionary is the result of a dictmerger of
 * an earlier weld_fused_for call: that call must have been enqueued on the same stream (or
 * have finished), its handle must stay alive until this call's weld_result_status() has
 * returned, and a build that failed (capacity) leaves a partial dictionary.  Fused mode only.
 */
enum { WELD_OP_KEYEXISTS = 29, WELD_OP_DICTLOOKUP = 30 };
typedef struct {
    weld_result_t* result; /* handle of the call that built the dictionary  */
    int32_t builder;       /* index of a dictmerger among that call's builders */
} weld_dict_ref_t;
#define WELD_MAX_DICT_INPUTS 4
weld_status_t weld_fused_for_probe(const weld_cols_t* cols, int64_t n, const weld_dict_ref_t* dicts, int32_t ndicts,
                                   const weld_body_t* body, const weld_builder_t* builder, weld_result_t** out);

/*
 * A scalar defined outside the loop as an operand of its body (Sec. 3.2: a loop's function is a
 * closure over the values in scope; Sec. 4.1: objects depend on other objects' results):
 *   WELD_OP_SCALAR : a = column index.  That entry of the column list points at ONE element of
 *                    its type in DEVICE memory, and every row reads that same value.
 * The typical scalar is the merger result of an earlier call on the same stream
 * (weld_result_data of that handle): it is read in stream order by the loop's kernel, so no host
 * copy and no wait lies between the two loops.  A column is read either by WELD_OP_COL or by
 * WELD_OP_SCALAR, not both; its pointer must be valid even when n is 0; it is accepted by
 * weld_fused_for (both modes), weld_fused_for_probe and weld_fused_for_static, not in the bodies of
 * weld_nested_for.
 */
enum { WELD_OP_SCALAR = 31 };

/* The DEVICE address of merger result idx, returned WITHOUT waiting for the call's work: what a
 * later loop on the same stream passes as the column that WELD_OP_SCALAR reads.  The handle must
 * stay alive until that later call's weld_result_status() has returned.  NULL if idx is not a
 * merger of this call. */
const void* weld_result_scalar(const weld_result_t* r, int32_t idx);

/*
 * weld_fused_for_static -- weld_fused_for for callers that cannot allocate device memory: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  It calls no
 * hipMalloc, hipFree, hipHostMalloc, event or module routine: the results go to buffers the CALLER
 * passes, and the workspace (control words, merger partials, scan descriptors, hash tables, spill
 * queues) is one fixed buffer of WELD_STATIC_SCRATCH_BYTES that the library holds on every GPU it
 * runs on until the process ends (its first 4 KiB are the arrival words of kernels that finish
 * their call themselves, see weld_tuning_t.single_launch; they are zero between calls).
 *
 *  cols, n, body, builder : as for weld_fused_for.  Fused mode only; merger, vecbuilder,
 *           dictmerger and vecmerger (a groupbuilder's workspace grows with n: WELD_ERR_UNSUPPORTED).
 *           conf.memory_limit is ignored: the limit is the fixed buffer.
 *  outs   : host array, one entry per builder, 16-byte aligned DEVICE buffers owned by the caller:
 *             merger     data = 8 bytes (the scalar is stored in its own type at offset 0)
 *             vecbuilder data = room for `capacity` >= n elements (a filter's selectivity is not
 *                        known in advance; what lies beyond the returned length is unspecified)
 *             vecmerger  data = room for `capacity` >= length 8-byte cells
 *             dictmerger data = packed key structs, data2 = packed value structs, room for
 *                        `capacity` >= the builder's capacity entries each; unordered
 *  status_dev : DEVICE array of 1 + WELD_MAX_BUILDERS int64 written behind the call's kernels:
 *           [0] = 0 or error bits (1: more distinct keys than a dictmerger's capacity, 2: a tile gave
 *           up its bounded wait, 4: vecmerger index out of range); [1 + b] = elements of builder b
 *           (merger 1, vecbuilder / vecmerger length, dictmerger entries).
 * The call only enqueues on conf.stream; the caller waits for the stream and reads status_dev.
 *
 * Errors: WELD_ERR_NOT_READY when this loop has no loaded kernel yet -- compiling and loading one
 * allocates, so run the same loop (body, builders, tuning, 16-byte alignment of the columns) once
 * through weld_fused_for beforehand; WELD_ERR_OOM when the workspace exceeds the fixed buffer (a
 * dictmerger of more than about 5e5 keys and one value field, or more than about 4e6 tiles of a
 * filter; spill queues shrink to what is left and full ones fall back to device atomics, so large
 * dictionaries get slower, not wrong); WELD_ERR_INVALID_ARG for a missing or too small output.
 * The first call on a device fetches the buffer's address (set-up, once per device; do it outside a
 * capture).  Every call on a GPU shares that GPU's one buffer: calls on one stream are ordered and
 * safe, calls that overlap on different streams or host threads RACE -- the caller serialises them.
 */
#define WELD_STATIC_SCRATCH_BYTES (32ll << 20)
typedef struct {
    void* data;       /* device */
    void* data2;      /* device; dictmerger values, NULL otherwise */
    int64_t capacity; /* elements / entries the buffers have room for */
} weld_out_t;
weld_status_t weld_fused_for_static(const weld_cols_t* cols, int64_t n, const weld_body_t* body,
                                    const weld_builder_t* builder, const weld_out_t* outs, int64_t* status_dev);

/* Evaluation point: waits for the call's work, reads back lengths and kernel-side error
 * flags.  WELD_OK, WELD_ERR_CAPACITY or WELD_ERR_DEVICE.  Idempotent. */
weld_status_t weld_result_status(weld_result_t* r);

/* Human-readable text of the last error on this handle ("" if none).  Never NULL
 * for a non-NULL handle; owned by the handle. */
const char* weld_result_error(const weld_result_t* r);

/* Pointer to builder `idx`'s result (Sec. 4.1: "queried for a pointer to the
 * returned data").  Calls weld_result_status() first; NULL on any error.
 *   merger     -> DEVICE pointer to one scalar of its type (8-byte aligned)
 *   vecbuilder, vecmerger -> HOST pointer to a weld_vec_t  (ptr inside is a device pointer)
 *   dictmerger -> HOST pointer to a weld_dict_t (device pointers inside)
 *   groupbuilder -> HOST pointer to a weld_groups_t (device pointers inside)
 * Valid until weld_result_free(). */
const void* weld_result_data(weld_result_t* r, int32_t idx);

/* Convenience for callers without a HIP runtime of their own: copy `bytes` bytes of
 * builder idx's payload, starting at byte `offset`, to `dst`.
 *   part 0: merger scalar / vecbuilder elements / dictmerger or groupbuilder keys;
 *   part 1: dictmerger values / groupbuilder offsets;  part 2: groupbuilder values.
 *   dst_is_device != 0: dst is a device pointer (copy stays on the GPU). */
weld_status_t weld_result_fetch(weld_result_t* r, int32_t idx, int32_t part, void* dst,
                                int64_t offset, int64_t bytes, int32_t dst_is_device);

/* Milliseconds between the first and last kernel of the call, from HIP events recorded
 * on conf.stream around the enqueued work (valid after weld_result_status()). */
weld_status_t weld_result_elapsed_ms(weld_result_t* r, float* ms);

/* Milliseconds the GPU was busy with the call: in unfused mode the sum, over the operator loops, of the
 * time between each loop's first and last kernel - without the host waits between the loops (a filter's
 * length is read back before the next loop is sized); in fused mode the same as weld_result_elapsed_ms. */
weld_status_t weld_result_busy_ms(weld_result_t* r, float* ms);

/* Same, for the main loop kernel alone (fused mode; -1 if the call ran none). */
weld_status_t weld_result_kernel_ms(weld_result_t* r, float* ms);

/* Name of the main loop kernel as profilers show it ("" in unfused mode); owned by the handle. */
const char* weld_result_kernel_name(const weld_result_t* r);

/* Number of kernels the call launched (1-2 in fused mode, one per operator unfused). */
int32_t weld_result_kernel_count(const weld_result_t* r);

/* Work-groups of the main loop kernel (fused mode; 0 if the call ran none). */
int64_t weld_result_grid(const weld_result_t* r);

/* Frees the results and returns workspace to the library's pool (Sec. 4.1 FreeWeldResult).
 * NULL is allowed. */
void weld_result_free(weld_result_t* r);

/* Compile (or load from the on-disk cache) the fused kernel for this loop without
 * running it and without touching a GPU; used to build kernels ahead of time.
 * col_types: ncols weld_type_t values. */
weld_status_t weld_precompile(const int32_t* col_types, int32_t ncols, const weld_body_t* body,
                              const weld_builder_t* builder);

/* Directory for compiled code objects (created if missing).  NULL/"" disables the
 * disk cache.  Default: $WELD_HIP_CACHE_DIR, else "kcache" next to the library. */
weld_status_t weld_set_cache_dir(const char* path);

/* Validation only (no GPU needed): the status weld_fused_for would return before
 * planning.  err/errlen: optional buffer for the message. */
weld_status_t weld_validate(const int32_t* col_types, int32_t ncols, const weld_body_t* body,
                            const weld_builder_t* builder, char* err, size_t errlen);

/* The HIP source the runtime compiler is given for this loop (for inspection);
 * returns bytes needed including the terminator, copies at most buflen. */
int64_t weld_generated_source(const int32_t* col_types, int32_t ncols, const weld_body_t* body,
                              const weld_builder_t* builder, char* buf, int64_t buflen);

/* Release every cached device allocation of the pool back to the device. */
void weld_pool_trim(void);
/* Bytes currently held by the pool (in use + cached). */
int64_t weld_pool_bytes(void);

/* Text of the last error of a call that returned no handle (thread-local). */
const char* weld_last_error(void);

/* Streaming-read probe: sums `bytes` bytes at `data` (device, 16-byte aligned) with
 * 128-bit loads; used to measure the attainable HBM read rate on the box.
 * Writes a 64-bit checksum to *checksum_dev (device pointer). */
weld_status_t weld_probe_read(const void* data, int64_t bytes, void* checksum_dev, void* stream);
/* Plain copy kernel of known size (device to device, one 16-byte vector per thread), used to scale the HBM
 * counters and as the box's ceiling for a stream of as many bytes written as read. */
weld_status_t weld_probe_copy(void* dst, const void* src, int64_t bytes, void* stream);

const char* weld_version(void);

#ifdef __cplusplus
}
#endif
#endif /* WELD_HIP_H */
