// Host-callable launchers of the ahead-of-time compiled helper kernels.
#pragma once

#include <hip/hip_runtime_api.h>

#include <cstdint>

namespace weld {

struct DictLayout {
    int nkeys;
    int key_size[4];
    int key_shift[4];
    int key_stride;
    int nvals;
    int val_size[8];
    int val_stride;
};
struct DictValues {
    const unsigned long long* p[8];
};

// One entry per merger of a call: combine `count` 8-byte partials with `func` in index
// order and store the result, narrowed to `elem_size` bytes for integer types.
struct MergerFinish {
    int n;
    const unsigned long long* partial[8];
    void* result[8];
    int func[8];
    int is_f64[8];
    int elem_size[8];
    int bits[8];
};
hipError_t launch_merger_finish(const MergerFinish& m, int count, hipStream_t stream);

hipError_t launch_fill64(void* p, int64_t count, uint64_t value, hipStream_t stream);
// Several fills in one launch (the workspace of a call: control words, scan descriptors, the
// keys and value columns of a dictionary table ...).
struct FillList {
    int n = 0;
    void* p[16];
    long long count[16];
    unsigned long long value[16];
    bool add(void* ptr, int64_t cnt, uint64_t val) {
        if (cnt <= 0) return true;
        if (n == 16) return false;
        p[n] = ptr; count[n] = cnt; value[n] = val; ++n;
        return true;
    }
};
// start / stop (may be null): events that take the dispatch's own start / end time (no packet of their own in the queue)
hipError_t launch_fill_list(const FillList& f, hipStream_t stream, hipEvent_t start = nullptr);
// slot_pos (may be null): receives, for every occupied slot (and the extra slot `slots`), the
// position its entry was written to.  skip_if (may be null): the kernel does nothing when *skip_if != 0
// (the entries were packed by the kernels that built the table).
hipError_t launch_dict_extract(const void* keys, const void* hdr, int64_t slots, const DictValues& vals,
                               const DictLayout& lay, int64_t capacity, void* out_keys, void* out_vals,
                               void* count, void* err, int* slot_pos, unsigned long long* kp32, unsigned int* kwide,
                               const unsigned int* skip_if, hipStream_t stream);

// groupbuilder, second half.  The loop kernel has counted the pairs of every key in a
// dictionary (extracted into `counts`, one int64 per group, *ngroups of them) and compacted
// the pairs' key fields and values into vectors of *npairs elements.
//   group_offsets: offsets[g] = sum of counts[0..g), offsets[ngroups] = total; cursor[g] = 0.
//   group_scatter: value j goes to values_out[offsets[g] + position], g = the group of its
//                  key (found through the dictionary's table and slot_pos), position handed
//                  out per group: per tile of pairs an LDS table counts the pairs of each group
//                  and one device atomic per (tile, group) reserves their places.
struct GroupScatter {
    const unsigned long long* npairs;      // device
    int nkeys;
    const void* key[4];
    int key_size[4];
    int key_shift[4];
    int key_sext32;                        // the one key field holds the low half of a 64-bit key (its sign extension is the key)
    const void* value;
    int value_size;
    const unsigned long long* table_keys;
    const unsigned int* hdr;
    long long slots;
    const int* slot_pos;
    // for every slot (and the extra one) low half = low half of its key, high half = its group number, -1 where the
    // slot is free; *kwide != 0: some key is not the sign extension of its low half (then slot_pos and table_keys serve)
    const unsigned long long* kp32;
    const unsigned int* kwide;
    long long capacity;
    const long long* offsets;
    unsigned long long* cursor;
    void* values_out;
    // two-pass form (many groups): the pairs are first partitioned by ranges of 2^log_bucket groups
    const unsigned long long* ngroups;     // device
    int log_bucket;
    int nbuckets;                          // <= 256
    unsigned long long* bcursor;           // one per bucket, zero on entry
    unsigned short* tmp_group;             // group of each partitioned pair, counted from its range's first
    unsigned long long* tmp_value;         // its value (bits)
};
// desc: one zeroed 8-byte word per 8192 groups of the capacity; err: the call's error word; max_blocks: work-groups resident at once
hipError_t launch_group_offsets(const void* counts, const void* ngroups, int64_t capacity, void* offsets, void* cursor,
                                void* desc, void* err, int max_blocks, hipStream_t stream);
hipError_t launch_group_scatter(const GroupScatter& g, int blocks, hipStream_t stream);
// The same in two kernels for dictionaries of many groups: partition the pairs by group range,
// then place every range's pairs (both read g.ngroups and the offsets on the device).
hipError_t launch_group_partition(const GroupScatter& g, int blocks, hipStream_t stream);
hipError_t launch_group_place(const GroupScatter& g, int blocks, hipStream_t stream);
// A vecmerger whose merges the loop kernel queued by range of 2^shift cells (spill_kernels.hip): work-group g of the
// loop kernel appended to segment [g][range] of `log` (cap entries, a multiple of 8, of entry_bytes: 2 = the cell within
// its range, the merged value being the constant const_bits; 10 = a segment is cap values of 8 bytes followed by cap
// cells of 2 bytes) and stored the segment lengths
// in qcnt[g * ranges + range].  One work-group per range merges the range's entries in LDS and combines the cells
// that were touched into out[range << shift ...] (it owns them: plain loads and stores).
struct VecmRanges {
    const void* log;
    const unsigned int* qcnt;
    int groups;
    int ranges;
    int shift;                 // <= 13
    long long cap;
    long long length;
    int func;                  // weld_func_t
    int is_f64;
    unsigned long long ident;
    int entry_bytes;
    int long_segments;         // 2-byte entries: segments of about a thousand entries and more are expected (read with 16-byte loads)
    unsigned long long const_bits;
    unsigned long long* out;
};
hipError_t launch_vecm_ranges(const VecmRanges& v, hipStream_t stream, hipEvent_t stop = nullptr);

// Aggregation of the key-partitioned spill queues of a large dictmerger (spill_kernels.hip).
// The loop kernel's work-group g appends to segment [g][partition] of `log` (cap entries of
// 1 + nvals 8-byte words each) and stores the segment lengths in qcnt[g * kSpillParts + partition].
constexpr int kSpillParts = 256;
struct SpillMerge {
    const unsigned long long* log;
    const unsigned int* qcnt;
    int groups;                    // work-groups of the loop kernel, <= 1024
    long long cap;
    int func;
    int is_f64[8];
    unsigned long long ident[8];
    unsigned long long* keys;      // the global table the loop kernel uses
    unsigned int* hdr;
    long long slots;
    unsigned long long* vals[8];
    int* err;
    // slice mode (launch_dict_slice_build): `parts` partitions = slices of the global table
    int parts;
    unsigned long long* overflow;        // entries (1 + nvals words) that found no room in their slice
    unsigned int* overflow_count;        // zero on entry
    long long overflow_cap;
    // 0: entries are 1 + nvals words; 1 / 2: one word per entry, low half = the key (zero- / sign-extended
    // to the packed 64-bit key), high half = the value, a signed 32-bit partial sum (nvals == 1, func = add)
    int compact;
    long long capacity;            // the dictmerger's declared capacity (sizes the aggregation's LDS tables)
    int table_slots, split;        // set by launch_dict_spill_merge
    // slice mode, pack != 0: a slice that starts from an empty table (no loop kernel inserted directly) also
    // writes its entries to the result's packed arrays while it has them in LDS, the entries of the list
    // follow, and *packed (zero on entry) is set: the extraction kernel behind then has nothing to do
    // (it would read the whole table again: 512 MiB for 2^25 slots)
    int pack;
    DictLayout lay;
    unsigned char* out_keys;
    unsigned char* out_vals;
    unsigned long long* out_count; // entries written so far (zero on entry)
    unsigned int* packed;
};
hipError_t launch_dict_spill_merge(const SpillMerge& a, int nvals, hipStream_t stream, hipEvent_t stop = nullptr);
// Dictionaries of millions of keys: partition p of the queues holds the keys whose home slot lies in
// the p-th of `parts` equal slices of the global table (slice = as many slots as an LDS table of this
// entry size has).  One work-group per slice loads the slice, merges the partition into it in LDS
// and stores it back; the few entries that probe past the end of their slice are inserted into
// the global table by a second small kernel afterwards.  a.slots == a.parts * slice slots.
hipError_t launch_dict_slice_build(const SpillMerge& a, int nvals, hipStream_t stream, hipEvent_t stop = nullptr);

// Nested loops.  is64: the start / end vectors hold 64-bit (else 32-bit) integers.
// segments_check raises bit 8 of *err unless start[0] == 0, start[i] <= end[i],
// end[i] == start[i+1] and end[n_outer-1] == n_inner.  tile_rows writes, for every tile t of
// `tile` inner elements, the last outer element whose range starts at or before the tile's
// first inner element (tile_row[ntiles] = n_outer - 1).  or_error ORs the error word of an
// earlier step's control block into a later one's.
hipError_t launch_segments_check(const void* start, const void* end, int is64, int64_t n_outer, int64_t n_inner,
                                 void* err, hipStream_t stream);
// ranges_offsets: offsets[i] = number of inner elements the outer elements before i visit (start, start +
// stride, ... below end; stride null = 1), offsets[n_outer] = *total = all of them; bit 8 of *err for a
// negative start, end < start, end > n_inner or stride < 1.  One work-group.
hipError_t launch_ranges_offsets(const void* start, const void* end, const void* stride, int is64, int64_t n_outer,
                                 int64_t n_inner, void* offsets, void* total, void* err, hipStream_t stream);
hipError_t launch_tile_rows(const void* start, int is64, int64_t n_outer, int64_t tile, int64_t ntiles,
                            void* tile_row, hipStream_t stream);
hipError_t launch_or_error(void* dst_ctl, const void* src_ctl, hipStream_t stream);
// 64 control words to pinned host memory; `done` (may be null) takes the dispatch's end time and is what the host waits for
hipError_t launch_ctl_to_host(const void* ctl, void* host, hipStream_t stream, hipEvent_t done);

// weld_fused_for_static (static_entry.hip): copies the error bits and the builders' lengths from a
// call's control block to the caller's device array (status[0] = error bits, status[1 + b] = length
// of builder b: known[b] if that is >= 0, else the count word the kernels left in the block).
struct StaticLengths {
    int count;
    long long known[8];
};
hipError_t launch_static_status(const void* ctl, const StaticLengths& lens, int64_t* status_dev, hipStream_t stream);

hipError_t launch_probe_read(const void* data, int64_t bytes, void* checksum, int blocks, hipStream_t stream);
hipError_t launch_probe_copy(void* dst, const void* src, int64_t bytes, hipStream_t stream);

}  // namespace weld
