// Second half of the large-dictionary path (dictmerger, Table 1 of the paper): merges that
// found no room in a work-group's LDS table were appended by the loop kernel to
// key-partitioned queues (segment [group][partition], `cap` entries of 1 + NV words:
// packed key, then one 8-byte cell per value field).  Here one 1024-thread work-group
// per partition aggregates its partition in an LDS hash table and then adds the table to
// the global one.  A partition holds about keys / 256 distinct keys, so its table fits LDS
// where the whole key set did not, and the random-address device atomics of the direct
// path (23.7 G/s on this part, the bound of that path) shrink to one per distinct key.
//
// The hash functions and the global-table insert are the ones of the loop kernels: both
// write the same table.
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>

#define W_BLOCK 1024
#define W_V 2
#define W_U 1
#define W_ALIGNED 1
#include "fused_prelude.hip.h"

#include "aot_kernels.h"

namespace weld {

// largest power of two with slots * 8 * (1 + NV) <= 128 KiB
template <int NV> struct SpillTable {
    static constexpr int kSlots = NV <= 1 ? 8192 : NV <= 3 ? 4096 : NV <= 7 ? 2048 : 1024;
    static constexpr int kBatch = NV <= 1 ? 4 : NV <= 3 ? 2 : 1;   // entries a thread holds in registers, twice
};

// One field of a packed key or value struct: a single store of the field's width where the address is
// aligned to it, byte by byte otherwise.
__device__ __forceinline__ void pack_field(unsigned char* p, u64 bits, int size) {
    if (size == 8 && ((uintptr_t)p & 7) == 0) *(u64*)p = bits;
    else if (size == 4 && ((uintptr_t)p & 3) == 0) *(u32*)p = (u32)bits;
    else
        for (int b = 0; b < size; ++b) p[b] = (unsigned char)(bits >> (8 * b));
}
// entry `pos` of the packed result arrays
template <int NV>
__device__ __forceinline__ void pack_entry(const SpillMerge& a, i64 pos, u64 key, const u64 (&v)[NV]) {
    unsigned char* ko = a.out_keys + pos * a.lay.key_stride;
    int off = 0;
    for (int k = 0; k < a.lay.nkeys; ++k) {
        pack_field(ko + off, key >> a.lay.key_shift[k], a.lay.key_size[k]);
        off += a.lay.key_size[k];
    }
    unsigned char* vo = a.out_vals + pos * a.lay.val_stride;
    off = 0;
#pragma unroll
    for (int k = 0; k < NV; ++k) {
        pack_field(vo + off, v[k], a.lay.val_size[k]);
        off += a.lay.val_size[k];
    }
}

// One value cell: the bits are an i64 or a double, FUNC is the dictmerger's merge function.
template <int FUNC> __device__ __forceinline__ void cell_combine(u64* p, u64 bits, int is_f64, const int agent) {
    if (is_f64) {
        double v;
        __builtin_memcpy(&v, &bits, 8);
        w_atomic<FUNC>(reinterpret_cast<double*>(p), v, agent);
    } else {
        w_atomic<FUNC>(reinterpret_cast<i64*>(p), (i64)bits, agent);
    }
}

// w_lds_slot with a probe loop that stays a loop (32 unrolled probes per call site made the
// kernel larger than the instruction cache)
__device__ __forceinline__ int lds_slot_looped(u64* keys, int slots, u64 kbits, int max_probe) {
    if (kbits == W_EMPTY_KEY) return -1;
    const int mask = slots - 1;
    int s = (int)w_hash_slot(kbits, (u32)slots);
#pragma unroll 1
    for (int probe = 0; probe < max_probe; ++probe) {
        u64 cur = __hip_atomic_load(keys + s, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        if (cur == kbits) return s;
        if (cur == W_EMPTY_KEY) {
            u64 expect = W_EMPTY_KEY;
            if (__hip_atomic_compare_exchange_strong(keys + s, &expect, kbits, __ATOMIC_RELAXED,
                                                     __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP))
                return s;
            if (expect == kbits) return s;
        }
        s = (s + 1) & mask;
    }
    return -1;
}

// COMPACT (NV == 1, FUNC == add): an entry is ONE word, low half the key (1: zero-extended, 2: sign-extended
// to the packed key), high half a signed 32-bit partial sum.
// The LDS table has a.table_slots slots (a power of two, sized by the host from the dictionary's
// capacity: a partition holds about 1/256 of the keys) and lies in dynamic LDS; a.split work-groups
// share a partition's entries, each with a table of its own, so that a dictionary of few keys per
// partition has two work-groups per compute unit at work instead of one.
template <int NV, int FUNC, int COMPACT = 0>
__global__ void __launch_bounds__(1024) dict_spill_merge_kernel(const SpillMerge a) {
    extern __shared__ u64 s_dyn[];
    const int S = a.table_slots;
    u64* const s_keys = s_dyn;
    u64* s_vals[NV];
#pragma unroll
    for (int k = 0; k < NV; ++k) s_vals[k] = s_dyn + (size_t)S * (1 + k);
    __shared__ u32 s_off[1025];
    __shared__ u32 s_wave[16];
    const int part = blockIdx.x / a.split;
    const int sub = blockIdx.x % a.split;
    const int tid = threadIdx.x;
    for (int q = tid; q < S; q += 1024) {
        s_keys[q] = W_EMPTY_KEY;
#pragma unroll
        for (int k = 0; k < NV; ++k) s_vals[k][q] = a.ident[k];
    }
    // exclusive prefix of the segment lengths of this partition over the groups (<= 1024)
    u32 mine = 0;
    if (tid < a.groups) {
        mine = a.qcnt[(size_t)tid * kSpillParts + part];
        if ((i64)mine > a.cap) mine = (u32)a.cap;
    }
    u32 incl = mine;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const u32 o = __shfl_up(incl, off, 64);
        if ((tid & 63) >= off) incl += o;
    }
    if ((tid & 63) == 63) s_wave[tid >> 6] = incl;
    __syncthreads();
    u32 before = 0;
    for (int w = 0; w < (tid >> 6); ++w) before += s_wave[w];
    s_off[tid + 1] = before + incl;
    if (tid == 0) s_off[0] = 0;
    __syncthreads();
    const u32 total = s_off[a.groups];
    const float guess = total ? (float)a.groups / (float)total : 0.f;

    // adds one entry to the global table: for what the LDS table cannot take, and for the
    // LDS table's own contents at the end
    auto to_global = [&](u64 key, const u64 (&w)[NV]) {
        const i64 g = w_table_slot(a.keys, a.hdr, a.slots, key, a.err);
        if (g >= 0) {
#pragma unroll
            for (int f = 0; f < NV; ++f) cell_combine<FUNC>(a.vals[f] + g, w[f], a.is_f64[f], 1);
        }
    };

    // ENT entries per thread and round, entry j of thread t at i0 + j * 1024 + t: the lanes of
    // a wavefront read neighbouring entries (one contiguous span per load when an entry is 16
    // bytes).  The loads of the next round are issued before the entries of this round are
    // merged, so the merges hide their latency.
    constexpr int ENT = SpillTable<NV>::kBatch;
    constexpr int WORDS = COMPACT ? 1 : 1 + NV;
    typedef u64 u64x2 __attribute__((ext_vector_type(2)));
    u64 kcur[ENT], knext[ENT];
    u64 vcur[ENT][NV], vnext[ENT][NV];
    auto fetch = [&](u32 i0, u64 (&k)[ENT], u64 (&w)[ENT][NV]) {
#pragma unroll
        for (int j = 0; j < ENT; ++j) {
            const u32 i = i0 + (u32)j * 1024u + (u32)tid;
            if (i < total) {
                // the segment of entry i: segments of one partition are about equally long, so
                // start from the proportional guess and walk (s_off[lo] <= i < s_off[lo + 1])
                // (the guess is a float product, not a 64-bit division per entry)
                int lo = (int)((float)i * guess);
                lo = lo < 0 ? 0 : (lo >= a.groups ? a.groups - 1 : lo);
                while (s_off[lo] > i) --lo;
                while (s_off[lo + 1] <= i) ++lo;
                const u64* e = a.log + (((size_t)lo * kSpillParts + part) * (size_t)a.cap + (i - s_off[lo])) * WORDS;
                u64 buf[WORDS];
                if (WORDS % 2 == 0) {               // entries are 16-byte aligned
                    const u64x2* e2 = reinterpret_cast<const u64x2*>(e);
#pragma unroll
                    for (int q = 0; q < WORDS / 2; ++q) {
                        const u64x2 t = e2[q];
                        buf[2 * q] = t.x;
                        buf[2 * q + 1] = t.y;
                    }
                } else {
#pragma unroll
                    for (int q = 0; q < WORDS; ++q) buf[q] = e[q];
                }
                if (COMPACT) {
                    // the word is taken apart where it is used: arithmetic on it here would make this
                    // load wait for its data on the spot, one load after the other (76 -> 63 us on C5)
                    k[j] = buf[0];
                    w[j][0] = 0;
                } else {
                    k[j] = buf[0];
#pragma unroll
                    for (int f = 0; f < NV; ++f) w[j][f] = buf[1 + f];
                }
            } else {
                k[j] = W_EMPTY_KEY;
#pragma unroll
                for (int f = 0; f < NV; ++f) w[j][f] = 0;
            }
        }
    };
    const u32 stride = 1024u * ENT * (u32)a.split;      // the partition's rounds are dealt to its work-groups in turn
    fetch((u32)sub * 1024u * ENT, kcur, vcur);
    for (u32 i0 = (u32)sub * 1024u * ENT; i0 < total; i0 += stride) {
        fetch(i0 + stride, knext, vnext);
        // first probe of all entries of the round side by side (one LDS latency instead of
        // one per entry); an entry whose first slot holds another key or nothing goes the
        // whole way (claim the free slot, or probe on)
        int sl[ENT];
        u64 first[ENT];
        if (COMPACT) {
#pragma unroll
            for (int j = 0; j < ENT; ++j) {
                const u64 word = kcur[j];
                const u32 lo = (u32)word;
                kcur[j] = COMPACT == 2 ? (u64)(i64)(int)lo : (u64)lo;
                vcur[j][0] = (u64)(i64)(int)(u32)(word >> 32);
            }
        }
#pragma unroll
        for (int j = 0; j < ENT; ++j) {
            sl[j] = (int)w_hash_slot(kcur[j], (u32)S);
            first[j] = __hip_atomic_load(s_keys + sl[j], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        }
#pragma unroll
        for (int j = 0; j < ENT; ++j) {
            const bool live = i0 + (u32)j * 1024u + (u32)tid < total;
            if (!live) sl[j] = -2;
            else if (first[j] != kcur[j] || kcur[j] == W_EMPTY_KEY) sl[j] = lds_slot_looped(s_keys, S, kcur[j], 32);
        }
#pragma unroll
        for (int j = 0; j < ENT; ++j) {
            if (sl[j] >= 0) {
#pragma unroll
                for (int f = 0; f < NV; ++f) cell_combine<FUNC>(&s_vals[f][sl[j]], vcur[j][f], a.is_f64[f], 0);
            } else if (sl[j] == -1) {
                // no room in this partition's table (or the one key equal to the free marker)
                to_global(kcur[j], vcur[j]);
            }
        }
#pragma unroll
        for (int j = 0; j < ENT; ++j) {
            kcur[j] = knext[j];
#pragma unroll
            for (int f = 0; f < NV; ++f) vcur[j][f] = vnext[j][f];
        }
    }
    __syncthreads();
    // occupied slots are few (a partition's distinct keys): list them first, so that the global
    // inserts - three dependent device-memory operations each - run side by side
    u32* const s_list = s_off;      // the prefix is not needed any more
    if (tid == 0) s_wave[0] = 0;
    __syncthreads();
    for (int q = tid; q < S; q += 1024) {
        if (s_keys[q] == W_EMPTY_KEY) continue;
        const u32 at = __hip_atomic_fetch_add(&s_wave[0], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        if (at < 1024) s_list[at] = (u32)q;
    }
    __syncthreads();
    const u32 occupied = s_wave[0];
    if (occupied <= 1024u) {
        if ((u32)tid < occupied) {
            const int q = (int)s_list[tid];
            u64 w[NV];
#pragma unroll
            for (int f = 0; f < NV; ++f) w[f] = s_vals[f][q];
            to_global(s_keys[q], w);
        }
    } else {                        // more than the list holds: every thread walks its slots
        for (int q = tid; q < S; q += 1024) {
            if (s_keys[q] == W_EMPTY_KEY) continue;
            u64 w[NV];
#pragma unroll
            for (int f = 0; f < NV; ++f) w[f] = s_vals[f][q];
            to_global(s_keys[q], w);
        }
    }
}

// ---------------------------------------------------------------- slices of the global table
// Dictionaries of millions of keys (the build side of a join): a partition's keys do not fit an
// LDS table, and every merge would be two device atomics at random addresses (23.7 G/s on this
// part: 1.3 ms for 1.5e7 keys).  Here the partitions ARE the table: partition p of the queues
// holds the keys whose home slot lies in slice p of the global table, a slice has as many slots
// as the LDS table of this entry size, and one work-group per slice loads the slice (it holds
// what loop kernels inserted directly when a queue segment was full), merges its partition into
// it with LDS atomics - linear probing as in the global table, but never past the end of the
// slice - and stores it back with plain coalesced stores.  What would probe past the end of
// its slice (and the one key equal to the free marker) goes to a short list that a second
// kernel inserts into the global table the usual way, after every slice is in place.
template <int NV, int FUNC>
__global__ void __launch_bounds__(1024) dict_slice_build_kernel(const SpillMerge a) {
    constexpr int S = SpillTable<NV>::kSlots;
    constexpr int WORDS = 1 + NV;
    __shared__ u64 s_keys[S];
    __shared__ u64 s_vals[NV][S];
    __shared__ u32 s_off[1025];
    __shared__ u32 s_wave[16];
    __shared__ unsigned short s_seg[4096];
    __shared__ u64 s_spare[128];           // where the merges of entries that are not there go: a key cell and a value cell per lane
    const int part = blockIdx.x;
    const int tid = threadIdx.x;
    const i64 base = (i64)part * S;
    // hdr[0] != 0: a loop kernel inserted into the global table directly (a queue segment was
    // full); otherwise the table is still as the fill kernel left it and need not be read
    const bool fresh = a.hdr[0] == 0;
    for (int q = tid; q < S; q += 1024) {
        s_keys[q] = fresh ? W_EMPTY_KEY : a.keys[base + q];
#pragma unroll
        for (int k = 0; k < NV; ++k) s_vals[k][q] = fresh ? a.ident[k] : a.vals[k][base + q];
    }
    u32 mine = 0;
    if (tid < a.groups) {
        mine = a.qcnt[(size_t)tid * a.parts + part];
        if ((i64)mine > a.cap) mine = (u32)a.cap;
    }
    u32 incl = mine;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const u32 o = __shfl_up(incl, off, 64);
        if ((tid & 63) >= off) incl += o;
    }
    if ((tid & 63) == 63) s_wave[tid >> 6] = incl;
    __syncthreads();
    u32 before = 0;
    for (int w = 0; w < (tid >> 6); ++w) before += s_wave[w];
    s_off[tid + 1] = before + incl;
    if (tid == 0) s_off[0] = 0;
    __syncthreads();
    const u32 total = s_off[a.groups];
    const u32 seg_lo = before + incl - mine, seg_hi = before + incl;        // this thread's segment among the partition's entries
    // 4096 entries a round, four per thread, all loaded before the first is merged.  Which segment an
    // entry lies in is written down by the segments' own threads first (a search through the offsets
    // by every entry - a guess and a walk of some thirty dependent LDS reads, the segments' lengths
    // being as uneven as they are - took a quarter of the kernel's time and slowed the merges of the
    // wavefronts that were already past it).
    for (u32 r0 = 0; r0 < total; r0 += 4096u) {
        if (r0) __syncthreads();               // the round before has read its segment numbers
        {
            const u32 lo = seg_lo > r0 ? seg_lo : r0, hi = seg_hi < r0 + 4096u ? seg_hi : r0 + 4096u;
            for (u32 i = lo; i < hi; ++i) s_seg[i - r0] = (unsigned short)tid;
        }
        __syncthreads();
        const u32 i0 = r0 + (u32)tid;
        u64 key[4], w[4][NV];
        bool live[4];
        // Every step below is written without a branch around it (an entry past the end re-reads the last
        // one and merges into a spare cell): a load or an LDS operation inside a branch is waited for at the
        // end of that branch, one entry after the other - four dependent round trips where one will do.
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            u32 i = i0 + (u32)q * 1024u;
            live[q] = i < total;
            i = live[q] ? i : total - 1u;
            const int lo = s_seg[i - r0];
            const u64* e = a.log + (((size_t)lo * a.parts + part) * (size_t)a.cap + (i - s_off[lo])) * WORDS;
            key[q] = e[0];
#pragma unroll
            for (int f = 0; f < NV; ++f) w[q][f] = e[1 + f];
        }
        // the home slots of all four are claimed at once (most are free: the table ends up half full)
        int sl[4];
        u64 seen[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const i64 s = (i64)w_table_hash_slot(key[q], (u32)a.slots) - base;      // the key's home slot, inside this slice
            const bool ok = live[q] && key[q] != W_EMPTY_KEY && s >= 0 && s < S;
            sl[q] = ok ? (int)s : -1;
            seen[q] = W_EMPTY_KEY;
            __hip_atomic_compare_exchange_strong(ok ? s_keys + s : s_spare + (tid & 63), &seen[q], ok ? key[q] : W_EMPTY_KEY, __ATOMIC_RELAXED,
                                                 __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        }
        // an entry whose home slot holds another key walks on (one in five, most of them one slot further)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            if (sl[q] < 0 || seen[q] == W_EMPTY_KEY || seen[q] == key[q]) continue;
            int t = sl[q] + 1;
            sl[q] = -1;
#pragma unroll 1
            for (; t < S; ++t) {
                const u64 cur = __hip_atomic_load(s_keys + t, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
                if (cur == key[q]) { sl[q] = t; break; }
                if (cur == W_EMPTY_KEY) {
                    u64 expect = W_EMPTY_KEY;
                    if (__hip_atomic_compare_exchange_strong(s_keys + t, &expect, key[q], __ATOMIC_RELAXED, __ATOMIC_RELAXED,
                                                             __HIP_MEMORY_SCOPE_WORKGROUP) || expect == key[q]) {
                        sl[q] = t;
                        break;
                    }
                }
            }
        }
#pragma unroll
        for (int q = 0; q < 4; ++q) {
#pragma unroll
            for (int f = 0; f < NV; ++f) cell_combine<FUNC>(sl[q] >= 0 ? &s_vals[f][sl[q]] : s_spare + 64 + (tid & 63), w[q][f], a.is_f64[f], 0);
        }
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            if (!live[q] || sl[q] >= 0) continue;
            // past the end of the slice, or the key equal to the free marker: to the list
            const u32 at = __hip_atomic_fetch_add(a.overflow_count, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if ((i64)at < a.overflow_cap) {
                u64* o = a.overflow + (size_t)at * WORDS;
                o[0] = key[q];
#pragma unroll
                for (int f = 0; f < NV; ++f) o[1 + f] = w[q][f];
            } else {
                atomicOr(a.err, 1);          // only a table far over its declared capacity gets here: the capacity error
            }
        }
    }
    __syncthreads();
    for (int q = tid; q < S; q += 1024) {
        a.keys[base + q] = s_keys[q];
#pragma unroll
        for (int k = 0; k < NV; ++k) a.vals[k][base + q] = s_vals[k][q];
    }
    // The result's packed arrays, while the slice is in LDS (a table that no loop kernel inserted into
    // directly: everything in it came through this kernel).  A thread's slots get neighbouring places, the
    // slice's places are reserved with one device atomic.
    if (a.pack && fresh) {
        u32 cnt = 0;
        for (int q = tid; q < S; q += 1024) cnt += s_keys[q] != W_EMPTY_KEY ? 1u : 0u;
        u32 inc = cnt;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const u32 o = __shfl_up(inc, off, 64);
            if ((tid & 63) >= off) inc += o;
        }
        __syncthreads();                       // (s_wave and s_off[0..1] are free again)
        if ((tid & 63) == 63) s_wave[tid >> 6] = inc;
        __syncthreads();
        u32 pre = 0, all = 0;
        for (int w = 0; w < 16; ++w) {
            if (w < (tid >> 6)) pre += s_wave[w];
            all += s_wave[w];
        }
        u64* const s_place = reinterpret_cast<u64*>(s_spare);
        if (tid == 0) {
            s_place[0] = all ? __hip_atomic_fetch_add(a.out_count, (u64)all, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : 0;
            if (blockIdx.x == 0) *a.packed = 1u;
        }
        __syncthreads();
        i64 pos = (i64)s_place[0] + pre + inc - cnt;
        for (int q = tid; q < S; q += 1024) {
            const u64 key = s_keys[q];
            if (key == W_EMPTY_KEY) continue;
            if (pos < a.capacity) {
                u64 v[NV];
#pragma unroll
                for (int k = 0; k < NV; ++k) v[k] = s_vals[k][q];
                pack_entry<NV>(a, pos, key, v);
            } else {
                atomicOr(a.err, 1);            // more keys than the declared capacity
            }
            ++pos;
        }
    }
}

template <int NV, int FUNC>
__global__ void __launch_bounds__(256) dict_overflow_insert_kernel(const SpillMerge a) {
    constexpr int WORDS = 1 + NV;
    i64 n = (i64)*a.overflow_count;
    if (n > a.overflow_cap) n = a.overflow_cap;
    const bool pack = a.pack && a.hdr[0] == 0;         // the slices packed their entries: the list's keys follow here
    for (i64 i = (i64)blockIdx.x * 256 + threadIdx.x; i < n; i += (i64)gridDim.x * 256) {
        u64* e = a.overflow + (size_t)i * WORDS;
        const u64 key = e[0];
        u64 w[NV];
#pragma unroll
        for (int f = 0; f < NV; ++f) w[f] = e[1 + f];
        // the key's slot, and whether THIS entry put the key there (one entry per key does: it reserves the
        // key's place in the packed arrays and writes the key; the value follows when all are merged)
        i64 g = -1;
        bool claimed = false;
        if (key == W_EMPTY_KEY) {
            claimed = __hip_atomic_exchange(a.hdr + 1, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == 0u;
            g = a.slots;
        } else {
            const i64 mask = a.slots - 1;
            i64 s = (i64)w_table_hash_slot(key, (u32)a.slots);
            for (i64 probe = 0; probe < a.slots; ++probe) {
                const u64 cur = __hip_atomic_load(a.keys + s, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                if (cur == key) { g = s; break; }
                if (cur == W_EMPTY_KEY) {
                    u64 expect = W_EMPTY_KEY;
                    if (__hip_atomic_compare_exchange_strong(a.keys + s, &expect, key, __ATOMIC_RELAXED, __ATOMIC_RELAXED,
                                                             __HIP_MEMORY_SCOPE_AGENT)) {
                        g = s;
                        claimed = true;
                        break;
                    }
                    if (expect == key) { g = s; break; }
                }
                s = (s + 1) & mask;
            }
            if (g < 0) atomicOr(a.err, 1);
        }
        if (g >= 0) {
#pragma unroll
            for (int f = 0; f < NV; ++f) cell_combine<FUNC>(a.vals[f] + g, w[f], a.is_f64[f], 1);
        }
        if (pack) {
            // the entry's own words now say where the key's value goes: slot, place (-1: another entry's business)
            i64 pos = -1;
            if (claimed) {
                pos = (i64)__hip_atomic_fetch_add(a.out_count, 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                if (pos >= a.capacity) {
                    atomicOr(a.err, 1);
                    pos = -1;
                }
            }
            e[0] = (u64)g;
            e[1] = (u64)pos;
        }
    }
}

// Behind the kernel above, when the entries are packed by the table's builders: the keys that came through the
// list get their (now final) values and their key fields.
template <int NV>
__global__ void __launch_bounds__(256) dict_overflow_pack_kernel(const SpillMerge a) {
    constexpr int WORDS = 1 + NV;
    if (!(a.pack && a.hdr[0] == 0)) return;
    i64 n = (i64)*a.overflow_count;
    if (n > a.overflow_cap) n = a.overflow_cap;
    for (i64 i = (i64)blockIdx.x * 256 + threadIdx.x; i < n; i += (i64)gridDim.x * 256) {
        const u64* e = a.overflow + (size_t)i * WORDS;
        const i64 g = (i64)e[0], pos = (i64)e[1];
        if (g < 0 || pos < 0) continue;
        u64 v[NV];
#pragma unroll
        for (int f = 0; f < NV; ++f) v[f] = a.vals[f][g];
        pack_entry<NV>(a, pos, g == a.slots ? W_EMPTY_KEY : a.keys[g], v);
    }
}

template <int NV, int FUNC>
static hipError_t launch_slices(const SpillMerge& a, hipStream_t stream, hipEvent_t stop) {
    if (a.slots != (long long)a.parts * SpillTable<NV>::kSlots || a.groups > 1024) return hipErrorInvalidValue;
    dict_slice_build_kernel<NV, FUNC><<<dim3((unsigned)a.parts), dim3(1024), 0, stream>>>(a);
    hipError_t h = hipGetLastError();
    if (h != hipSuccess) return h;
    if (!a.pack) {
        if (stop) hipExtLaunchKernelGGL((dict_overflow_insert_kernel<NV, FUNC>), dim3(64), dim3(256), 0, stream, nullptr, stop, 0, a);
        else dict_overflow_insert_kernel<NV, FUNC><<<dim3(64), dim3(256), 0, stream>>>(a);
        return hipGetLastError();
    }
    dict_overflow_insert_kernel<NV, FUNC><<<dim3(64), dim3(256), 0, stream>>>(a);
    h = hipGetLastError();
    if (h != hipSuccess) return h;
    if (stop) hipExtLaunchKernelGGL(dict_overflow_pack_kernel<NV>, dim3(64), dim3(256), 0, stream, nullptr, stop, 0, a);
    else dict_overflow_pack_kernel<NV><<<dim3(64), dim3(256), 0, stream>>>(a);
    return hipGetLastError();
}
template <int NV>
static hipError_t launch_slices_nv(const SpillMerge& a, hipStream_t stream, hipEvent_t stop) {
    switch (a.func) {
        case W_FUNC_ADD: return launch_slices<NV, W_FUNC_ADD>(a, stream, stop);
        case W_FUNC_MUL: return launch_slices<NV, W_FUNC_MUL>(a, stream, stop);
        case W_FUNC_MIN: return launch_slices<NV, W_FUNC_MIN>(a, stream, stop);
        case W_FUNC_MAX: return launch_slices<NV, W_FUNC_MAX>(a, stream, stop);
        default: return hipErrorInvalidValue;
    }
}
hipError_t launch_dict_slice_build(const SpillMerge& a, int nvals, hipStream_t stream, hipEvent_t stop) {
    switch (nvals) {
        case 1: return launch_slices_nv<1>(a, stream, stop);
        case 2: return launch_slices_nv<2>(a, stream, stop);
        case 3: return launch_slices_nv<3>(a, stream, stop);
        case 4: return launch_slices_nv<4>(a, stream, stop);
        case 5: return launch_slices_nv<5>(a, stream, stop);
        case 6: return launch_slices_nv<6>(a, stream, stop);
        case 7: return launch_slices_nv<7>(a, stream, stop);
        case 8: return launch_slices_nv<8>(a, stream, stop);
        default: return hipErrorInvalidValue;
    }
}

template <int NV>
static hipError_t launch_nv(const SpillMerge& in, hipStream_t stream, hipEvent_t stop) {
    SpillMerge a = in;
    // table: four slots per key the partition is expected to hold (capacity / 256), at least 1024, at
    // most what 128 KiB take; two work-groups per partition where two such tables fit a compute unit
    // (more work-groups per partition gained nothing: they do not start any sooner)
    constexpr int kMax = SpillTable<NV>::kSlots;
    int slots = 1024;
    while (slots < kMax && (long long)slots * kSpillParts < 4 * a.capacity) slots *= 2;
    if (slots > kMax) slots = kMax;
    a.table_slots = slots;
    a.split = kMax / slots >= 2 ? 2 : 1;
    const dim3 grid(kSpillParts * a.split), block(1024);
    const size_t lds = (size_t)slots * 8 * (1 + NV);
    auto go = [&](void (*kern)(const SpillMerge)) -> hipError_t {
        if (lds > 65536) {      // more dynamic LDS than a kernel gets without asking
            const hipError_t he = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
            if (he != hipSuccess) return he;
        }
        if (stop) hipExtLaunchKernelGGL(kern, grid, block, lds, stream, nullptr, stop, 0, a);
        else kern<<<grid, block, lds, stream>>>(a);
        return hipGetLastError();
    };
    if (a.compact) {
        if (NV != 1 || a.func != W_FUNC_ADD) return hipErrorInvalidValue;
        return a.compact == 2 ? go(dict_spill_merge_kernel<1, W_FUNC_ADD, 2>) : go(dict_spill_merge_kernel<1, W_FUNC_ADD, 1>);
    }
    switch (a.func) {
        case W_FUNC_ADD: return go(dict_spill_merge_kernel<NV, W_FUNC_ADD>);
        case W_FUNC_MUL: return go(dict_spill_merge_kernel<NV, W_FUNC_MUL>);
        case W_FUNC_MIN: return go(dict_spill_merge_kernel<NV, W_FUNC_MIN>);
        case W_FUNC_MAX: return go(dict_spill_merge_kernel<NV, W_FUNC_MAX>);
        default: return hipErrorInvalidValue;
    }
}

// ---------------------------------------------------------------- queued vecmerger
// One work-group per range of cells.  The range's cells start at the identity in LDS; a wavefront takes the range's
// segment of one loop work-group at a time (lanes read neighbouring entries) and merges with LDS atomics; at the
// end every cell that left the identity is combined into the result, which the work-group owns for its range.
// LONG (2-byte entries): the host expects segments of a thousand entries and more; the kernel then reads them with
// 16-byte loads.  (One kernel with both ways of reading ran the other, one entry per lane and load, 8-17 % slower.)
template <int FUNC, int ENTRY, bool LONG>
__global__ void __launch_bounds__(1024) vecm_ranges_kernel(const VecmRanges a) {
    __shared__ u64 s_cell[8192];
    __shared__ u32 s_len[2048];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int r = blockIdx.x;
    const int cells = 1 << a.shift;
    for (int q = tid; q < cells; q += 1024) s_cell[q] = a.ident;
    // the lengths of the range's segments, read side by side (one memory round trip for all of them)
    for (int g = tid; g < a.groups; g += 1024) s_len[g] = a.qcnt[(i64)g * a.ranges + r];
    __syncthreads();
    for (int g = wave; g < a.groups; g += 16) {
        const i64 len = (i64)s_len[g] < a.cap ? (i64)s_len[g] : a.cap;
        const i64 seg = ((i64)g * a.ranges + r) * a.cap;
        // eight loads of a lane in flight (no branch around a load: an entry past the end re-reads the last one)
        if (ENTRY == 2) {
            const unsigned short* e = (const unsigned short*)a.log + seg;
            const bool merge_as_one = len >= a.cap && ((FUNC == 0 && !a.is_f64) || FUNC == 2 || FUNC == 3);
            if (LONG && !merge_as_one) {
                // A lane takes eight neighbouring entries with one 16-byte load (a segment begins at a 16-byte address
                // and holds a multiple of eight entries; those past `len` are read and not used), four such loads
                // in flight: with one 2-byte entry per lane and load a wavefront had 1 KB in flight, a compute unit
                // 16 KB, and the kernel read its 0.2 GB at 2.2 TB/s.  For long segments only (up to 2^21 cells with
                // 1e8 rows): a segment of 200 entries would keep 25 lanes busy.
                typedef u32 u32x4 __attribute__((ext_vector_type(4)));
                const u32x4* e16 = (const u32x4*)e;
                const i64 nvec = (len + 7) / 8;
                for (i64 v0 = 0; v0 < nvec; v0 += 256) {
                    u32x4 x[4];
#pragma unroll
                    for (int k = 0; k < 4; ++k) {
                        const i64 vi = v0 + k * 64 + lane;
                        x[k] = __builtin_nontemporal_load(e16 + (vi < nvec ? vi : nvec - 1));
                    }
#pragma unroll
                    for (int k = 0; k < 4; ++k) {
                        const i64 vi = v0 + k * 64 + lane;
                        if (vi >= nvec) continue;
#pragma unroll
                        for (int q = 0; q < 8; ++q) {
                            const u32 c = (x[k][q >> 1] >> (16 * (q & 1))) & 0xffffu;
                            if (vi * 8 + q < len && c < (u32)cells) cell_combine<FUNC>(s_cell + c, a.const_bits, a.is_f64, 0);
                        }
                    }
                }
                continue;
            }
            for (i64 i0 = 0; i0 < len; i0 += 512) {
                u32 c[8];
#pragma unroll
                for (int k = 0; k < 8; ++k) {
                    const i64 i = i0 + k * 64 + lane;
                    c[k] = (u32)__builtin_nontemporal_load(e + (i < len ? i : len - 1));
                }
                if (!merge_as_one) {
#pragma unroll
                    for (int k = 0; k < 8; ++k)
                        if (i0 + k * 64 + lane < len && c[k] < (u32)cells) cell_combine<FUNC>(s_cell + c[k], a.const_bits, a.is_f64, 0);
                    continue;
                }
                // A segment that is full: a hot cell.  Most lanes of a load then hold the same cell, and 64 LDS atomics
                // on one address run one after the other; the lanes that hold the first valid lane's cell merge as one
                // where that gives the same bits (integer sums: the constant times their number; minima and maxima:
                // the constant once).  Segments with room take the forms above: the ballots cost a quarter of the
                // kernel's time on uniform indices.
                const bool as_one = true;
#pragma unroll
                for (int k = 0; k < 8; ++k) {
                    const bool valid = i0 + k * 64 + lane < len && c[k] < (u32)cells;
                    const u64 vm = __builtin_amdgcn_ballot_w64(valid);
                    if (vm == 0) continue;
                    const int leader = (int)__builtin_ctzll(vm);
                    const u32 lead = (u32)__shfl((int)c[k], leader, 64);
                    const bool same = as_one && valid && c[k] == lead;
                    const u64 sm = __builtin_amdgcn_ballot_w64(same);
                    if (same) {
                        if (lane == leader)
                            cell_combine<FUNC>(s_cell + lead, FUNC == 0 ? a.const_bits * (u64)__popcll(sm) : a.const_bits, a.is_f64, 0);
                    } else if (valid) {
                        cell_combine<FUNC>(s_cell + c[k], a.const_bits, a.is_f64, 0);
                    }
                }
            }
        } else {
            // (a segment's values, 8 bytes each, then its cells, 2 bytes each: cap is a multiple of 8)
            const char* sg = (const char*)a.log + seg * 10;
            const u64* ev = (const u64*)sg;
            const unsigned short* ec = (const unsigned short*)(sg + 8 * a.cap);
            for (i64 i0 = 0; i0 < len; i0 += 512) {
                u64 c[8], v[8];
#pragma unroll
                for (int k = 0; k < 8; ++k) {
                    const i64 i = i0 + k * 64 + lane;
                    const i64 ic = i < len ? i : len - 1;
                    c[k] = (u64)__builtin_nontemporal_load(ec + ic);
                    v[k] = __builtin_nontemporal_load(ev + ic);
                }
#pragma unroll
                for (int k = 0; k < 8; ++k)
                    if (i0 + k * 64 + lane < len && c[k] < (u64)cells) cell_combine<FUNC>(s_cell + c[k], v[k], a.is_f64, 0);
            }
        }
    }
    __syncthreads();
    const i64 first = (i64)r << a.shift;
    for (int q = tid; q < cells; q += 1024) {
        const u64 x = s_cell[q];
        if (x == a.ident || first + q >= a.length) continue;
        u64* p = a.out + first + q;
        if (a.is_f64) {
            double cur, add;
            const u64 cb = *p;
            __builtin_memcpy(&cur, &cb, 8);
            __builtin_memcpy(&add, &x, 8);
            const double res = w_combine<FUNC>(cur, add);
            u64 rb;
            __builtin_memcpy(&rb, &res, 8);
            *p = rb;
        } else {
            *p = (u64)w_combine<FUNC>((i64)*p, (i64)x);
        }
    }
}

template <int FUNC>
static hipError_t launch_vecm_func(const VecmRanges& v, hipStream_t stream, hipEvent_t stop) {
    if (v.entry_bytes == 2 && v.long_segments)
        hipExtLaunchKernelGGL((vecm_ranges_kernel<FUNC, 2, true>), dim3((unsigned)v.ranges), dim3(1024), 0, stream, nullptr, stop, 0, v);
    else if (v.entry_bytes == 2)
        hipExtLaunchKernelGGL((vecm_ranges_kernel<FUNC, 2, false>), dim3((unsigned)v.ranges), dim3(1024), 0, stream, nullptr, stop, 0, v);
    else
        hipExtLaunchKernelGGL((vecm_ranges_kernel<FUNC, 10, false>), dim3((unsigned)v.ranges), dim3(1024), 0, stream, nullptr, stop, 0, v);
    return hipGetLastError();
}
hipError_t launch_vecm_ranges(const VecmRanges& v, hipStream_t stream, hipEvent_t stop) {
    if (v.ranges < 1 || v.shift < 0 || v.shift > 13 || v.groups < 1 || v.groups > 2048 || v.cap < 0 ||
        (v.entry_bytes != 2 && v.entry_bytes != 10) || (v.cap & 7) || ((long long)v.ranges << v.shift) < v.length)
        return hipErrorInvalidValue;
    switch (v.func) {
        case 0: return launch_vecm_func<0>(v, stream, stop);
        case 1: return launch_vecm_func<1>(v, stream, stop);
        case 2: return launch_vecm_func<2>(v, stream, stop);
        case 3: return launch_vecm_func<3>(v, stream, stop);
        default: return hipErrorInvalidValue;
    }
}

hipError_t launch_dict_spill_merge(const SpillMerge& a, int nvals, hipStream_t stream, hipEvent_t stop) {
    switch (nvals) {
        case 1: return launch_nv<1>(a, stream, stop);
        case 2: return launch_nv<2>(a, stream, stop);
        case 3: return launch_nv<3>(a, stream, stop);
        case 4: return launch_nv<4>(a, stream, stop);
        case 5: return launch_nv<5>(a, stream, stop);
        case 6: return launch_nv<6>(a, stream, stop);
        case 7: return launch_nv<7>(a, stream, stop);
        case 8: return launch_nv<8>(a, stream, stop);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace weld
