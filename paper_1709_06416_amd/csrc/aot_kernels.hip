// Ahead-of-time compiled helper kernels (gfx950): workspace fills, dictionary
// result extraction, and the two memory probes used for roofline measurements.
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>

#include "aot_kernels.h"

namespace weld {

typedef unsigned long long u64;
typedef long long i64;
typedef unsigned int u32;
typedef u32 u32x4 __attribute__((ext_vector_type(4)));
typedef i64 i64x2 __attribute__((ext_vector_type(2)));

static const u64 kEmptyKey = 0x8000000000000000ull;

// ---------------------------------------------------------------- fill
// Workspace is cleared with a kernel rather than a memset node so that a caller may
// capture the whole call into a HIP graph.
__global__ void __launch_bounds__(256) fill64_kernel(u64* p, i64 count, u64 value) {
    for (i64 i = (i64)blockIdx.x * 256 + threadIdx.x; i < count; i += (i64)gridDim.x * 256) p[i] = value;
}

hipError_t launch_fill64(void* p, int64_t count, uint64_t value, hipStream_t stream) {
    if (count <= 0) return hipSuccess;
    int64_t blocks = (count + 255) / 256;
    if (blocks > 4096) blocks = 4096;
    fill64_kernel<<<dim3((unsigned)blocks), dim3(256), 0, stream>>>((u64*)p, count, value);
    return hipGetLastError();
}

__global__ void __launch_bounds__(256) fill_list_kernel(const FillList f) {
    for (int k = 0; k < f.n; ++k) {
        u64* const p = (u64*)f.p[k];
        const u64 v = f.value[k];
        for (i64 i = (i64)blockIdx.x * 256 + threadIdx.x; i < f.count[k]; i += (i64)gridDim.x * 256) p[i] = v;
    }
}

hipError_t launch_fill_list(const FillList& f, hipStream_t stream, hipEvent_t start) {
    if (f.n == 0) return hipSuccess;
    long long most = 0;
    for (int k = 0; k < f.n; ++k) most = f.count[k] > most ? f.count[k] : most;
    int64_t blocks = (most + 255) / 256;
    if (blocks > 4096) blocks = 4096;
    if (start) hipExtLaunchKernelGGL(fill_list_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, start, nullptr, 0, f);
    else fill_list_kernel<<<dim3((unsigned)blocks), dim3(256), 0, stream>>>(f);
    return hipGetLastError();
}

// ---------------------------------------------------------------- merger result
// Fixed-order combination of the per-work-group partials of every merger of a call
// (one work-group per merger).  Thread j folds partials j, j+256, ... in that order,
// then the 256 per-thread values are combined by a fixed butterfly and in wavefront
// order, so the result is the same on every run.
// (min / max of anything with a NaN is NaN, as in the loop kernels: `b != b` is never true for integers)
template <class T> __device__ T combine(int func, T a, T b) {
    switch (func) {
        case 0: return a + b;
        case 1: return a * b;
        case 2: return b != b ? b : (b < a ? b : a);
        default: return b != b ? b : (b > a ? b : a);
    }
}
template <class T> __device__ T block_combine(int func, T v, T ident, T* scratch) {
    for (int off = 32; off > 0; off >>= 1) v = combine(func, v, (T)__shfl_xor(v, off, 64));
    if ((threadIdx.x & 63) == 0) scratch[threadIdx.x >> 6] = v;
    __syncthreads();
    T r = ident;
    for (int w = 0; w < 4; ++w) r = combine(func, r, scratch[w]);
    return r;
}

__global__ void __launch_bounds__(256) merger_finish_kernel(MergerFinish m, int count) {
    __shared__ u64 scratch[4];
    const int b = blockIdx.x;
    const int func = m.func[b];
    const u64* part = m.partial[b];
    if (m.is_f64[b]) {
        const double ident = func == 0 ? 0.0 : func == 1 ? 1.0 : func == 2 ? __builtin_huge_val() : -__builtin_huge_val();
        double v = ident;
        for (int i = threadIdx.x; i < count; i += 256) v = combine(func, v, __longlong_as_double((i64)part[i]));
        v = block_combine(func, v, ident, (double*)scratch);
        if (threadIdx.x == 0) *(double*)m.result[b] = v;
    } else {
        const int bits = m.bits[b];
        const i64 ident = func == 0 ? 0 : func == 1 ? 1 : func == 2 ? (i64)((1ull << (bits - 1)) - 1) : -(i64)(1ull << (bits - 1));
        i64 v = ident;
        for (int i = threadIdx.x; i < count; i += 256) {
            const i64 x = (i64)part[i];
            v = func == 1 ? (i64)((u64)v * (u64)x) : func == 0 ? (i64)((u64)v + (u64)x) : combine(func, v, x);
        }
        // wrapping arithmetic through the unsigned type inside the tree as well
        for (int off = 32; off > 0; off >>= 1) {
            const i64 o = __shfl_xor(v, off, 64);
            v = func == 1 ? (i64)((u64)v * (u64)o) : func == 0 ? (i64)((u64)v + (u64)o) : combine(func, v, o);
        }
        i64* sc = (i64*)scratch;
        if ((threadIdx.x & 63) == 0) sc[threadIdx.x >> 6] = v;
        __syncthreads();
        i64 r = ident;
        for (int w = 0; w < 4; ++w) r = func == 1 ? (i64)((u64)r * (u64)sc[w]) : func == 0 ? (i64)((u64)r + (u64)sc[w]) : combine(func, r, sc[w]);
        if (threadIdx.x == 0) {
            unsigned char* out = (unsigned char*)m.result[b];
            for (int k = 0; k < m.elem_size[b]; ++k) out[k] = (unsigned char)((u64)r >> (8 * k));
        }
    }
}

hipError_t launch_merger_finish(const MergerFinish& m, int count, hipStream_t stream) {
    if (m.n <= 0) return hipSuccess;
    merger_finish_kernel<<<dim3((unsigned)m.n), dim3(256), 0, stream>>>(m, count);
    return hipGetLastError();
}

// ---------------------------------------------------------------- dictionary result
// One field of a packed struct: a single store of the field's width where the address is aligned
// to it (always so for a struct of one field, or of 8-byte fields), byte by byte otherwise.
__device__ __forceinline__ void store_field(unsigned char* p, u64 bits, int size) {
    if (size == 8 && ((uintptr_t)p & 7) == 0) *(u64*)p = bits;
    else if (size == 4 && ((uintptr_t)p & 3) == 0) *(u32*)p = (u32)bits;
    else
        for (int b = 0; b < size; ++b) p[b] = (unsigned char)(bits >> (8 * b));
}

// Walks the open-addressing table and writes every occupied slot as one (key struct,
// value struct) pair in C packed layout (Sec. 4.2 of the paper).  Entry order is
// unspecified (the paper's dict is unordered).  Entries beyond `capacity` raise the
// capacity error instead of being written.
template <int J>
__global__ void __launch_bounds__(256) dict_extract_kernel(const u64* keys, const u32* hdr, i64 slots,
                                                           DictValues vals, DictLayout lay, i64 capacity,
                                                           unsigned char* out_keys, unsigned char* out_vals,
                                                           u64* count, int* err, int* slot_pos, u64* kp32, u32* kwide,
                                                           const u32* skip_if) {
    if (skip_if && *skip_if != 0) return;
    // A work-group takes 256 * J slots at a time, a wavefront 64 * J consecutive ones (load j of lane
    // l: slot (wave * J + j) * 64 + l).  The occupied slots are counted, their output positions
    // reserved with ONE device atomic (a same-address atomic costs about 12 ns here, serialised: one
    // per entry would dominate large dictionaries, and for tables of millions of slots even one per
    // 2048 slots shows - those take 8192 a round) and handed out in slot order, so that the 64
    // lanes of a store write neighbouring entries.
    __shared__ u32 s_wave[4];
    __shared__ u64 s_base;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const i64 total = slots + 1;                       // the extra slot holds the key equal to the free marker
    const bool marker_key = hdr[1] != 0;               // (read once: the loops below would reload it for every slot)
    bool wide = false;
    for (i64 base = (i64)blockIdx.x * 256 * J; base < total; base += (i64)gridDim.x * 256 * J) {
        u64 kb[J];
        u32 used = 0;                                  // bit j: slot j of this thread is occupied
        u32 mine = 0;                                  // occupied slots of the wavefront
#pragma unroll
        for (int j = 0; j < J; ++j) {                  // all loads first: they are in flight together
            const i64 s = base + (i64)(wave * J + j) * 64 + lane;
            kb[j] = s < slots ? __builtin_nontemporal_load(keys + s) : kEmptyKey;
        }
#pragma unroll
        for (int j = 0; j < J; ++j) {
            const i64 s = base + (i64)(wave * J + j) * 64 + lane;
            const bool u = s < slots ? (kb[j] != kEmptyKey) : (s == slots && marker_key);
            used |= (u ? 1u : 0u) << j;
            mine += (u32)__popcll(__builtin_amdgcn_ballot_w64(u));
        }
        if (lane == 0) s_wave[wave] = mine;
        __syncthreads();
        u32 before = 0, all = 0;
        for (int w = 0; w < 4; ++w) {
            if (w < wave) before += s_wave[w];
            all += s_wave[w];
        }
        if (tid == 0) s_base = all ? atomicAdd(count, (u64)all) : 0;
        __syncthreads();
        u64 run = s_base + before;
        // eight slots per lane at a time: their value cells are loaded side by side before any is
        // stored (a store through a byte pointer may alias anything, so the compiler keeps every
        // load behind the store before it: one memory round trip per slot otherwise)
#pragma unroll
        for (int j0 = 0; j0 < J; j0 += 8) {
            i64 at[8];
#pragma unroll
            for (int q = 0; q < 8; ++q) {
                const int j = j0 + q;
                const bool u = (used >> j) & 1u;
                const u64 bal = __builtin_amdgcn_ballot_w64(u);
                at[q] = (i64)(run + (u64)__builtin_amdgcn_mbcnt_hi((u32)(bal >> 32), __builtin_amdgcn_mbcnt_lo((u32)bal, 0)));
                run += (u64)__popcll(bal);
                const i64 s = base + (i64)(wave * J + j) * 64 + lane;
                if (!u) {
                    if (kp32 && s < total) kp32[s] = 0xffffffff00000000ull;     // a free slot
                    at[q] = -1;
                    continue;
                }
                if (slot_pos) slot_pos[s] = at[q] < capacity ? (int)at[q] : -1;
                if (kp32) {
                    // the slot's group number beside the low half of its key: one 8-byte read answers a look-up
                    // as long as every key is the sign extension of its low half (`wide` says whether)
                    const u64 kfull = s < slots ? kb[j] : kEmptyKey;
                    kp32[s] = ((u64)(u32)(at[q] < capacity ? (int)at[q] : -1) << 32) | (u32)kfull;
                    wide |= (i64)kfull != (i64)(int)(u32)kfull;
                }
                if (at[q] >= capacity) {
                    atomicOr(err, 1);
                    at[q] = -1;
                    continue;
                }
                unsigned char* ko = out_keys + at[q] * lay.key_stride;
                int off = 0;
                for (int k = 0; k < lay.nkeys; ++k) {
                    store_field(ko + off, kb[j] >> lay.key_shift[k], lay.key_size[k]);
                    off += lay.key_size[k];
                }
            }
            int off = 0;
            for (int k = 0; k < lay.nvals; ++k) {
                u64 cell[8];
#pragma unroll
                for (int q = 0; q < 8; ++q) {
                    const i64 s = base + (i64)(wave * J + j0 + q) * 64 + lane;
                    cell[q] = at[q] >= 0 ? vals.p[k][s] : 0;
                }
#pragma unroll
                for (int q = 0; q < 8; ++q)
                    if (at[q] >= 0) store_field(out_vals + at[q] * lay.val_stride + off, cell[q], lay.val_size[k]);
                off += lay.val_size[k];
            }
        }
        __syncthreads();                               // s_wave / s_base are reused by the next round
    }
    if (kwide && __builtin_amdgcn_ballot_w64(wide) != 0 && lane == 0) atomicOr(kwide, 1u);
}

hipError_t launch_dict_extract(const void* keys, const void* hdr, int64_t slots, const DictValues& vals,
                               const DictLayout& lay, int64_t capacity, void* out_keys, void* out_vals,
                               void* count, void* err, int* slot_pos, unsigned long long* kp32, unsigned int* kwide,
                               const unsigned int* skip_if, hipStream_t stream) {
    const bool big = slots >= (1ll << 22);
    const int64_t round = big ? 8192 : 2048;
    int64_t blocks = (slots + 1 + round - 1) / round;
    if (blocks > 2048) blocks = 2048;
    if (big)
        dict_extract_kernel<32><<<dim3((unsigned)blocks), dim3(256), 0, stream>>>(
            (const u64*)keys, (const u32*)hdr, slots, vals, lay, capacity, (unsigned char*)out_keys,
            (unsigned char*)out_vals, (u64*)count, (int*)err, slot_pos, (u64*)kp32, kwide, skip_if);
    else
        dict_extract_kernel<8><<<dim3((unsigned)blocks), dim3(256), 0, stream>>>(
            (const u64*)keys, (const u32*)hdr, slots, vals, lay, capacity, (unsigned char*)out_keys,
            (unsigned char*)out_vals, (u64*)count, (int*)err, slot_pos, (u64*)kp32, kwide, skip_if);
    return hipGetLastError();
}

// ---------------------------------------------------------------- groupbuilder
// Exclusive prefix sums of the group sizes, 8192 groups a round, one round per work-group at a time:
// a thread loads eight neighbouring sizes, the 1024 partial sums are scanned across the work-group, the
// round's total is published in `desc` and the sum of the rounds before it collected from there
// (decoupled look-back: bits 63..62 of a descriptor = 0 nothing yet, 1 the round's own total, 2 the
// total of all rounds up to it), and the thread writes its eight offsets.  The grid never exceeds
// what is resident at once, so a round only waits for work-groups that are running; the wait is
// bounded all the same (error bit 2, the call then reports a device error).
__global__ void __launch_bounds__(1024) group_offsets_kernel(const i64* counts, const u64* ngroups, i64 capacity,
                                                             i64* offsets, u64* cursor, u64* desc, int* err) {
    __shared__ i64 s_wave[16];
    __shared__ i64 s_carry;
    const int tid = threadIdx.x;
    i64 n = (i64)*ngroups;
    if (n > capacity) n = capacity;
    const bool aligned16 = (((uintptr_t)counts | (uintptr_t)offsets | (uintptr_t)cursor) & 15) == 0;
    if (n == 0 && blockIdx.x == 0 && tid == 0) offsets[0] = 0;
    for (i64 round = blockIdx.x; round * 8192 < n; round += gridDim.x) {
        const i64 base = round * 8192;
        i64 c[8];
        i64 mine = 0;
        const bool whole = base + 8192 <= n && aligned16;      // every thread's eight groups exist
        if (whole) {
            // 16-byte loads: a lane's eight sizes are 64 contiguous bytes, lanes are 64 bytes apart, so
            // every load instruction of a wavefront touches 32 cache lines whatever its width
            const i64x2* p = (const i64x2*)(counts + base + (i64)tid * 8);
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const i64x2 v = p[q];
                c[2 * q] = v.x;
                c[2 * q + 1] = v.y;
            }
#pragma unroll
            for (int k = 0; k < 8; ++k) mine += c[k];
        } else {
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                const i64 g = base + (i64)tid * 8 + k;
                c[k] = g < n ? counts[g] : 0;
                mine += c[k];
            }
        }
        i64 incl = mine;
        for (int off = 1; off < 64; off <<= 1) {
            const i64 o = __shfl_up(incl, off, 64);
            if ((tid & 63) >= off) incl += o;
        }
        if ((tid & 63) == 63) s_wave[tid >> 6] = incl;
        __syncthreads();
        if (tid < 64) {
            i64 total = 0;
#pragma unroll
            for (int w = 0; w < 16; ++w) total += s_wave[w];
            // publish, then walk back over the rounds before this one, 64 at a time
            i64 excl = 0;
            if (round == 0) {
                if (tid == 0) __hip_atomic_store(desc, (2ull << 62) | (u64)total, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            } else {
                if (tid == 0) __hip_atomic_store(desc + round, (1ull << 62) | (u64)total, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                i64 j = round - 1, spins = 0;
                bool failed = false;
                for (;;) {
                    const i64 idx = j - tid;
                    const u64 d = idx >= 0 ? __hip_atomic_load(desc + idx, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : (2ull << 62);
                    const u32 state = (u32)(d >> 62);
                    const u64 unpublished = __ballot(state == 0);
                    const u64 have_prefix = __ballot(state == 2);
                    const int first = have_prefix ? (int)__builtin_ctzll(have_prefix) : 64;
                    const u64 need = first >= 63 ? ~0ull : ((2ull << first) - 1);
                    if (unpublished & need) {
                        if (++spins > (1 << 22)) { failed = true; break; }
                        __builtin_amdgcn_s_sleep(2);
                        continue;
                    }
                    i64 part = (tid <= first) ? (i64)(d & ((1ull << 62) - 1)) : 0;
                    for (int off = 32; off > 0; off >>= 1) part += __shfl_xor(part, off, 64);
                    excl += part;
                    if (first < 64) break;
                    j -= 64;
                }
                if (failed) {
                    if (tid == 0) atomicOr(err, 2);
                    excl = 0;
                }
                if (tid == 0) __hip_atomic_store(desc + round, (2ull << 62) | (u64)(excl + total), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
            if (tid == 0) {
                s_carry = excl;
                if (base + 8192 >= n) offsets[n] = excl + total;     // the last round closes the array
            }
        }
        __syncthreads();
        i64 run = s_carry + incl - mine;
        for (int w = 0; w < (tid >> 6); ++w) run += s_wave[w];
        if (whole) {
            i64x2* po = (i64x2*)(offsets + base + (i64)tid * 8);
            i64x2* pc = (i64x2*)(cursor + base + (i64)tid * 8);
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                i64x2 o;
                o.x = run;
                o.y = run + c[2 * q];
                run = o.y + c[2 * q + 1];
                po[q] = o;
                const i64x2 zero = {0, 0};
                pc[q] = zero;
            }
        } else {
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                const i64 g = base + (i64)tid * 8 + k;
                if (g < n) {
                    offsets[g] = run;
                    cursor[g] = 0;
                }
                run += c[k];
            }
        }
        __syncthreads();
    }
}

hipError_t launch_group_offsets(const void* counts, const void* ngroups, int64_t capacity, void* offsets, void* cursor,
                                void* desc, void* err, int max_blocks, hipStream_t stream) {
    int64_t blocks = (capacity + 8191) / 8192;
    if (blocks > max_blocks) blocks = max_blocks;
    if (blocks < 1) blocks = 1;
    group_offsets_kernel<<<dim3((unsigned)blocks), dim3(1024), 0, stream>>>((const i64*)counts, (const u64*)ngroups, capacity,
                                                                              (i64*)offsets, (u64*)cursor, (u64*)desc, (int*)err);
    return hipGetLastError();
}

// Element i of a vector that is read once, front to back (the compacted pairs of a groupbuilder):
// loaded with the streaming hint, so that it does not push the dictionary's table, which every pair
// looks its key up in, out of the L2.
__device__ __forceinline__ u64 load_bits(const void* p, i64 i, int size) {
    switch (size) {
        case 1: return (u64)__builtin_nontemporal_load((const unsigned char*)p + i);
        case 4: return (u64)__builtin_nontemporal_load((const u32*)p + i);
        default: return __builtin_nontemporal_load((const u64*)p + i);
    }
}
// the hash of the work-groups' own LDS caches (one multiplication), and the hash of the dictionaries'
// global tables, the same as the loop kernels' (both probe the same tables: a second multiplication
// for tables of 2^21 slots and more)
__device__ __forceinline__ u32 cache_hash_slot(u64 k, u32 slots) {
    const u32 x = (u32)k ^ ((u32)(k >> 32) * 0x85ebca6bu);
    return (x * 0x9e3779b1u) >> (__builtin_clz(slots) + 1);
}
__device__ __forceinline__ u32 table_hash_slot(u64 k, u32 slots) {
    const u32 x = (u32)k ^ ((u32)(k >> 32) * 0x85ebca6bu);
    u32 h = x * 0x9e3779b1u;
    if (slots >= (1u << 21)) {
        asm volatile("");
        h ^= h >> 15;
        h *= 0x2c1b3c6du;
        h ^= h >> 13;
    }
    return h >> (__builtin_clz(slots) + 1);
}

#define GROUP_TILE 4096
#define GROUP_LDS 8192
__global__ void __launch_bounds__(1024) group_scatter_kernel(const GroupScatter a) {
    // one 8-byte entry per group met in the tile: first (group : u32, pairs of it in this tile :
    // u32), then, once the places are reserved, overwritten by where those pairs start in
    // values_out.  64 KiB, so that two work-groups share a CU.
    __shared__ u64 s_ent[GROUP_LDS];
    u32* const s_half = reinterpret_cast<u32*>(s_ent);
#define s_gid(e) s_half[2 * (e)]
#define s_cnt(e) s_half[2 * (e) + 1]
    const int tid = threadIdx.x;
    const i64 npairs = (i64)*a.npairs;
    const i64 ntiles = (npairs + GROUP_TILE - 1) / GROUP_TILE;
    for (int q = tid; q < GROUP_LDS; q += 1024) s_ent[q] = 0xffffffffull;
    __syncthreads();
    for (i64 t = blockIdx.x; t < ntiles; t += gridDim.x) {
        int entry[4];
        u32 rank[4];
        u64 val[4], kb[4], first[4];
        i64 slot[4];
        int gid[4];
        bool live[4];
        // the four pairs of a thread go through every step side by side, so that their loads
        // (pair, first table probe, group of the slot) are in flight together
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const i64 i = t * GROUP_TILE + j * 1024 + tid;
            live[j] = i < npairs;
            kb[j] = 0;
            val[j] = 0;
            if (live[j]) {
                for (int k = 0; k < a.nkeys; ++k) kb[j] |= load_bits(a.key[k], i, a.key_size[k]) << a.key_shift[k];
                if (a.key_sext32) kb[j] = (u64)(i64)(int)(u32)kb[j];
                val[j] = load_bits(a.value, i, a.value_size);
            }
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            slot[j] = (i64)table_hash_slot(kb[j], (u32)a.slots);
            first[j] = live[j] ? a.table_keys[slot[j]] : kEmptyKey;
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            // the key's slot in the dictionary (every key is there unless the capacity overflowed)
            if (!live[j]) { slot[j] = -1; continue; }
            if (kb[j] == kEmptyKey) { slot[j] = a.hdr[1] ? a.slots : -1; continue; }
            if (first[j] == kb[j]) continue;
            i64 s = slot[j], found = -1;
            u64 cur = first[j];
            for (i64 probe = 1; probe < a.slots && cur != kEmptyKey; ++probe) {
                s = (s + 1) & (a.slots - 1);
                cur = a.table_keys[s];
                if (cur == kb[j]) { found = s; break; }
            }
            slot[j] = found;
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) gid[j] = slot[j] >= 0 ? a.slot_pos[slot[j]] : -1;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            entry[j] = -1;
            rank[j] = 0;
            if (gid[j] < 0) continue;                           // not extracted: the call fails with the capacity error
            // this tile's entry for the group, and the pair's rank inside it
            u32 e = ((u32)gid[j] * 0x9e3779b1u) >> (32 - 13);
            for (;;) {                                          // at most GROUP_TILE groups in 2 * GROUP_TILE entries
                const u32 cur = __hip_atomic_load(&s_gid(e), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
                if (cur == (u32)gid[j]) break;
                if (cur == ~0u) {
                    u32 expect = ~0u;
                    if (__hip_atomic_compare_exchange_strong(&s_gid(e), &expect, (u32)gid[j], __ATOMIC_RELAXED, __ATOMIC_RELAXED,
                                                             __HIP_MEMORY_SCOPE_WORKGROUP) || expect == (u32)gid[j])
                        break;
                }
                e = (e + 1) & (GROUP_LDS - 1);
            }
            entry[j] = (int)e;
            rank[j] = __hip_atomic_fetch_add(&s_cnt(e), 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        }
        __syncthreads();
        {
            // one device atomic per (tile, group) reserves the group's places; the eight entries a
            // thread looks at are handled side by side (a returning atomic takes microseconds)
            u32 g8[GROUP_LDS / 1024], c8[GROUP_LDS / 1024];
            i64 off8[GROUP_LDS / 1024];
            u64 cur8[GROUP_LDS / 1024];
#pragma unroll
            for (int q = 0; q < GROUP_LDS / 1024; ++q) {
                const u64 ent = s_ent[q * 1024 + tid];
                g8[q] = (u32)ent;
                c8[q] = (u32)(ent >> 32);
            }
#pragma unroll
            for (int q = 0; q < GROUP_LDS / 1024; ++q) {
                off8[q] = 0;
                cur8[q] = 0;
                if (g8[q] != ~0u) {
                    off8[q] = a.offsets[g8[q]];
                    cur8[q] = __hip_atomic_fetch_add(&a.cursor[g8[q]], (u64)c8[q], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                }
            }
#pragma unroll
            for (int q = 0; q < GROUP_LDS / 1024; ++q)
                if (g8[q] != ~0u) s_ent[q * 1024 + tid] = (u64)(off8[q] + (i64)cur8[q]);
        }
        __syncthreads();
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            if (entry[j] < 0) continue;
            const i64 dst = (i64)s_ent[entry[j]] + rank[j];
            // cached stores: the places of one (tile, group) are neighbours, L2 merges them
            // (non-temporal stores wrote 3.7 GB instead of 2.4 GB for 0.72 GB of values)
            switch (a.value_size) {
                case 1: ((unsigned char*)a.values_out)[dst] = (unsigned char)val[j]; break;
                case 4: ((u32*)a.values_out)[dst] = (u32)val[j]; break;
                default: ((u64*)a.values_out)[dst] = val[j]; break;
            }
        }
        __syncthreads();
        for (int q = tid; q < GROUP_LDS; q += 1024) s_ent[q] = 0xffffffffull;
        __syncthreads();
    }
#undef s_gid
#undef s_cnt
}

hipError_t launch_group_scatter(const GroupScatter& g, int blocks, hipStream_t stream) {
    group_scatter_kernel<<<dim3((unsigned)blocks), dim3(1024), 0, stream>>>(g);
    return hipGetLastError();
}

// Many groups: the kernel above pays one device atomic per (tile, group), and with a heavy-tailed
// key set nearly every pair of a rare group is alone in its tile - C5's zip codes: 5.5e7 atomics
// for 9e7 pairs, which is what its 2.3 ms were.  Two kernels instead:
//  * group_partition_kernel partitions the pairs by RANGES of 2^log_bucket consecutive groups (at
//    most 256 ranges; a range's pairs go to the same index range of the scratch arrays that its
//    values will occupy in the result, so the group offsets double as range boundaries): one
//    device atomic per (tile, range);
//  * group_place_kernel takes a range 8192 pairs at a time and moves every value into its
//    group's vector, counting per group in a directly indexed LDS array: one device atomic per
//    (chunk, group), with a few hundred groups per chunk instead of 1e5.
// The first sorts its 4096 pairs in LDS before it writes, so that consecutive threads store to
// consecutive addresses (runs of one range): 1.25 -> 1.1 ms; the same in the second kernel, whose
// runs are shorter, cost more than it saved (0.6 -> 0.8 ms).  Counting a work-group's whole share
// first, to reserve once per destination, was slower too: the second look-up of every key cost
// more than the atomics it saved (1.8 against 1.1 ms).
#define PART_CACHE 2048

// Groups of four pairs per thread: (key bits, live) -> group number or -1.  Which group a key
// belongs to is a probe of the dictionary's table plus a read of the slot's group number: two
// random 8- and 4-byte reads that each move a whole cache line to the CU.  The work-group
// remembers the groups of the keys it has looked up in a directly mapped LDS cache (no eviction:
// with a heavy-tailed key set the frequent keys get there first and then answer most lookups).
// An entry is claimed by writing its key; its group number follows, and until then reads of the
// entry count as misses.
__device__ __forceinline__ void groups_of_keys(const GroupScatter& a, bool narrow, u64* s_ck, u32* s_cg, const u64 (&kb)[4],
                                               const bool (&live)[4], int (&gid)[4]) {
    u32 ce[4];
    u64 first[4], ck[4];
    i64 slot[4];
    bool miss[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        ce[j] = cache_hash_slot(kb[j], PART_CACHE);
        ck[j] = __hip_atomic_load(&s_ck[ce[j]], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        gid[j] = -1;
        miss[j] = live[j];
        if (live[j] && ck[j] == kb[j] && kb[j] != kEmptyKey) {
            const u32 g = __hip_atomic_load(&s_cg[ce[j]], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
            if (g != ~0u) {
                gid[j] = (int)g;
                miss[j] = false;
            }
        }
    }
    if (narrow) {
        // Every key of the dictionary is the sign extension of its low half: the look-up reads ONE 8-byte
        // word per slot, the low half of the slot's key beside its group number (written at extraction), and a
        // table of 2^18 slots is 2 MB of such words instead of 2 MB of keys and 1 MB of numbers read one after
        // the other.  The four first reads of a thread are issued side by side (slot 0 where none is needed).
        u64 e[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            slot[j] = (i64)table_hash_slot(kb[j], (u32)a.slots);
            e[j] = a.kp32[miss[j] ? slot[j] : 0];
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            if (!miss[j]) continue;
            const u32 k32 = (u32)kb[j];
            int g = -1;
            if ((i64)kb[j] == (i64)(int)k32) {                   // (a wide key is in no such dictionary)
                u64 cur = e[j];
                i64 s = slot[j];
                for (i64 probe = 0; probe < a.slots; ++probe) {
                    const int pos = (int)(cur >> 32);
                    if (pos < 0) break;                          // a free slot (or an entry beyond the capacity): not there
                    if ((u32)cur == k32) { g = pos; break; }
                    s = (s + 1) & (a.slots - 1);
                    cur = a.kp32[s];
                }
            }
            gid[j] = g;
        }
    } else {
    // (requesting the home slot's group number together with its key, to save the second read its wait,
    // costs more in cache lines moved than it saves: 1.07 -> 1.17 ms)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        slot[j] = (i64)table_hash_slot(kb[j], (u32)a.slots);
        first[j] = miss[j] ? a.table_keys[slot[j]] : kEmptyKey;
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        if (!miss[j]) { slot[j] = -1; continue; }
        if (kb[j] == kEmptyKey) { slot[j] = a.hdr[1] ? a.slots : -1; continue; }
        if (first[j] == kb[j]) continue;
        i64 s = slot[j], found = -1;
        u64 cur = first[j];
        for (i64 probe = 1; probe < a.slots && cur != kEmptyKey; ++probe) {
            s = (s + 1) & (a.slots - 1);
            cur = a.table_keys[s];
            if (cur == kb[j]) { found = s; break; }
        }
        slot[j] = found;
    }
    // (the four group numbers are read side by side, from slot 0 where none is needed: behind a branch each
    // read would be waited for before the next is issued)
    int sp[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) sp[j] = a.slot_pos[miss[j] && slot[j] >= 0 ? slot[j] : 0];
#pragma unroll
    for (int j = 0; j < 4; ++j)
        if (miss[j]) gid[j] = slot[j] >= 0 ? sp[j] : -1;
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        if (!miss[j] || gid[j] < 0 || kb[j] == kEmptyKey || ck[j] != kEmptyKey) continue;
        u64 expect = kEmptyKey;
        if (__hip_atomic_compare_exchange_strong(&s_ck[ce[j]], &expect, kb[j], __ATOMIC_RELAXED, __ATOMIC_RELAXED,
                                                 __HIP_MEMORY_SCOPE_WORKGROUP))
            __hip_atomic_store(&s_cg[ce[j]], (u32)gid[j], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    }
#pragma unroll
    for (int j = 0; j < 4; ++j)
        if (gid[j] >= 0 && (gid[j] >> a.log_bucket) >= a.nbuckets) gid[j] = -1;     // (capacity error: not extracted)
}

// WIDE: one 8-byte key field and 8-byte values.  Their loads then stand in the code without a branch
// around them (a pair past the end re-reads the last one and is not used), which is what lets the next
// tile's loads stay in flight while this tile is ranked, sorted and stored: a load inside a branch -
// `if (i < npairs)`, or a switch over the field's size - is waited for at the end of that branch, and the
// eight loads of a thread then took eight memory round trips, one after the other, before anything else ran.
// WIDE == 4: the same with the key's low half in a 4-byte column.
template <int WIDE>
__global__ void __launch_bounds__(1024) group_partition_kernel(const GroupScatter a) {
    __shared__ u32 s_cnt[256];        // pairs of the tile per range
    __shared__ i64 s_cur[256];        // where the tile's pairs of a range go
    __shared__ u64 s_ck[PART_CACHE];
    __shared__ u32 s_cg[PART_CACHE];
    __shared__ u32 s_off[257];
    __shared__ u32 s_sg[GROUP_TILE];
    __shared__ u64 s_sv[GROUP_TILE];
    const int tid = threadIdx.x;
    const i64 npairs = (i64)*a.npairs;
    const i64 ntiles = (npairs + GROUP_TILE - 1) / GROUP_TILE;
    const bool narrow = a.kp32 && *a.kwide == 0;      // (uniform: every key of the dictionary fits 32 bits)
    if (tid < 256) s_cnt[tid] = 0;
    for (int q = tid; q < PART_CACHE; q += 1024) {
        s_ck[q] = kEmptyKey;
        s_cg[q] = ~0u;
    }
    __syncthreads();
    // the pairs of the work-group's next tile are loaded while this tile is ranked, sorted and stored
    u64 nval[4], nkb[4];
    auto load_tile = [&](i64 t) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const i64 i = t * GROUP_TILE + j * 1024 + tid;
            if (WIDE) {
                const i64 ic = i < npairs ? i : npairs - 1;
                if (WIDE == 4) nkb[j] = (u64)(i64)(int)__builtin_nontemporal_load((const u32*)a.key[0] + ic);
                else nkb[j] = __builtin_nontemporal_load((const u64*)a.key[0] + ic);
                nval[j] = __builtin_nontemporal_load((const u64*)a.value + ic);
            } else {
                nkb[j] = 0;
                nval[j] = 0;
                if (i < npairs) {
                    for (int k = 0; k < a.nkeys; ++k) nkb[j] |= load_bits(a.key[k], i, a.key_size[k]) << a.key_shift[k];
                    if (a.key_sext32) nkb[j] = (u64)(i64)(int)(u32)nkb[j];
                    nval[j] = load_bits(a.value, i, a.value_size);
                }
            }
        }
    };
    if ((i64)blockIdx.x < ntiles) load_tile(blockIdx.x);
    for (i64 t = blockIdx.x; t < ntiles; t += gridDim.x) {
        u32 rank[4];
        u64 val[4], kb[4];
        int gid[4];
        bool live[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            live[j] = t * GROUP_TILE + j * 1024 + tid < npairs;
            kb[j] = nkb[j];
            val[j] = nval[j];
        }
        // (the next tile's loads before this tile's look-ups, although the look-ups' answers then queue behind them:
        // with the look-ups first the kernel took 0.85 ms instead of 0.75)
        if (t + gridDim.x < ntiles) load_tile(t + gridDim.x);
        groups_of_keys(a, narrow, s_ck, s_cg, kb, live, gid);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            rank[j] = 0;
            if (gid[j] >= 0)
                rank[j] = __hip_atomic_fetch_add(&s_cnt[gid[j] >> a.log_bucket], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        }
        __syncthreads();
        if (tid < 64) {
            // exclusive prefix of the 256 counts: four per lane, then across the wavefront
            u32 c[4], mine = 0;
#pragma unroll
            for (int k = 0; k < 4; ++k) { c[k] = s_cnt[tid * 4 + k]; mine += c[k]; }
            u32 incl = mine;
            for (int o = 1; o < 64; o <<= 1) {
                const u32 up = __shfl_up(incl, o, 64);
                if (tid >= o) incl += up;
            }
            u32 run = incl - mine;
#pragma unroll
            for (int k = 0; k < 4; ++k) { s_off[tid * 4 + k] = run; run += c[k]; }
            if (tid == 63) s_off[256] = run;
        } else if (tid - 64 < a.nbuckets && s_cnt[tid - 64] != 0) {
            // one device atomic per (tile, range); a pair of the range exists, so its first group does
            const int b = tid - 64;
            s_cur[b] = a.offsets[(i64)b << a.log_bucket] +
                       (i64)__hip_atomic_fetch_add(&a.bcursor[b], (u64)s_cnt[b], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        __syncthreads();
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            if (gid[j] < 0) continue;
            const u32 p = s_off[gid[j] >> a.log_bucket] + rank[j];
            s_sg[p] = (u32)gid[j];
            s_sv[p] = val[j];
        }
        __syncthreads();
        const u32 placed = s_off[256];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const u32 p = j * 1024 + tid;
            if (p >= placed) continue;
            const u32 g = s_sg[p];
            const int b = (int)(g >> a.log_bucket);
            const i64 dst = s_cur[b] + (i64)(p - s_off[b]);
            if (dst < 0 || dst >= npairs) continue;     // only after a capacity error (sizes and pairs then disagree)
            a.tmp_group[dst] = (unsigned short)(g & (((u32)1 << a.log_bucket) - 1));      // (a range holds at most 4096 groups)
            a.tmp_value[dst] = s_sv[p];
        }
        __syncthreads();
        if (tid < 256) s_cnt[tid] = 0;
        __syncthreads();
    }
}

#define PLACE_CHUNK 8192
#define PLACE_MAX_BUCKET 4096
__global__ void __launch_bounds__(1024) group_place_kernel(const GroupScatter a) {
    __shared__ i64 s_first[257];                  // chunks before each range
    __shared__ i64 s_begin[257];                  // where each range's pairs begin in the scratch arrays (s_begin[b + 1]: where they end)
    __shared__ u32 s_cnt[PLACE_MAX_BUCKET];       // pairs of the chunk per group of the range
    __shared__ i64 s_base[PLACE_MAX_BUCKET];      // where they go
    const int tid = threadIdx.x;
    const i64 npairs = (i64)*a.npairs;
    i64 G = (i64)*a.ngroups;
    if (G > a.capacity) G = a.capacity;
    const i64 B = (i64)1 << a.log_bucket;
    // Where the ranges begin, read by 257 threads at once and kept (one thread reading them one after the
    // other was a hundred memory round trips in front of every work-group's first chunk, and read again
    // when a chunk is looked up they were a round trip of their own in front of every chunk's loads).
    if (tid <= 256) {
        const i64 b = tid < a.nbuckets ? tid : a.nbuckets;
        s_begin[tid] = a.offsets[b * B < G ? b * B : G];
    }
    __syncthreads();
    if (tid < 64) {
        // chunks before each range: exclusive prefix of the ranges' chunk counts, four ranges per lane
        i64 c[4], mine = 0;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            c[k] = (s_begin[tid * 4 + k + 1] - s_begin[tid * 4 + k] + PLACE_CHUNK - 1) / PLACE_CHUNK;
            mine += c[k];
        }
        i64 incl = mine;
        for (int o = 1; o < 64; o <<= 1) {
            const i64 up = __shfl_up(incl, o, 64);
            if (tid >= o) incl += up;
        }
        i64 run = incl - mine;
#pragma unroll
        for (int k = 0; k < 4; ++k) { s_first[tid * 4 + k] = run; run += c[k]; }
        if (tid == 63) s_first[256] = run;
    }
    for (int q = tid; q < PLACE_MAX_BUCKET; q += 1024) s_cnt[q] = 0;
    __syncthreads();
    const i64 total = s_first[256];
    // the chunk after this one is loaded while this one is counted and stored
    // (loads without a branch around them: a pair past the range's end re-reads the range's last one
    // and is marked in `ndead`, not by a value put in place of the load's, which would wait for the load)
    u32 ngrp[8];
    u64 nval[8];
    u32 ndead = 0;
    i64 n_lo = 0, n_hi = 0;
    auto load_chunk = [&](i64 w) {
        int b = 0;                                 // last range with s_first[b] <= w
        for (int step = 128; step > 0; step >>= 1)
            if (b + step < 256 && s_first[b + step] <= w) b += step;
        n_lo = (i64)b * B < G ? (i64)b * B : G;
        n_hi = (i64)(b + 1) * B < G ? (i64)(b + 1) * B : G;
        const i64 start = s_begin[b] + (w - s_first[b]) * PLACE_CHUNK;
        const i64 stop = s_begin[b + 1];
        ndead = 0;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const i64 i = start + j * 1024 + tid;
            ndead |= (i < stop ? 0u : 1u) << j;
            const i64 ic = i < stop ? i : stop - 1;        // (a chunk exists only where its range has pairs: start < stop)
            ngrp[j] = (u32)__builtin_nontemporal_load(a.tmp_group + ic);
            nval[j] = __builtin_nontemporal_load(a.tmp_value + ic);
        }
    };
    if ((i64)blockIdx.x < total) load_chunk(blockIdx.x);
    for (i64 w = blockIdx.x; w < total; w += gridDim.x) {
        const i64 lo_g = n_lo, hi_g = n_hi;
        u32 rank[8], local[8];
        u64 val[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            local[j] = (ndead >> j) & 1u ? ~0u : ngrp[j];
            val[j] = nval[j];
        }
        if (w + gridDim.x < total) load_chunk(w + gridDim.x);
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            rank[j] = 0;
            if (local[j] >= (u32)(hi_g - lo_g)) { local[j] = ~0u; continue; }   // (scratch left unwritten after a capacity error)
            rank[j] = __hip_atomic_fetch_add(&s_cnt[local[j]], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        }
        __syncthreads();
        for (int q = tid; q < (int)B; q += 1024) {
            const u32 c = s_cnt[q];
            if (c != 0)
                s_base[q] = a.offsets[lo_g + q] + (i64)__hip_atomic_fetch_add(&a.cursor[lo_g + q], (u64)c, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        __syncthreads();
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            if (local[j] == ~0u) continue;
            // the places of one (chunk, group) are neighbours: L2 merges these stores into lines
            const i64 dst = s_base[local[j]] + rank[j];
            if (dst < 0 || dst >= npairs) continue;
            switch (a.value_size) {
                case 1: ((unsigned char*)a.values_out)[dst] = (unsigned char)val[j]; break;
                case 4: ((u32*)a.values_out)[dst] = (u32)val[j]; break;
                default: ((u64*)a.values_out)[dst] = val[j]; break;
            }
        }
        __syncthreads();
        for (int q = tid; q < (int)B; q += 1024) s_cnt[q] = 0;
        __syncthreads();
    }
}

hipError_t launch_group_partition(const GroupScatter& g, int blocks, hipStream_t stream) {
    if (g.nbuckets < 1 || g.nbuckets > 256 || g.log_bucket < 0 || (1ll << g.log_bucket) > PLACE_MAX_BUCKET) return hipErrorInvalidValue;
    if (g.nkeys == 1 && g.key_size[0] == 8 && g.key_shift[0] == 0 && g.value_size == 8)
        group_partition_kernel<8><<<dim3((unsigned)blocks), dim3(1024), 0, stream>>>(g);
    else if (g.nkeys == 1 && g.key_sext32 && g.key_size[0] == 4 && g.key_shift[0] == 0 && g.value_size == 8)
        group_partition_kernel<4><<<dim3((unsigned)blocks), dim3(1024), 0, stream>>>(g);
    else
        group_partition_kernel<0><<<dim3((unsigned)blocks), dim3(1024), 0, stream>>>(g);
    return hipGetLastError();
}
hipError_t launch_group_place(const GroupScatter& g, int blocks, hipStream_t stream) {
    if (g.nbuckets < 1 || g.nbuckets > 256 || g.log_bucket < 0 || (1ll << g.log_bucket) > PLACE_MAX_BUCKET) return hipErrorInvalidValue;
    group_place_kernel<<<dim3((unsigned)blocks), dim3(1024), 0, stream>>>(g);
    return hipGetLastError();
}

// ---------------------------------------------------------------- nested loops
template <class T>
__global__ void __launch_bounds__(256) segments_check_kernel(const T* start, const T* end, i64 n_outer, i64 n_inner, int* err) {
    bool bad = false;
    for (i64 i = (i64)blockIdx.x * 256 + threadIdx.x; i < n_outer; i += (i64)gridDim.x * 256) {
        const i64 s = (i64)start[i], e = (i64)end[i];
        if (s < 0 || e < s || e > n_inner) bad = true;
        if (i == 0 && s != 0) bad = true;
        if (i == n_outer - 1 && e != n_inner) bad = true;
        if (i + 1 < n_outer && e != (i64)start[i + 1]) bad = true;
    }
    if (bad) atomicOr(err, 8);
}

hipError_t launch_segments_check(const void* start, const void* end, int is64, int64_t n_outer, int64_t n_inner,
                                 void* err, hipStream_t stream) {
    if (n_outer <= 0) return hipSuccess;
    int64_t blocks = (n_outer + 255) / 256;
    if (blocks > 2048) blocks = 2048;
    if (is64)
        segments_check_kernel<i64><<<dim3((unsigned)blocks), dim3(256), 0, stream>>>((const i64*)start, (const i64*)end, n_outer, n_inner, (int*)err);
    else
        segments_check_kernel<int><<<dim3((unsigned)blocks), dim3(256), 0, stream>>>((const int*)start, (const int*)end, n_outer, n_inner, (int*)err);
    return hipGetLastError();
}

// Ranges with strides, possibly overlapping or with gaps: outer element i visits start[i],
// start[i] + stride[i], ... below end[i], count[i] = ceil((end - start) / stride) inner elements.
// offsets[i] = count[0] + ... + count[i-1], offsets[n_outer] = the total, which is also written to
// *total (8 bytes of the control block, so that one copy brings it to the host with the error
// word).  One work-group: eight consecutive elements per thread and round, a work-group scan per
// round.  Raises bit 8 of *err for start < 0, end < start, end > n_inner or stride < 1.
template <class T>
__global__ void __launch_bounds__(1024) ranges_offsets_kernel(const T* start, const T* end, const T* stride, i64 n_outer,
                                                              i64 n_inner, i64* offsets, i64* total, int* err) {
    __shared__ i64 s_wave[16];
    __shared__ i64 s_carry;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    if (tid == 0) s_carry = 0;
    __syncthreads();
    bool bad = false;
    for (i64 base = 0; base < n_outer; base += 8192) {
        i64 cnt[8];
        i64 mine = 0;
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            const i64 r = base + (i64)tid * 8 + k;
            i64 c = 0;
            if (r < n_outer) {
                const i64 s = (i64)start[r], e = (i64)end[r], st = stride ? (i64)stride[r] : 1;
                if (s < 0 || e < s || e > n_inner || st < 1) bad = true;
                else c = (e - s + st - 1) / st;
            }
            cnt[k] = c;
            mine += c;
        }
        i64 incl = mine;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const i64 o = __shfl_up(incl, off, 64);
            if (lane >= off) incl += o;
        }
        if (lane == 63) s_wave[wave] = incl;
        __syncthreads();
        i64 before = s_carry;
        for (int w = 0; w < wave; ++w) before += s_wave[w];
        i64 run = before + incl - mine;
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            const i64 r = base + (i64)tid * 8 + k;
            if (r < n_outer) offsets[r] = run;
            run += cnt[k];
        }
        __syncthreads();
        if (tid == 1023) s_carry = run;
        __syncthreads();
    }
    if (tid == 0) {
        offsets[n_outer] = s_carry;
        *total = s_carry;
    }
    if (bad) atomicOr(err, 8);
}

hipError_t launch_ranges_offsets(const void* start, const void* end, const void* stride, int is64, int64_t n_outer,
                                 int64_t n_inner, void* offsets, void* total, void* err, hipStream_t stream) {
    if (is64)
        ranges_offsets_kernel<i64><<<dim3(1), dim3(1024), 0, stream>>>((const i64*)start, (const i64*)end, (const i64*)stride, n_outer,
                                                                      n_inner, (i64*)offsets, (i64*)total, (int*)err);
    else
        ranges_offsets_kernel<int><<<dim3(1), dim3(1024), 0, stream>>>((const int*)start, (const int*)end, (const int*)stride, n_outer,
                                                                      n_inner, (i64*)offsets, (i64*)total, (int*)err);
    return hipGetLastError();
}

template <class T>
__global__ void __launch_bounds__(256) tile_rows_kernel(const T* start, i64 n_outer, i64 tile, i64 ntiles, int* tile_row) {
    const i64 t = (i64)blockIdx.x * 256 + threadIdx.x;
    if (t > ntiles) return;
    if (t == ntiles) {
        tile_row[t] = (int)(n_outer - 1);
        return;
    }
    const i64 e0 = t * tile;
    i64 lo = 0, hi = n_outer;              // start[lo] <= e0 (start[0] == 0), "start[n_outer]" > e0
    while (hi - lo > 1) {
        const i64 mid = (lo + hi) >> 1;
        if ((i64)start[mid] <= e0) lo = mid; else hi = mid;
    }
    tile_row[t] = (int)lo;
}

hipError_t launch_tile_rows(const void* start, int is64, int64_t n_outer, int64_t tile, int64_t ntiles,
                            void* tile_row, hipStream_t stream) {
    if (n_outer <= 0) return hipSuccess;
    const int64_t blocks = (ntiles + 1 + 255) / 256;
    if (is64)
        tile_rows_kernel<i64><<<dim3((unsigned)blocks), dim3(256), 0, stream>>>((const i64*)start, n_outer, tile, ntiles, (int*)tile_row);
    else
        tile_rows_kernel<int><<<dim3((unsigned)blocks), dim3(256), 0, stream>>>((const int*)start, n_outer, tile, ntiles, (int*)tile_row);
    return hipGetLastError();
}

__global__ void or_error_kernel(u32* dst_ctl, const u32* src_ctl) {
    if (threadIdx.x == 0 && src_ctl[2]) atomicOr(dst_ctl + 2, src_ctl[2]);
}

hipError_t launch_or_error(void* dst_ctl, const void* src_ctl, hipStream_t stream) {
    or_error_kernel<<<dim3(1), dim3(64), 0, stream>>>((u32*)dst_ctl, (const u32*)src_ctl);
    return hipGetLastError();
}

// The call's 64 control words to the result handle's pinned host copy, written by a kernel: a
// device-to-host copy command of 256 bytes takes the copy engine's detour (about 10 us on the
// stream); `done`, the event the host waits for, is this dispatch's own end.
__global__ void ctl_to_host_kernel(const u32* ctl, u32* host) { host[threadIdx.x] = ctl[threadIdx.x]; }

hipError_t launch_ctl_to_host(const void* ctl, void* host, hipStream_t stream, hipEvent_t done) {
    hipExtLaunchKernelGGL(ctl_to_host_kernel, dim3(1), dim3(64), 0, stream, nullptr, done, 0, (const u32*)ctl, (u32*)host);
    return hipGetLastError();
}

// ---------------------------------------------------------------- probes
// Pure streaming read with 16-byte loads, in the shape the loop kernels read their columns in: a
// work-group takes contiguous 56 KB tiles round-robin and has a whole tile's loads (fourteen per
// thread) in flight before it uses the first; one work-group per compute unit is what that rate
// wants.  This is the attainable HBM read rate on the box.
#define PROBE_LOADS 14
__global__ void __launch_bounds__(256) probe_read_kernel(const u32x4* p, i64 n16, u64* checksum) {
    u32 a = 0, b = 0, c = 0, d = 0;
    const i64 tile = (i64)PROBE_LOADS * 256;
    const i64 ntiles = n16 / tile;
    for (i64 t = blockIdx.x; t < ntiles; t += gridDim.x) {
        u32x4 v[PROBE_LOADS];
#pragma unroll
        for (int j = 0; j < PROBE_LOADS; ++j) v[j] = __builtin_nontemporal_load(p + t * tile + j * 256 + threadIdx.x);
#pragma unroll
        for (int j = 0; j < PROBE_LOADS; ++j) { a += v[j].x; b += v[j].y; c += v[j].z; d += v[j].w; }
    }
    for (i64 i = ntiles * tile + (i64)blockIdx.x * 256 + threadIdx.x; i < n16; i += (i64)gridDim.x * 256) {
        const u32x4 v = __builtin_nontemporal_load(p + i);
        a += v.x; b += v.y; c += v.z; d += v.w;
    }
    u64 s = (u64)a + b + c + d;
    for (int off = 32; off > 0; off >>= 1) s += __shfl_xor(s, off, 64);
    if ((threadIdx.x & 63) == 0) atomicAdd(checksum, s);
}

hipError_t launch_probe_read(const void* data, int64_t bytes, void* checksum, int blocks, hipStream_t stream) {
    probe_read_kernel<<<dim3((unsigned)blocks), dim3(256), 0, stream>>>((const u32x4*)data, bytes / 16, (u64*)checksum);
    return hipGetLastError();
}

// Plain copy of known size: bytes read == bytes written == `bytes`.  One 16-byte vector per thread,
// streaming loads and stores, as many work-groups as that takes: the shape that moves the most on this
// part (6.4 TB/s of read + write; the same copy by eight resident work-groups per compute unit that walk
// the buffer moves 5.7, by one per unit 3.0 - what a one-to-one stream can reach depends on how many
// wavefronts have accesses in flight).
__global__ void __launch_bounds__(256) probe_copy_kernel(u32x4* dst, const u32x4* src, i64 n16) {
    const i64 i = (i64)blockIdx.x * 256 + threadIdx.x;
    if (i < n16) __builtin_nontemporal_store(__builtin_nontemporal_load(src + i), dst + i);
}

hipError_t launch_probe_copy(void* dst, const void* src, int64_t bytes, hipStream_t stream) {
    const i64 n16 = bytes / 16;
    if (n16 <= 0) return hipSuccess;
    if ((n16 + 255) / 256 > 0x7fffffffll) return hipErrorInvalidValue;
    probe_copy_kernel<<<dim3((unsigned)((n16 + 255) / 256)), dim3(256), 0, stream>>>((u32x4*)dst, (const u32x4*)src, n16);
    return hipGetLastError();
}

}  // namespace weld
