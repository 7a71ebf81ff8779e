// Device-side building blocks of the fused `for` loop kernels (gfx950, wave64).
//
// This text is compiled at run time together with a generated row function and
// kernel skeleton, once per distinct loop (the paper's backends also generate
// one fused kernel per program, Sec. 5 "Partial GPU Backend").  Everything in
// here is written for 64-wide wavefronts: ballots are 64-bit, a work-group is
// W_WAVES wavefronts, and each wavefront owns contiguous runs of rows so that
// one load instruction of a wavefront covers one contiguous 64*16-byte span.
//
// Macros the generated code defines before this text:
//   W_BLOCK  work-group size (multiple of 64)     W_V  rows per lane per load
//   W_U      loads in flight per lane and column  W_ALIGNED 1 = 16-byte loads legal
#define W_WAVES (W_BLOCK / 64)
#define W_UNIT (64 * W_V)            /* rows one wavefront covers with one load   */
#define W_WAVE_ROWS (W_UNIT * W_U)   /* contiguous rows owned by a wavefront      */
#define W_TILE (W_WAVE_ROWS * W_WAVES)

typedef unsigned long long u64;
typedef long long i64;
typedef unsigned int u32;

#define W_FUNC_ADD 0
#define W_FUNC_MUL 1
#define W_FUNC_MIN 2
#define W_FUNC_MAX 3

#define W_EMPTY_KEY 0x8000000000000000ull

// ---------------------------------------------------------------- column loader
template <class T, int V> struct wvec { T e[V]; };
template <int BYTES> struct w_carrier;
template <> struct w_carrier<1> { typedef unsigned char t; };
template <> struct w_carrier<2> { typedef unsigned short t; };
template <> struct w_carrier<4> { typedef unsigned int t; };
template <> struct w_carrier<8> { typedef unsigned long long t; };
template <> struct w_carrier<16> { typedef unsigned int t __attribute__((ext_vector_type(4))); };

// One lane reads V consecutive elements with a single wide load (16 bytes when
// sizeof(T)*V == 16); a wavefront thereby reads one contiguous span.
template <class T, int V>
__device__ __forceinline__ wvec<T, V> w_load(const T* __restrict__ p) {
    wvec<T, V> r;
#if W_ALIGNED
    if constexpr (sizeof(T) < 4 && sizeof(T) * V <= 16) {
        // vectors of one- and two-byte elements go through an integer of their size: as element
        // vectors they are loaded without the streaming hint, and such loads displace what
        // earlier kernels wrote from the memory-side cache, write-backs included
        typedef typename w_carrier<sizeof(T) * V>::t ct;
        const ct x = __builtin_nontemporal_load(reinterpret_cast<const ct*>(p));
        __builtin_memcpy(r.e, &x, sizeof(T) * V);
    } else {
        typedef T vt __attribute__((ext_vector_type(V)));
        const vt x = __builtin_nontemporal_load(reinterpret_cast<const vt*>(p));
#pragma unroll
        for (int k = 0; k < V; ++k) r.e[k] = x[k];
    }
#else
#pragma unroll
    for (int k = 0; k < V; ++k) r.e[k] = p[k];
#endif
    return r;
}

template <class T, int V>
__device__ __forceinline__ void w_store(T* __restrict__ p, const wvec<T, V>& v) {
#if W_ALIGNED
    if constexpr (sizeof(T) < 4 && sizeof(T) * V <= 16) {
        typedef typename w_carrier<sizeof(T) * V>::t ct;
        ct x;
        __builtin_memcpy(&x, v.e, sizeof(T) * V);
        __builtin_nontemporal_store(x, reinterpret_cast<ct*>(p));
    } else {
        typedef T vt __attribute__((ext_vector_type(V)));
        vt x;
#pragma unroll
        for (int k = 0; k < V; ++k) x[k] = v.e[k];
        __builtin_nontemporal_store(x, reinterpret_cast<vt*>(p));
    }
#else
#pragma unroll
    for (int k = 0; k < V; ++k) p[k] = v.e[k];
#endif
}

// ---------------------------------------------------------------- 8-bit products
// The product of two i8 values wraps to 8 bits; it is formed in a 32-bit register that the
// optimiser cannot see through.  Written as plain 8-bit arithmetic, the compiler merged the
// multiply with a following addition into a byte dot product (v_dot4_u32_u8) and got the addend
// wrong where it was the rounding term of a signed division or remainder: (x * x) % 2 of an i8
// column came out as 89.
__device__ __forceinline__ signed char w_mul_i8(signed char a, signed char b) {
    int r = (int)a * (int)b;
    asm("" : "+v"(r));
    return (signed char)r;
}

// ---------------------------------------------------------------- edge values
// Where the paper is silent, the library fixes (and its tests pin) one behaviour:
//   min / max of anything with a NaN is NaN (the operator and the merge function alike);
//   an integer x / 0 is 0 and x % 0 is 0; the most negative value over -1 wraps to itself, remainder 0;
//   a cast of f64 to an integer truncates, NaN gives 0, values beyond the 64-bit range its nearest end.
__device__ __forceinline__ double w_min_f64(double a, double b) {
    const double r = b < a ? b : a;
    return b != b ? b : r;                  // (a NaN in `a` is already what the compare leaves)
}
__device__ __forceinline__ double w_max_f64(double a, double b) {
    const double r = b > a ? b : a;
    return b != b ? b : r;
}
template <class T> __device__ __forceinline__ T w_div_int(T a, T b) {
    typedef typename w_carrier<sizeof(T)>::t U;
    if (b == 0) return 0;
    if (b == (T)-1) return (T)((U)0 - (U)a);
    return (T)(a / b);
}
template <class T> __device__ __forceinline__ T w_mod_int(T a, T b) {
    if (b == 0 || b == (T)-1) return 0;
    return (T)(a % b);
}
__device__ __forceinline__ i64 w_f64_to_i64(double x) {
    if (x != x) return 0;
    if (x >= 9223372036854775808.0) return 0x7fffffffffffffffll;
    if (x < -9223372036854775808.0) return (i64)0x8000000000000000ull;
    return (i64)x;
}

// ---------------------------------------------------------------- merge functions
template <int F> __device__ __forceinline__ double w_combine(double a, double b) {
    if (F == W_FUNC_ADD) return a + b;
    if (F == W_FUNC_MUL) return a * b;
    if (F == W_FUNC_MIN) return w_min_f64(a, b);
    return w_max_f64(a, b);
}
// integers wrap: sums and products go through the unsigned type
template <int F> __device__ __forceinline__ i64 w_combine(i64 a, i64 b) {
    if (F == W_FUNC_ADD) return (i64)((u64)a + (u64)b);
    if (F == W_FUNC_MUL) return (i64)((u64)a * (u64)b);
    if (F == W_FUNC_MIN) return b < a ? b : a;
    return b > a ? b : a;
}
template <int F> __device__ __forceinline__ double w_identity_f64() {
    if (F == W_FUNC_ADD) return 0.0;
    if (F == W_FUNC_MUL) return 1.0;
    if (F == W_FUNC_MIN) return __builtin_huge_val();
    return -__builtin_huge_val();
}
// identity of an integer merger whose declared width is BITS (accumulated in 64 bits)
template <int F, int BITS> __device__ __forceinline__ i64 w_identity_int() {
    if (F == W_FUNC_ADD) return 0;
    if (F == W_FUNC_MUL) return 1;
    if (F == W_FUNC_MIN) return (i64)((1ull << (BITS - 1)) - 1);
    return (i64)(~0ull << (BITS - 1));
}

// ---------------------------------------------------------------- erf
// The library's own erf for f64 (the device math library's costs about 100 vector
// instructions, two of them per row made the Black-Scholes loop compute bound): a degree-9
// Taylor polynomial per interval of width 1/16 on [0, 6), coefficients from a table that the
// build step computes in 80-digit arithmetic (paper_1709_06416_amd/erf_table.py: remainder
// below 4e-18; interval 0 is expanded about 0 and so keeps the relative accuracy of small
// arguments; 1 from 6 on, where erf has long rounded to 1).  The table is copied to LDS once
// per work-group: lanes index it with their own interval.
#ifdef W_USE_ERF
__device__ const double w_erf_table[960] = {
@W_ERF_TABLE@
};
__shared__ double w_erf_lds[960];
__device__ __forceinline__ void w_erf_init() {
    for (int q = threadIdx.x; q < 960; q += W_BLOCK) w_erf_lds[q] = w_erf_table[q];
    __syncthreads();
}
__device__ __forceinline__ double w_erf(double x) {
    const double a = __builtin_fabs(x);
    int k = (int)(a * 16.0);
    k = k > 95 ? 95 : k;
    const double c = k ? ((double)k + 0.5) * 0.0625 : 0.0;
    const double h = a - c;
    const double* t = w_erf_lds + k * 10;
    double p = t[9];
#pragma unroll
    for (int j = 8; j >= 0; --j) p = __builtin_fma(p, h, t[j]);
    p = a >= 6.0 ? 1.0 : p;
    return __builtin_copysign(p, x);
}
#endif

// ---------------------------------------------------------------- log, exp
// The library's own log and exp for f64 (the device math library's take about 94 and 38 vector
// instructions; these take about 40 and 30).  Tables and constants come from the build step
// (paper_1709_06416_amd/logexp_table.py, 80-digit arithmetic); both stay within about one unit
// in the last place of the correctly rounded result.
//   log: x = 2^e * m, m in [181/256, 362/256); per interval of width 1/128 the table holds R, the
//        double nearest the reciprocal of the interval's centre, and -ln R in two doubles;
//        r = fma(m, R, -1), log x = e ln2 - ln R + (r - r^2/2 + ... - r^8/8).  Around 1, R = 1:
//        r = m - 1 exactly, so the result keeps its relative accuracy there.
//   exp: n = rint(x * 64/ln2), r = x - n ln2/64 in two pieces, e^x = 2^(n>>6) * T[n&63] * e^r.
// Special values as the C library's: log(+-0) = -inf, log(x<0) = NaN, log(inf) = inf; exp
// overflows to inf and underflows through the denormals to 0; NaN in, NaN out.
#if defined(W_USE_LOG) || defined(W_USE_EXP)
@W_LOGEXP_CONSTS@
#endif
#ifdef W_USE_LOG
__device__ const double w_log_table[273] = {
@W_LOG_TABLE@
};
__shared__ double w_log_lds[273];
__device__ __forceinline__ void w_log_init() {
    for (int q = threadIdx.x; q < 273; q += W_BLOCK) w_log_lds[q] = w_log_table[q];
    __syncthreads();
}
__device__ __forceinline__ double w_log(double x) {
    double m = __builtin_amdgcn_frexp_mant(x);          // [0.5, 1); 0, inf and NaN come back as they are
    int e = __builtin_amdgcn_frexp_exp(x);
    const bool low = m < 0.70703125;                    // 181/256
    m = low ? m * 2.0 : m;
    e = low ? e - 1 : e;
    int i = (int)(m * 128.0) - 90;
    i = i < 0 ? 0 : (i > 90 ? 90 : i);                  // (only special values get clamped)
    const double* t = w_log_lds + 3 * i;
    const double r = __builtin_fma(m, t[0], -1.0);
    double p = W_LOG_C8;
    p = __builtin_fma(p, r, W_LOG_C7);
    p = __builtin_fma(p, r, W_LOG_C6);
    p = __builtin_fma(p, r, W_LOG_C5);
    p = __builtin_fma(p, r, W_LOG_C4);
    p = __builtin_fma(p, r, W_LOG_C3);
    p = __builtin_fma(p, r, W_LOG_C2);
    const double fe = (double)e;
    const double hi = __builtin_fma(fe, W_LN2_HI, t[1]);
    const double lo = __builtin_fma(fe, W_LN2_LO, t[2]);
    double res = hi + (r + __builtin_fma(p, r * r, lo));
    res = x < 0.0 ? __builtin_nan("") : res;
    res = x == 0.0 ? -__builtin_huge_val() : res;
    res = x == __builtin_huge_val() ? x : res;          // (the polynomial of an infinite r is inf - inf)
    return res;
}
#endif
#ifdef W_USE_EXP
__device__ const double w_exp_table[128] = {
@W_EXP_TABLE@
};
__shared__ double w_exp_lds[128];
__device__ __forceinline__ void w_exp_init() {
    for (int q = threadIdx.x; q < 128; q += W_BLOCK) w_exp_lds[q] = w_exp_table[q];
    __syncthreads();
}
__device__ __forceinline__ double w_exp(double x) {
    double xc = x < -1000.0 ? -1000.0 : x;              // keeps n inside an int; the result is 0 / inf either way
    xc = xc > 1000.0 ? 1000.0 : xc;
    const double fn = __builtin_rint(xc * W_INV_L64);
    const int n = (int)fn;
    double r = __builtin_fma(-fn, W_L64_HI, xc);
    r = __builtin_fma(-fn, W_L64_LO, r);
    const double* t = w_exp_lds + 2 * (n & 63);
    double p = W_EXP_C6;
    p = __builtin_fma(p, r, W_EXP_C5);
    p = __builtin_fma(p, r, W_EXP_C4);
    p = __builtin_fma(p, r, W_EXP_C3);
    p = __builtin_fma(p, r, W_EXP_C2);
    p = __builtin_fma(p, r * r, r);                     // e^r - 1
    const double s = t[0] + __builtin_fma(t[0], p, t[1]);
    const double res = __builtin_ldexp(s, n >> 6);
    return x != x ? x : res;
}
#endif

// ---------------------------------------------------------------- lookup
// lookup(v, ix) of a nested loop's inner body: an index outside the vector raises error
// bit 4 (the call then fails) and yields 0 instead of reading out of bounds.
template <class T>
__device__ __forceinline__ T w_lookup(const T* __restrict__ v, i64 len, i64 ix, int* err) {
    if ((u64)ix < (u64)len) return v[ix];
    atomicOr(err, 4);
    return (T)0;
}

// ---------------------------------------------------------------- wavefront level
__device__ __forceinline__ int w_lane() {
    return (int)__builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u));
}
// number of set bits of a 64-bit ballot below this lane
__device__ __forceinline__ int w_rank_below(u64 ballot) {
    return (int)__builtin_amdgcn_mbcnt_hi((u32)(ballot >> 32),
                                          __builtin_amdgcn_mbcnt_lo((u32)ballot, 0u));
}
__device__ __forceinline__ u64 w_ballot(bool p) { return __builtin_amdgcn_ballot_w64(p); }

// butterfly reduction over the 64 lanes; every lane ends with the same value, and
// the combination order is fixed, so the result does not depend on scheduling
// Sum of an int over the 64 lanes of the wavefront, returned to all of them (data-parallel-primitive
// adds inside the 16-lane rows, then the rows' last lanes are passed on: no LDS traffic).
__device__ __forceinline__ int w_wave_sum(int v) {
    v += __builtin_amdgcn_update_dpp(0, v, 0x111, 0xf, 0xf, true);   // lane - 1 of the row
    v += __builtin_amdgcn_update_dpp(0, v, 0x112, 0xf, 0xf, true);   // lane - 2
    v += __builtin_amdgcn_update_dpp(0, v, 0x114, 0xf, 0xf, true);   // lane - 4
    v += __builtin_amdgcn_update_dpp(0, v, 0x118, 0xf, 0xf, true);   // lane - 8: lane 15 of a row holds the row's sum
    v += __builtin_amdgcn_update_dpp(0, v, 0x142, 0xa, 0xf, true);   // rows 1 and 3 add lane 15 of the row before
    v += __builtin_amdgcn_update_dpp(0, v, 0x143, 0xc, 0xf, true);   // rows 2 and 3 add lane 31
    return __builtin_amdgcn_readlane(v, 63);
}

template <int F, class T> __device__ __forceinline__ T w_wave_reduce(T v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v = w_combine<F>(v, __shfl_xor(v, off, 64));
    return v;
}

// work-group reduction: wavefront butterfly, then W_WAVES partials through LDS,
// combined in wavefront order.  `scratch` has W_WAVES slots.  All threads call it;
// all threads return the total.
template <int F, class T>
__device__ __forceinline__ T w_block_reduce(T v, T* scratch, T ident) {
    v = w_wave_reduce<F>(v);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) scratch[threadIdx.x >> 6] = v;
    __syncthreads();
    T r = ident;
#pragma unroll
    for (int w = 0; w < W_WAVES; ++w) r = w_combine<F>(r, scratch[w]);
    return r;
}

// ---------------------------------------------------------------- device-scope access
// The eight XCDs have separate L2s: words other work-groups must see are read and
// written with agent-scope atomics.
__device__ __forceinline__ u64 w_ld_agent(const u64* p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void w_st_agent(u64* p, u64 v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// ---------------------------------------------------------------- merger finish
// Every work-group stores one partial per merger (index = its work-group id).  A
// small second kernel combines the partials in index order, so the result does not
// depend on the order in which work-groups ran, and no cross-XCD release/acquire
// fence is needed inside the loop kernel (such a fence writes back and invalidates
// the whole L2 of the XCD: measured at about 0.25 us per work-group, serialised).
template <class T> __device__ __forceinline__ void w_store_partial(u64* partial, T v) {
    u64 bits;
    __builtin_memcpy(&bits, &v, 8);
    partial[blockIdx.x] = bits;
}

// Single-launch form: the loop kernel combines the partials itself.  A partial is exchanged into its
// slot at device scope (performed once the old value is back), a work-group counts itself in after
// every one of its wavefronts has had its device-scope writes acknowledged, and the work-group that
// finds all others counted reads the partials back at device scope: nothing here relies on one
// XCD's L2 being written back or another's being invalidated.
template <class T> __device__ __forceinline__ void w_publish_partial(u64* partial, T v) {
    u64 bits;
    __builtin_memcpy(&bits, &v, 8);
    const u64 old = __hip_atomic_exchange(partial + blockIdx.x, bits, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    asm volatile("" ::"v"(old));
}
// True in every thread of the work-group that finishes last.  All threads call it.  Additions to one
// word are performed one after the other (about 15 ns apiece: 7 us for 500 work-groups), so a
// work-group counts itself in at one of up to 32 leaves (word 16 * (1 + leaf): a cache line each), and
// only the last one at a leaf - which puts the leaf back to zero - goes on to the root (word 0).
__device__ __forceinline__ bool w_arrive_last(u32* arrive) {
    __shared__ u32 s_last;
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (threadIdx.x == 0) {
        const u32 leaves = gridDim.x < 32u ? gridDim.x : 32u;
        const u32 leaf = blockIdx.x % leaves;
        const u32 members = (gridDim.x - leaf + leaves - 1u) / leaves;
        u32* const cell = arrive + 16u * (1u + leaf);
        u32 last = 0;
        if (__hip_atomic_fetch_add(cell, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == members - 1u) {
            __hip_atomic_store(cell, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            last = __hip_atomic_fetch_add(arrive, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == leaves - 1u ? 1u : 0u;
        }
        s_last = last;
    }
    __syncthreads();
    return s_last != 0;
}
// Thread j folds partials j, j + W_BLOCK, ... in that order, then the work-group's fixed reduction:
// the result is the same on every run, whichever work-group does it.
template <int F, class T> __device__ __forceinline__ T w_fold_partials(const u64* partial, u32 count, T* scratch, T ident) {
    T v = ident;
    for (u32 i = threadIdx.x; i < count; i += W_BLOCK) {
        const u64 bits = w_ld_agent(partial + i);
        T x;
        __builtin_memcpy(&x, &bits, 8);
        v = w_combine<F>(v, x);
    }
    return w_block_reduce<F>(v, scratch, ident);
}
// The call's status words (64 of them; word 2 = the error bits collected in arrive[2]), written whole,
// and the arrival words back to zero for the next call that uses them.
__device__ __forceinline__ void w_finish_status(u32* ctl, u32* arrive) {
    if (threadIdx.x < 64) {
        const u32 e = __hip_atomic_load(arrive + 2, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        ctl[threadIdx.x] = threadIdx.x == 2 ? e : 0u;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        __hip_atomic_store(arrive, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_store(arrive + 2, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
}

// ---------------------------------------------------------------- vecbuilder scan
// Decoupled look-back over tile descriptors: bits 63..62 = state, 61..0 = count.
//   0 = not yet published, 1 = this tile's own count, 2 = inclusive prefix.
// Tiles are numbered by an atomic ticket in the order they START, so a tile only
// ever waits for tiles that are already running.  Called by the 64 lanes of one
// wavefront.  Returns the number of elements appended by all earlier tiles.
// The wait is bounded: after `spin_limit` polls without progress the error flag is
// raised and 0 is returned (writes then stay inside the output, the call reports
// a device error), so the kernel always terminates.
#define W_DESC_AGG (1ull << 62)
#define W_DESC_PFX (2ull << 62)
#define W_DESC_VAL ((1ull << 62) - 1)

__device__ __forceinline__ i64 w_lookback(u64* desc, i64 tile, i64 own, i64 spin_limit, int* err) {
    const int lane = w_lane();
    if (tile == 0) {
        if (lane == 0) w_st_agent(desc, W_DESC_PFX | (u64)own);
        return 0;
    }
    if (lane == 0) w_st_agent(desc + tile, W_DESC_AGG | (u64)own);
    i64 excl = 0;
    i64 j = tile - 1;                       // nearest predecessor of the current window
    i64 spins = 0;
    bool failed = false;
    for (;;) {
        const i64 idx = j - lane;
        const u64 d = idx >= 0 ? w_ld_agent(desc + idx) : W_DESC_PFX;
        const u32 state = (u32)(d >> 62);
        const u64 unpublished = w_ballot(state == 0);
        const u64 have_prefix = w_ballot(state == 2);
        const int first = have_prefix ? (int)__builtin_ctzll(have_prefix) : 64;
        const u64 need = first >= 63 ? ~0ull : ((2ull << first) - 1);
        if (unpublished & need) {
            if (++spins > spin_limit) { failed = true; break; }
            __builtin_amdgcn_s_sleep(2);
            continue;
        }
        const i64 mine = (lane <= first) ? (i64)(d & W_DESC_VAL) : 0;
        excl += w_wave_reduce<W_FUNC_ADD>(mine);
        if (first < 64) break;
        j -= 64;
    }
    if (failed) {
        if (lane == 0) atomicOr(err, 2);
        excl = 0;
    }
    if (lane == 0) w_st_agent(desc + tile, W_DESC_PFX | (u64)(excl + own));
    return excl;
}

// The same look-back in two steps, for loops that overlap tiles: a tile publishes its own count as
// soon as it is known and collects the sum of its predecessors later (after its merges), when the
// tiles in front have had time to publish theirs.  Called by one whole wavefront each.
__device__ __forceinline__ void w_lookback_publish(u64* desc, i64 tile, i64 own) {
    if (w_lane() == 0) w_st_agent(desc + tile, (tile == 0 ? W_DESC_PFX : W_DESC_AGG) | (u64)own);
}
__device__ __forceinline__ i64 w_lookback_resolve(u64* desc, i64 tile, i64 own, i64 spin_limit, int* err) {
    const int lane = w_lane();
    if (tile == 0) return 0;
    i64 excl = 0;
    i64 j = tile - 1;
    i64 spins = 0;
    bool failed = false;
    for (;;) {
        const i64 idx = j - lane;
        const u64 d = idx >= 0 ? w_ld_agent(desc + idx) : W_DESC_PFX;
        const u32 state = (u32)(d >> 62);
        const u64 unpublished = w_ballot(state == 0);
        const u64 have_prefix = w_ballot(state == 2);
        const int first = have_prefix ? (int)__builtin_ctzll(have_prefix) : 64;
        const u64 need = first >= 63 ? ~0ull : ((2ull << first) - 1);
        if (unpublished & need) {
            if (++spins > spin_limit) { failed = true; break; }
            __builtin_amdgcn_s_sleep(2);
            continue;
        }
        const i64 mine = (lane <= first) ? (i64)(d & W_DESC_VAL) : 0;
        excl += w_wave_reduce<W_FUNC_ADD>(mine);
        if (first < 64) break;
        j -= 64;
    }
    if (failed) {
        if (lane == 0) atomicOr(err, 2);
        excl = 0;
    }
    if (lane == 0) w_st_agent(desc + tile, W_DESC_PFX | (u64)(excl + own));
    return excl;
}

// ---------------------------------------------------------------- atomics on builders
template <int F> __device__ __forceinline__ void w_atomic_f64(double* p, double v, const int scope_agent) {
    if (F == W_FUNC_ADD) {
        if (scope_agent) __hip_atomic_fetch_add(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        else __hip_atomic_fetch_add(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    } else {
        u64* q = reinterpret_cast<u64*>(p);
        u64 old = scope_agent ? __hip_atomic_load(q, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)
                              : __hip_atomic_load(q, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        for (;;) {
            double cur;
            __builtin_memcpy(&cur, &old, 8);
            const double nxt = w_combine<F>(cur, v);
            u64 nb;
            __builtin_memcpy(&nb, &nxt, 8);
            if (nb == old) break;
            const bool ok = scope_agent
                ? __hip_atomic_compare_exchange_strong(q, &old, nb, __ATOMIC_RELAXED, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)
                : __hip_atomic_compare_exchange_strong(q, &old, nb, __ATOMIC_RELAXED, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
            if (ok) break;
        }
    }
}
template <int F> __device__ __forceinline__ void w_atomic_i64(i64* p, i64 v, const int scope_agent) {
    if (F == W_FUNC_ADD) {
        if (scope_agent) __hip_atomic_fetch_add(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        else __hip_atomic_fetch_add(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    } else if (F == W_FUNC_MIN) {
        if (scope_agent) __hip_atomic_fetch_min(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        else __hip_atomic_fetch_min(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    } else if (F == W_FUNC_MAX) {
        if (scope_agent) __hip_atomic_fetch_max(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        else __hip_atomic_fetch_max(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    } else {
        i64 old = scope_agent ? __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)
                              : __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        for (;;) {
            const i64 nxt = (i64)((u64)old * (u64)v);
            const bool ok = scope_agent
                ? __hip_atomic_compare_exchange_strong(p, &old, nxt, __ATOMIC_RELAXED, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)
                : __hip_atomic_compare_exchange_strong(p, &old, nxt, __ATOMIC_RELAXED, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
            if (ok) break;
        }
    }
}
template <int F> __device__ __forceinline__ void w_atomic(double* p, double v, const int agent) { w_atomic_f64<F>(p, v, agent); }
template <int F> __device__ __forceinline__ void w_atomic(i64* p, i64 v, const int agent) { w_atomic_i64<F>(p, v, agent); }

// A merge of a queued vecmerger that found its segment full (skewed indices: a hot cell fills its range's segment
// many times over).  Straight to the result it would be one device atomic per merge on the hot cell's address,
// about 12 ns each and serialised; instead the work-group combines such merges in a small directly mapped LDS
// table (tag = the cell's index, W_VQ_NONE where free; the values start at the identity) and sends every
// occupied entry to the result once, at its end.  An index that finds four entries in a row taken by others goes
// straight to the result (with one entry to try, a cell with 2 % of all merges lost its entry to a neighbour of
// its range in one work-group in nine, and those work-groups' device atomics on its address tripled the time).
#define W_VQ_OVERFLOW 1024
#define W_VQ_NONE 0xffffffffu
template <int F, class T>
__device__ __forceinline__ void w_vecm_overflow(u32* tags, T* vals, u32 ix, T v, T* out) {
    const u32 home = (ix * 0x9e3779b1u) >> 22;
#pragma unroll 1
    for (u32 probe = 0; probe < 4; ++probe) {
        const u32 h = (home + probe) & (W_VQ_OVERFLOW - 1);
        u32 cur = __hip_atomic_load(tags + h, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        if (cur == W_VQ_NONE) {
            u32 expect = W_VQ_NONE;
            cur = __hip_atomic_compare_exchange_strong(tags + h, &expect, ix, __ATOMIC_RELAXED, __ATOMIC_RELAXED,
                                                       __HIP_MEMORY_SCOPE_WORKGROUP) ? ix : expect;
        }
        if (cur == ix) {
            w_atomic<F>(vals + h, v, 0);
            return;
        }
    }
    w_atomic<F>(out + ix, v, 1);
}

// ---------------------------------------------------------------- division by a constant
// x / D and x % D for a 64-bit x and a compile-time D in [2, 2^31): the compiler turns them
// into a 64 x 64 -> 128-bit multiplication (ten quarter-rate 32-bit multiplications with the
// correction); when every lane of the wavefront holds 0 <= x < 2^32 - columns of codes, dates
// and identifiers mostly do - a 32-bit one does.  `live` = the row needs the result at all:
// the other lanes do not force the long path.  CONV = all 64 lanes make the call together;
// the wavefront-wide decision is only taken then.  In the guarded code of a ragged tile, where
// lanes past the end sit out, the long form is used: with the ballot-controlled branch nested
// in that divergent code, merges of LATER statements lost lanes (seen on the GPU; both
// branches return the same value, so the source gave no reason for it).
template <i64 D, bool CONV> __device__ __forceinline__ i64 w_div_const(i64 x, bool live) {
    if (CONV) {
        if (!live) x = 0;
        if (__builtin_expect(w_ballot((u64)x >> 32 != 0) == 0, 1)) return (i64)((u32)x / (u32)D);
    }
    return x / D;
}
template <i64 D, bool CONV> __device__ __forceinline__ i64 w_mod_const(i64 x, bool live) {
    if (CONV) {
        if (!live) x = 0;
        if (__builtin_expect(w_ballot((u64)x >> 32 != 0) == 0, 1)) return (i64)((u32)x % (u32)D);
    }
    return x % D;
}

// ---------------------------------------------------------------- hash tables
// 32-bit multiplicative (Fibonacci) hash of the folded key: a handful of 32-bit
// instructions; callers take the HIGH bits (w_hash(k) >> (32 - log2 slots)).
__device__ __forceinline__ u32 w_hash(u64 k) {
    const u32 x = (u32)k ^ ((u32)(k >> 32) * 0x85ebca6bu);
    return x * 0x9e3779b1u;
}
__device__ __forceinline__ u32 w_hash_slot(u64 k, u32 slots) {   // slots is a power of two >= 2
    return w_hash(k) >> (__builtin_clz(slots) + 1);
}
// Second hash (admission filter bits, spill partition), all of whose bits depend on all of
// w_hash's: given the high bits that pick a table slot, it still takes every value.  One more
// 32-bit multiplication - these run at a quarter of the rate of other vector instructions,
// which is what the loops over large dictionaries are bound by.
__device__ __forceinline__ u32 w_hash2(u64 k) {
    u32 h = w_hash(k);
    h ^= h >> 15;
    h *= 0x2c1b3c6du;
    return h ^ (h >> 13);
}
// Home slot in a GLOBAL table (every dictionary's final table, and the tables other loops probe).
// Tables of 2^21 slots and more lie beyond every cache, and each step of a probe is a trip to
// memory: they take the second hash.  Under one multiplication, keys with a stride keep enough
// structure to stack on few slots - order numbers times four, 4e6 of them in 2^23 slots: 3.3 keys
// per occupied home slot, and 70 % of all inserts and lookups find another key there first; a random
// function gives 1.26 and 21 %, and so does the second hash for strides 1 to 1024.  Smaller tables
// (their probes stay in the L2) and the LDS tables keep the single multiplication: multiplications
// run at a quarter of the rate, and the kernels that look keys up in such tables are bound by the
// instructions they issue (groupbuilder's partition step: 1.03 -> 1.26 ms with the second hash).
// Which hash a table uses follows from its size alone, so everything that probes it agrees.
__device__ __forceinline__ u32 w_table_hash_slot(u64 k, u32 slots) {   // slots is a power of two >= 2
    u32 h = w_hash(k);
    if (slots >= (1u << 21)) {
        asm volatile("");                  // (keeps the branch: slots is uniform, and both sides computed cost the multiplication)
        h ^= h >> 15;
        h *= 0x2c1b3c6du;
        h ^= h >> 13;
    }
    return h >> (__builtin_clz(slots) + 1);
}

// Global open-addressing table (linear probing, power-of-two slot count, keys packed
// into 64 bits, W_EMPTY_KEY marks a free slot).  The one key whose packed bits equal
// the marker lives in the extra slot `slots` and is flagged in hdr[1].
// Returns the slot, or -1 (and raises the capacity error) if the table is full.
__device__ __forceinline__ i64 w_table_slot(u64* keys, u32* hdr, i64 slots, u64 kbits, int* err) {
    if (kbits == W_EMPTY_KEY) {
        __hip_atomic_store(hdr + 1, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        return slots;
    }
    const i64 mask = slots - 1;
    i64 s = (i64)w_table_hash_slot(kbits, (u32)slots);
    for (i64 probe = 0; probe < slots; ++probe) {
        // a key cell changes once, from the marker to its key: a cached copy that already
        // shows the key is final, and a stale marker is resolved by the compare-and-swap
        u64 cur = keys[s];
        if (cur == kbits) return s;
        if (cur == W_EMPTY_KEY) {
            u64 expect = W_EMPTY_KEY;
            if (__hip_atomic_compare_exchange_strong(keys + s, &expect, kbits, __ATOMIC_RELAXED,
                                                     __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT))
                return s;
            if (expect == kbits) return s;
        }
        s = (s + 1) & mask;
    }
    atomicOr(err, 1);
    return -1;
}

// Read-only probe of a table that an earlier loop built (the probe side of a hash join):
// the slot of `kbits`, or -1 if the key is absent.
// `live` = the row needs the answer at all.  The first probe is a load that EVERY row issues
// (rows that do not need it read slot 0, one cached line for the whole wavefront), so that
// the loads of the rows a lane holds are independent straight-line code and go out together;
// behind a branch per row each would wait for the one before (a selective join's probe: 0.39 ->
// 0.3 ms).  Only a key that does not sit in its home slot walks on, in a loop of its own.
__device__ __forceinline__ i64 w_table_find(const u64* __restrict__ keys, const u32* __restrict__ hdr, i64 slots, u64 kbits,
                                            bool live) {
    const i64 mask = slots - 1;
    const i64 home = live ? (i64)w_table_hash_slot(kbits, (u32)slots) : 0;
    const u64 first = keys[home];
    if (!live) return -1;
    if (kbits == W_EMPTY_KEY) return hdr[1] ? slots : -1;
    if (first == kbits) return home;
    if (first == W_EMPTY_KEY) return -1;
    i64 s = (home + 1) & mask;
    for (i64 probe = 1; probe < slots; ++probe) {
        const u64 cur = keys[s];
        if (cur == kbits) return s;
        if (cur == W_EMPTY_KEY) return -1;
        s = (s + 1) & mask;
    }
    return -1;
}
// one field of the value struct found there (cells are 8 bytes: i64 or double accumulators); again a
// load that every row issues (slot 0 when there is nothing to fetch)
template <class T, class A>
__device__ __forceinline__ T w_table_value(const A* __restrict__ cells, i64 slot) {
    const A cell = cells[slot >= 0 ? slot : 0];
    return slot >= 0 ? (T)cell : (T)0;
}

// Work-group private table in LDS: same scheme, at most `max_probe` probes; -1 means
// "no room here", and the caller sends that merge to the global table instead.
__device__ __forceinline__ int w_lds_slot(u64* keys, int slots, u64 kbits, int max_probe) {
    if (kbits == W_EMPTY_KEY) return -1;
    const int mask = slots - 1;
    int s = (int)w_hash_slot(kbits, (u32)slots);
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

// Same, with an admission filter for key sets much larger than the table: a key may take a
// free slot only the second time this work-group sees it (a bit per hashed key in `door`
// remembers the first time).  Keys that occur once per work-group - most of a heavy-tailed
// key set - then never occupy slots that the frequent keys need.
__device__ __forceinline__ int w_lds_slot_filtered(u64* keys, int slots, u64 kbits, int max_probe,
                                                   u32* door, u32 door_words) {
    if (kbits == W_EMPTY_KEY) return -1;
    const int mask = slots - 1;
    int s = (int)w_hash_slot(kbits, (u32)slots);
    for (int probe = 0; probe < max_probe; ++probe) {
        u64 cur = __hip_atomic_load(keys + s, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        if (cur == kbits) return s;
        if (cur == W_EMPTY_KEY) {
            const u32 h2 = w_hash2(kbits);
            const u32 bit = 1u << (h2 & 31);
            const u32 seen = __hip_atomic_fetch_or(door + ((h2 >> 5) & (door_words - 1)), bit, __ATOMIC_RELAXED,
                                                   __HIP_MEMORY_SCOPE_WORKGROUP);
            if (!(seen & bit)) return -1;
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

// Compact cells: a dictmerger[K,V,+] whose packed key is the zero or sign extension of its low 32
// bits and whose single value is a 32-bit partial sum keeps a 4-byte key and a 4-byte sum per slot
// (two arrays, so that the 64 lanes of an access spread over all banks): the same LDS holds twice
// the slots of the general table, and the entries that leave through the spill queues are 8 bytes
// instead of 16.  W_EMPTY_KEY32 marks a free slot; the one key with those low bits never enters the
// table (its merges take the miss path).  The slot hash is private to the table: one multiplication.
// (Tried and dropped: buckets of four slots read with one 16-byte load, rows whose bucket is full going
// straight to the spill queue - the wide random LDS reads cost more than the probe sequence saved.)
#define W_EMPTY_KEY32 0x80000000u
__device__ __forceinline__ u32 w_hash_slot32(u32 k, u32 slots) {
    return (k * 0x9e3779b1u) >> (__builtin_clz(slots) + 1);
}
__device__ __forceinline__ u64 w_compact_entry(u64 kbits, i64 v) {
    return (u64)(u32)kbits | ((u64)(u32)v << 32);
}
// The slots of the probe sequence (at most four) are read side by side, one LDS round trip instead of one per step;
// what was read may be out of date by the time it is looked at, which only matters for a slot read as free, and that
// one is taken by compare-and-swap, which tells (a slot once occupied keeps its key: nothing is ever deleted).
__device__ __forceinline__ int w_lds_slot32(u32* keys, int slots, u64 kbits, int max_probe) {
    const u32 k = (u32)kbits;
    if (k == W_EMPTY_KEY32) return -1;
    const int mask = slots - 1;
    const int s0 = (int)w_hash_slot32(k, (u32)slots);
    u32 cur[4];
#pragma unroll
    for (int probe = 0; probe < 4; ++probe)
        cur[probe] = __hip_atomic_load(keys + ((s0 + (probe < max_probe ? probe : 0)) & mask), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
#pragma unroll
    for (int probe = 0; probe < 4; ++probe) {
        if (probe >= max_probe) break;
        const int s = (s0 + probe) & mask;
        if (cur[probe] == k) return s;
        if (cur[probe] == W_EMPTY_KEY32) {
            u32 expect = W_EMPTY_KEY32;
            if (__hip_atomic_compare_exchange_strong(keys + s, &expect, k, __ATOMIC_RELAXED,
                                                     __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP))
                return s;
            if (expect == k) return s;
        }
    }
    return -1;
}
__device__ __forceinline__ void w_lds_add32(u32* vals, int slot, i64 v) {
    __hip_atomic_fetch_add(vals + slot, (u32)v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
}

// Spill queues of a large dictionary.  A merge that found no room in the LDS table is
// appended to segment [work-group][partition] of a log in global memory instead of
// going to the global table with device atomics; the partition is taken from a hash that
// is independent of the table hashes.  `qn` are the work-group's W_SPILL_PARTS segment
// lengths (LDS), `cap` the entries a segment holds, `words` = 1 + value fields.  Returns
// the word offset of the entry in the log (key word first), or -1 if the segment is full:
// the caller then falls back to the global table.  A second kernel aggregates partition by
// partition in LDS.
// With W_SPILL_BY_SLOT the partition is instead the slice of the global table that the key's
// home slot lies in (W_SPILL_PARTS slices, up to 4096): dictionaries of millions of keys, whose
// table a second kernel then builds slice by slice in LDS.
#ifndef W_SPILL_PARTS
#define W_SPILL_PARTS 256
#endif
__device__ __forceinline__ u32 w_spill_part(u64 kbits) {
#ifdef W_SPILL_BY_SLOT
    // the slice of the table the key's home slot lies in (slices of 2^W_SPILL_SLICE_BITS slots)
    return w_table_hash_slot(kbits, (u32)W_SPILL_PARTS << W_SPILL_SLICE_BITS) >> W_SPILL_SLICE_BITS;
#else
    return w_hash2(kbits) >> 24;
#endif
}
__device__ __forceinline__ i64 w_spill_entry(u32 part, u32 pos, i64 cap, int words);
__device__ __forceinline__ i64 w_spill_index(u32* qn, i64 cap, int words, u64 kbits) {
    const u32 part = w_spill_part(kbits);
    const u32 pos = __hip_atomic_fetch_add(qn + part, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    return w_spill_entry(part, pos, cap, words);
}
// word offset of entry `pos` of this work-group's segment of partition `part`, -1 past the segment's end
__device__ __forceinline__ i64 w_spill_entry(u32 part, u32 pos, i64 cap, int words) {
    if (pos >= (u32)cap) return -1;
#ifdef W_SPILL_BY_SLOT
    const u64 local = (u64)part * (u64)(u32)cap + pos;
#else
    // cap < 2^23 (the host sees to it): the entry's index inside the work-group's block of
    // segments fits 32 bits and takes a 24-bit multiplication; the block's base is scalar
    const u64 local = __umul24(part, (u32)cap) + pos;
#endif
    return (i64)(((u64)blockIdx.x * W_SPILL_PARTS * (u64)cap + local) * (u64)words);
}
// Stores to device memory that say so (a pointer that went through a select or a helper is
// otherwise stored through with flat instructions, which also count as LDS operations and
// make every later wait on LDS wait for memory as well).
typedef u64 w_u64x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ void w_gstore1(u64* p, u64 x) {
    *(__attribute__((address_space(1))) u64*)p = x;
}
__device__ __forceinline__ void w_gstore_u16(unsigned short* p, unsigned short x) {
    *(__attribute__((address_space(1))) unsigned short*)p = x;
}
__device__ __forceinline__ void w_gstore2(u64* p, u64 x, u64 y) {   // p is 16-byte aligned
    const w_u64x2 v = {x, y};
    *(__attribute__((address_space(1))) w_u64x2*)p = v;
}
__device__ __forceinline__ u64 w_bits(double v) {
    u64 b;
    __builtin_memcpy(&b, &v, 8);
    return b;
}
__device__ __forceinline__ u64 w_bits(i64 v) { return (u64)v; }
template <class T> __device__ __forceinline__ T w_from_bits(u64 b) {
    T v;
    __builtin_memcpy(&v, &b, 8);
    return v;
}

// Register-slot dictionary for a handful of groups: the work-group keeps the list
// of keys it has met in LDS (append-only); every lane accumulates each group in
// registers.  Returns the slot of `kbits`, appending it if new; -1 if the list is
// full (capacity error).
template <int S>
__device__ __forceinline__ int w_slot_list_insert(u64* s_keys, u64 kbits, int* err) {
#pragma unroll
    for (int s = 0; s < S; ++s) {
        u64 cur = __hip_atomic_load(s_keys + s, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        if (cur == kbits) return s;
        if (cur == W_EMPTY_KEY) {
            u64 expect = W_EMPTY_KEY;
            if (__hip_atomic_compare_exchange_strong(s_keys + s, &expect, kbits, __ATOMIC_RELAXED,
                                                     __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP))
                return s;
            if (expect == kbits) return s;
        }
    }
    atomicOr(err, 1);
    return -1;
}
