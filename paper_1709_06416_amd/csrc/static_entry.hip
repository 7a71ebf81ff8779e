// weld_fused_for_static: the fused loop for callers that cannot allocate device memory (code under
// HIP graph capture, tight serving loops, harnesses that forbid hipMalloc).
//
// The ordinary entry point takes one pool block per call for its control words, workspace and
// results.  Here the results go to buffers the caller passes and the workspace is a fixed device
// array of this file, one copy per GPU, held until the process ends.  The kernels are the same: they
// take the workspace as pointer arguments either way.
//
// In host code the array's NAME is only a stand-in for the device symbol, not a device address; the
// address on the current device comes from hipGetSymbolAddress, once per device, and that pointer is
// what every launch and fill below is given.
#include <hip/hip_runtime.h>

#include <mutex>

#include "aot_kernels.h"
#include "weld_internal.h"

// (No `used` attribute here: the compiler gives a static device variable that host code refers to a
// global symbol in the code object, which is how the runtime finds it; `used` kept it local and
// hipGetSymbolAddress aborted the process.)
static __device__ __align__(256) unsigned char scratch[WELD_STATIC_SCRATCH_BYTES];

namespace weld {
namespace {

constexpr int kMaxDevices = 64;
std::mutex g_mu;
unsigned char* g_scratch_ptr[kMaxDevices] = {nullptr};   // per device: each GPU holds its own copy of the array

// The workspace's address on the current device (set-up on the first call per device).
Error static_scratch(unsigned char** out) {
    int dev = -1;
    hipError_t h = hipGetDevice(&dev);
    if (h != hipSuccess) {
        Error e; e.status = WELD_ERR_DEVICE; e.text = std::string("hipGetDevice: ") + hipGetErrorString(h);
        return e;
    }
    if (dev < 0 || dev >= kMaxDevices) {
        Error e; e.status = WELD_ERR_DEVICE; e.text = "device index out of range";
        return e;
    }
    std::lock_guard<std::mutex> lk(g_mu);
    if (!g_scratch_ptr[dev]) {
        unsigned char* ptr = nullptr;
        h = hipGetSymbolAddress((void**)&ptr, HIP_SYMBOL(scratch));
        if (h != hipSuccess || !ptr) {
            (void)hipGetLastError();
            Error e; e.status = WELD_ERR_DEVICE;
            e.text = std::string("hipGetSymbolAddress of the fixed workspace: ") + hipGetErrorString(h);
            return e;
        }
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return Error();
}

__global__ void static_status_kernel(const unsigned int* ctl, const StaticLengths lens, long long* status) {
    const int t = threadIdx.x;
    if (t == 0) status[0] = (long long)ctl[2];
    if (t >= 1 && t <= WELD_MAX_BUILDERS) {
        const int b = t - 1;
        long long v = 0;
        if (b < lens.count)
            v = lens.known[b] >= 0 ? lens.known[b] : *(const long long*)((const char*)ctl + 16 + 8 * b);
        status[t] = v;
    }
}

}  // namespace

hipError_t launch_static_status(const void* ctl, const StaticLengths& lens, int64_t* status_dev, hipStream_t stream) {
    static_status_kernel<<<dim3(1), dim3(64), 0, stream>>>((const unsigned int*)ctl, lens, (long long*)status_dev);
    return hipGetLastError();
}

}  // namespace weld

using namespace weld;

extern "C" weld_status_t weld_fused_for_static(const weld_cols_t* cols, int64_t n, const weld_body_t* body,
                                               const weld_builder_t* builder, const weld_out_t* outs, int64_t* status_dev) {
    if (!cols || !body || !builder || !status_dev) { set_last_error("null argument"); return WELD_ERR_INVALID_ARG; }
    if (n < 0) { set_last_error("negative row count"); return WELD_ERR_INVALID_ARG; }
    if (cols->ncols < 0 || cols->ncols > WELD_MAX_COLS || (cols->ncols > 0 && !cols->col)) {
        set_last_error("bad column list");
        return WELD_ERR_INVALID_ARG;
    }
    if (builder->conf.mode != WELD_MODE_FUSED) {
        set_last_error("the call that allocates nothing runs the fused loop only");
        return WELD_ERR_UNSUPPORTED;
    }
    int32_t types[WELD_MAX_COLS];
    for (int c = 0; c < cols->ncols; ++c) types[c] = cols->col[c].type;
    Loop L;
    Error e = validate(types, cols->ncols, body, builder, &L);
    if (!e.ok()) { set_last_error(e.text); return e.status; }
    ColRef refs[WELD_MAX_COLS];
    for (int c = 0; c < cols->ncols; ++c) {
        if (((n > 0 && L.col_used[c]) || L.col_scalar[c]) && !cols->col[c].data) { set_last_error("null column pointer"); return WELD_ERR_INVALID_ARG; }
        if ((uintptr_t)cols->col[c].data % (uintptr_t)type_size(L.col_type[c])) {
            set_last_error("column pointer not aligned to its element size");
            return WELD_ERR_INVALID_ARG;
        }
        refs[c].data = cols->col[c].data;
        refs[c].type = cols->col[c].type;
    }
    if (!L.builders.empty() && !outs) { set_last_error("no output buffers"); return WELD_ERR_INVALID_ARG; }
    for (size_t b = 0; b < L.builders.size(); ++b) {
        const weld_builder_spec_t& s = L.builders[b];
        const weld_out_t& o = outs[b];
        int64_t need = 0;
        switch (s.kind) {
            case WELD_MERGER: need = 1; break;
            case WELD_VECBUILDER: need = L.merge_of[b] >= 0 ? n : 0; break;
            case WELD_VECMERGER: need = s.length; break;
            case WELD_DICTMERGER: need = s.capacity; break;
            default:
                set_last_error("groupbuilders need workspace in proportion to the rows: not in the call that allocates nothing");
                return WELD_ERR_UNSUPPORTED;
        }
        const bool missing = need > 0 && (!o.data || (s.kind == WELD_DICTMERGER && !o.data2));
        if (missing || (s.kind != WELD_MERGER && o.capacity < need) || ((uintptr_t)o.data & 15) || ((uintptr_t)o.data2 & 15)) {
            set_last_error("output " + std::to_string(b) + ": needs 16-byte aligned device buffers with room for " +
                           std::to_string(need) + " elements");
            return WELD_ERR_INVALID_ARG;
        }
    }
    unsigned char* ptr = nullptr;
    e = static_scratch(&ptr);
    if (!e.ok()) { set_last_error(e.text); return e.status; }
    StaticTarget st;
    // the array's first 4 KiB are never part of a call's workspace: they are zero from the start, and
    // the kernels that count their work-groups in there leave them zero
    st.arrive = (uint32_t*)ptr;
    st.scratch = (char*)ptr + 4096;
    st.scratch_bytes = (size_t)WELD_STATIC_SCRATCH_BYTES - 4096;
    st.outs = outs;
    st.status_dev = status_dev;
    e = run_fused_static(L, refs, n, builder->conf, st);
    if (!e.ok()) { set_last_error(e.text); return e.status; }
    return WELD_OK;
}
