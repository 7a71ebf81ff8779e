// Device memory pool: results and workspace of a call come from here and go back
// on weld_result_free (Sec. 4.3 of the paper: values allocated during execution are
// owned by the runtime and released after evaluation).  Blocks are cached by size so
// that repeated evaluations of the same loop allocate nothing.
#include <hip/hip_runtime_api.h>

#include <map>
#include <mutex>

#include "weld_internal.h"

namespace weld {
namespace {
std::mutex g_mu;
std::multimap<size_t, void*> g_free;  // cached blocks by size
std::map<void*, size_t> g_live;       // blocks handed out
int64_t g_total = 0;

size_t round_up(size_t b) {
    const size_t g = b < (1u << 20) ? 4096 : (1u << 20);
    return (b + g - 1) / g * g;
}
}  // namespace

Error pool_alloc(size_t bytes, void** out) {
    std::lock_guard<std::mutex> lk(g_mu);
    const size_t sz = round_up(bytes ? bytes : 1);
    auto it = g_free.lower_bound(sz);
    if (it != g_free.end() && it->first <= sz + sz / 8) {
        *out = it->second;
        g_live[it->second] = it->first;
        g_free.erase(it);
        return Error();
    }
    void* p = nullptr;
    hipError_t h = hipMalloc(&p, sz);
    if (h != hipSuccess) {
        // give cached blocks back to the device and retry once
        for (auto& kv : g_free) { (void)hipFree(kv.second); g_total -= (int64_t)kv.first; }
        g_free.clear();
        (void)hipGetLastError();
        h = hipMalloc(&p, sz);
    }
    if (h != hipSuccess) {
        (void)hipGetLastError();
        Error e;
        e.status = WELD_ERR_OOM;
        e.text = std::string("hipMalloc of ") + std::to_string(sz) + " bytes failed: " + hipGetErrorString(h);
        return e;
    }
    g_total += (int64_t)sz;
    g_live[p] = sz;
    *out = p;
    return Error();
}

void pool_free(void* p) {
    if (!p) return;
    std::lock_guard<std::mutex> lk(g_mu);
    auto it = g_live.find(p);
    if (it == g_live.end()) return;
    g_free.insert({it->second, p});
    g_live.erase(it);
}

void pool_trim() {
    std::lock_guard<std::mutex> lk(g_mu);
    for (auto& kv : g_free) { (void)hipFree(kv.second); g_total -= (int64_t)kv.first; }
    g_free.clear();
}

int64_t pool_bytes() {
    std::lock_guard<std::mutex> lk(g_mu);
    return g_total;
}

}  // namespace weld
