// Run-time compilation of generated kernels for gfx950, with an in-memory and an
// on-disk cache of code objects.
//
// The paper's system compiles each combined program once at its evaluation point
// (Sec. 7.8 reports 62-257 ms per program); here the compiler is hiprtc and a loop
// that was seen before, in this process or an earlier one, costs a hash lookup.
// Compilation needs no GPU, so kernels can be built ahead of time on a build host.
#include <dlfcn.h>
#include <hip/hip_runtime_api.h>
#include <hip/hip_ext.h>
#include <hip/hiprtc.h>
#include <sys/stat.h>
#include <unistd.h>

#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <fstream>
#include <map>
#include <mutex>

#include "weld_internal.h"

namespace weld {

struct Kernel {
    std::vector<char> code;
    hipModule_t mod = nullptr;
    hipFunction_t fn = nullptr;
    bool loaded = false;
};

namespace {

std::mutex g_mu;
std::map<std::string, Kernel*> g_kernels;  // keyed by full source text
std::string g_cache_dir;
bool g_cache_dir_set = false;

const char* const kOptions[] = {
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-ffp-contract=off",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
};
const int kNumOptions = sizeof(kOptions) / sizeof(kOptions[0]);

uint64_t fnv(const std::string& s, uint64_t h) {
    for (unsigned char c : s) { h ^= c; h *= 0x100000001b3ull; }
    return h;
}

std::string default_cache_dir() {
    const char* env = getenv("WELD_HIP_CACHE_DIR");
    if (env && *env) return env;
    Dl_info info;
    if (dladdr((void*)&default_cache_dir, &info) && info.dli_fname) {
        std::string p = info.dli_fname;
        size_t slash = p.rfind('/');
        if (slash != std::string::npos) return p.substr(0, slash) + "/kcache";
    }
    return "";
}

std::string cache_path(const std::string& source) {
    if (!g_cache_dir_set) { g_cache_dir = default_cache_dir(); g_cache_dir_set = true; }
    if (g_cache_dir.empty()) return "";
    std::string opts;
    for (int i = 0; i < kNumOptions; ++i) { opts += kOptions[i]; opts += ' '; }
    int rtc_major = 0, rtc_minor = 0;
    hiprtcVersion(&rtc_major, &rtc_minor);
    opts += std::to_string(rtc_major) + "." + std::to_string(rtc_minor);
    const uint64_t h1 = fnv(opts, fnv(source, 0xcbf29ce484222325ull));
    const uint64_t h2 = fnv(source, fnv(opts, 0x84222325cbf29ce4ull));
    char name[64];
    snprintf(name, sizeof name, "/%016llx%016llx.hsaco", (unsigned long long)h1, (unsigned long long)h2);
    return g_cache_dir + name;
}

Error err(weld_status_t st, const std::string& text) {
    Error e;
    e.status = st;
    e.text = text;
    return e;
}

Error compile(const std::string& source, std::vector<char>* code) {
    hiprtcProgram prog;
    hiprtcResult r = hiprtcCreateProgram(&prog, source.c_str(), "weld_fused.hip", 0, nullptr, nullptr);
    if (r != HIPRTC_SUCCESS) return err(WELD_ERR_DEVICE, std::string("hiprtcCreateProgram: ") + hiprtcGetErrorString(r));
    r = hiprtcCompileProgram(prog, kNumOptions, const_cast<const char**>(kOptions));
    if (r != HIPRTC_SUCCESS) {
        size_t n = 0;
        hiprtcGetProgramLogSize(prog, &n);
        std::string log(n, '\0');
        if (n) hiprtcGetProgramLog(prog, &log[0]);
        hiprtcDestroyProgram(&prog);
        if (log.size() > 4000) log.resize(4000);
        return err(WELD_ERR_DEVICE, std::string("kernel compilation failed: ") + hiprtcGetErrorString(r) + "\n" + log);
    }
    size_t n = 0;
    hiprtcGetCodeSize(prog, &n);
    code->resize(n);
    hiprtcGetCode(prog, code->data());
    hiprtcDestroyProgram(&prog);
    return Error();
}

}  // namespace

Error set_cache_dir(const char* path) {
    std::lock_guard<std::mutex> lk(g_mu);
    g_cache_dir = path ? path : "";
    g_cache_dir_set = true;
    if (!g_cache_dir.empty()) mkdir(g_cache_dir.c_str(), 0755);
    return Error();
}

Error jit_get(const std::string& source, const std::string& kernel_name, bool load_on_device, Kernel** out) {
    std::lock_guard<std::mutex> lk(g_mu);
    Kernel* k = nullptr;
    auto it = g_kernels.find(source);
    if (it != g_kernels.end()) {
        k = it->second;
    } else {
        k = new Kernel();
        const std::string path = cache_path(source);
        bool have = false;
        if (!path.empty()) {
            std::ifstream in(path, std::ios::binary);
            if (in) {
                k->code.assign(std::istreambuf_iterator<char>(in), std::istreambuf_iterator<char>());
                have = k->code.size() > 64;
            }
        }
        if (!have) {
            Error e = compile(source, &k->code);
            if (!e.ok()) { delete k; return e; }
            if (!path.empty()) {
                mkdir(g_cache_dir.c_str(), 0755);
                const std::string tmp = path + ".tmp" + std::to_string((long)getpid());
                std::ofstream o(tmp, std::ios::binary);
                if (o) {
                    o.write(k->code.data(), (std::streamsize)k->code.size());
                    o.close();
                    if (rename(tmp.c_str(), path.c_str()) != 0) unlink(tmp.c_str());
                }
            }
        }
        g_kernels[source] = k;
    }
    if (load_on_device && !k->loaded) {
        hipError_t h = hipModuleLoadData(&k->mod, k->code.data());
        if (h != hipSuccess) return err(WELD_ERR_DEVICE, std::string("hipModuleLoadData: ") + hipGetErrorString(h));
        h = hipModuleGetFunction(&k->fn, k->mod, kernel_name.c_str());
        if (h != hipSuccess) return err(WELD_ERR_DEVICE, std::string("hipModuleGetFunction: ") + hipGetErrorString(h));
        k->loaded = true;
    }
    *out = k;
    return Error();
}

int jit_blocks_per_cu(Kernel* k, int block) {
    int nb = 0;
    if (hipModuleOccupancyMaxActiveBlocksPerMultiprocessor(&nb, k->fn, block, 0) != hipSuccess) {
        (void)hipGetLastError();
        return 0;
    }
    return nb;
}

Error jit_launch(Kernel* k, unsigned grid, unsigned block, void* args, size_t args_bytes, void* stream, void* start_event,
                 void* stop_event) {
    void* extra[] = {HIP_LAUNCH_PARAM_BUFFER_POINTER, args, HIP_LAUNCH_PARAM_BUFFER_SIZE, &args_bytes,
                     HIP_LAUNCH_PARAM_END};
    hipError_t h;
    if (start_event || stop_event) {
        // the events take the dispatch's own start and end times: no packets of their own in the queue
        // (an event record is a barrier packet, about 4.5 us during which the queue starts nothing)
        h = hipExtModuleLaunchKernel(k->fn, grid * block, 1, 1, block, 1, 1, 0, (hipStream_t)stream, nullptr, extra,
                                     (hipEvent_t)start_event, (hipEvent_t)stop_event, 0);
    } else {
        h = hipModuleLaunchKernel(k->fn, grid, 1, 1, block, 1, 1, 0, (hipStream_t)stream, nullptr, extra);
    }
    if (h != hipSuccess) return err(WELD_ERR_DEVICE, std::string("hipModuleLaunchKernel: ") + hipGetErrorString(h));
    return Error();
}

}  // namespace weld
