// Launch-shape tuning of one loop on its own data.
//
// How many work-groups a streaming loop should keep in flight is not something the kernel's
// resource use decides.  Measured on MI355X: a loop that reads 28 bytes a row and does little
// else runs best with ONE 256-thread work-group per compute unit (57 KB of loads in flight per
// unit; 3 % slower with the eight that fit), a loop with seven columns and a register dictionary
// wants two (4 % slower with the three that fit, 20 % with four), and a loop that spends as long
// computing as loading wants more work-groups than are resident at once, so that they drift apart
// and one group's arithmetic overlaps another's loads (9 % faster than a resident grid that
// marches in step).  So the host program may ask: run the loop a few times per candidate grid,
// keep the fastest.  The result is a tuning record to pass to later calls; a loop keeps the
// same record afterwards, so its results stay reproducible from call to call (a merger's
// partial sums are grouped by work-group).
#include <hip/hip_runtime_api.h>

#include <algorithm>
#include <string>
#include <vector>

#include "weld_internal.h"

using namespace weld;

extern "C" weld_status_t weld_tune_launch(const weld_cols_t* cols, int64_t n, const weld_body_t* body,
                                          const weld_builder_t* builder, weld_tuning_t* best, float* best_ms,
                                          float* default_ms) {
    if (!cols || !body || !builder || !best || n < 0) {
        set_last_error("weld_tune_launch: null argument or negative row count");
        return WELD_ERR_INVALID_ARG;
    }
    if (builder->conf.mode != WELD_MODE_FUSED) {
        set_last_error("weld_tune_launch: fused mode only");
        return WELD_ERR_UNSUPPORTED;
    }
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess ||
        cus <= 0) {
        (void)hipGetLastError();
        set_last_error("weld_tune_launch: no usable HIP device");
        return WELD_ERR_DEVICE;
    }
    // work-groups per compute unit; 0 stands for the library's own choice and is tried first
    static const int kPerUnit[] = {0, 1, 2, 3, 4, 6, 8, 12, 16, 32, 64};
    const int kRuns = 6;      // the first one warms up (code object load, pool blocks)
    *best = builder->conf.tune;
    float best_time = -1.0f, first_time = -1.0f;
    std::vector<int64_t> tried;           // grids as launched (the library clamps what it is asked for)
    for (int per_unit : kPerUnit) {
        weld_builder_t b = *builder;
        b.conf.tune.grid_blocks = per_unit * cus;
        std::vector<float> ms;
        bool seen_before = false;
        for (int run = 0; run < kRuns && !seen_before; ++run) {
            weld_result_t* r = nullptr;
            weld_status_t st = weld_fused_for(cols, n, body, &b, &r);
            if (st != WELD_OK) return st;
            st = weld_result_status(r);
            float t = -1.0f;
            if (st == WELD_OK) st = weld_result_kernel_ms(r, &t);
            if (st != WELD_OK) {
                set_last_error(std::string("weld_tune_launch: ") + weld_result_error(r));
                weld_result_free(r);
                return st;
            }
            const int64_t launched = r->grid;
            weld_result_free(r);
            if (run == 0) {
                seen_before = std::find(tried.begin(), tried.end(), launched) != tried.end();
                tried.push_back(launched);
            } else if (t >= 0.0f) {
                ms.push_back(t);
            }
        }
        if (seen_before || ms.empty()) continue;
        std::sort(ms.begin(), ms.end());
        const float t = ms[ms.size() / 2];
        if (per_unit == 0) first_time = t;
        // another grid must win by more than run-to-run noise
        if (best_time < 0.0f || t < 0.975f * best_time) {
            best_time = t;
            best->grid_blocks = b.conf.tune.grid_blocks;
        }
    }
    if (best_ms) *best_ms = best_time;
    if (default_ms) *default_ms = first_time;
    return WELD_OK;
}
