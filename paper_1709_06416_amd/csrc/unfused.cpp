// Operator-at-a-time execution (placeholder until the per-operator kernels land).
#include "weld_internal.h"

namespace weld {

Error run_unfused(const Loop&, const weld_cols_t*, int64_t, const weld_builder_t*, weld_result*) {
    Error e;
    e.status = WELD_ERR_UNSUPPORTED;
    e.text = "unfused mode is not built yet";
    return e;
}

}  // namespace weld
