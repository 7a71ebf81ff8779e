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

hipError_t launch_fill64(void* p, int64_t count, uint64_t value, hipStream_t stream);
hipError_t launch_dict_extract(const void* keys, const void* hdr, int64_t slots, const DictValues& vals,
                               const DictLayout& lay, int64_t capacity, void* out_keys, void* out_vals,
                               void* count, void* err, hipStream_t stream);
hipError_t launch_probe_read(const void* data, int64_t bytes, void* checksum, int blocks, hipStream_t stream);
hipError_t launch_probe_copy(void* dst, const void* src, int64_t bytes, int blocks, hipStream_t stream);

}  // namespace weld
