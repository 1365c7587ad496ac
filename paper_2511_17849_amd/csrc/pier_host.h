// Host-side helpers shared by the source files of libpier that implement the C ABI.
// Not part of the ABI.
#pragma once
#include "../../include/pier.h"

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace pier {

// Records the calling thread's error text (pier_last_error) and returns st.
pier_status fail(pier_status st, const char* fmt, ...) __attribute__((format(printf, 2, 3)));

// A pointer handed over as "device memory": must be non-null, aligned to its element, and
// lie with its whole extent inside one allocation of GPU `device`.
pier_status check_device_range(const void* ptr, int64_t numel, size_t elem, int device, const char* what,
                               int tensor);

}  // namespace pier

#define PIER_HIP(call)                                                                             \
    do {                                                                                           \
        hipError_t e_ = (call);                                                                    \
        if (e_ != hipSuccess)                                                                      \
            return ::pier::fail(e_ == hipErrorOutOfMemory ? PIER_ERR_OOM : PIER_ERR_HIP, "%s: %s", \
                                #call, hipGetErrorString(e_));                                     \
    } while (0)
