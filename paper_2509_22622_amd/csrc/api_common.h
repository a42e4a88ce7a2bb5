// Shared by the translation units that implement the C-ABI (include/longlive.h): error reporting, argument checks
// and the process-wide kernel-variant selection.
#pragma once
#include "../../include/longlive.h"

#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdint>
#include <string>
#include <vector>

#include "cache_index.h"
#include "kernels.h"

namespace ll_api {

// Record a message for ll_last_error() (thread-local) and return `s`.
ll_status fail(ll_status s, const char* fmt, ...);
ll_status hip_fail(hipError_t e, const char* what);

// the kernels move 16 bytes per lane
inline bool aligned16(const void* a, const void* b = nullptr, const void* c = nullptr, const void* d = nullptr) {
    return ((reinterpret_cast<uintptr_t>(a) | reinterpret_cast<uintptr_t>(b) | reinterpret_cast<uintptr_t>(c) |
             reinterpret_cast<uintptr_t>(d)) & 15) == 0;
}

extern int g_variant;   // ll_set_attn_variant: 0 = default for the shape

}  // namespace ll_api
