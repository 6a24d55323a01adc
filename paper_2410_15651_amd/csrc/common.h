// Internal helpers shared by the library's translation units (host side):
// status/error plumbing and HIP call checking.  Not part of the public ABI.
#pragma once

#include <hip/hip_runtime.h>

#include <cstdarg>
#include <cstdint>
#include <cstdio>

#include "rlhf_rollout.h"

namespace rlhf {

// Stores printf-style text for rlhf_last_error_string() and returns `code`.
int fail(int code, const char *fmt, ...) __attribute__((format(printf, 2, 3)));

void clear_error();

inline int elem_bytes(int dtype)
{
    return dtype == RLHF_F32 ? 4 : 2;
}

}  // namespace rlhf

#define RLHF_HIP_TRY(expr)                                                                 \
    do {                                                                                   \
        hipError_t _e = (expr);                                                            \
        if (_e != hipSuccess)                                                              \
            return ::rlhf::fail(RLHF_ERR_DEVICE, "%s failed: %s (%s:%d)", #expr,           \
                                hipGetErrorString(_e), __FILE__, __LINE__);                \
    } while (0)

// After a kernel launch: pick up launch-configuration errors without synchronising.
#define RLHF_LAUNCH_CHECK(name)                                                            \
    do {                                                                                   \
        hipError_t _e = hipGetLastError();                                                 \
        if (_e != hipSuccess)                                                              \
            return ::rlhf::fail(RLHF_ERR_DEVICE, "launch of %s failed: %s", name,          \
                                hipGetErrorString(_e));                                    \
    } while (0)
