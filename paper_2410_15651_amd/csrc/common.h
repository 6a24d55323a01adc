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

// The runtime forms a launch's size per grid dimension as workgroups x lanes
// in 32 bits and reports no error when that wraps (a grid of 2^24 + 3
// workgroups of 256 lanes runs three of them).  Every launch keeps each
// dimension at or below this count.
constexpr int64_t max_workgroups(int lanes_per_workgroup)
{
    return 0xffffffffLL / lanes_per_workgroup;
}

// Kernels with one workgroup per row spread the rows over grid.x and grid.y:
// row = blockIdx.y * kRowSlab + blockIdx.x, and workgroups past the last row
// leave at once.  2^20 x 1024 lanes stays below the 32-bit limit and 65,535
// slabs cover any int32 row count.
constexpr int64_t kRowSlab = 1 << 20;

inline dim3 row_grid(int64_t n_rows, unsigned z = 1)
{
    const int64_t x = n_rows < kRowSlab ? n_rows : kRowSlab;
    return dim3((unsigned)x, (unsigned)((n_rows + kRowSlab - 1) / kRowSlab), z);
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
