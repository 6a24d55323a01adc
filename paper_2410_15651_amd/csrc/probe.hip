// Streaming-read probe: what a plain kernel that only reads can pull from HBM
// on this device.  The decode-attention and log-prob kernels are bound by HBM
// reads; the benchmark reports their rates against the published peak and,
// beside it, against this measured ceiling (same 16-byte non-temporal loads,
// nothing else in the kernel).
//
// Matrix-rate probe: what a kernel that only issues the prefill kernel's matrix
// instruction reaches, and at which shader clock, on operands the caller
// supplies.  The device lowers its clock under matrix load by an amount that
// depends on the data (zeros switch fewer wires than random mantissas), so the
// published peak is not what any kernel can reach on real data; the benchmark
// sets the prefill kernel's rate beside this figure.
#include <hip/hip_runtime.h>

#include <algorithm>

#include "common.h"
#include "device_ops.h"
#include "mfma_ops.h"

namespace rlhf {
namespace {

constexpr int kThreads = 256;
constexpr int kUnroll = 4;

__global__ __launch_bounds__(kThreads) void read_probe_kernel(const uint4 *__restrict__ p, int64_t n_vec,
                                                              uint32_t *__restrict__ sink)
{
    int64_t i = (int64_t)blockIdx.x * kThreads * kUnroll + threadIdx.x;
    const int64_t stride = (int64_t)gridDim.x * kThreads * kUnroll;
    uint32_t acc = 0;
    for (; i + (kUnroll - 1) * kThreads < n_vec; i += stride) {
        uint4 v[kUnroll];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u)
            v[u] = load16(p + i + u * kThreads);
#pragma unroll
        for (int u = 0; u < kUnroll; ++u)
            acc ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
    }
    for (; i < n_vec; i += kThreads) {  // the last, partly filled group of a workgroup
        const uint4 v = load16(p + i);
        acc ^= v.x ^ v.y ^ v.z ^ v.w;
    }
    // keeps the loads alive; practically never taken, and harmless when it is
    if (acc == 0x9E3779B9u && sink)
        *sink = acc;
}

constexpr int kMatrixThreads = 768;  // three wavefronts per SIMD, as the prefill kernel
constexpr int kMatrixPerIter = 8;

// Every lane takes sixteen 16-byte operand registers from the buffer (wrapping
// around its end) and then issues iterations x 8 products 32x32x16 (bf16) into
// four independent accumulators.
__global__ __launch_bounds__(kMatrixThreads) void matrix_probe_kernel(const uint4 *__restrict__ operands,
                                                                      int64_t n_vec, int iterations,
                                                                      unsigned long long *__restrict__ ticks)
{
    uint4 a[8], b[8];
    const int64_t first = ((int64_t)blockIdx.x * kMatrixThreads + threadIdx.x) * 16;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        a[i] = operands[(first + i) % n_vec];
        b[i] = operands[(first + 8 + i) % n_vec];
    }
    f32x16_t c[4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 16; ++j)
            c[i][j] = 0.f;
    const unsigned long long wall0 = __builtin_amdgcn_s_memrealtime(), clk0 = __builtin_readcyclecounter();
    for (int it = 0; it < iterations; ++it) {
#pragma unroll
        for (int i = 0; i < kMatrixPerIter; ++i)
            c[i % 4] = mfma_32x32<RLHF_BF16>(a[i], b[(3 * i + 1) & 7], c[i % 4]);
    }
    const unsigned long long wall1 = __builtin_amdgcn_s_memrealtime(), clk1 = __builtin_readcyclecounter();
    float sum = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 16; ++j)
            sum += c[i][j];
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        ticks[0] = wall1 - wall0;  // 100 MHz
        ticks[1] = clk1 - clk0;    // shader cycles
    }
    if (sum == 12345.678f)  // keeps the products alive; practically never taken, and harmless when it is
        ticks[2] = 1;
}

}  // namespace
}  // namespace rlhf

extern "C" int rlhf_probe_matrix_rate(const void *operands, size_t bytes, int32_t iterations,
                                      int32_t n_workgroups, uint64_t *ticks, void *stream)
{
    using namespace rlhf;
    if (!operands || (uintptr_t)operands % 16 || bytes < 16)
        return fail(RLHF_ERR_INVALID, "operands must be a 16-byte aligned device buffer of at least 16 bytes");
    if (!ticks || (uintptr_t)ticks % 8)
        return fail(RLHF_ERR_INVALID, "ticks must be a device array of three uint64");
    if (iterations < 0 || n_workgroups <= 0 || n_workgroups > (1 << 20))
        return fail(RLHF_ERR_INVALID, "iterations %d, n_workgroups %d", iterations, n_workgroups);
    hipLaunchKernelGGL(matrix_probe_kernel, dim3((unsigned)n_workgroups), dim3(kMatrixThreads), 0,
                       (hipStream_t)stream, (const uint4 *)operands, (int64_t)(bytes / 16), (int)iterations,
                       (unsigned long long *)ticks);
    RLHF_LAUNCH_CHECK("matrix_probe_kernel");
    return RLHF_OK;
}

extern "C" int rlhf_probe_stream_read(const void *buffer, size_t bytes, uint32_t *sink, void *stream)
{
    using namespace rlhf;
    if (!buffer || (uintptr_t)buffer % 16)
        return fail(RLHF_ERR_INVALID, "buffer must be a 16-byte aligned device pointer");
    const int64_t n_vec = (int64_t)(bytes / 16);
    if (n_vec == 0)
        return RLHF_OK;
    const int64_t per_group = (int64_t)kThreads * kUnroll;
    const int64_t groups = (n_vec + per_group - 1) / per_group;
    const unsigned grid = (unsigned)std::min<int64_t>(groups, 16384);
    hipLaunchKernelGGL(read_probe_kernel, dim3(grid), dim3(kThreads), 0, (hipStream_t)stream,
                       (const uint4 *)buffer, n_vec, sink);
    RLHF_LAUNCH_CHECK("read_probe_kernel");
    return RLHF_OK;
}
