/* Plain-copy yardstick for the benchmark and the counter runs (libzipccl_yardstick.so); see zipccl_yardstick.h. */
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "zipccl_yardstick.h"

namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
constexpr uint32_t kThreads = 256;

__global__ __launch_bounds__(kThreads) void k_copy(const u32x4* __restrict__ src, u32x4* __restrict__ dst, uint64_t n16)
{
    const uint64_t i = (uint64_t)blockIdx.x * kThreads + threadIdx.x;
    if (i < n16) dst[i] = src[i];
}

} // namespace

extern "C" int zipccl_yardstick_copy(void* d_dst, const void* d_src, size_t bytes, void* stream)
{
    if (!d_dst || !d_src || (reinterpret_cast<uintptr_t>(d_dst) % 16) || (reinterpret_cast<uintptr_t>(d_src) % 16) ||
        (bytes % 16) || bytes / 16 / kThreads > 0x7FFFFFFFull)
        return 1;
    const uint64_t n16 = bytes / 16;
    if (n16 == 0) return 0;
    const uint64_t blocks = (n16 + kThreads - 1) / kThreads;
    hipLaunchKernelGGL(k_copy, dim3((uint32_t)blocks), dim3(kThreads), 0, (hipStream_t)stream,
                       static_cast<const u32x4*>(d_src), static_cast<u32x4*>(d_dst), n16);
    return hipGetLastError() == hipSuccess ? 0 : 5;
}
