// Plain device-to-device copy with known traffic: the yardstick for hardware
// counters and for the copy bandwidth the machine reaches.
#include "irm_internal.hpp"

__global__ __launch_bounds__(256) void calibrate_copy(u32x4 *__restrict__ dst, const u32x4 *__restrict__ src,
                                                      uint64_t n_vec)
{
    const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
    uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    // four independent 16-byte accesses in flight per lane
    for (; i + 3 * stride < n_vec; i += 4 * stride) {
        const u32x4 a = __builtin_nontemporal_load(src + i);
        const u32x4 b = __builtin_nontemporal_load(src + i + stride);
        const u32x4 c = __builtin_nontemporal_load(src + i + 2 * stride);
        const u32x4 d = __builtin_nontemporal_load(src + i + 3 * stride);
        __builtin_nontemporal_store(a, dst + i);
        __builtin_nontemporal_store(b, dst + i + stride);
        __builtin_nontemporal_store(c, dst + i + 2 * stride);
        __builtin_nontemporal_store(d, dst + i + 3 * stride);
    }
    for (; i < n_vec; i += stride) __builtin_nontemporal_store(__builtin_nontemporal_load(src + i), dst + i);
}

extern "C" irm_status irm_calibrate_copy(void *d_dst, const void *d_src, uint64_t bytes, uint32_t grid,
                                         void *stream)
{
    if (!d_dst || !d_src || bytes < 16 || (bytes & 15) || ((uintptr_t)d_dst & 15) || ((uintptr_t)d_src & 15))
        return IRM_ERR_INVALID_ARG;
    if (grid == 0) grid = 256 * 8;
    if (grid > (1u << 20)) return IRM_ERR_INVALID_ARG;
    hipLaunchKernelGGL(calibrate_copy, dim3(grid), dim3(256), 0, (hipStream_t)stream, (u32x4 *)d_dst,
                       (const u32x4 *)d_src, bytes / 16);
    return irm_launch_status();
}
