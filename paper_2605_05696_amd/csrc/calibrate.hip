// Plain kernels with known traffic: the yardsticks for hardware counters and for the
// bandwidth the machine reaches on a stream that only reads, only writes, or copies.
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

// Shaped streams.  Every workgroup owns one contiguous range and walks it in steps of
// lanes * U 16-byte vectors: U loads per lane are issued, then U stores (mode copy), or the
// loads are only folded into a value that is never stored (mode read), or a pattern is stored
// (mode write).  Non-temporal accesses, like the row kernels.
template <int U, int MODE>
__global__ void yardstick(u32x4 *__restrict__ dst, const u32x4 *__restrict__ src, uint64_t vec_per_wg, uint32_t xcd)
{
    // xcd: workgroups are dealt round-robin to the 8 XCDs, so range (x % 8) * grid / 8 + x / 8 gives
    // every XCD one contiguous eighth of the buffers, as the row kernels do
    const uint32_t range = xcd ? (blockIdx.x & 7u) * (gridDim.x >> 3) + (blockIdx.x >> 3) : blockIdx.x;
    const uint64_t base = (uint64_t)range * vec_per_wg + threadIdx.x;
    const uint64_t step = (uint64_t)blockDim.x * U;
    const uint32_t n_steps = (uint32_t)(vec_per_wg / step);
    u32x4 acc = {0u, 0u, 0u, 0u};
#pragma nounroll
    for (uint32_t t = 0; t < n_steps; ++t) {
        u32x4 r[U];
        if (MODE != 2) {
#pragma unroll
            for (int i = 0; i < U; ++i)
                r[i] = __builtin_nontemporal_load(src + base + t * step + (uint64_t)i * blockDim.x);
        }
        if (MODE == 0) {
#pragma unroll
            for (int i = 0; i < U; ++i)
                __builtin_nontemporal_store(r[i], dst + base + t * step + (uint64_t)i * blockDim.x);
        } else if (MODE == 1) {
#pragma unroll
            for (int i = 0; i < U; ++i) acc ^= r[i];
        } else {
            const u32x4 pattern = {t, threadIdx.x, range, 0x5A5A5A5Au};
#pragma unroll
            for (int i = 0; i < U; ++i)
                __builtin_nontemporal_store(pattern, dst + base + t * step + (uint64_t)i * blockDim.x);
        }
    }
    // never true for the data the bench fills the source with; keeps the loads alive
    if (MODE == 1 && acc.x == 0x9E3779B9u && acc.y == 0x7F4A7C15u && acc.z == 0x0u && acc.w == 0xFFFFFFFFu)
        dst[base] = acc;
}

template <int MODE>
static bool yardstick_launch(uint32_t u, dim3 grid, dim3 block, hipStream_t s, u32x4 *dst, const u32x4 *src,
                             uint64_t vec_per_wg, uint32_t xcd)
{
    switch (u) {
    case 1: hipLaunchKernelGGL((yardstick<1, MODE>), grid, block, 0, s, dst, src, vec_per_wg, xcd); return true;
    case 2: hipLaunchKernelGGL((yardstick<2, MODE>), grid, block, 0, s, dst, src, vec_per_wg, xcd); return true;
    case 4: hipLaunchKernelGGL((yardstick<4, MODE>), grid, block, 0, s, dst, src, vec_per_wg, xcd); return true;
    case 9: hipLaunchKernelGGL((yardstick<9, MODE>), grid, block, 0, s, dst, src, vec_per_wg, xcd); return true;
    case 18: hipLaunchKernelGGL((yardstick<18, MODE>), grid, block, 0, s, dst, src, vec_per_wg, xcd); return true;
    case 36: hipLaunchKernelGGL((yardstick<36, MODE>), grid, block, 0, s, dst, src, vec_per_wg, xcd); return true;
    default: return false;
    }
}

extern "C" irm_status irm_yardstick(void *d_dst, const void *d_src, uint64_t bytes, uint32_t mode, uint32_t grid,
                                    uint32_t lanes, uint32_t vectors_per_lane, void *stream)
{
    const uint32_t xcd = mode & IRM_YARDSTICK_XCD_RANGES ? 1u : 0u;
    mode &= ~(uint32_t)IRM_YARDSTICK_XCD_RANGES;
    if (!d_dst || !d_src || ((uintptr_t)d_dst & 15) || ((uintptr_t)d_src & 15) || mode > IRM_YARDSTICK_WRITE)
        return IRM_ERR_INVALID_ARG;
    if (xcd && (grid & 7u)) return IRM_ERR_INVALID_ARG;
    if (grid < 1 || grid > (1u << 20) || lanes < 64 || lanes > 1024 || (lanes & 63)) return IRM_ERR_INVALID_ARG;
    // every workgroup's range must be a whole number of steps: no tail, no bounds check in the loop
    const uint64_t step_bytes = (uint64_t)lanes * vectors_per_lane * 16u;
    if (!step_bytes || bytes % ((uint64_t)grid * step_bytes) != 0) return IRM_ERR_INVALID_ARG;
    const uint64_t vec_per_wg = bytes / 16u / grid;
    if (vec_per_wg / ((uint64_t)lanes * vectors_per_lane) > 0xFFFFFFFFull) return IRM_ERR_INVALID_ARG;
    hipStream_t s = (hipStream_t)stream;
    bool ok;
    if (mode == IRM_YARDSTICK_COPY)
        ok = yardstick_launch<0>(vectors_per_lane, dim3(grid), dim3(lanes), s, (u32x4 *)d_dst, (const u32x4 *)d_src,
                                 vec_per_wg, xcd);
    else if (mode == IRM_YARDSTICK_READ)
        ok = yardstick_launch<1>(vectors_per_lane, dim3(grid), dim3(lanes), s, (u32x4 *)d_dst, (const u32x4 *)d_src,
                                 vec_per_wg, xcd);
    else
        ok = yardstick_launch<2>(vectors_per_lane, dim3(grid), dim3(lanes), s, (u32x4 *)d_dst, (const u32x4 *)d_src,
                                 vec_per_wg, xcd);
    if (!ok) return IRM_ERR_INVALID_ARG;
    return irm_launch_status();
}
