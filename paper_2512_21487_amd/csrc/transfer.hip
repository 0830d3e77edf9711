// Stand-in for the A2E / E2A transfers (Sec. 2.2; Eq. a2e_detail) in pinned-host mode: a chunk
// of activations crosses the host link in a copy kernel that reads (or writes) the pinned
// host buffer directly.  A kernel launch never blocks the host thread and costs a few
// microseconds, where the runtime's asynchronous memcpy was measured to take 25-50 us per
// call and to block for milliseconds now and then, which serialised the chunk pipeline.
// 16 bytes per lane, four independent loads per lane in flight; the grid is small (the link,
// not the CUs, is the bottleneck) so the copy shares the GPU with the expert GEMMs.
#include "common.h"
#include "kernels.h"

namespace moe_ep {

// U independent loads per lane in flight; any block size up to 256
template <typename V, int U>
__global__ __launch_bounds__(256) void copy_kernel(const V* __restrict__ src, V* __restrict__ dst, size_t n)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    for (; i + (U - 1) * stride < n; i += U * stride) {
        V v[U];
#pragma unroll
        for (int u = 0; u < U; ++u) v[u] = src[i + u * stride];
#pragma unroll
        for (int u = 0; u < U; ++u) dst[i + u * stride] = v[u];
    }
    for (; i < n; i += stride) dst[i] = src[i];
}

// grid workgroups of `threads` lanes, `unroll` loads in flight per lane (1, 2 or 4)
hipError_t launch_copy(void* dst, const void* src, size_t bytes, int grid, hipStream_t s, int threads, int unroll)
{
    if (bytes == 0) return hipSuccess;
    if (threads < 64 || threads > 256 || threads % 64) return hipErrorInvalidValue;
    const bool a16 = ((reinterpret_cast<uintptr_t>(dst) | reinterpret_cast<uintptr_t>(src) | bytes) & 15) == 0;
    if (a16) {
        auto* sp = static_cast<const uint4*>(src);
        auto* dp = static_cast<uint4*>(dst);
        if (unroll >= 4) hipLaunchKernelGGL((copy_kernel<uint4, 4>), dim3(grid), dim3(threads), 0, s, sp, dp, bytes / 16);
        else if (unroll >= 2) hipLaunchKernelGGL((copy_kernel<uint4, 2>), dim3(grid), dim3(threads), 0, s, sp, dp, bytes / 16);
        else hipLaunchKernelGGL((copy_kernel<uint4, 1>), dim3(grid), dim3(threads), 0, s, sp, dp, bytes / 16);
    } else {  // 4-byte granularity (gate scores of a chunk need not start on a 16-byte boundary)
        hipLaunchKernelGGL((copy_kernel<uint32_t, 4>), dim3(grid), dim3(threads), 0, s, static_cast<const uint32_t*>(src),
                           static_cast<uint32_t*>(dst), bytes / 4);
    }
    return hipGetLastError();
}

// Stand-in for an attention-group task of a given duration (Sec. 2.3: the attention of a
// micro-batch runs on other GPUs; here only its place in the schedule matters): one wavefront that
// sleeps until the constant 100 MHz wall clock has advanced by `ticks`, or until `max_polls` polls
// have passed, whichever comes first, so that the kernel ends whatever the clock does.
__global__ __launch_bounds__(64) void busy_kernel(long long ticks, int max_polls)
{
    const long long t0 = wall_clock64();
    for (int i = 0; i < max_polls && wall_clock64() - t0 < ticks; ++i) __builtin_amdgcn_s_sleep(32);
}

hipError_t launch_busy(double microseconds, hipStream_t s)
{
    if (!(microseconds > 0.0)) return hipSuccess;
    if (microseconds > 1e6) return hipErrorInvalidValue;
    const long long ticks = (long long)(microseconds * 100.0);
    // a poll (s_sleep 32 = about 2048 cycles) takes at least half a microsecond at any clock the part runs at
    const int max_polls = (int)(microseconds * 4.0) + 64;
    hipLaunchKernelGGL(busy_kernel, dim3(1), dim3(64), 0, s, ticks, max_polls);
    return hipGetLastError();
}

}  // namespace moe_ep
