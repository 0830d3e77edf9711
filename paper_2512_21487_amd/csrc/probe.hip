// What this GPU sustains, measured next to the layer: a register-only MFMA loop (no LDS, no
// memory) on random or all-zero bf16 operands, and a streaming device-to-device copy.  The
// fractions of the vendor peaks that the layer's kernels reach are read against these: the part
// trades clock for matrix-pipe activity under its power limit, so the 2.5 PFLOP/s figure, which
// assumes the maximum clock, is not a corner real operands reach.  Measurement aid only: nothing
// on the path calls it; it is built into a library of its own (libmoe_ep_probe.so) for the benchmark.
#include <cmath>
#include <cstring>
#include <vector>

#include "common.h"
#include "moe_ep_probe.h"

namespace moe_ep {

constexpr int kProbeSets = 1, kProbeBlocks = 8;  // operand registers of one 32-wide step of a 128 x 128 wave tile

// Every wavefront multiplies the same 8 + 8 operand fragments into 64 accumulator blocks of 16 x 16 with
// v_mfma_f32_16x16x32_bf16, the instruction the grouped GEMM multiplies with, in the order a K step issues
// them: row blocks down one column of blocks and up the next, so one operand changes per instruction and
// an accumulator is revisited every 64 instructions.  (The same loop out of v_mfma_f32_32x32x16_bf16
// sustains about 5 % fewer flops under the package power limit.)
__global__ __launch_bounds__(256) void mfma_probe_kernel(const uint4* __restrict__ in, float* __restrict__ out,
                                                         int iters, long long* __restrict__ clk)
{
    f32x4_t acc[kProbeBlocks][kProbeBlocks];
#pragma unroll
    for (int i = 0; i < kProbeBlocks; ++i)
#pragma unroll
        for (int j = 0; j < kProbeBlocks; ++j)
#pragma unroll
            for (int r = 0; r < 4; ++r) acc[i][j][r] = 0.f;
    bf16x8_t a[kProbeBlocks], b[kProbeBlocks];
#pragma unroll
    for (int i = 0; i < kProbeBlocks; ++i) {
        a[i] = __builtin_bit_cast(bf16x8_t, in[i * 256 + threadIdx.x]);
        b[i] = __builtin_bit_cast(bf16x8_t, in[(kProbeBlocks + i) * 256 + threadIdx.x]);
    }
    const long long c0 = clock64(), w0 = wall_clock64();
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int q = 0; q < kProbeBlocks * kProbeBlocks; ++q) {
            const int j = q / kProbeBlocks, i = (j & 1) ? kProbeBlocks - 1 - q % kProbeBlocks : q % kProbeBlocks;
            acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(b[j], a[i], acc[i][j], 0, 0, 0);
        }
    }
    const long long c1 = clock64(), w1 = wall_clock64();
    float sum = 0.f;
#pragma unroll
    for (int i = 0; i < kProbeBlocks; ++i)
#pragma unroll
        for (int j = 0; j < kProbeBlocks; ++j)
#pragma unroll
            for (int r = 0; r < 4; ++r) sum += acc[i][j][r];
    out[blockIdx.x * 256 + threadIdx.x] = sum;  // keeps the loop alive
    if (threadIdx.x == 0) {
        clk[2 * blockIdx.x] = c1 - c0;       // shader cycles
        clk[2 * blockIdx.x + 1] = w1 - w0;   // ticks of the constant 100 MHz clock
    }
}

__global__ __launch_bounds__(256) void copy_probe_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst, size_t n)
{
    const size_t stride = (size_t)gridDim.x * 256;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += stride) dst[i] = src[i];
}

namespace {

struct Buffers {
    void* p[4] = {nullptr, nullptr, nullptr, nullptr};
    ~Buffers() { for (void* q : p) if (q) (void)hipFree(q); }
};

uint16_t to_bf16(float f)
{
    uint32_t u;
    memcpy(&u, &f, 4);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

}  // namespace
}  // namespace moe_ep

using namespace moe_ep;

extern "C" int moe_ep_probe_device(int32_t device, int32_t zero_operands, double* mfma_tflops, double* mfma_ghz,
                                   double* copy_gbs)
{
    if (device < 0 || !mfma_tflops || !mfma_ghz || !copy_gbs) return -1;
#define PROBE_TRY(call) do { if ((call) != hipSuccess) { (void)hipGetLastError(); return -3; } } while (0)
    PROBE_TRY(hipSetDevice(device));
    hipDeviceProp_t prop;
    PROBE_TRY(hipGetDeviceProperties(&prop, device));
    const int n_cu = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;

    // operands: standard normal values rounded to bf16 (Box-Muller over a fixed linear congruential
    // sequence), or zeros
    const size_t n_in = (size_t)kProbeSets * 2 * kProbeBlocks * 256 * 8;
    std::vector<uint16_t> h(n_in, 0);
    if (!zero_operands) {
        uint32_t state = 12345u;
        auto uni = [&]() { state = state * 1664525u + 1013904223u; return ((state >> 8) + 1.0f) / 16777218.0f; };
        for (uint16_t& v : h) v = to_bf16(sqrtf(-2.0f * logf(uni())) * cosf(6.2831853f * uni()));
    }
    const size_t copy_bytes = (size_t)1 << 29;  // twice the 256 MB memory-side cache
    Buffers buf;
    PROBE_TRY(hipMalloc(&buf.p[0], n_in * 2));
    PROBE_TRY(hipMalloc(&buf.p[1], (size_t)n_cu * 256 * 4));
    PROBE_TRY(hipMalloc(&buf.p[2], (size_t)n_cu * 16));
    PROBE_TRY(hipMalloc(&buf.p[3], 2 * copy_bytes));
    PROBE_TRY(hipMemcpy(buf.p[0], h.data(), n_in * 2, hipMemcpyHostToDevice));
    hipEvent_t e0 = nullptr, e1 = nullptr;
    PROBE_TRY(hipEventCreate(&e0));
    if (hipEventCreate(&e1) != hipSuccess) { (void)hipEventDestroy(e0); return -3; }
    int rc = 0;
    float ms = 0.f;
    do {
        // the first launch brings the clock controller to its steady state for this load, the second is timed
        const int iters = 40000;  // x 64 MFMAs: about 22 ms per launch
        auto* in = static_cast<const uint4*>(buf.p[0]);
        auto* out = static_cast<float*>(buf.p[1]);
        auto* clk = static_cast<long long*>(buf.p[2]);
        hipLaunchKernelGGL(mfma_probe_kernel, dim3(n_cu), dim3(256), 0, 0, in, out, iters, clk);
        if (hipEventRecord(e0, 0) != hipSuccess) { rc = -3; break; }
        hipLaunchKernelGGL(mfma_probe_kernel, dim3(n_cu), dim3(256), 0, 0, in, out, iters, clk);
        if (hipEventRecord(e1, 0) != hipSuccess || hipEventSynchronize(e1) != hipSuccess ||
            hipEventElapsedTime(&ms, e0, e1) != hipSuccess || hipGetLastError() != hipSuccess) { rc = -3; break; }
        std::vector<long long> hc((size_t)2 * n_cu);
        if (hipMemcpy(hc.data(), clk, (size_t)n_cu * 16, hipMemcpyDeviceToHost) != hipSuccess) { rc = -3; break; }
        double cycles = 0.0, ticks = 0.0;
        for (int i = 0; i < n_cu; ++i) { cycles += (double)hc[2 * i]; ticks += (double)hc[2 * i + 1]; }
        const double flop = (double)n_cu * 4.0 * iters * (kProbeSets * kProbeBlocks * kProbeBlocks) * 2.0 * 16 * 16 * 32;
        *mfma_tflops = flop / (ms * 1e-3) / 1e12;
        *mfma_ghz = ticks > 0.0 ? cycles / ticks * 0.1 : 0.0;

        // streaming copy of 512 MiB: bytes read + bytes written per second
        auto* src = static_cast<uint4*>(buf.p[3]);
        auto* dst = reinterpret_cast<uint4*>(static_cast<char*>(buf.p[3]) + copy_bytes);
        if (hipMemsetAsync(src, 1, copy_bytes, 0) != hipSuccess) { rc = -3; break; }
        hipLaunchKernelGGL(copy_probe_kernel, dim3(n_cu * 8), dim3(256), 0, 0, src, dst, copy_bytes / 16);
        if (hipEventRecord(e0, 0) != hipSuccess) { rc = -3; break; }
        hipLaunchKernelGGL(copy_probe_kernel, dim3(n_cu * 8), dim3(256), 0, 0, src, dst, copy_bytes / 16);
        if (hipEventRecord(e1, 0) != hipSuccess || hipEventSynchronize(e1) != hipSuccess ||
            hipEventElapsedTime(&ms, e0, e1) != hipSuccess || hipGetLastError() != hipSuccess) { rc = -3; break; }
        *copy_gbs = 2.0 * (double)copy_bytes / (ms * 1e-3) / 1e9;
    } while (false);
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
#undef PROBE_TRY
    return rc;
}
