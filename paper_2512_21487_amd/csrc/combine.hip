// Weighted aggregation of the selected experts' outputs (Sec. 2.1), added to the shared experts'
// output that the shared down projection has already written into the output rows.  Token-major gather-reduce: a wavefront owns an output row, walks the row's
// kept slots in slot order, and accumulates in fp32; every load and store is 16 bytes per
// lane and contiguous over the wavefront.  No atomics, so the result is deterministic.
#include "common.h"
#include "kernels.h"

namespace moe_ep {

__device__ __forceinline__ void fma8(float* acc, float ws, const uint4& v) {
    acc[0] = fmaf(ws, bf16_lo(v.x), acc[0]); acc[1] = fmaf(ws, bf16_hi(v.x), acc[1]);
    acc[2] = fmaf(ws, bf16_lo(v.y), acc[2]); acc[3] = fmaf(ws, bf16_hi(v.y), acc[3]);
    acc[4] = fmaf(ws, bf16_lo(v.z), acc[4]); acc[5] = fmaf(ws, bf16_hi(v.z), acc[5]);
    acc[6] = fmaf(ws, bf16_lo(v.w), acc[6]); acc[7] = fmaf(ws, bf16_hi(v.w), acc[7]);
}

// 8 fp32 values of an expert's output row, weighted into the accumulator
__device__ __forceinline__ void fma8f(float* acc, float ws, const f32x4_t& lo, const f32x4_t& hi) {
    acc[0] = fmaf(ws, lo[0], acc[0]); acc[1] = fmaf(ws, lo[1], acc[1]);
    acc[2] = fmaf(ws, lo[2], acc[2]); acc[3] = fmaf(ws, lo[3], acc[3]);
    acc[4] = fmaf(ws, hi[0], acc[4]); acc[5] = fmaf(ws, hi[1], acc[5]);
    acc[6] = fmaf(ws, hi[2], acc[6]); acc[7] = fmaf(ws, hi[3], acc[7]);
}

// YMODE: 0 = y holds bf16 expert outputs, 1 = fp32 expert outputs (rows of M floats), 2 = bf16
// expert outputs that already carry their routing weight (the sum then uses weight 1)
template <int YMODE>
__global__ __launch_bounds__(256) void combine_kernel(
    const uint4* __restrict__ y, const int32_t* __restrict__ pos, const float* __restrict__ w, int Tn,
    int k, int M8, bool accumulate, bool all_rows, const uint4* out_src, uint4* out)
{
    const int lane = threadIdx.x & 63;
    const int gw = (blockIdx.x * 256 + threadIdx.x) >> 6, nw = gridDim.x * 4;
    for (int t = gw; t < Tn; t += nw) {
        const int my_pos = (lane < k) ? pos[(size_t)t * k + lane] : -1;
        const float my_w = (lane < k) ? w[(size_t)t * k + lane] : 0.f;
        // accumulate: the row already holds the shared experts' output; a token with no kept
        // slot keeps it as it is
        // (all_rows: the rows are written somewhere else than they are read from -- straight to the
        // caller's host buffer -- so a row that only carries the shared experts' output moves too)
        if (accumulate && !all_rows && __ballot(my_pos >= 0) == 0ull) continue;
        // the column loop runs the same number of times in every lane: the slot broadcasts below
        // read lanes 0..k-1, which must not have left the loop when a row is shorter than a trip
        for (int c0 = 0; c0 < M8; c0 += 128) {
            // two 16-byte column chunks per lane and trip: twice the loads in flight
            const int ca = c0 + lane, cb = c0 + 64 + lane;
            const bool in_a = ca < M8, in_b = cb < M8;
            float acc_a[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
            float acc_b[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
            for (int s = 0; s < k; ++s) {
                const int p = __shfl(my_pos, s, 64);  // uniform over the wavefront
                const float ws = YMODE == 2 ? 1.0f : __shfl(my_w, s, 64);
                if (p >= 0) {
                    if (YMODE == 1) {
                        const f32x4_t* yf = reinterpret_cast<const f32x4_t*>(y) + (size_t)p * M8 * 2;
                        f32x4_t a0, a1, b0, b1;
                        if (in_a) { a0 = yf[2 * ca]; a1 = yf[2 * ca + 1]; }
                        if (in_b) { b0 = yf[2 * cb]; b1 = yf[2 * cb + 1]; }
                        if (in_a) fma8f(acc_a, ws, a0, a1);
                        if (in_b) fma8f(acc_b, ws, b0, b1);
                    } else {
                        uint4 va, vb;
                        if (in_a) va = y[(size_t)p * M8 + ca];
                        if (in_b) vb = y[(size_t)p * M8 + cb];
                        if (in_a) fma8(acc_a, ws, va);
                        if (in_b) fma8(acc_b, ws, vb);
                    }
                }
            }
            if (in_a) {
                if (accumulate) fma8(acc_a, 1.0f, out_src[(size_t)t * M8 + ca]);
                uint4 o;
                o.x = pack_bf16x2(acc_a[0], acc_a[1]); o.y = pack_bf16x2(acc_a[2], acc_a[3]);
                o.z = pack_bf16x2(acc_a[4], acc_a[5]); o.w = pack_bf16x2(acc_a[6], acc_a[7]);
                out[(size_t)t * M8 + ca] = o;
            }
            if (in_b) {
                if (accumulate) fma8(acc_b, 1.0f, out_src[(size_t)t * M8 + cb]);
                uint4 o;
                o.x = pack_bf16x2(acc_b[0], acc_b[1]); o.y = pack_bf16x2(acc_b[2], acc_b[3]);
                o.z = pack_bf16x2(acc_b[4], acc_b[5]); o.w = pack_bf16x2(acc_b[6], acc_b[7]);
                out[(size_t)t * M8 + cb] = o;
            }
        }
    }
}

hipError_t launch_combine(const void* y, const int32_t* pos, const float* w, int Tn, int k, int M,
                          bool accumulate, int y_mode, const void* out_src, void* out, int grid, hipStream_t s)
{
    if (Tn <= 0) return hipSuccess;
    if (y_mode < 0 || y_mode > 2) return hipErrorInvalidValue;
    auto* yy = static_cast<const uint4*>(y);
    auto* oo = static_cast<uint4*>(out);
    auto* src = static_cast<const uint4*>(out_src ? out_src : out);
    const bool all_rows = out_src != nullptr && out_src != out;
    if (y_mode == 0) hipLaunchKernelGGL(combine_kernel<0>, dim3(grid), dim3(256), 0, s, yy, pos, w, Tn, k, M / 8, accumulate, all_rows, src, oo);
    else if (y_mode == 1) hipLaunchKernelGGL(combine_kernel<1>, dim3(grid), dim3(256), 0, s, yy, pos, w, Tn, k, M / 8, accumulate, all_rows, src, oo);
    else hipLaunchKernelGGL(combine_kernel<2>, dim3(grid), dim3(256), 0, s, yy, pos, w, Tn, k, M / 8, accumulate, all_rows, src, oo);
    return hipGetLastError();
}

}  // namespace moe_ep
