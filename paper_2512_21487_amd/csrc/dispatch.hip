// Partition of the kept assignments by local expert (Sec. 2.1; Sec. 3.1 "The MoE Part"):
// a deterministic, stable counting sort in three steps.
//   scan     per expert, exclusive prefix over the 64-token workgroups of the router's
//            bit-mask populations -> first row of every (workgroup, expert) pair, the
//            per-expert counts and their prefix sum
//   permute  every assignment finds its row: expert base + workgroup base + number of
//            earlier tokens of the workgroup with the same expert (a popcount)
//   gather   the token rows are copied into expert-grouped order, 16 bytes per lane
#include "common.h"
#include "kernels.h"

namespace moe_ep {

__global__ __launch_bounds__(1024) void dispatch_scan_kernel(
    const unsigned long long* __restrict__ blk_mask, int nblk, int El,
    int32_t* __restrict__ blk_off, int32_t* __restrict__ count, int32_t* __restrict__ offset)
{
    __shared__ int s_count[512];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    for (int e = wave; e < El; e += 16) {
        int carry = 0;
        for (int b0 = 0; b0 < nblk; b0 += 64) {
            const int b = b0 + lane;
            const int c = (b < nblk) ? __popcll(blk_mask[(size_t)b * El + e]) : 0;
            int x = c;
#pragma unroll
            for (int d = 1; d < 64; d <<= 1) {
                const int y = __shfl_up(x, d, 64);
                if (lane >= d) x += y;
            }
            if (b < nblk) blk_off[(size_t)b * El + e] = carry + x - c;
            carry += __shfl(x, 63, 64);
        }
        if (lane == 0) s_count[e] = carry;
    }
    __syncthreads();
    if (wave == 0) {
        // El <= 512: lane owns 8 consecutive experts
        int c[8], rows = 0;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int e = lane * 8 + i;
            c[i] = (e < El) ? s_count[e] : 0;
            rows += c[i];
        }
        int xr = rows;
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            const int yr = __shfl_up(xr, d, 64);
            if (lane >= d) xr += yr;
        }
        int r = xr - rows;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int e = lane * 8 + i;
            if (e < El) { count[e] = c[i]; offset[e] = r; }
            if (e == El) offset[e] = r;
            r += c[i];
        }
        if (El == 512 && lane == 63) offset[El] = r;
    }
}

__global__ __launch_bounds__(256) void dispatch_permute_kernel(
    const int32_t* __restrict__ idx, const unsigned long long* __restrict__ blk_mask,
    const int32_t* __restrict__ blk_off, const int32_t* __restrict__ offset, int Tn, int k, int e0,
    int El, int32_t* __restrict__ pos, int32_t* __restrict__ perm)
{
    extern __shared__ unsigned long long smem[];
    unsigned long long* smask = smem;
    int* sbase = reinterpret_cast<int*>(smem + El);
    const int tid = threadIdx.x, blk = blockIdx.x;
    for (int i = tid; i < El; i += 256) {
        smask[i] = blk_mask[(size_t)blk * El + i];
        sbase[i] = offset[i] + blk_off[(size_t)blk * El + i];
    }
    __syncthreads();
    const int t_begin = blk * kTokPerBlock;
    const int n_tok = min(kTokPerBlock, Tn - t_begin);
    for (int a = tid; a < n_tok * k; a += 256) {
        const int tl = a / k;
        const size_t ga = (size_t)t_begin * k + a;  // global assignment id = t*k + slot
        const int e = idx[ga] - e0;
        int p = -1;
        if (e >= 0 && e < El) {
            p = sbase[e] + __popcll(smask[e] & ((1ull << tl) - 1ull));
            perm[p] = (int32_t)ga;
        }
        pos[ga] = p;
    }
}

__global__ __launch_bounds__(256) void gather_rows_kernel(
    const uint4* __restrict__ tokens, const int32_t* __restrict__ perm,
    const int32_t* __restrict__ n_rows_ptr, int k, int M8, uint4* __restrict__ xp)
{
    const int A = *n_rows_ptr;
    const int lane = threadIdx.x & 63;
    const int gw = (blockIdx.x * 256 + threadIdx.x) >> 6, nw = gridDim.x * 4;
    for (int p = gw; p < A; p += nw) {
        const int t = perm[p] / k;
        const uint4* src = tokens + (size_t)t * M8;
        uint4* dst = xp + (size_t)p * M8;
        int c = lane;
        for (; c + 192 < M8; c += 256) {
            const uint4 a0 = src[c], a1 = src[c + 64], a2 = src[c + 128], a3 = src[c + 192];
            dst[c] = a0; dst[c + 64] = a1; dst[c + 128] = a2; dst[c + 192] = a3;
        }
        for (; c < M8; c += 64) dst[c] = src[c];
    }
}

hipError_t launch_dispatch_scan(const unsigned long long* blk_mask, int nblk, int El,
                                int32_t* blk_off, int32_t* count, int32_t* offset, hipStream_t s)
{
    hipLaunchKernelGGL(dispatch_scan_kernel, dim3(1), dim3(1024), 0, s, blk_mask, nblk, El,
                       blk_off, count, offset);
    return hipGetLastError();
}

hipError_t launch_dispatch_permute(const int32_t* idx, const unsigned long long* blk_mask,
                                   const int32_t* blk_off, const int32_t* offset, int Tn, int k,
                                   int e0, int El, int32_t* pos, int32_t* perm, hipStream_t s)
{
    if (Tn <= 0) return hipSuccess;
    const int nblk = (Tn + kTokPerBlock - 1) / kTokPerBlock;
    hipLaunchKernelGGL(dispatch_permute_kernel, dim3(nblk), dim3(256),
                       El * (sizeof(unsigned long long) + sizeof(int)), s, idx, blk_mask, blk_off,
                       offset, Tn, k, e0, El, pos, perm);
    return hipGetLastError();
}

hipError_t launch_gather_rows(const void* tokens, const int32_t* perm, const int32_t* n_rows_ptr,
                              int k, int M, void* xp, int grid, hipStream_t s)
{
    hipLaunchKernelGGL(gather_rows_kernel, dim3(grid), dim3(256), 0, s,
                       static_cast<const uint4*>(tokens), perm, n_rows_ptr, k, M / 8,
                       static_cast<uint4*>(xp));
    return hipGetLastError();
}

}  // namespace moe_ep
