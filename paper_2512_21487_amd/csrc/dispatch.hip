// Partition of the kept assignments by local expert (Sec. 2.1; Sec. 3.1 "The MoE Part"):
// a deterministic, stable counting sort.
//   permute  from the router's per-workgroup bit masks (one bit per token and expert) every
//            64-token workgroup derives the per-expert counts, their prefix sum and the rows its
//            own tokens start at; every assignment then finds its row: expert base + rows of
//            earlier workgroups + number of earlier tokens of the workgroup with the same expert
//            (a popcount)
//   gather   the token rows are copied into expert-grouped order, 16 bytes per lane (only when
//            the gate/up projection does not gather them itself)
#include "common.h"
#include "kernels.h"

namespace moe_ep {

// One launch: every workgroup (64 tokens) sums the populations of all workgroups' masks itself --
// per expert the total and the part that lies before it -- instead of waiting for a scan kernel
// (nblk * El popcounts per workgroup, from L2; a launch boundary costs more).  Workgroup 0 also
// writes the per-expert counts and their prefix sum for the GEMMs.
__global__ __launch_bounds__(256) void dispatch_permute_kernel(
    const int32_t* __restrict__ idx, const unsigned long long* __restrict__ blk_mask, int nblk, int Tn, int k,
    int e0, int El, int32_t* __restrict__ count, int32_t* __restrict__ offset, int32_t* __restrict__ pos,
    int32_t* __restrict__ perm)
{
    extern __shared__ unsigned long long smem[];
    unsigned long long* smask = smem;
    int* sbase = reinterpret_cast<int*>(smem + El);   // rows of this workgroup's tokens before it, then the row base
    int* stotal = sbase + El;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, blk = blockIdx.x;
    for (int e = wave; e < El; e += 4) {
        int total = 0, before = 0;
        for (int b0 = 0; b0 < nblk; b0 += 64) {
            const int b = b0 + lane;
            const unsigned long long m = (b < nblk) ? blk_mask[(size_t)b * El + e] : 0ull;
            const int c = __popcll(m);
            total += c;
            before += (b < blk) ? c : 0;
            if (b == blk) smask[e] = m;
        }
#pragma unroll
        for (int d = 32; d >= 1; d >>= 1) {
            total += __shfl_xor(total, d, 64);
            before += __shfl_xor(before, d, 64);
        }
        if (lane == 0) { stotal[e] = total; sbase[e] = before; }
    }
    __syncthreads();
    if (wave == 0) {
        // exclusive prefix of the totals over the experts; El <= 512: a lane owns 8 consecutive experts
        int c[8], rows = 0;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int e = lane * 8 + i;
            c[i] = (e < El) ? stotal[e] : 0;
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
            if (e < El) {
                sbase[e] += r;
                if (blk == 0) { count[e] = c[i]; offset[e] = r; }
            }
            if (e == El && blk == 0) offset[e] = r;
            r += c[i];
        }
        if (El == 512 && lane == 63 && blk == 0) offset[El] = r;
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

// no tokens: the counts and their prefix sum are zeros
__global__ void dispatch_empty_kernel(int El, int32_t* __restrict__ count, int32_t* __restrict__ offset)
{
    for (int e = threadIdx.x; e <= El; e += blockDim.x) {
        if (e < El) count[e] = 0;
        offset[e] = 0;
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

hipError_t launch_dispatch(const int32_t* idx, const unsigned long long* blk_mask, int Tn, int k, int e0, int El,
                           int32_t* count, int32_t* offset, int32_t* pos, int32_t* perm, hipStream_t s)
{
    if (Tn <= 0) {
        hipLaunchKernelGGL(dispatch_empty_kernel, dim3(1), dim3(256), 0, s, El, count, offset);
        return hipGetLastError();
    }
    const int nblk = (Tn + kTokPerBlock - 1) / kTokPerBlock;
    hipLaunchKernelGGL(dispatch_permute_kernel, dim3(nblk), dim3(256),
                       El * (sizeof(unsigned long long) + 2 * sizeof(int)), s, idx, blk_mask, nblk, Tn, k, e0, El,
                       count, offset, pos, perm);
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
