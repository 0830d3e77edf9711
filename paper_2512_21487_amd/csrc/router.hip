// Gate: per token, the top-k of E routing scores and their renormalised softmax weights
// (Sec. 2.1).  One 64-lane wavefront owns a token at a time (four tokens in turn, their scores
// all requested up front): lane l holds scores l, l+64, ... in registers, each of the k rounds
// is a lane-local scan plus a 6-step butterfly arg-max.
// The same workgroup (64 tokens) also records, per local expert, a 64-bit mask of the
// tokens that selected it; the partition kernels derive counts and stable ranks from it,
// so no atomically allocated slot ever decides an order.
#include "common.h"
#include "kernels.h"

namespace moe_ep {

constexpr int kMaxEpl = 8;  // scores per lane: E <= 512

constexpr int kRouterThreads = 1024;                                   // 16 wavefronts per 64-token workgroup
constexpr int kTokPerWave = kTokPerBlock / (kRouterThreads / 64);      // 4 tokens per wavefront

__global__ __launch_bounds__(kRouterThreads) void router_topk_kernel(
    const float* __restrict__ logits, int Tn, int E, int k, int e0, int El,
    int32_t* __restrict__ idx, float* __restrict__ w, unsigned long long* __restrict__ blk_mask)
{
    extern __shared__ unsigned long long smask[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    for (int i = tid; i < El; i += kRouterThreads) smask[i] = 0ull;
    __syncthreads();

    const int epl = (E + 63) >> 6;
    // all of this wavefront's scores are requested before the first one is used
    float v[kTokPerWave][kMaxEpl];
#pragma unroll
    for (int j = 0; j < kTokPerWave; ++j) {
        const int t = blockIdx.x * kTokPerBlock + wave * kTokPerWave + j;
        const float* row = logits + (size_t)min(t, Tn - 1) * E;
#pragma unroll
        for (int i = 0; i < kMaxEpl; ++i) {
            const int e = lane + 64 * i;
            v[j][i] = (i < epl && e < E) ? row[e] : 0.f;
        }
    }
    // the four tokens advance through the k selection rounds together: their arg-max chains are
    // independent, so the cross-lane exchanges of one token hide behind those of the others
    unsigned taken[kTokPerWave];
    int my_idx[kTokPerWave];
    float my_val[kTokPerWave];
#pragma unroll
    for (int j = 0; j < kTokPerWave; ++j) {
        taken[j] = 0; my_idx[j] = 0; my_val[j] = 0.f;
#pragma unroll
        for (int i = 0; i < kMaxEpl; ++i)
            if (!(i < epl && lane + 64 * i < E)) taken[j] |= 1u << i;
    }
    for (int s = 0; s < k; ++s) {
        float bv[kTokPerWave];
        int bi[kTokPerWave];
#pragma unroll
        for (int j = 0; j < kTokPerWave; ++j) {
            // lane-local best: larger score first, equal scores keep the lower index
            bv[j] = -INFINITY; bi[j] = INT_MAX;
#pragma unroll
            for (int i = 0; i < kMaxEpl; ++i)
                if (!((taken[j] >> i) & 1u) && (bi[j] == INT_MAX || v[j][i] > bv[j])) { bv[j] = v[j][i]; bi[j] = lane + 64 * i; }
        }
#pragma unroll
        for (int d = 32; d >= 1; d >>= 1) {
#pragma unroll
            for (int j = 0; j < kTokPerWave; ++j) {
                const float ov = __shfl_xor(bv[j], d, 64);
                const int oi = __shfl_xor(bi[j], d, 64);
                if (ov > bv[j] || (ov == bv[j] && oi < bi[j])) { bv[j] = ov; bi[j] = oi; }
            }
        }
#pragma unroll
        for (int j = 0; j < kTokPerWave; ++j) {
            if ((bi[j] & 63) == lane) taken[j] |= 1u << (bi[j] >> 6);
            if (lane == s) { my_idx[j] = bi[j]; my_val[j] = bv[j]; }
        }
    }
#pragma unroll
    for (int j = 0; j < kTokPerWave; ++j) {
        const int tl = wave * kTokPerWave + j;
        const int t = blockIdx.x * kTokPerBlock + tl;
        if (t >= Tn) break;  // uniform over the wavefront
        // softmax restricted to the selection = full softmax renormalised over it
        const float v0 = __shfl(my_val[j], 0, 64);
        const float ex = (lane < k) ? expf(my_val[j] - v0) : 0.f;
        float sum = ex;
#pragma unroll
        for (int d = 32; d >= 1; d >>= 1) sum += __shfl_xor(sum, d, 64);
        if (lane < k) {
            idx[(size_t)t * k + lane] = my_idx[j];
            w[(size_t)t * k + lane] = ex / sum;
            const int el = my_idx[j] - e0;
            if (el >= 0 && el < El) atomicOr(&smask[el], 1ull << tl);
        }
    }
    __syncthreads();
    unsigned long long* dst = blk_mask + (size_t)blockIdx.x * El;
    for (int i = tid; i < El; i += kRouterThreads) dst[i] = smask[i];
}

hipError_t launch_router(const float* logits, int Tn, int E, int k, int e0, int El, int32_t* idx,
                         float* w, unsigned long long* blk_mask, hipStream_t s)
{
    if (Tn <= 0) return hipSuccess;
    const int nblk = (Tn + kTokPerBlock - 1) / kTokPerBlock;
    hipLaunchKernelGGL(router_topk_kernel, dim3(nblk), dim3(kRouterThreads), El * sizeof(unsigned long long), s,
                       logits, Tn, E, k, e0, El, idx, w, blk_mask);
    return hipGetLastError();
}

}  // namespace moe_ep
