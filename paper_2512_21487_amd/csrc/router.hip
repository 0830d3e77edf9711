// Gate: per token, the top-k of E routing scores and their renormalised softmax weights
// (Sec. 2.1).  A token is owned by one 16-lane row of a wavefront, so a wavefront advances four
// tokens at once: lane l of the row holds scores l, l+16, ... in registers, and each of the k
// selection rounds is a lane-local scan plus a four-step arg-max over the row done with DPP
// lane exchanges (quad swaps and row mirrors: register moves, no LDS traffic).
// The same workgroup (64 tokens) also records, per local expert, a 64-bit mask of the
// tokens that selected it; the partition kernels derive counts and stable ranks from it,
// so no atomically allocated slot ever decides an order.
#include "common.h"
#include "kernels.h"

namespace moe_ep {

constexpr int kRouterThreads = 1024;  // 16 wavefronts x 4 rows = the 64 tokens of a workgroup

// the value lane (lane ^ pattern) of the same 16-lane row holds; ctrl is a DPP control:
// 0xB1 / 0x4E swap neighbours / pairs inside a quad, 0x141 / 0x140 mirror a half row / a row
template <int CTRL>
__device__ __forceinline__ int row_exchange(int x) { return __builtin_amdgcn_update_dpp(x, x, CTRL, 0xF, 0xF, false); }

// larger score first, equal scores keep the lower expert index
__device__ __forceinline__ void keep_better(float& bv, int& bi, float ov, int oi)
{
    if (ov > bv || (ov == bv && oi < bi)) { bv = ov; bi = oi; }
}

template <int CTRL>
__device__ __forceinline__ void row_argmax_step(float& bv, int& bi)
{
    const float ov = __builtin_bit_cast(float, row_exchange<CTRL>(__builtin_bit_cast(int, bv)));
    const int oi = row_exchange<CTRL>(bi);
    keep_better(bv, bi, ov, oi);
}

template <int EPL>  // scores per lane: E <= 16 * EPL
__global__ __launch_bounds__(kRouterThreads) void router_topk_kernel(
    const float* __restrict__ logits, int Tn, int E, int k, int e0, int El,
    int32_t* __restrict__ idx, float* __restrict__ w, unsigned long long* __restrict__ blk_mask)
{
    extern __shared__ unsigned long long smask[];                  // [El] token masks of the local experts
    int* s_idx = reinterpret_cast<int*>(smask + El);               // [64][k] selected experts
    float* s_ex = reinterpret_cast<float*>(s_idx + kTokPerBlock * k);  // [64][k] exp(score - best score)
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int sub = lane & 15, tl = wave * 4 + (lane >> 4);        // lane inside the row; token inside the block
    for (int i = tid; i < El; i += kRouterThreads) smask[i] = 0ull;
    __syncthreads();

    const int t = blockIdx.x * kTokPerBlock + tl;
    const bool live = t < Tn;
    const float* row = logits + (size_t)min(t, Tn - 1) * E;
    float v[EPL];
    unsigned taken = 0;  // bit i: score i of this lane is out of range or already selected
#pragma unroll
    for (int i = 0; i < EPL; ++i) {
        const int e = sub + 16 * i;
        if (e < E) v[i] = row[e]; else { v[i] = 0.f; taken |= 1u << i; }
    }
    float v0 = 0.f, sum = 0.f;
    for (int s = 0; s < k; ++s) {
        float bv = -INFINITY;
        int bi = INT_MAX;
#pragma unroll
        for (int i = 0; i < EPL; ++i)  // ascending index inside a lane: a strict > keeps the lower one
            if (!((taken >> i) & 1u) && (bi == INT_MAX || v[i] > bv)) { bv = v[i]; bi = sub + 16 * i; }
        row_argmax_step<0xB1>(bv, bi);
        row_argmax_step<0x4E>(bv, bi);
        row_argmax_step<0x141>(bv, bi);
        row_argmax_step<0x140>(bv, bi);   // every lane of the row now holds the round's winner
        if ((bi & 15) == sub) taken |= 1u << (bi >> 4);
        if (s == 0) v0 = bv;
        // softmax restricted to the selection = full softmax renormalised over it
        const float ex = expf(bv - v0);
        sum += ex;
        if (sub == 0 && live) {
            s_idx[tl * k + s] = bi;
            s_ex[tl * k + s] = ex;
            const int el = bi - e0;
            if (el >= 0 && el < El) atomicOr(&smask[el], 1ull << tl);
        }
    }
    __syncthreads();
    if (live)
        for (int s = sub; s < k; s += 16) {
            idx[(size_t)t * k + s] = s_idx[tl * k + s];
            w[(size_t)t * k + s] = s_ex[tl * k + s] / sum;
        }
    unsigned long long* dst = blk_mask + (size_t)blockIdx.x * El;
    for (int i = tid; i < El; i += kRouterThreads) dst[i] = smask[i];
}

hipError_t launch_router(const float* logits, int Tn, int E, int k, int e0, int El, int32_t* idx,
                         float* w, unsigned long long* blk_mask, hipStream_t s)
{
    if (Tn <= 0) return hipSuccess;
    if (E < 1 || E > 512 || k < 1 || k > 64) return hipErrorInvalidValue;
    const int nblk = (Tn + kTokPerBlock - 1) / kTokPerBlock;
    const size_t lds = El * sizeof(unsigned long long) + (size_t)kTokPerBlock * k * 8;
#define MOE_EP_ROUTER(EPL)                                                                          \
    hipLaunchKernelGGL(router_topk_kernel<EPL>, dim3(nblk), dim3(kRouterThreads), lds, s, logits, Tn, E, k, e0, \
                       El, idx, w, blk_mask)
    if (E <= 16) MOE_EP_ROUTER(1);
    else if (E <= 32) MOE_EP_ROUTER(2);
    else if (E <= 64) MOE_EP_ROUTER(4);
    else if (E <= 128) MOE_EP_ROUTER(8);
    else if (E <= 160) MOE_EP_ROUTER(10);
    else if (E <= 256) MOE_EP_ROUTER(16);
    else MOE_EP_ROUTER(32);
#undef MOE_EP_ROUTER
    return hipGetLastError();
}

}  // namespace moe_ep
