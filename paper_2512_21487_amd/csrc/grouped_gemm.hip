// Expert projections as a grouped bf16 GEMM on the CDNA4 matrix cores
// (Sec. 3.1: z_gate = W_gate h, z_up = W_up h, z_down = W_down act; Eq. moe_detail,
// Eq. shared_detail).
//
// Both operands are K-contiguous in memory (activations [rows, K], weights [N, K]), which is
// exactly what v_mfma_f32_32x32x16_bf16 wants per lane: 8 consecutive K values of one row.
// The weight rows feed the instruction's first operand and the token rows the second, so a
// lane ends up with 4 consecutive output columns of one token row -> 8-byte bf16 stores.
//
// One launch covers all experts.  Workgroups are persistent and walk a tile list that is
// defined by device-side prefix sums (the host never learns the routing): tile id ->
// (expert, column tile, row tile), row tiles fastest so that the workgroups of one XCD
// share a weight panel through that XCD's L2.  The id -> workgroup map hands each XCD
// contiguous runs of tile ids (workgroup b runs on XCD b mod 8).
//
// LDS tiles are [rows][64] bf16 (128 B per row, eight 16-byte chunks) with the chunk index
// XOR-ed by bits 1..3 of the row, which makes both the 16-byte staging stores and the
// MFMA fragment loads conflict-free.  Two stages: global -> registers for step kt+1 is in
// flight while step kt is multiplied out of LDS; one barrier per step.
//
// SwiGLU: the weight tile holds BN/2 rows of W_gate and the matching BN/2 rows of W_up; a
// wavefront's accumulator blocks pair a gate block with the up block of the same columns,
// so act = silu(z_gate) * z_up is formed in registers and only act is written.
#include "common.h"
#include "kernels.h"

namespace moe_ep {

constexpr int kBM = 128;  // rows per tile, shared by all variants (the scan kernel counts row tiles with it)

template <int BM, int BN, int WGM, int WGN, bool SWIGLU>
struct GemmCfg {
    static constexpr int BK = 64;
    static constexpr int THREADS = WGM * WGN * 64;
    static constexpr int WTM = BM / WGM, WTN = BN / WGN;
    static constexpr int MB = WTM / 32, NB = WTN / 32;
    static constexpr int XL = BM * 8 / THREADS, WL = BN * 8 / THREADS;
    static constexpr int ROWS_PER_PASS = THREADS / 8;
    static constexpr int STAGE_CHUNKS = (BM + BN) * 8;
    static constexpr int LDS_BYTES = 2 * STAGE_CHUNKS * 16;
    static constexpr int BN_OUT = SWIGLU ? BN / 2 : BN;
    static_assert(BM % (WGM * 32) == 0 && BN % (WGN * 32) == 0, "wave tiles are 32x32 blocks");
    static_assert(!SWIGLU || NB % 2 == 0, "gate/up blocks pair up inside a wavefront");
    static_assert((BM * 8) % THREADS == 0 && (BN * 8) % THREADS == 0, "whole staging passes");
};

__device__ __forceinline__ float silu_f(float g) { return g / (1.0f + __expf(-g)); }

template <int BM, int BN, int WGM, int WGN, bool SWIGLU, bool RAGGED>
__global__ __launch_bounds__(WGM* WGN * 64) void grouped_gemm_kernel(GemmArgs a)
{
    using Cfg = GemmCfg<BM, BN, WGM, WGN, SWIGLU>;
    constexpr int MB = Cfg::MB, NB = Cfg::NB, XL = Cfg::XL, WL = Cfg::WL;
    constexpr int THREADS = Cfg::THREADS, BN_OUT = Cfg::BN_OUT;
    extern __shared__ uint4 lds[];
    __shared__ int s_pref[513];
    __shared__ int s_off[513];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WGN, wn = wave % WGN;
    constexpr bool ragged = RAGGED;  // routed experts: ragged groups from device prefix sums; shared: dense
    const int NT = (a.N + BN_OUT - 1) / BN_OUT;
    int mt_total, mt_per = 0;
    if (ragged) {
        for (int i = tid; i <= a.G; i += THREADS) { s_pref[i] = a.mt_prefix[i]; s_off[i] = a.offset[i]; }
        __syncthreads();
        mt_total = s_pref[a.G];
    } else {
        mt_per = (a.dense_rows + BM - 1) / BM;
        mt_total = mt_per * a.G;
    }
    const int total = mt_total * NT;
    const int per_xcd = gridDim.x >> 3;
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    const int KT = a.K / Cfg::BK;

    // staging geometry of this thread: chunk column c, first row r0, swizzled LDS chunk
    const int c_ld = tid & 7, r0_ld = tid >> 3;
    const int st_chunk = r0_ld * 8 + (c_ld ^ ((r0_ld >> 1) & 7));
    // fragment geometry of this lane
    const int fr_row = lane & 31, fr_sw = (lane >> 1) & 7, fr_kh = lane >> 5;

    for (int it = 0;; ++it) {
        const int L = (it * 8 + xcd) * per_xcd + slot;
        if (L >= total) break;
        int g, mi, ni, row0, nrows;
        if (ragged) {
            int lo = 0, hi = a.G;
            while (hi - lo > 1) {
                const int mid = (lo + hi) >> 1;
                if (s_pref[mid] * NT <= L) lo = mid; else hi = mid;
            }
            g = lo;
            const int mt_g = s_pref[g + 1] - s_pref[g];
            const int l = L - s_pref[g] * NT;
            ni = l / mt_g; mi = l - ni * mt_g;
            row0 = s_off[g] + mi * BM;
            nrows = min(BM, s_off[g + 1] - row0);
        } else {
            const int per_g = mt_per * NT;
            g = L / per_g;
            const int l = L - g * per_g;
            ni = l / mt_per; mi = l - ni * mt_per;
            row0 = mi * BM;
            nrows = min(BM, a.dense_rows - row0);
        }
        const int n0 = ni * BN_OUT;
        const uint16_t* Wg = a.W + (size_t)g * a.w_group_stride;

        // row pointers of the chunks this thread stages (rows past the end re-read the last valid row)
        const uint16_t* xptr[XL];
        const uint16_t* wptr[WL];
#pragma unroll
        for (int i = 0; i < XL; ++i) {
            const int r = min(r0_ld + i * Cfg::ROWS_PER_PASS, nrows - 1);
            xptr[i] = a.A + (size_t)(row0 + r) * a.lda + c_ld * 8;
        }
#pragma unroll
        for (int i = 0; i < WL; ++i) {
            const int j = r0_ld + i * Cfg::ROWS_PER_PASS;  // row of the LDS weight tile
            int n;
            const uint16_t* base = Wg;
            if (SWIGLU) {
                if (j < BN / 2) n = n0 + j; else { n = n0 + j - BN / 2; base = Wg + a.w_up_offset; }
            } else {
                n = n0 + j;
            }
            n = min(n, a.N - 1);
            wptr[i] = base + (size_t)n * a.ldw + c_ld * 8;
        }

        f32x16_t acc[MB][NB];
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
#pragma unroll
            for (int nb = 0; nb < NB; ++nb)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[mb][nb][r] = 0.f;

        uint4 xreg[XL], wreg[WL];
        auto load_global = [&](int kt) {
            const int k = kt * Cfg::BK;
            const int seg = k / a.kseg_len;
            const size_t wk = (size_t)seg * a.w_kseg_stride + (k - seg * a.kseg_len);
#pragma unroll
            for (int i = 0; i < XL; ++i) xreg[i] = *reinterpret_cast<const uint4*>(xptr[i] + k);
#pragma unroll
            for (int i = 0; i < WL; ++i) wreg[i] = *reinterpret_cast<const uint4*>(wptr[i] + wk);
        };
        auto store_lds = [&](int buf) {
            uint4* sX = lds + buf * Cfg::STAGE_CHUNKS;
            uint4* sW = sX + BM * 8;
#pragma unroll
            for (int i = 0; i < XL; ++i) sX[st_chunk + i * Cfg::ROWS_PER_PASS * 8] = xreg[i];
#pragma unroll
            for (int i = 0; i < WL; ++i) sW[st_chunk + i * Cfg::ROWS_PER_PASS * 8] = wreg[i];
        };

        load_global(0);
        store_lds(0);
        __syncthreads();
        for (int kt = 0; kt < KT; ++kt) {
            const int buf = kt & 1;
            if (kt + 1 < KT) load_global(kt + 1);
            const uint4* sX = lds + buf * Cfg::STAGE_CHUNKS;
            const uint4* sW = sX + BM * 8;
#pragma unroll
            for (int kk = 0; kk < 4; ++kk) {
                const int csw = (kk * 2 + fr_kh) ^ fr_sw;
                bf16x8_t xf[MB], wf[NB];
#pragma unroll
                for (int mb = 0; mb < MB; ++mb) {
                    const int row = wm * Cfg::WTM + mb * 32 + fr_row;
                    xf[mb] = __builtin_bit_cast(bf16x8_t, sX[row * 8 + csw]);
                }
#pragma unroll
                for (int nb = 0; nb < NB; ++nb) {
                    int rb;
                    if (SWIGLU) rb = (nb < NB / 2) ? wn * (Cfg::WTN / 2) + nb * 32
                                                   : BN / 2 + wn * (Cfg::WTN / 2) + (nb - NB / 2) * 32;
                    else rb = wn * Cfg::WTN + nb * 32;
                    wf[nb] = __builtin_bit_cast(bf16x8_t, sW[(rb + fr_row) * 8 + csw]);
                }
#pragma unroll
                for (int nb = 0; nb < NB; ++nb)
#pragma unroll
                    for (int mb = 0; mb < MB; ++mb)
                        acc[mb][nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[nb], xf[mb], acc[mb][nb], 0, 0, 0);
            }
            if (kt + 1 < KT) store_lds(buf ^ 1);
            __syncthreads();
        }

        // epilogue: lane holds token row (lane & 31) of each block and, per register quad q,
        // output columns 8q + 4*(lane >> 5) + {0..3} of the block
        uint16_t* Cg = a.C + (size_t)g * a.c_group_col_stride;
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) {
            const int m = wm * Cfg::WTM + mb * 32 + fr_row;
            if (m >= nrows) continue;
            uint16_t* crow = Cg + (size_t)(row0 + m) * a.ldc;
            if (SWIGLU) {
#pragma unroll
                for (int nb = 0; nb < NB / 2; ++nb)
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const int n = n0 + wn * (Cfg::WTN / 2) + nb * 32 + q * 8 + fr_kh * 4;
                        if (n >= a.N) continue;
                        float h[4];
#pragma unroll
                        for (int i = 0; i < 4; ++i)
                            h[i] = silu_f(acc[mb][nb][q * 4 + i]) * acc[mb][nb + NB / 2][q * 4 + i];
                        uint2 o;
                        o.x = pack_bf16x2(h[0], h[1]); o.y = pack_bf16x2(h[2], h[3]);
                        *reinterpret_cast<uint2*>(crow + n) = o;
                    }
            } else {
#pragma unroll
                for (int nb = 0; nb < NB; ++nb)
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const int n = n0 + wn * Cfg::WTN + nb * 32 + q * 8 + fr_kh * 4;
                        if (n >= a.N) continue;
                        uint2 o;
                        o.x = pack_bf16x2(acc[mb][nb][q * 4 + 0], acc[mb][nb][q * 4 + 1]);
                        o.y = pack_bf16x2(acc[mb][nb][q * 4 + 2], acc[mb][nb][q * 4 + 3]);
                        *reinterpret_cast<uint2*>(crow + n) = o;
                    }
            }
        }
    }
}

template <int BM, int BN, int WGM, int WGN, bool SWIGLU, bool RAGGED>
static hipError_t launch_variant(const GemmArgs& a, int n_cu, int max_row_tiles, hipStream_t s)
{
    using Cfg = GemmCfg<BM, BN, WGM, WGN, SWIGLU>;
    const int NT = (a.N + Cfg::BN_OUT - 1) / Cfg::BN_OUT;
    const long long max_tiles = (long long)max_row_tiles * NT;
    if (max_tiles <= 0) return hipSuccess;
    const int occ = (160 * 1024) / Cfg::LDS_BYTES >= 2 ? 2 : 1;
    long long grid = (long long)n_cu * occ;
    if (grid > max_tiles) grid = max_tiles;
    grid = (grid + 7) / 8 * 8;
    hipLaunchKernelGGL((grouped_gemm_kernel<BM, BN, WGM, WGN, SWIGLU, RAGGED>), dim3((unsigned)grid),
                       dim3(Cfg::THREADS), Cfg::LDS_BYTES, s, a);
    return hipGetLastError();
}

template <int BM, int BN, int WGM, int WGN, bool SWIGLU, bool RAGGED>
static hipError_t raise_lds_limit()
{
    using Cfg = GemmCfg<BM, BN, WGM, WGN, SWIGLU>;
    return hipFuncSetAttribute(
        reinterpret_cast<const void*>(&grouped_gemm_kernel<BM, BN, WGM, WGN, SWIGLU, RAGGED>),
        hipFuncAttributeMaxDynamicSharedMemorySize, Cfg::LDS_BYTES);
}

template <int BN>
static hipError_t raise_all()
{
    hipError_t e;
    if ((e = raise_lds_limit<kBM, BN, 2, 2, true, true>()) != hipSuccess) return e;
    if ((e = raise_lds_limit<kBM, BN, 2, 2, true, false>()) != hipSuccess) return e;
    if ((e = raise_lds_limit<kBM, BN, 2, 2, false, true>()) != hipSuccess) return e;
    return raise_lds_limit<kBM, BN, 2, 2, false, false>();
}

hipError_t grouped_gemm_init()
{
    hipError_t e = raise_all<256>();
    return e != hipSuccess ? e : raise_all<128>();
}

int grouped_gemm_row_tile() { return kBM; }

template <int BN>
static hipError_t launch_bn(const GemmArgs& a, bool swiglu, int n_cu, int max_row_tiles, hipStream_t s)
{
    const bool ragged = a.offset != nullptr;
    if (swiglu) return ragged ? launch_variant<kBM, BN, 2, 2, true, true>(a, n_cu, max_row_tiles, s)
                              : launch_variant<kBM, BN, 2, 2, true, false>(a, n_cu, max_row_tiles, s);
    return ragged ? launch_variant<kBM, BN, 2, 2, false, true>(a, n_cu, max_row_tiles, s)
                  : launch_variant<kBM, BN, 2, 2, false, false>(a, n_cu, max_row_tiles, s);
}

hipError_t launch_grouped_gemm(const GemmArgs& a, bool swiglu, int variant, int n_cu,
                               int max_row_tiles, hipStream_t s)
{
    if (variant == 1) return launch_bn<128>(a, swiglu, n_cu, max_row_tiles, s);
    return launch_bn<256>(a, swiglu, n_cu, max_row_tiles, s);
}

}  // namespace moe_ep
