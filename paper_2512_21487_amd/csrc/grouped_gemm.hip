// Expert projections as a grouped bf16 GEMM on the CDNA4 matrix cores
// (Sec. 3.1: z_gate = W_gate h, z_up = W_up h, z_down = W_down act; Eq. moe_detail,
// Eq. shared_detail).
//
// Both operands are K-contiguous in memory (activations [rows, K], weights [N, K]), which is
// exactly what the bf16 matrix instructions want per lane: 8 consecutive K values of one row.
// The weight rows feed the instruction's first operand and the token rows the second, so a
// lane ends up with 4 consecutive output columns of one token row.  Two instruction shapes are
// built (template argument MI): v_mfma_f32_16x16x32_bf16 for the shapes the library picks by
// itself -- at the package power limit, where these launches run, it does the same work in the
// same number of cycles at a higher clock, because a 16 x 16 block moves fewer accumulator
// registers per multiply-add -- and v_mfma_f32_32x32x16_bf16.  The two give the same bits.
//
// One launch covers all experts.  Workgroups are persistent and walk a tile list that is
// defined by device-side prefix sums (the host never learns the routing): tile id ->
// (expert, band of row tiles, column tile, row tile in the band), so that the workgroups of
// one XCD share a few weight panels and a few row panels through that XCD's L2.  The id ->
// workgroup map hands each XCD contiguous runs of tile ids (workgroup b runs on XCD b mod 8).
//
// Data movement: global_load_lds_dwordx4 moves 16 bytes per lane from global memory straight
// into LDS (no staging registers, no ds_write), into a ring of STAGES K-steps: while step kt
// is multiplied, the loads of the next STAGES-1 steps are in flight.  One wave instruction
// fills 1 KB of LDS in lane order; LDS rows are BK bf16 wide and their 16-byte chunks are
// XOR-swizzled by the row so that MFMA fragment reads are bank-conflict free.  The swizzle
// is applied on the global side: lane l fetches the chunk that belongs at physical slot l.
// The loads are asynchronous: each wavefront counts its own with s_waitcnt vmcnt(n), then a
// raw s_barrier publishes every wavefront's rows (one barrier per K step).
//
// SwiGLU: the weight tile holds BN/2 rows of W_gate and the matching BN/2 rows of W_up; a
// wavefront's accumulator blocks pair a gate block with the up block of the same columns,
// so act = silu(z_gate) * z_up is formed in registers and only act is written.
#include <type_traits>

#include "common.h"
#include "kernels.h"

namespace moe_ep {

template <int BM, int BN, int BK_, int STAGES_, int WGM, int WGN, bool SWIGLU>
struct GemmCfg {
    static constexpr int BK = BK_, STAGES = STAGES_;
    static constexpr int CPR = BK / 8;             // 16-byte chunks per LDS row
    static constexpr int RP = 16 / CPR;            // LDS rows per 256 bytes (one sweep over all banks)
    static constexpr int RPR = 64 / CPR;           // LDS rows per 1 KB region (one wave load instruction)
    static constexpr int KKW = BK / 16;            // MFMA k16 steps per K step
    static constexpr int NW = WGM * WGN, THREADS = NW * 64;
    static constexpr int WTM = BM / WGM, WTN = BN / WGN;
    static constexpr int MB = WTM / 32, NB = WTN / 32;
    static constexpr int REGIONS = (BM + BN) / RPR;
    static constexpr int RPW = REGIONS / NW;       // regions each wavefront loads per stage
    static constexpr int XRPW = (BM / RPR) / NW;   // of which activation regions
    static constexpr int STAGE_CHUNKS = (BM + BN) * CPR;
    static constexpr int LDS_BYTES = STAGES * STAGE_CHUNKS * 16;
    static constexpr int BN_OUT = SWIGLU ? BN / 2 : BN;
    static_assert(BK == 32 || BK == 64, "LDS rows are 64 or 128 bytes");
    static_assert(BM % (WGM * 32) == 0 && BN % (WGN * 32) == 0, "wave tiles are 32x32 blocks");
    static_assert(!SWIGLU || NB % 2 == 0, "gate/up blocks pair up inside a wavefront");
    static_assert((BM / RPR) % NW == 0 && (BN / RPR) % NW == 0, "regions split evenly over wavefronts");
    static_assert(STAGES >= 2 && STAGES <= 5 && (STAGES - 2) * RPW <= 63, "ring depth and vmcnt budget");
    static_assert(KKW % 2 == 0, "a K step starts and ends on fragment set 0 / 1");
    // MFMAs between two hand-overs, and over how many of them (counted from the hand-over that
    // frees the slot) a wavefront spreads the RPW loads of one K step: a load blocks the
    // wavefront's instruction stream until the CU's memory pipeline takes it, so loads issued
    // faster than that pipeline drains stall the MFMAs queued behind them.  The last k16 step
    // before the next hand-over stays free: in a two-slot ring the last load needs that time to
    // land, and the deeper rings measure about 1 % faster with it than with the whole K step.
#ifndef MOE_EP_ISSUE_WINDOW
#define MOE_EP_ISSUE_WINDOW (KKW * MB * NB - MB * NB > RPW ? KKW * MB * NB - MB * NB : RPW)
#endif
    static constexpr int SLOTS = KKW * MB * NB;
    static constexpr int WINDOW = MOE_EP_ISSUE_WINDOW;
    static_assert(WINDOW >= RPW && WINDOW <= SLOTS, "at most one load per MFMA between two hand-overs");
    // the load issued behind MFMA number p after a hand-over, or -1
    static constexpr int load_at(int p)
    {
        const int l = (p * RPW + WINDOW - 1) / WINDOW;
        return (l < RPW && (l * WINDOW) / RPW == p) ? l : -1;
    }
    // The same K step out of v_mfma_f32_16x16x32_bf16 (MI == 16 below): a wavefront's tile is MB16 x NB16
    // blocks of 16 x 16, a K step is KK32 steps of 32, the hand-over sits TAIL16 MFMAs before the end of the
    // K step's SLOTS16 MFMAs and the loads are spread over the WINDOW16 MFMAs that follow it.
    static constexpr int MB16 = WTM / 16, NB16 = WTN / 16, KK32 = BK / 32;
    // Measured (DeepSeek-V2-shaped share): one row of four wavefronts (the routed experts' 160-row tiles) runs
    // 1-2 % faster with the hand-over an eighth before the K step's end and the loads spread over seven eighths,
    // two rows of two wavefronts (256-row tiles) 1-2 % faster with a quarter and three quarters.
    static constexpr int SLOTS16 = KK32 * MB16 * NB16;
    static constexpr int TAIL16_ = WGM == 1 ? SLOTS16 / 8 : SLOTS16 / 4;
    static constexpr int TAIL16 = TAIL16_ > MB16 + NB16 ? TAIL16_ : MB16 + NB16;
    static constexpr int HO16 = SLOTS16 - TAIL16;
    static constexpr int WINDOW16_ = WGM == 1 ? SLOTS16 * 7 / 8 : SLOTS16 * 3 / 4;
    static constexpr int WINDOW16 = WINDOW16_ > RPW ? WINDOW16_ : RPW;
#ifndef MOE_EP_RD16_STRIDE
#define MOE_EP_RD16_STRIDE 2
#endif
    static constexpr int RD16 = MOE_EP_RD16_STRIDE * (MB16 + NB16) <= MB16 * NB16 ? MOE_EP_RD16_STRIDE : MB16 * NB16 / (MB16 + NB16);
    static constexpr int load_at16(int p)
    {
        const int l = (p * RPW + WINDOW16 - 1) / WINDOW16;
        return (l < RPW && (l * WINDOW16) / RPW == p) ? l : -1;
    }
};

// g * sigmoid(g) from the hardware's exp2 and reciprocal (about 1 ulp each: far below the bf16
// rounding of the result); exp2 saturates to +inf / 0 at the ends, which give -0 and g
__device__ __forceinline__ float silu_f(float g)
{
    return g * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(g * -1.4426950408889634f));
}

// s_waitcnt vmcnt(n) lgkmcnt(0): all but the newest n vector-memory loads have landed and every LDS
// read has returned (gfx9 encoding: vmcnt[3:0] | expcnt[6:4] | lgkmcnt[11:8] | vmcnt[5:4] << 14)
#define MOE_EP_WAIT_VMCNT_LGKM0(n) __builtin_amdgcn_s_waitcnt(((n) & 15) | (((n) >> 4) << 14) | 0x0070)

constexpr int kMaxGroups = 512;
constexpr int kTileCache = 32;  // tiles per workgroup whose coordinates are decoded ahead (4 ints each)
constexpr int kLdsPerWorkgroup = 160 * 1024;

// Behind the ring, in the same dynamic LDS allocation: the tile coordinate cache and, for ragged
// groups, three tables of G + 1 ints (sized by the launch, so that a deep ring of large tiles and
// a few groups fit the 160 KB together).
struct LdsTables { int *tile, *pref, *row0, *rowend; };
__device__ __forceinline__ LdsTables lds_tables(uint4* lds, int ring_bytes, int G)
{
    LdsTables t;
    t.tile = reinterpret_cast<int*>(reinterpret_cast<char*>(lds) + ring_bytes);
    t.pref = t.tile + 4 * kTileCache;
    t.row0 = t.pref + (G + 1);
    t.rowend = t.row0 + (G + 1);
    return t;
}
// Row tiles of ragged groups are cut to fit the group, not to a fixed height.  A tile is hb "units"
// tall, a unit being one 32-row accumulator block for each of the workgroup's WGM rows of wavefronts
// (unit_rows = 32 * WGM); a group of n rows has u = ceil(n / unit_rows) units and gets
// ceil(u / max_units) tiles whose heights differ by at most one unit: 616 rows in units of 32 with
// at most 8 per tile are tiles of 7, 7 and 6 units, not 256 + 256 + 104 rows.  A wavefront skips the
// MFMAs of the blocks a tile does not have, so a group costs ceil(n / unit_rows) units of matrix
// work whatever max_units is; max_units (a launch argument, at most the MB the kernel was
// compiled for) only trades tile count against operand bytes per flop.
struct TileCut { int tiles, base, rem; };   // tiles of base units, the first rem of them one more
__host__ __device__ __forceinline__ TileCut cut_group(int rows, int unit_rows, int max_units)
{
    TileCut c;
    const int u = (rows + unit_rows - 1) / unit_rows;
    c.tiles = (u + max_units - 1) / max_units;
    c.base = c.tiles ? u / c.tiles : 0;
    c.rem = c.tiles ? u - c.base * c.tiles : 0;
    return c;
}

// The tables of a launch over ragged groups, built by the workgroup's first wavefront from the group
// offsets alone (the host never learns them): first and last row of every group and the prefix sum
// of the groups' tile counts, 9 groups per lane and a scan over the lanes.
__device__ __forceinline__ void fill_tables(const GemmArgs& a, const LdsTables& t, int unit_rows, int max_units)
{
    static_assert(9 * 64 > kMaxGroups, "one wavefront covers every group and the total");
    const int tid = threadIdx.x;
    __syncthreads();
    if (tid < 64) {
        int cnt[9], sum = 0;
#pragma unroll
        for (int j = 0; j < 9; ++j) {
            const int g = tid * 9 + j;
            int c = 0;
            if (g < a.G) {
                const int r0 = a.offset[g], r1 = a.offset[g + 1];
                t.row0[g] = r0;
                t.rowend[g] = r1;
                c = cut_group(r1 - r0, unit_rows, max_units).tiles;
            }
            cnt[j] = sum;
            sum += c;
        }
        int incl = sum;
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            const int up = __shfl_up(incl, d, 64);
            if (tid >= d) incl += up;
        }
        const int base = incl - sum;
#pragma unroll
        for (int j = 0; j < 9; ++j) {
            const int g = tid * 9 + j;
            if (g <= a.G) t.pref[g] = base + cnt[j];
        }
    }
    __syncthreads();
}

static int lds_table_bytes(bool ragged, int G) { return (4 * kTileCache + (ragged ? 3 * (G + 1) : 0)) * 4; }
static int lds_cap(int bytes) { return bytes < kLdsPerWorkgroup ? bytes : kLdsPerWorkgroup; }

// All tiles that a workgroup owns.  Ragged mode reads the groups from LDS tables the caller has
// filled: s_pref[g] = row tiles before group g (s_pref[G] = all of them), s_row0[g] / s_rowend[g] =
// the rows of group g; its tiles are at most max_units units tall (cut_group).
// EPI, what the epilogue writes (the down projection of the routed experts only; 0 everywhere else):
// 0 bf16 results; 1 fp32 results (the experts' outputs are then not rounded before the aggregation);
// 2 bf16 results already multiplied by the routing weight of the row's assignment (Sec. 2.1: the
// aggregation then only adds)
template <int BM, int BN, int BK, int STAGES, int WGM, int WGN, bool SWIGLU, bool RAGGED, int EPI = 0, bool PACKED = false, int MI = 32>
__device__ __forceinline__ void gemm_tiles(const GemmArgs& a, uint4* lds, const int* s_pref, const int* s_row0,
                                           const int* s_rowend, int* s_tile, int max_units)
{
    using Cfg = GemmCfg<BM, BN, BK, STAGES, WGM, WGN, SWIGLU>;
    constexpr int MB = Cfg::MB, NB = Cfg::NB, RPW = Cfg::RPW, XRPW = Cfg::XRPW, NW = Cfg::NW;
    constexpr int THREADS = Cfg::THREADS, BN_OUT = Cfg::BN_OUT, CPR = Cfg::CPR, RP = Cfg::RP;
    constexpr int RPR = Cfg::RPR, KKW = Cfg::KKW;
    constexpr int MB16 = Cfg::MB16, NB16 = Cfg::NB16, KK32 = Cfg::KK32, SLOTS16 = Cfg::SLOTS16, HO16 = Cfg::HO16;
    static_assert(MI == 32 || MI == 16, "v_mfma_f32_32x32x16_bf16 or v_mfma_f32_16x16x32_bf16");
    static_assert(MI == 32 || (BK == 64 && Cfg::RPW <= Cfg::WINDOW16 && Cfg::WINDOW16 <= SLOTS16 && MB16 + NB16 <= Cfg::TAIL16 && NB16 % 2 == 0 &&
                               (!SWIGLU || NB16 % 4 == 0)),
                  "16 x 16 blocks: a K step is two steps of 32 (fragment sets 0 and 1), its loads and the next K step's "
                  "first fragment reads fit their windows, column blocks pair up for the stores");
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // uniform: LDS destinations stay scalar
    const int wn = wave % WGN, wm = wave / WGN;
    const int NT = (a.N + BN_OUT - 1) / BN_OUT;
    int mt_total, mt_per = 0;
    if (RAGGED) {  // routed experts: ragged groups, tables in LDS
        mt_total = s_pref[a.G];
    } else {       // shared experts: every group multiplies the same dense rows
        mt_per = (a.dense_rows + BM - 1) / BM;
        mt_total = mt_per * a.G;
    }
    const int total = mt_total * NT;
    // A launch lasts as many tiles as its busiest workgroup works through: rounds = ceil(total /
    // workgroups).  Only as many workgroups as it takes to finish in that many rounds stay: the
    // others would run one tile less and then wait (984 tiles on 256 compute units are 4 rounds on 248
    // as well; no measurable change in time, less work for the power budget).  The count is a multiple
    // of 8 so that every XCD (workgroup id mod 8) keeps the same number of workgroups.
    const int rounds = (total + (int)gridDim.x - 1) / (int)gridDim.x;
    const int active = rounds > 0 ? min((int)gridDim.x, (((total + rounds - 1) / rounds) + 7) & ~7) : 0;
    const int per_xcd = active >> 3;
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    if (slot >= per_xcd) return;   // the whole workgroup leaves, before any barrier of the tile pass
    const int KT = a.K / BK;
    // fragment geometry of this lane: row inside a 32-row block, swizzle term, k half
    // (16 x 16 blocks: row inside a 16-row block, swizzle term, which 8 of a step's 32 k values)
    const int fr_row = MI == 16 ? lane & 15 : lane & 31, fr_sw = (fr_row / RP) % CPR, fr_kh = MI == 16 ? lane >> 4 : lane >> 5;
    // load geometry of this lane: row inside a 1 KB region, physical chunk slot
    const int ld_row = lane / CPR, ld_p = lane % CPR;

    // Coordinates of a tile (wavefront-uniform) and, separately, the issue side: where the
    // direct-to-LDS loads of the tile whose K steps are being fetched come from.  The two differ at
    // the end of a tile, when the ring already takes in the next tile's first K steps.
    // hb: accumulator blocks per wavefront this tile has (MB in dense mode and for a full-height tile);
    // the rows of a tile are dealt to the WGM rows of wavefronts hb * 32 at a time
    struct Tile { int g, row0, nrows, n0, hb; };
    const bool mapped = RAGGED && a.a_row_map != nullptr;   // token rows gathered by the tile loads
    // weights in tile order (kernels.h): a K step's weight tile is one contiguous block
    constexpr bool packed = PACKED;
    static_assert(!PACKED || (BN == kPackRows && BK == kPackK), "the tile-order copy is laid out for one weight tile shape");
    const uint16_t* Xi = a.A;
    const uint16_t* Wi = a.W;
    // per region this wavefront loads: the lane's global source (row, swizzled chunk) as a byte
    // offset from the tile's activation rows Xi or the group's weights Wi (one group's matrices
    // and one activation panel are checked by the launcher to span less than 2^32 bytes)
    uint32_t goff[RPW];

    // tile number it of this workgroup -> coordinates; false past the last tile
    auto decode_tile = [&](int it, int& g, int& row0, int& nrows, int& n0, int& hb) -> bool {
        const int L = (it * 8 + xcd) * per_xcd + slot;
        if (L >= total) return false;
        // tile id -> (group, row tile, column tile): inside a group the row tiles are taken in bands
        // of kBand; inside a band the row tile runs fastest, then the column tile.  A run of 32
        // consecutive ids (one XCD's share) then covers about kBand row panels x 32/kBand
        // weight panels instead of 32 x 1, which is what that XCD's L2 has to fetch.
        constexpr int kBand = 8;
        int mi, ni, mt_g, l;
        if (RAGGED) {
            int lo = 0, hi = a.G;
            while (hi - lo > 1) {
                const int mid = (lo + hi) >> 1;
                if (s_pref[mid] * NT <= L) lo = mid; else hi = mid;
            }
            g = lo;
            mt_g = s_pref[g + 1] - s_pref[g];
            l = L - s_pref[g] * NT;
        } else {
            const int per_g = mt_per * NT;
            g = L / per_g;
            mt_g = mt_per;
            l = L - g * per_g;
        }
        {
            const int band = l / (kBand * NT);
            const int band_h = min(kBand, mt_g - band * kBand);
            const int lb = l - band * kBand * NT;
            ni = lb / band_h;
            mi = band * kBand + (lb - ni * band_h);
        }
        if (RAGGED) {
            const TileCut c = cut_group(s_rowend[g] - s_row0[g], 32 * WGM, max_units);
            hb = c.base + (mi < c.rem ? 1 : 0);
            row0 = s_row0[g] + (mi * c.base + min(mi, c.rem)) * (32 * WGM);
            nrows = min(hb * 32 * WGM, s_rowend[g] - row0);
        } else {
            hb = MB;
            row0 = mi * BM;
            nrows = min(BM, a.dense_rows - row0);
        }
        n0 = ni * BN_OUT;
        return true;
    };
    // The search and the divisions of a tile's coordinates would sit in the middle of a K loop, once
    // per tile and wavefront, with the matrix pipe waiting: the workgroup's first kTileCache tiles
    // are decoded once, one per thread, before the first tile starts.
    for (int it = tid; it < kTileCache; it += THREADS) {
        int g = -1, row0 = 0, nrows = 0, n0 = 0, hb = 0;
        if (!decode_tile(it, g, row0, nrows, n0, hb)) g = -1;
        s_tile[4 * it + 0] = g; s_tile[4 * it + 1] = row0; s_tile[4 * it + 2] = nrows | (hb << 16); s_tile[4 * it + 3] = n0;
    }
    __syncthreads();
    // tile number it of this workgroup -> coordinates, Xi / Wi / goff; false past the last tile
    auto setup_tile = [&](int it, Tile& t) __attribute__((always_inline)) -> bool {
        int g, row0, nrows, n0, hb;
        if (it < kTileCache) {
            g = s_tile[4 * it + 0]; row0 = s_tile[4 * it + 1]; n0 = s_tile[4 * it + 3];
            nrows = s_tile[4 * it + 2] & 0xffff; hb = s_tile[4 * it + 2] >> 16;
            if (g < 0) return false;
        } else if (!decode_tile(it, g, row0, nrows, n0, hb)) {
            return false;
        }
        // the coordinates came through LDS; telling the compiler they are wavefront-uniform keeps
        // base addresses in scalar registers and leaves the lanes 32-bit offsets only
        t.g = __builtin_amdgcn_readfirstlane(g);
        t.row0 = __builtin_amdgcn_readfirstlane(row0);
        t.nrows = __builtin_amdgcn_readfirstlane(nrows);
        t.n0 = __builtin_amdgcn_readfirstlane(n0);
        t.hb = __builtin_amdgcn_readfirstlane(hb);
        if (packed) Wi = a.Wp + ((size_t)t.g * NT + t.n0 / BN_OUT) * ((size_t)KT * BN * BK);
        else Wi = a.W + (size_t)t.g * a.w_group_stride;
        Xi = mapped ? a.A : a.A + (size_t)t.row0 * a.lda;
        // activation regions first: the tile row each lane fetches, and with gathered token rows the
        // row map's entries for all of them in one go (the loads are independent; one wait for the lot
        // instead of one memory round trip per region in the middle of a K loop)
        int src_row[XRPW > 0 ? XRPW : 1];
#pragma unroll
        for (int i = 0; i < XRPW; ++i) {
            const int r = (wave + NW * i) * RPR + ld_row;
            // LDS row r belongs to wavefront row r / WTM, which holds tile rows
            // [(r / WTM) * hb * 32, +hb * 32); blocks the tile does not have and rows past its
            // end re-read the last valid row (one cache line for the whole region)
            const int within = r % Cfg::WTM;
            int rr = (RAGGED && WGM > 1) ? (r / Cfg::WTM) * t.hb * 32 + within : r;
            if (RAGGED && within >= t.hb * 32) rr = t.nrows - 1;
            src_row[i] = min(rr, t.nrows - 1);
        }
        if (mapped) {
#pragma unroll
            for (int i = 0; i < XRPW; ++i) src_row[i] = a.a_row_map[t.row0 + src_row[i]];
            asm volatile("" ::: "memory");   // all of them are in flight before the first is used
#pragma unroll
            for (int i = 0; i < XRPW; ++i) src_row[i] /= a.a_row_div;
        }
#pragma unroll
        for (int i = 0; i < RPW; ++i) {
            const int j = wave + NW * i;                 // region index inside a stage
            const int r = j * RPR + ld_row;              // row in the stacked [activations; weights] tile
            const int c = ld_p ^ ((r / RP) % CPR);       // logical chunk stored at physical slot ld_p
            if (i < XRPW) {
                goff[i] = ((uint32_t)src_row[i < XRPW ? i : 0] * (uint32_t)a.lda + c * 8) * 2u;
            } else {
                const int jw = r - BM;                   // row of the weight tile
                int n;
                uint32_t base = 0;
                if (SWIGLU) {
                    if (jw < BN / 2) n = t.n0 + jw; else { n = t.n0 + jw - BN / 2; base = (uint32_t)a.w_up_offset; }
                } else {
                    n = t.n0 + jw;
                }
                n = min(n, a.N - 1);
                goff[i] = packed ? (uint32_t)(jw * BK + c * 8) * 2u
                                 : (base + (uint32_t)n * (uint32_t)a.ldw + c * 8) * 2u;
            }
        }
        return true;
    };

    // first LDS row of accumulator column block nb of this wavefront (stacked tile coordinates)
    auto w_row_base = [&](int nb) -> int {
        if (SWIGLU) return BM + ((nb < NB / 2) ? wn * (Cfg::WTN / 2) + nb * 32
                                               : BN / 2 + wn * (Cfg::WTN / 2) + (nb - NB / 2) * 32);
        return BM + wn * Cfg::WTN + nb * 32;
    };
    f32x16_t acc[MI == 32 ? MB : 1][MI == 32 ? NB : 1];
    bf16x8_t xf[2][MI == 32 ? MB : 1], wf[2][MI == 32 ? NB : 1];
    // 16 x 16 blocks (MI == 16): a lane's four accumulators of a block are four consecutive output columns of
    // one token row; fragments are 16 rows by 32 k, 8 k per lane
    auto w_row_base16 = [&](int nb) -> int {
        if (SWIGLU) return BM + ((nb < NB16 / 2) ? wn * (Cfg::WTN / 2) + nb * 16
                                                 : BN / 2 + wn * (Cfg::WTN / 2) + (nb - NB16 / 2) * 16);
        return BM + wn * Cfg::WTN + nb * 16;
    };
    f32x4_t acc16[MI == 16 ? MB16 : 1][MI == 16 ? NB16 : 1];
    bf16x8_t xf16[2][MI == 16 ? MB16 : 1], wf16[2][MI == 16 ? NB16 : 1];
    // one LDS fragment read of a 16-row block from ring slot base sT_, step kk_ of 32: f < MB16 an activation
    // block, f >= MB16 a weight block
#define MOE_EP_FRAG16(sT_, kk_, set_, f_)                                                         \
    {                                                                                             \
        const int csw_ = ((kk_) * 4 + fr_kh) ^ fr_sw;                                             \
        if ((f_) < MB16) xf16[set_][(f_) < MB16 ? (f_) : 0] = __builtin_bit_cast(bf16x8_t,        \
            (sT_)[(wm * Cfg::WTM + (f_) * 16 + fr_row) * CPR + csw_]);                            \
        else wf16[set_][(f_) >= MB16 ? (f_) - MB16 : 0] = __builtin_bit_cast(bf16x8_t,            \
            (sT_)[(w_row_base16((f_) >= MB16 ? (f_) - MB16 : 0) + fr_row) * CPR + csw_]);         \
    }
    // one LDS fragment read from ring slot base sT_: index f < MB is an activation block,
    // f >= MB a weight block
#define MOE_EP_FRAG1(sT_, kk_, set_, f_)                                                          \
    {                                                                                             \
        const int csw_ = ((kk_) * 2 + fr_kh) ^ fr_sw;                                             \
        if ((f_) < MB) xf[set_][(f_) < MB ? (f_) : 0] = __builtin_bit_cast(bf16x8_t,              \
            (sT_)[(wm * Cfg::WTM + (f_) * 32 + fr_row) * CPR + csw_]);                            \
        else wf[set_][(f_) >= MB ? (f_) - MB : 0] = __builtin_bit_cast(bf16x8_t,                  \
            (sT_)[(w_row_base((f_) >= MB ? (f_) - MB : 0) + fr_row) * CPR + csw_]);               \
    }
    // one direct-to-LDS load of the issue-side tile: region i of this wavefront, K step ks_, ring slot stage_
#define MOE_EP_ISSUE1(ks_, stage_, i_)                                                            \
    {                                                                                             \
        const int k_ = (ks_) * BK;                                                                \
        const int seg_ = k_ / a.kseg_len;                                                         \
        const size_t wk_ = packed ? (size_t)(ks_) * (BN * BK)                                     \
                                  : (size_t)seg_ * a.w_kseg_stride + (k_ - seg_ * a.kseg_len);    \
        uint4* dst_ = lds + (stage_) * Cfg::STAGE_CHUNKS + wave * 64 + NW * 64 * (i_);            \
        __builtin_amdgcn_global_load_lds(                                                         \
            reinterpret_cast<const uint4*>(reinterpret_cast<const char*>(                         \
                (i_) < XRPW ? Xi + k_ : Wi + wk_) + goff[i_]),                                    \
            dst_, 16, 0, 0);                                                                      \
    }
#define SB() __builtin_amdgcn_sched_barrier(0)
    // The hand-over of a ring slot to the MFMAs: this wavefront's loads into it have landed (all
    // but the newest pending_ loads), its own LDS reads of older slots have returned, and after
    // the barrier the same holds for every wavefront, so the slot may be read and the slot read
    // before it may be refilled.
#define MOE_EP_HANDOVER(pending_)                                                                 \
    {                                                                                             \
        MOE_EP_WAIT_VMCNT_LGKM0(pending_);                                                        \
        __builtin_amdgcn_s_barrier();                                                             \
        asm volatile("" ::: "memory");                                                            \
    }
    // One K step of the tile being computed.  The source order below is the issue order:
    // sched_barrier(0) after every MFMA keeps the compiler from regrouping.  A K step is KKW k16
    // steps; k16 step i works out of fragment set i & 1 while the LDS reads of step i+1 are slipped
    // between its MFMAs.  The hand-over of the next ring slot sits in front of the LAST k16 step:
    // the fragments of the next K step's first k16 step are read during that step (prefetch_; not
    // at the end of a tile, whose epilogue would have to keep them alive), so the LDS latency after
    // a barrier hides behind MB*NB MFMAs.  The same barrier frees the slot this K step has been
    // reading - every wavefront's last reads of it have returned - and the loads of the K step
    // STAGES ahead (ki on the issue side) start into it at once and carry on through the first
    // k16 steps of the following K step, spread evenly behind the MFMAs (GemmCfg::load_at).  When the issue side has used up its
    // tile it moves to the workgroup's next one just before that.  Fragment reads are ordered so
    // that the first MFMA needs only the first two.
#define MOE_EP_FRAG_ORDER(f_) ((f_) == 0 ? MB : (f_) <= MB ? (f_) - 1 : (f_))
#define MOE_EP_STEP(prefetch_)                                                                    \
    {                                                                                             \
        const uint4* sT = lds + stage * Cfg::STAGE_CHUNKS;                                        \
        const int st_next = stage == STAGES - 1 ? 0 : stage + 1;                                  \
        const uint4* sN = lds + st_next * Cfg::STAGE_CHUNKS;                                      \
        const int st_prev = stage == 0 ? STAGES - 1 : stage - 1;                                  \
        _Pragma("unroll") for (int i = 0; i < KKW; ++i) {                                         \
            if (i == KKW - 1) {                                                                   \
                if (ki == KT) {                                                                   \
                    if (!issue_end) {                                                             \
                        has_nxt = setup_tile(it_issue + 1, nxt);                                  \
                        if (has_nxt) ++it_issue; else issue_end = true;                           \
                    }                                                                             \
                    ki = 0;                                                                       \
                }                                                                                 \
                MOE_EP_HANDOVER((STAGES - 2) * RPW)                                               \
            }                                                                                     \
            _Pragma("unroll") for (int q = 0; q < MB * NB; ++q) {                                 \
                /* row blocks run down and up in turn: one operand changes per MFMA, never both */ \
                const int nb = q / MB, mb = (nb & 1) ? MB - 1 - q % MB : q % MB;                  \
                acc[mb][nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[i & 1][nb], xf[i & 1][mb], acc[mb][nb], 0, 0, 0); \
                _Pragma("unroll") for (int f = q; f < MB + NB; f += MB * NB) {                    \
                    if (i + 1 < KKW) MOE_EP_FRAG1(sT, i + 1, (i + 1) & 1, MOE_EP_FRAG_ORDER(f))   \
                    else if (prefetch_) MOE_EP_FRAG1(sN, 0, 0, MOE_EP_FRAG_ORDER(f))              \
                }                                                                                 \
                if (i + 1 < KKW) {  /* the rest of the load group that started a K step ago */    \
                    const int l_ = Cfg::load_at((i + 1) * MB * NB + q);                           \
                    if (l_ >= 0) MOE_EP_ISSUE1(ki - 1, st_prev, l_ < 0 ? 0 : l_)                  \
                } else {                                                                          \
                    const int l_ = Cfg::load_at(q);                                               \
                    if (l_ >= 0) MOE_EP_ISSUE1(ki, stage, l_ < 0 ? 0 : l_)                        \
                }                                                                                 \
                SB();                                                                             \
            }                                                                                     \
        }                                                                                         \
        ++ki;                                                                                     \
        stage = st_next;                                                                          \
    }

    // The same K step out of 16 x 16 x 32 MFMAs: KK32 steps of 32, step j out of fragment set j & 1 while the
    // reads of step j + 1 are slipped behind every second of its first MFMAs.  The hand-over sits in front of
    // MFMA HO16; the next K step's first fragments are read behind the MFMAs that follow it, the loads of
    // the K step STAGES ahead start there and carry on into the following K step (GemmCfg::load_at16).
#define MOE_EP_FRAG_ORDER16(f_) ((f_) == 0 ? MB16 : (f_) <= MB16 ? (f_) - 1 : (f_))
#define MOE_EP_STEP16(prefetch_)                                                                  \
    {                                                                                             \
        const uint4* sT = lds + stage * Cfg::STAGE_CHUNKS;                                        \
        const int st_next = stage == STAGES - 1 ? 0 : stage + 1;                                  \
        const uint4* sN = lds + st_next * Cfg::STAGE_CHUNKS;                                      \
        const int st_prev = stage == 0 ? STAGES - 1 : stage - 1;                                  \
        constexpr int RS_ = Cfg::TAIL16 / (MB16 + NB16);   /* MFMAs per prefetch read */          \
        _Pragma("unroll") for (int j = 0; j < KK32; ++j) {                                        \
            _Pragma("unroll") for (int q = 0; q < MB16 * NB16; ++q) {                             \
                const int m_ = j * MB16 * NB16 + q;                                               \
                if (m_ == HO16) {                                                                 \
                    if (ki == KT) {                                                               \
                        if (!issue_end) {                                                         \
                            has_nxt = setup_tile(it_issue + 1, nxt);                              \
                            if (has_nxt) ++it_issue; else issue_end = true;                       \
                        }                                                                         \
                        ki = 0;                                                                   \
                    }                                                                             \
                    MOE_EP_HANDOVER((STAGES - 2) * RPW)                                           \
                }                                                                                 \
                const int nb = q / MB16, mb = (nb & 1) ? MB16 - 1 - q % MB16 : q % MB16;          \
                /* written out so that the block is updated in place, in accumulator registers: through the  \
                   builtin the register allocator moves blocks between two K steps and through vector registers */ \
                asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0"                             \
                             : "+a"(acc16[mb][nb]) : "v"(wf16[j & 1][nb]), "v"(xf16[j & 1][mb])); \
                if (j + 1 < KK32) {                                                               \
                    if (q % Cfg::RD16 == 0 && q / Cfg::RD16 < MB16 + NB16)                        \
                        MOE_EP_FRAG16(sT, j + 1, (j + 1) & 1, MOE_EP_FRAG_ORDER16(q / Cfg::RD16)) \
                } else if (prefetch_) {                                                           \
                    const int f_ = m_ - HO16;                                                     \
                    if (f_ >= 0 && f_ % RS_ == 0 && f_ / RS_ < MB16 + NB16)                       \
                        MOE_EP_FRAG16(sN, 0, 0, MOE_EP_FRAG_ORDER16(f_ / RS_))                    \
                }                                                                                 \
                if (m_ >= HO16) {                                                                 \
                    const int l_ = Cfg::load_at16(m_ - HO16);                                     \
                    if (l_ >= 0) MOE_EP_ISSUE1(ki, stage, l_ < 0 ? 0 : l_)                        \
                } else {  /* the rest of the load group that started a K step ago */              \
                    const int l_ = Cfg::load_at16(m_ + SLOTS16 - HO16);                           \
                    if (l_ >= 0) MOE_EP_ISSUE1(ki - 1, st_prev, l_ < 0 ? 0 : l_)                  \
                }                                                                                 \
                SB();                                                                             \
            }                                                                                     \
        }                                                                                         \
        ++ki;                                                                                     \
        stage = st_next;                                                                          \
    }

    Tile cur, nxt;
    if (!setup_tile(0, cur)) return;
    // The ring never drains between tiles: the issue side runs STAGES K steps ahead of the MFMAs and
    // simply crosses into the workgroup's next tile (the launcher guarantees KT >= STAGES, so it is
    // never more than one tile ahead), and the epilogue's stores overlap the next tile's loads.
    // After the last tile it wraps around to that tile's own first K steps: a few wasted loads at
    // the very end keep every step of the loop alike.
    int stage = 0, it_issue = 0;
    bool has_nxt = false, issue_end = false;
    // K steps 0 .. STAGES-2 go in flight, the first is handed over, and K step STAGES-1 starts
    // the way every later one does: behind a hand-over
#pragma unroll
    for (int p = 0; p < STAGES - 1; ++p)
#pragma unroll
        for (int i = 0; i < RPW; ++i) MOE_EP_ISSUE1(p, p, i)
    MOE_EP_HANDOVER((STAGES - 2) * RPW)
    if constexpr (MI == 32) {
#pragma unroll
        for (int p = 0; p < MB * NB; ++p)
            if (Cfg::load_at(p) >= 0) MOE_EP_ISSUE1(STAGES - 1, STAGES - 1, Cfg::load_at(p) < 0 ? 0 : Cfg::load_at(p))
    } else {
#pragma unroll
        for (int p = 0; p < SLOTS16 - HO16; ++p)
            if (Cfg::load_at16(p) >= 0) MOE_EP_ISSUE1(STAGES - 1, STAGES - 1, Cfg::load_at16(p) < 0 ? 0 : Cfg::load_at16(p))
    }
    int ki = STAGES;  // K step of the issue-side tile whose loads start at the next hand-over
    {   // the first tile's first K step has been handed over: its first fragments.  Every later K
        // step, the first of a following tile included, gets them from the step before it.
        const uint4* s0 = lds + stage * Cfg::STAGE_CHUNKS;
        if constexpr (MI == 32) {
#pragma unroll
            for (int f = 0; f < MB + NB; ++f) MOE_EP_FRAG1(s0, 0, 0, MOE_EP_FRAG_ORDER(f))
        } else {
#pragma unroll
            for (int f = 0; f < MB16 + NB16; ++f) MOE_EP_FRAG16(s0, 0, 0, MOE_EP_FRAG_ORDER16(f))
        }
        SB();
    }
    for (;;) {
        // one loop shape for every K step: the last one of a tile hands the next tile's first K
        // step over and reads its first fragments, which wait in registers through the epilogue
        if constexpr (MI == 32) {
#pragma unroll
            for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                for (int nb = 0; nb < NB; ++nb)
#pragma unroll
                    for (int r = 0; r < 16; ++r) acc[mb][nb][r] = 0.f;
            for (int kt = 0; kt < KT; ++kt) MOE_EP_STEP(true)
        } else {
#pragma unroll
            for (int mb = 0; mb < MB16; ++mb)
#pragma unroll
                for (int nb = 0; nb < NB16; ++nb)
#pragma unroll
                    for (int r = 0; r < 4; ++r) acc16[mb][nb][r] = 0.f;
            // the compiler does not know the hand-written MFMAs' latencies: wait states between the zeroing moves
            // and the first MFMA that reads them, and between the last MFMAs and the epilogue's accumulator reads
            SB();
            asm volatile("s_nop 7");
            SB();
            for (int kt = 0; kt < KT; ++kt) MOE_EP_STEP16(true)
            SB();
            asm volatile("s_nop 15");
            asm volatile("s_nop 15");
            SB();
        }

        // epilogue: a lane holds token row (lane & 31) of each block and, per register quad q,
        // output columns 8q + 4*(lane >> 5) + {0..3} of the block.  Two quads are exchanged between
        // the half-wavefronts (v_permlane32_swap) so that a lane stores 8 consecutive columns with
        // one 16-byte store: every store instruction then carries 32 bytes per token row instead of
        // 16, and the store path of the CU, which is what the epilogue waits for, sees half the
        // requests.  A tile whose columns all lie inside N (the usual case, decided once per tile)
        // stores without per-store column tests.
        if constexpr (MI == 16) {
            // 16 x 16 blocks: a lane holds token row (lane & 15) of each block and output columns
            // 4 * (lane >> 4) + {0..3} of it.  Two neighbouring column blocks exchange halves between the
            // rows of 16 lanes (v_permlane16_swap: rows 1 and 3 of the first operand against rows 0 and 2 of
            // the second), after which a lane holds 8 consecutive columns of one of the two blocks and a
            // store instruction carries 64 contiguous bytes per token row.
            const int g4 = fr_kh;
            const int n_wave = cur.n0 + wn * (SWIGLU ? Cfg::WTN / 2 : Cfg::WTN);
            uint16_t* Cg = a.C + (size_t)cur.g * a.c_group_col_stride + n_wave;
            auto store_tile16 = [&](auto guard_n) {
                constexpr bool GUARD_N = decltype(guard_n)::value;
#pragma unroll
                for (int mb = 0; mb < MB16; ++mb) {
                    // a row of blocks is pinned in its accumulator registers right before its turn
                    if constexpr (NB16 == 8)
                        asm volatile("; accumulator row %8" : "+a"(acc16[mb][0]), "+a"(acc16[mb][1]), "+a"(acc16[mb][2]), "+a"(acc16[mb][3]),
                                     "+a"(acc16[mb][NB16 > 4 ? 4 : 0]), "+a"(acc16[mb][NB16 > 5 ? 5 : 1]), "+a"(acc16[mb][NB16 > 6 ? 6 : 2]), "+a"(acc16[mb][NB16 > 7 ? 7 : 3]) : "n"(mb));
                    else if constexpr (NB16 == 4)
                        asm volatile("; accumulator row %4" : "+a"(acc16[mb][0]), "+a"(acc16[mb][1]), "+a"(acc16[mb][2]), "+a"(acc16[mb][3]) : "n"(mb));
                    if (RAGGED && mb >= 2 * cur.hb) continue;
                    const int m = (RAGGED ? wm * cur.hb * 32 : wm * Cfg::WTM) + mb * 16 + fr_row;
                    if (m >= cur.nrows) continue;  // the same for the lanes of an exchange (they share lane & 15)
                    if (EPI == 1) {
                        float* frow = reinterpret_cast<float*>(a.C) + (size_t)cur.g * a.c_group_col_stride +
                                      (size_t)(cur.row0 + m) * a.ldc + cur.n0 + wn * Cfg::WTN + g4 * 4;
#pragma unroll
                        for (int nb = 0; nb < NB16; ++nb) {
                            if (GUARD_N && cur.n0 + wn * Cfg::WTN + g4 * 4 + nb * 16 >= a.N) continue;
                            *reinterpret_cast<f32x4_t*>(frow + nb * 16) = acc16[mb][nb];
                        }
                        continue;
                    }
                    const float rw = EPI == 2 ? a.row_weight[a.row_assignment[cur.row0 + m]] : 1.0f;
                    uint16_t* crow = Cg + (size_t)(cur.row0 + m) * a.ldc;
#pragma unroll
                    for (int nb = 0; nb < (SWIGLU ? NB16 / 2 : NB16); nb += 2) {
                        uint32_t pk[2][2];  // [block nb, nb + 1][column pair]
#pragma unroll
                        for (int j = 0; j < 2; ++j) {
                            float h[4];
#pragma unroll
                            for (int i = 0; i < 4; ++i)
                                h[i] = SWIGLU ? silu_f(acc16[mb][nb + j][i]) * acc16[mb][nb + j + NB16 / 2][i]
                                     : EPI == 2 ? rw * acc16[mb][nb + j][i]
                                                : acc16[mb][nb + j][i];
                            pk[j][0] = pack_bf16x2(h[0], h[1]);
                            pk[j][1] = pack_bf16x2(h[2], h[3]);
                        }
                        const auto s0 = __builtin_amdgcn_permlane16_swap(pk[0][0], pk[1][0], false, false);
                        const auto s1 = __builtin_amdgcn_permlane16_swap(pk[0][1], pk[1][1], false, false);
                        // rows of lanes 0 / 2 now hold columns 0..7 / 8..15 of block nb, rows 1 / 3 those of block nb + 1
                        const int col = (nb + (g4 & 1)) * 16 + (g4 >> 1) * 8;
                        if (GUARD_N && n_wave + col >= a.N) continue;
                        uint4 o;
                        o.x = s0[0]; o.y = s1[0]; o.z = s0[1]; o.w = s1[1];
                        *reinterpret_cast<uint4*>(crow + col) = o;
                    }
                }
            };
            if (cur.n0 + Cfg::BN_OUT <= a.N) store_tile16(std::false_type{});
            else store_tile16(std::true_type{});
        } else {
            const int n_lane = cur.n0 + wn * (SWIGLU ? Cfg::WTN / 2 : Cfg::WTN) + fr_kh * 8;
            uint16_t* Cg = a.C + (size_t)cur.g * a.c_group_col_stride + n_lane;
            auto store_tile = [&](auto guard_n) {
                constexpr bool GUARD_N = decltype(guard_n)::value;
#pragma unroll
                for (int mb = 0; mb < MB; ++mb) {
                    // a row of blocks is pinned in its accumulator registers right before its turn
                    if (NB == 4) asm volatile("; accumulator row %4" : "+a"(acc[mb][0]), "+a"(acc[mb][1]), "+a"(acc[mb][NB > 2 ? 2 : 0]), "+a"(acc[mb][NB > 3 ? 3 : 1]) : "n"(mb));
                    else if (NB == 2) asm volatile("; accumulator row %2" : "+a"(acc[mb][0]), "+a"(acc[mb][1]) : "n"(mb));
                    if (RAGGED && mb >= cur.hb) continue;
                    const int m = (RAGGED ? wm * cur.hb * 32 : wm * Cfg::WTM) + mb * 32 + fr_row;
                    if (m >= cur.nrows) continue;  // the same for both lanes of an exchange
                    if (EPI == 1) {
                        // fp32 results: a lane's register quad is 4 consecutive columns = one 16-byte store
                        float* frow = reinterpret_cast<float*>(a.C) + (size_t)cur.g * a.c_group_col_stride +
                                      (size_t)(cur.row0 + m) * a.ldc + cur.n0 + wn * Cfg::WTN + fr_kh * 4;
#pragma unroll
                        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
                            for (int q = 0; q < 4; ++q) {
                                if (GUARD_N && cur.n0 + wn * Cfg::WTN + fr_kh * 4 + nb * 32 + q * 8 >= a.N) continue;
                                f32x4_t o = {acc[mb][nb][q * 4], acc[mb][nb][q * 4 + 1], acc[mb][nb][q * 4 + 2], acc[mb][nb][q * 4 + 3]};
                                *reinterpret_cast<f32x4_t*>(frow + nb * 32 + q * 8) = o;
                            }
                        continue;
                    }
                    // EPI == 2: the routing weight of the assignment this grouped row belongs to
                    const float rw = EPI == 2 ? a.row_weight[a.row_assignment[cur.row0 + m]] : 1.0f;
                    uint16_t* crow = Cg + (size_t)(cur.row0 + m) * a.ldc;
#pragma unroll
                    for (int nb = 0; nb < (SWIGLU ? NB / 2 : NB); ++nb) {
                        // the block stays in its accumulator registers until here: without the
                        // pin the compiler copies all accumulators out during the last K step,
                        // spills, and every spill reload waits for all stores before it
#pragma unroll
                        for (int q = 0; q < 4; q += 2) {
                            uint32_t pk[2][2];  // [quad q, q+1][column pair]
#pragma unroll
                            for (int j = 0; j < 2; ++j) {
                                float h[4];
#pragma unroll
                                for (int i = 0; i < 4; ++i)
                                    h[i] = SWIGLU ? silu_f(acc[mb][nb][(q + j) * 4 + i]) * acc[mb][nb + NB / 2][(q + j) * 4 + i]
                                         : EPI == 2 ? rw * acc[mb][nb][(q + j) * 4 + i]
                                                    : acc[mb][nb][(q + j) * 4 + i];
                                pk[j][0] = pack_bf16x2(h[0], h[1]);
                                pk[j][1] = pack_bf16x2(h[2], h[3]);
                            }
                            // lanes 32..63 of quad q  <->  lanes 0..31 of quad q+1
                            const auto s0 = __builtin_amdgcn_permlane32_swap(pk[0][0], pk[1][0], false, false);
                            const auto s1 = __builtin_amdgcn_permlane32_swap(pk[0][1], pk[1][1], false, false);
                            if (GUARD_N && n_lane + nb * 32 + q * 8 >= a.N) continue;
                            uint4 o;
                            o.x = s0[0]; o.y = s1[0]; o.z = s0[1]; o.w = s1[1];
                            *reinterpret_cast<uint4*>(crow + nb * 32 + q * 8) = o;
                        }
                    }
                }
            };
            if (cur.n0 + Cfg::BN_OUT <= a.N) store_tile(std::false_type{});
            else store_tile(std::true_type{});
        }
        if (!has_nxt) break;
        cur = nxt;
        has_nxt = false;
    }
    // loads still on their way write into this workgroup's LDS: they must land before it is given up
    MOE_EP_WAIT_VMCNT_LGKM0(0);
#undef MOE_EP_HANDOVER
#undef MOE_EP_STEP
#undef MOE_EP_STEP16
#undef MOE_EP_FRAG_ORDER
#undef MOE_EP_FRAG_ORDER16
#undef MOE_EP_FRAG16
#undef SB
#undef MOE_EP_ISSUE1
#undef MOE_EP_FRAG1
}


template <int BM, int BN, int BK, int STAGES, int WGM, int WGN, bool SWIGLU, bool RAGGED, int EPI = 0, bool PACKED = false, int MI = 32>
__global__ __launch_bounds__(WGM* WGN * 64) void grouped_gemm_kernel(GemmArgs a)
{
    extern __shared__ uint4 lds[];
    using Cfg = GemmCfg<BM, BN, BK, STAGES, WGM, WGN, SWIGLU>;
    const LdsTables t = lds_tables(lds, Cfg::LDS_BYTES, a.G);
    const int max_units = (a.max_units > 0 && a.max_units < Cfg::MB) ? a.max_units : Cfg::MB;
    if (RAGGED) fill_tables(a, t, 32 * WGM, max_units);
    gemm_tiles<BM, BN, BK, STAGES, WGM, WGN, SWIGLU, RAGGED, EPI, PACKED, MI>(a, lds, t.pref, t.row0, t.rowend, t.tile, max_units);
}

// what every kernel here assumes of its arguments beyond the shapes the caller has checked
static bool args_fit(const GemmArgs& a, bool swiglu, bool ragged, int bm)
{
    // lanes address with 32-bit byte offsets inside one group's weights and one activation panel
    const long long w_span = ((swiglu ? a.w_up_offset : 0) + (long long)a.N * a.ldw) * 2;
    const long long x_span = (long long)(a.a_row_map ? a.a_src_rows : bm) * a.lda * 2;
    if (a.a_row_map && (!ragged || a.a_row_div < 1 || a.a_src_rows < 1)) return false;
    if (w_span >= (1ll << 32) || x_span >= (1ll << 32) || w_span < 0) return false;
    if (a.G < 1 || a.G > kMaxGroups) return false;
    // the epilogue stores 8 output columns (16 bytes) per lane
    return !(a.N % 8 || a.ldc % 8 || a.c_group_col_stride % 8 || (reinterpret_cast<uintptr_t>(a.C) & 15));
}

template <int BM, int BN, int BK, int STAGES, int WGM, int WGN, bool SWIGLU, bool RAGGED, int EPI = 0, bool PACKED = false, int MI = 32>
static hipError_t launch_one(const GemmArgs& a, int n_cu, long long max_rows, hipStream_t s)
{
    using Cfg = GemmCfg<BM, BN, BK, STAGES, WGM, WGN, SWIGLU>;
    const int NT = (a.N + Cfg::BN_OUT - 1) / Cfg::BN_OUT;
    // an upper bound of the row tiles the device-side tables can describe
    const int tile_rows = 32 * WGM * ((a.max_units > 0 && a.max_units < Cfg::MB) ? a.max_units : Cfg::MB);
    const long long max_row_tiles = RAGGED ? (max_rows + tile_rows - 1) / tile_rows + a.G
                                           : (long long)((a.dense_rows + BM - 1) / BM) * a.G;
    const long long max_tiles = max_row_tiles * NT;
    if (max_tiles <= 0) return hipSuccess;
    if (!args_fit(a, SWIGLU, RAGGED, BM)) return hipErrorInvalidValue;
    const int lds_bytes = Cfg::LDS_BYTES + lds_table_bytes(RAGGED, a.G);
    if (lds_bytes > kLdsPerWorkgroup) return hipErrorInvalidValue;  // launch_grouped_gemm has checked
    // workgroups per CU: LDS and 8 wavefront slots
    int occ = kLdsPerWorkgroup / lds_bytes;
    const int by_waves = 8 / Cfg::NW;
    if (occ > by_waves) occ = by_waves;
    if (occ < 1) occ = 1;
    long long grid = (long long)n_cu * occ;
    if (grid > max_tiles) grid = max_tiles;
    grid = (grid + 7) / 8 * 8;
    hipLaunchKernelGGL((grouped_gemm_kernel<BM, BN, BK, STAGES, WGM, WGN, SWIGLU, RAGGED, EPI, PACKED, MI>),
                       dim3((unsigned)grid), dim3(Cfg::THREADS), lds_bytes, s, a);
    return hipGetLastError();
}

template <int BM, int BN, int BK, int STAGES, int WGM, int WGN, bool PACKED, int MI>
static hipError_t raise_all()
{
    hipError_t e;
#define R(SW, RG, EPI)                                                                                  \
    if ((e = hipFuncSetAttribute(                                                                       \
             reinterpret_cast<const void*>(&grouped_gemm_kernel<BM, BN, BK, STAGES, WGM, WGN, SW, RG, EPI, PACKED, MI>), \
             hipFuncAttributeMaxDynamicSharedMemorySize,                                                \
             lds_cap(GemmCfg<BM, BN, BK, STAGES, WGM, WGN, SW>::LDS_BYTES +                             \
                     lds_table_bytes(RG, kMaxGroups)))) != hipSuccess) return e;
    R(true, true, 0) R(true, false, 0) R(false, true, 0) R(false, false, 0) R(false, true, 1) R(false, true, 2)
#undef R
    return hipSuccess;
}

// PK: the variant also exists for weights in tile order (its weight tile is kPackRows x kPackK)
template <int BM, int BN, int BK, int STAGES, int WGM, int WGN, bool PK, int MI>
static hipError_t launch_cfg(const GemmArgs& a, bool swiglu, int n_cu, long long max_rows, hipStream_t s)
{
    const bool ragged = a.offset != nullptr;
    if (swiglu && a.epi != 0) return hipErrorInvalidValue;
    // only the routed down projection has other epilogues
    if (a.epi != 0 && (!ragged || a.epi < 0 || a.epi > 2 || (a.epi == 2 && (!a.row_weight || !a.row_assignment))))
        return hipErrorInvalidValue;
    auto go = [&](auto packed) -> hipError_t {
        constexpr bool P = decltype(packed)::value;
        if (swiglu) return ragged ? launch_one<BM, BN, BK, STAGES, WGM, WGN, true, true, 0, P, MI>(a, n_cu, max_rows, s)
                                  : launch_one<BM, BN, BK, STAGES, WGM, WGN, true, false, 0, P, MI>(a, n_cu, max_rows, s);
        if (a.epi == 1) return launch_one<BM, BN, BK, STAGES, WGM, WGN, false, true, 1, P, MI>(a, n_cu, max_rows, s);
        if (a.epi == 2) return launch_one<BM, BN, BK, STAGES, WGM, WGN, false, true, 2, P, MI>(a, n_cu, max_rows, s);
        return ragged ? launch_one<BM, BN, BK, STAGES, WGM, WGN, false, true, 0, P, MI>(a, n_cu, max_rows, s)
                      : launch_one<BM, BN, BK, STAGES, WGM, WGN, false, false, 0, P, MI>(a, n_cu, max_rows, s);
    };
    if constexpr (PK) {
        if (a.Wp != nullptr) return go(std::true_type{});
    }
    return go(std::false_type{});
}

// tile variants: id, BM, BN, BK, ring slots, wavefronts in m, in n, fall-back, tile-order weights, block rows
// (0: short row tiles; with exactly 16 rows per expert they stream the weights 13 % faster than
// the 128-row tiles, with the ragged counts of real routing they do not, so nothing selects them by
// default).  BM is the tallest tile of a variant: over ragged groups the tiles are cut to fit the group
// (cut_group) in units of 32 rows per row of wavefronts.  A ring of S slots needs K >= S * BK; for a
// shorter K the launcher takes the two-slot variant with 32-wide K steps (K is a multiple of 64)
// listed in the eighth column.  Ninth column: the variant is also built for weights in tile
// order (kernels.h: the shapes the library picks by itself; the others read the caller's layout).
// Last column: rows of the matrix instruction's block, 32 (v_mfma_f32_32x32x16_bf16) or 16
// (v_mfma_f32_16x16x32_bf16; 64-wide K steps only, so their fall-backs for a short K are 32-row
// variants).  21, 22 and 31 are 1, 2 and 11 with 16-row blocks: what the library picks by itself.
#define MOE_EP_VARIANTS(X)         \
    X(0, 64, 128, 64, 2, 1, 2, 8, false, 32)  \
    X(1, 128, 256, 64, 3, 2, 2, 6, true, 32) \
    X(2, 256, 256, 64, 2, 2, 2, 9, true, 32) \
    X(6, 128, 256, 32, 2, 2, 2, 6, false, 32) \
    X(8, 64, 128, 32, 2, 1, 2, 8, false, 32)  \
    X(9, 256, 256, 32, 2, 2, 2, 9, false, 32)  \
    X(11, 160, 256, 64, 3, 1, 4, 12, true, 32) \
    X(12, 160, 256, 32, 2, 1, 2, 12, false, 32) \
    X(13, 224, 256, 64, 2, 1, 4, 12, false, 32) \
    X(14, 256, 256, 64, 2, 1, 4, 12, false, 32) \
    X(21, 128, 256, 64, 3, 2, 2, 6, true, 16) \
    X(22, 256, 256, 64, 2, 2, 2, 9, true, 16) \
    X(31, 160, 256, 64, 3, 1, 4, 12, true, 16)

hipError_t grouped_gemm_init()
{
    hipError_t e;
#define X(id, BM, BN, BK, ST, WGM, WGN, FB, PK, MI)                                      \
    if ((e = raise_all<BM, BN, BK, ST, WGM, WGN, false, MI>()) != hipSuccess) return e;  \
    if constexpr (PK) if ((e = raise_all<BM, BN, BK, ST, WGM, WGN, PK, MI>()) != hipSuccess) return e;
    MOE_EP_VARIANTS(X)
#undef X
    return hipSuccess;
}

bool grouped_gemm_variant_shape(int variant, int K, bool ragged, int G, int shape[8])
{
    switch (variant) {
#define X(id, BM, BN, BK, ST, WGM, WGN, FB, PK, MI)                                                  \
        case id:                                                                                    \
            if (K / BK < ST || GemmCfg<BM, BN, BK, ST, WGM, WGN, false>::LDS_BYTES +                \
                                       lds_table_bytes(ragged, G) > kLdsPerWorkgroup) {              \
                if (FB == id) return false;                                                         \
                return grouped_gemm_variant_shape(FB, K, ragged, G, shape);                         \
            }                                                                                       \
            shape[0] = BM; shape[1] = BN; shape[2] = BK; shape[3] = ST; shape[4] = WGM; shape[5] = WGN; \
            shape[6] = PK; shape[7] = MI;                                                           \
            return true;
        MOE_EP_VARIANTS(X)
#undef X
        default: return false;
    }
}

int grouped_gemm_variant_mfma16(int variant)
{
    return variant == 1 ? 21 : variant == 2 ? 22 : variant == 11 ? 31 : variant;
}

hipError_t launch_grouped_gemm(const GemmArgs& a, bool swiglu, int variant, int n_cu,
                               long long max_rows, hipStream_t s)
{
    if (a.K < 64 || a.K % 64) return hipErrorInvalidValue;
    if (a.offset ? max_rows <= 0 : a.dense_rows <= 0) return hipSuccess;
    switch (variant) {
#define X(id, BM, BN, BK, ST, WGM, WGN, FB, PK, MI)                                                  \
        case id:                                                                                    \
            if (a.K / BK < ST || GemmCfg<BM, BN, BK, ST, WGM, WGN, false>::LDS_BYTES +              \
                                         lds_table_bytes(a.offset != nullptr, a.G) > kLdsPerWorkgroup) { \
                if (FB == id) return hipErrorInvalidValue;                                          \
                return launch_grouped_gemm(a, swiglu, FB, n_cu, max_rows, s);                  \
            }                                                                                       \
            return launch_cfg<BM, BN, BK, ST, WGM, WGN, PK, MI>(a, swiglu, n_cu, max_rows, s);
        MOE_EP_VARIANTS(X)
#undef X
        default: return hipErrorInvalidValue;
    }
}

// ---- weights in tile order (kernels.h)
__global__ __launch_bounds__(256) void pack_weights_kernel(GemmArgs a, bool swiglu, uint4* __restrict__ dst, size_t chunks)
{
    const int bn_out = swiglu ? kPackRows / 2 : kPackRows;
    const int NT = (a.N + bn_out - 1) / bn_out, KT = a.K / kPackK;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < chunks; i += (size_t)gridDim.x * blockDim.x) {
        const int c = (int)(i % 8);                       // 16-byte chunk of the 128-byte row
        size_t r = i / 8;
        const int jw = (int)(r % kPackRows); r /= kPackRows;
        const int ks = (int)(r % KT); r /= KT;
        const int nt = (int)(r % NT);
        const int g = (int)(r / NT);
        int n = nt * bn_out + jw;
        long long base = 0;
        if (swiglu && jw >= kPackRows / 2) { n = nt * bn_out + jw - kPackRows / 2; base = a.w_up_offset; }
        n = min(n, a.N - 1);
        const int k = ks * kPackK + c * 8;
        const int seg = k / a.kseg_len;
        const uint16_t* src = a.W + (size_t)g * a.w_group_stride + base + (size_t)n * a.ldw +
                              (size_t)seg * a.w_kseg_stride + (k - seg * a.kseg_len);
        dst[i] = *reinterpret_cast<const uint4*>(src);
    }
}

size_t packed_weight_elems(const GemmArgs& a, bool swiglu)
{
    const int bn_out = swiglu ? kPackRows / 2 : kPackRows;
    const size_t NT = (a.N + bn_out - 1) / bn_out;
    return (size_t)a.G * NT * kPackRows * (size_t)a.K;
}

hipError_t launch_pack_weights(const GemmArgs& a, bool swiglu, uint16_t* dst, int grid, hipStream_t s)
{
    if (a.K < kPackK || a.K % kPackK || a.kseg_len % 8 || a.ldw % 8 || a.w_group_stride % 8 || a.w_up_offset % 8 ||
        a.w_kseg_stride % 8 || (reinterpret_cast<uintptr_t>(a.W) & 15) || (reinterpret_cast<uintptr_t>(dst) & 15))
        return hipErrorInvalidValue;
    const size_t chunks = packed_weight_elems(a, swiglu) / 8;
    if (chunks == 0) return hipSuccess;
    hipLaunchKernelGGL(pack_weights_kernel, dim3(grid), dim3(256), 0, s, a, swiglu, reinterpret_cast<uint4*>(dst), chunks);
    return hipGetLastError();
}

}  // namespace moe_ep
