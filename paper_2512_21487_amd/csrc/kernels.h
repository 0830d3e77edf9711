// Host-side launchers of the HIP kernels (internal to the library; the public boundary is moe_ep.h).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace moe_ep {

// tokens per router / permute workgroup: one bit each in a 64-bit mask per expert
constexpr int kTokPerBlock = 64;

// ---- gate: softmax + top-k (Sec. 2.1) and per-workgroup expert bit masks for the partition
hipError_t launch_router(const float* logits, int Tn, int E, int k, int e0, int El, int32_t* idx,
                         float* w, unsigned long long* blk_mask, hipStream_t s);

// ---- partition by expert (Sec. 2.1; Sec. 3.1 "The MoE Part")
// count [El], offset [El + 1], pos [Tn * k] (row of an assignment or -1), perm [rows] (row -> assignment)
hipError_t launch_dispatch(const int32_t* idx, const unsigned long long* blk_mask, int Tn, int k, int e0, int El,
                           int32_t* count, int32_t* offset, int32_t* pos, int32_t* perm, hipStream_t s);
hipError_t launch_gather_rows(const void* tokens, const int32_t* perm, const int32_t* n_rows_ptr,
                              int k, int M, void* xp, int grid, hipStream_t s);

// ---- weighted aggregation (Sec. 2.1)
// y_mode: 0 bf16 expert outputs, weighted here; 1 fp32 expert outputs, weighted here; 2 bf16 expert
// outputs that already carry their routing weight
// accumulate: the rows at out_src already hold the shared experts' output and the sum is added to
// them.  out_src == NULL or == out: in place (rows with nothing kept are then left alone); else
// every row is read at out_src and written at out (which may be the caller's pinned host buffer)
hipError_t launch_combine(const void* y, const int32_t* pos, const float* w, int Tn, int k, int M,
                          bool accumulate, int y_mode, const void* out_src, void* out, int grid, hipStream_t s);

// ---- chunk transfers over the host link (pinned-host mode); bytes must be a multiple of 4
hipError_t launch_copy(void* dst, const void* src, size_t bytes, int grid, hipStream_t s, int threads = 256, int unroll = 4);
// a one-wavefront kernel that lasts about `microseconds` (at most 1 s): stand-in for a task that
// runs on other hardware
hipError_t launch_busy(double microseconds, hipStream_t s);

// ---- expert projections as one grouped GEMM launch (Sec. 3.1, Eq. moe_detail / shared_detail)
struct GemmArgs {
    const uint16_t* A;         // activations, bf16 [rows, lda]
    const uint16_t* W;         // first group's weight matrix, bf16 rows of length ldw
    uint16_t* C;               // output, bf16 [rows, ldc]
    const int32_t* offset;     // ragged mode: [G+1] first row of each group (device); NULL = dense
    int G;                     // groups (experts)
    int dense_rows;            // dense mode: every group multiplies rows [0, dense_rows) of A
    int K;                     // reduction length, multiple of 64
    int N;                     // output columns per group (SwiGLU: activation columns)
    int lda, ldc, ldw;
    long long w_group_stride;  // elements from one group's matrix to the next group's
    long long w_up_offset;     // SwiGLU: elements from W_gate to W_up
    int kseg_len;              // K is split into segments of this length ...
    long long w_kseg_stride;   // ... whose weight blocks are this many elements apart
    int c_group_col_stride;    // dense mode: group g writes columns starting at g * this
    // ragged mode, optional: grouped row p is not row p of A but row a_row_map[p] / a_row_div of A
    // (the partition's row -> assignment map with a_row_div = top_k: the token rows are then
    // gathered by the tile loads themselves); a_src_rows = rows A holds.  NULL = rows are in place.
    const int32_t* a_row_map;
    int a_row_div;
    int a_src_rows;
    // ragged mode: tallest row tile, in units of 32 rows per row of wavefronts of the variant
    // (0 or more than the variant holds = the variant's full height); every group's tiles are cut
    // to equal heights below this
    int max_units;
    // what the epilogue writes (ragged, no SwiGLU only; see grouped_gemm.hip): 0 bf16, 1 fp32 (C then
    // points at floats, ldc counts floats), 2 bf16 scaled by row_weight[row_assignment[grouped row]]
    int epi;
    const float* row_weight;
    const int32_t* row_assignment;
    // optional: the same weights in tile order (pack_weights), or NULL.  Used by the variants whose
    // weight tile is kPackRows rows by kPackK reduction steps; the others read W.
    const uint16_t* Wp;
};
// Weights in tile order: for every group, column tile and K step of kPackK, the kPackRows x kPackK
// block the GEMM's weight tile holds at that step (SwiGLU: kPackRows / 2 rows of W_gate, then the
// matching rows of W_up; rows past N repeat row N - 1), contiguous (32 KB), blocks in (group, column
// tile, K step) order.  a.W etc. describe the source as for a launch; a.Wp is ignored.
constexpr int kPackRows = 256, kPackK = 64;
size_t packed_weight_elems(const GemmArgs& a, bool swiglu);
hipError_t launch_pack_weights(const GemmArgs& a, bool swiglu, uint16_t* dst, int grid, hipStream_t s);
// variant: index into the tile-shape table of grouped_gemm.hip; max_rows: ragged mode, an upper
// bound of the rows of all groups together (the kernel cuts them into row tiles itself, from
// `offset`; the bound only sizes the grid); ignored in dense mode
hipError_t launch_grouped_gemm(const GemmArgs& a, bool swiglu, int variant, int n_cu,
                               long long max_rows, hipStream_t s);
hipError_t grouped_gemm_init();   // raises the dynamic-LDS limit of every instantiation once
// the shape a launch of `variant` really runs (after the fall-backs for a short K or many groups):
// shape[] = tallest tile rows, weight rows per tile, K step, ring slots, wavefronts in m, in n,
// whether it reads weights in tile order when the launch has them (GemmArgs::Wp), and the rows of the
// matrix instruction's block (32: v_mfma_f32_32x32x16_bf16, 16: v_mfma_f32_16x16x32_bf16); false for an
// unknown variant
bool grouped_gemm_variant_shape(int variant, int K, bool ragged, int G, int shape[8]);
// the variant of the same tile shape that multiplies with the 16 x 16 x 32 instruction, or `variant` itself
int grouped_gemm_variant_mfma16(int variant);

}  // namespace moe_ep
