/*
 * moe_ep.h -- C ABI of the expert-group side of one MoE layer on one MI355X.
 *
 * The library runs, for the experts one GPU of the expert group holds, the
 * part of a mixture-of-experts layer that fine-grained disaggregated expert
 * parallelism schedules: gate softmax + top-k (Sec. 2.1), partition of the
 * tokens by expert (Sec. 2.1; Sec. 3.1 "The MoE Part"), the three projections
 * of each routed expert (Sec. 3.1, Eq. moe_detail), the weighted aggregation
 * of the selected experts' outputs (Sec. 2.1), the optional shared experts
 * (Sec. 3.1, Eq. shared_detail), all cut along the token dimension into
 * r_2 = r_chunks pieces (Sec. 2.3) whose transfers and compute overlap.
 *
 * Plain C: no C++ types, no exceptions, nothing from PyTorch crosses this
 * boundary.  Every function returns a moe_ep_status (0 = OK, negative = error)
 * unless stated otherwise, never aborts, and validates its arguments before
 * anything is launched or allocated.
 *
 * Notation (Table "Notations"): M hidden size, H expert intermediate size,
 * E global experts, top_k experts per token, r_2 chunks.
 */
#ifndef MOE_EP_H
#define MOE_EP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct moe_ep_ctx moe_ep_ctx; /* opaque, owned by the library */

typedef enum {
    MOE_EP_OK = 0,
    MOE_EP_EINVAL = -1, /* bad argument; nothing was launched               */
    MOE_EP_ENOMEM = -2, /* host or device allocation failed                 */
    MOE_EP_EHIP = -3,   /* a HIP call failed (see moe_ep_last_error)        */
    MOE_EP_ESTATE = -4  /* call not valid in the context's current state    */
} moe_ep_status;

/* Where the shared experts run relative to the routed chunks (Sec. 4.2,
 * "Determine the order of Attention and Shared Expert", reduced to the one
 * GPU this library drives).  The result does not depend on the order. */
typedef enum {
    MOE_EP_ORDER_SHARED_FIRST = 0, /* shared experts on all tokens, then the routed chunks:
                                      the shared expert treated as part of what precedes the
                                      transfer (Sec. 2.3, first limitation)                 */
    MOE_EP_ORDER_INTERLEAVED = 1   /* shared experts of chunk j issued next to routed chunk j */
} moe_ep_order;

/* Where tokens / gate_logits / out live.  Weights are always in device memory. */
typedef enum {
    MOE_EP_IO_DEVICE = 0,     /* device pointers; no copies are made                        */
    MOE_EP_IO_PINNED_HOST = 1 /* pinned host pointers; each chunk crosses the host link in and
                                 out, standing in for the A2E / E2A transfers (Sec. 2.2; Eq.
                                 a2e_detail): inbound as a copy on a stream of the context
                                 (a chunk's gate scores first: gate and partition run while its
                                 token rows are still on the link),
                                 outbound as the aggregation's own stores into the host buffer
                                 (moe_ep_forward; the environment variable MOE_EP_FUSED_OUT=0
                                 makes it a copy on a second stream) or as such a copy
                                 (moe_ep_forward_dep)                                       */
} moe_ep_io;

typedef struct {
    int32_t hidden;       /* M; multiple of 64                                              */
    int32_t inter;        /* H of a routed expert; multiple of 64; hidden * inter < 2^30    */
    int32_t n_experts;    /* E, size of the gate's expert axis; 1..512                      */
    int32_t local_begin;  /* first expert held here; experts [local_begin, +n_local)        */
    int32_t n_local;      /* E/eg experts held here; >= 1                                   */
    int32_t n_shared;     /* N_shared; 0 = no shared expert                                 */
    int32_t shared_inter; /* H of each shared expert; multiple of 64 (ignored if none)      */
    int32_t max_tokens;   /* largest n_tokens of a forward; sizes the workspaces            */
    int32_t max_top_k;    /* largest top_k of a forward; 1..min(E, 64)                      */
    int32_t max_chunks;   /* largest r_chunks of a forward; 1..64                           */
    int32_t io_mode;      /* moe_ep_io                                                      */
    int32_t device;       /* HIP device ordinal                                             */
} moe_ep_config;

/* Pure host checks of a layer's shape (the quantities of the paper's notation table: M, H, E, the
 * E / eg experts of a device, top_k, N_shared) and of a forward's arguments, usable without a GPU.
 * Return MOE_EP_OK or MOE_EP_EINVAL; if `why` is not NULL it receives a static string naming the
 * first violated rule. */
int moe_ep_validate_config(const moe_ep_config *cfg, const char **why);
int moe_ep_validate_forward(const moe_ep_config *cfg, const void *tokens,
                            const float *gate_logits, const void *routed_w,
                            const void *shared_w, int32_t top_k, int32_t r_chunks,
                            int32_t order, int32_t n_tokens, const void *out,
                            const char **why);

/* Device bytes moe_ep_create will allocate for this configuration (0 if invalid). */
size_t moe_ep_workspace_bytes(const moe_ep_config *cfg);

/* Create a context: selects cfg->device, allocates all workspaces, streams and
 * events once.  *out_ctx is set only on success.  Not thread-safe per context. */
int moe_ep_create(const moe_ep_config *cfg, moe_ep_ctx **out_ctx);

/*
 * One pass of the layer over n_tokens tokens.
 *
 *   tokens      bf16 [n_tokens, M] row-major
 *   gate_logits fp32 [n_tokens, E] row-major: routing scores over the GLOBAL expert axis.
 *               Per token the top_k largest scores are selected (equal scores: lower
 *               expert index first), their softmax weights renormalised to sum 1;
 *               assignments to experts outside [local_begin, local_begin + n_local) are
 *               dropped without renormalising (they belong to another GPU).
 *               NaN / Inf scores are not supported.
 *   routed_w    bf16, device: for each local expert, contiguous, W_gate [H, M],
 *               W_up [H, M], W_down [M, H], all row-major (Sec. 3.1); experts contiguous.
 *               (A pointer that moe_ep_prepare_weights has seen is read from the context's
 *               tile-order copy instead; the same holds for shared_w.)
 *   shared_w    bf16, device: the same triple for each shared expert with H = shared_inter;
 *               NULL exactly when n_shared == 0.
 *   top_k       1..min(E, max_top_k);   r_chunks 1..max_chunks (0 = chosen from the context's
 *               timing model, see moe_ep_set_pipeline_model): the token range is cut
 *               into r_chunks contiguous pieces of ceil(n_tokens / r_chunks) tokens (the
 *               last ones may be short or empty);   order: moe_ep_order (ignored when
 *               n_shared == 0).
 *   out         bf16 [n_tokens, M]: sum over kept slots of weight * expert(token) plus the
 *               sum of the shared experts; tokens with nothing kept and no shared expert
 *               get zeros.  Must not overlap tokens or gate_logits.  Accumulation is fp32; the activation between the up and down
 *               projections and each expert's output are rounded to bf16 once.
 *   stream      hipStream_t (NULL = the default stream).  The call only enqueues work: every
 *               kernel runs on `stream`, after what is already there; in pinned-host mode the
 *               chunk copies run on streams of the context and `stream` is made to wait
 *               for the last of them.  Buffers must stay valid until `stream` reaches that point.
 *               In device mode the call allocates nothing, sets no memory and never waits on the
 *               host, so it may be recorded into a HIP graph (stream capture) and replayed.
 *
 * tokens / gate_logits / out are device pointers in MOE_EP_IO_DEVICE mode and pinned host
 * pointers in MOE_EP_IO_PINNED_HOST mode.  Before anything is enqueued the runtime is asked what
 * each of the five pointers points at: one that is not GPU-addressable memory of the kind the mode
 * needs, or that lies in an allocation which ends before the bytes the forward will touch, gives
 * MOE_EP_EINVAL and a message naming the argument (the environment variable
 * MOE_EP_CHECK_POINTERS=0, read by moe_ep_create, skips the device-side queries; a bad pointer is
 * then a GPU memory fault).  The caller owns every buffer passed in; the
 * library owns its workspaces.  n_tokens == 0 is a no-op.  Results are deterministic:
 * the same inputs give the same bits, for every r_chunks and order.
 */
int moe_ep_forward(moe_ep_ctx *ctx, const void *tokens, const float *gate_logits,
                   const void *routed_w, const void *shared_w, int32_t top_k,
                   int32_t r_chunks, int32_t order, int32_t n_tokens, void *out,
                   void *stream);

/*
 * Expert weights in tile order (Sec. 3.1, "The MoE Part" and Eq. shared_detail: W_gate, W_up and W_down
 * of an expert are the same in every call, only the tokens change).  moe_ep_prepare_weights makes, in
 * device memory the context owns, a copy of the weights at routed_w and / or shared_w (either may be
 * NULL; layouts as for moe_ep_forward) in the order the projections' weight tiles read them: for every
 * expert, block of 256 output rows (gate/up: 128 rows of W_gate and the same 128 of W_up) and 64
 * reduction steps, one contiguous 32 KB block.  From then on every forward of this context that is
 * handed the same pointer reads the copy instead (the same kernels with another address pattern: the
 * same bits; 2-5 % less time on the prefill shapes, 19 % on the gate/up weight stream of the decode
 * shapes).  A pointer that has not been prepared is read where it is, as before.
 *
 *   stream   the copy kernels are enqueued here and the call returns; a forward that uses the copy must
 *            be ordered after them (same stream, or an event).
 *   memory   moe_ep_prepared_weight_bytes(cfg, routed, shared) bytes of device memory for the pointers
 *            given (about the size of the weights themselves), allocated by this call: MOE_EP_ENOMEM
 *            if there is not enough.  Preparing a pointer again refreshes its copy in place.
 *   stale    the copy is keyed by the pointer: a caller that rewrites the weights behind a prepared
 *            pointer prepares it again, or forgets it.
 * moe_ep_forget_weights frees the copies of the given pointers (both NULL: all of them) after waiting
 * for the device; moe_ep_destroy frees what is left.  MOE_EP_EINVAL: no pointer given, shared_w for a
 * configuration without shared experts, a pointer the GPU cannot read over the weights' extent.
 * moe_ep_prepared_weight_bytes: routed / shared non-zero = count that set; 0 for an invalid cfg.
 */
int moe_ep_prepare_weights(moe_ep_ctx *ctx, const void *routed_w, const void *shared_w, void *stream);
int moe_ep_forget_weights(moe_ep_ctx *ctx, const void *routed_w, const void *shared_w);
size_t moe_ep_prepared_weight_bytes(const moe_ep_config *cfg, int32_t routed, int32_t shared);

/*
 * moe_ep_forward for callers that cannot allocate device memory: code running under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  There is no context: the
 * workspaces a context would own (routing arrays, activation, expert outputs; the layout
 * moe_ep_workspace_bytes(cfg) describes) live in one array of MOE_EP_NOALLOC_SCRATCH_BYTES bytes that
 * is part of the library's device image, so every GPU the library runs on holds it from the first
 * use until the process ends.  The call allocates and frees nothing, on the host or on the device,
 * creates no stream or event, sets no memory and never waits on the host; it runs the same kernels
 * as moe_ep_forward and produces the same bits.
 *
 *   cfg       as for moe_ep_create; io_mode must be MOE_EP_IO_DEVICE, device < 16, and
 *             moe_ep_workspace_bytes(cfg) <= MOE_EP_NOALLOC_SCRATCH_BYTES (size max_tokens, max_top_k
 *             and max_chunks to the call itself: e.g. 256 tokens of the 4096-wide, top-8 decode
 *             shape need 23 MiB), else MOE_EP_EINVAL
 *   r_chunks  1..max_chunks (0 is not accepted: there is no context to hold a timing model)
 *   why       may be NULL; receives a string naming the first violated rule or the failed HIP call
 *             (valid until the next call for the same device)
 *   all other arguments, layouts, ownership and determinism as for moe_ep_forward.
 *
 * Every call on a GPU uses that GPU's one array, which keeps the previous call's contents (nothing
 * in it has to start at zero: each forward overwrites what it reads).  Two calls that overlap on one
 * GPU -- from two host threads, or on two streams without an order between them -- race; calls
 * on one stream, or ordered by events, are safe.  The first call on a device looks up the array's
 * address on that device and raises the kernels' LDS limit.
 */
#define MOE_EP_NOALLOC_SCRATCH_BYTES (32u << 20)
int moe_ep_forward_noalloc(const moe_ep_config *cfg, const void *tokens, const float *gate_logits,
                           const void *routed_w, const void *shared_w, int32_t top_k,
                           int32_t r_chunks, int32_t order, int32_t n_tokens, void *out,
                           void *stream, const char **why);

/*
 * Test / inspection surface: host copies of what the last forward computed for chunk
 * `chunk` (synchronises the context's streams; after moe_ep_forward_dep chunk = i * r_2 + j for
 * chunk j of micro-batch i).  Any pointer may be NULL.  With Tn the tokens of this chunk:
 *   idx    int32 [Tn, top_k] selected global expert ids, best first
 *   w      fp32  [Tn, top_k] routing weights
 *   pos    int32 [Tn, top_k] row of the assignment in the grouped input, -1 if dropped
 *   count  int32 [n_local]   rows per local expert
 *   offset int32 [n_local+1] exclusive prefix sum of count
 *   perm   int32 [offset[n_local]] row -> assignment id (chunk-local token * top_k + slot);
 *          rows are grouped by expert and ascend by token inside an expert
 * The caller sizes perm for Tn * top_k entries.  Returns MOE_EP_ESTATE before any forward.
 */
int moe_ep_get_routing(moe_ep_ctx *ctx, int32_t chunk, int32_t *idx, float *w, int32_t *pos,
                       int32_t *count, int32_t *offset, int32_t *perm);

/*
 * Per-stage device time, in milliseconds, measured with HIP events on the streams the stages
 * run on (the task times t_e, t_s, t_a2e that Sec. 4.1 fits its linear models to).  moe_ep_set_profiling(ctx, depth) makes the next `depth` forwards (0..256; 0 = off)
 * record an event before and after every stage; this serialises nothing.
 * moe_ep_get_stage_ms synchronises, returns the per-forward AVERAGE over the forwards recorded
 * since the last call, and opens a new window of `depth` forwards:
 *   ms[0] gate  ms[1] partition (permute + row gather)  ms[2] routed gate/up GEMM
 *   ms[3] routed down GEMM  ms[4] shared gate/up GEMM  ms[5] shared down GEMM
 *   ms[6] aggregation  ms[7] whole forward (first enqueue to last completion)
 *   ms[8] inbound copies  ms[9] outbound copies (MOE_EP_IO_PINNED_HOST only, else 0)
 *   ms[10] attention stand-ins (moe_ep_forward_dep only, else 0)
 * each summed over the chunks of a forward.  n = floats the caller provides (<= 11 written).
 * Returns MOE_EP_ESTATE when nothing was recorded.
 */
int moe_ep_set_profiling(moe_ep_ctx *ctx, int32_t depth);
/* Restricts the events to the stages whose bit (1 << index into ms[]) is set in `mask`; the default
 * is every stage.  Events between all stages cost a few percent of a forward (more for small
 * calls); timing only one stage leaves the rest of the forward undisturbed. */
int moe_ep_set_profiling_stages(moe_ep_ctx *ctx, uint32_t mask);
int moe_ep_get_stage_ms(moe_ep_ctx *ctx, float *ms, int32_t n);
/*
 * The measured schedule: for every timed stage instance of the forwards recorded in the current
 * window (call it before moe_ep_get_stage_ms, which closes the window), in issue order, its stage
 * (index into ms[] above), the forward it belongs to (0-based inside the window) and its start and
 * end in milliseconds after that forward's first enqueue.  With r_2 chunks a stage appears r_2 times;
 * this is the timeline the start times tau of Sec. 3.2 describe.  Arrays (host, any may be NULL) hold
 * max_spans entries; *n_spans receives the number written.
 */
int moe_ep_get_timeline(moe_ep_ctx *ctx, int32_t *stage, int32_t *forward, float *begin_ms, float *end_ms,
                        int32_t max_spans, int32_t *n_spans);

/*
 * Timing model of the chunk pipeline and the choice of r_2 (Sec. 4.1 linear task models; Sec. 4.2
 * layer-0 timeline and "Determine r_2 and m_e"; Theorem 4).  Every task time is alpha + beta * m
 * with m = tokens per chunk; times in any one unit (milliseconds in this repository).
 */
typedef struct {
    double alpha_in, beta_in;   /* inbound transfer (A2E stand-in)  */
    double alpha_e, beta_e;     /* expert compute of a chunk        */
    double alpha_out, beta_out; /* outbound transfer (E2A stand-in) */
    /* The same three tasks while the other resources are active.  The paper's resources are separate
     * hardware (Sec. 3.2); where they share a GPU a transfer in flight slows the compute beside it and
     * the reverse, so coefficients fitted from forwards with r_chunks > 1 go here.  All six zero = the
     * resources are independent (the paper's model).  When set, one chunk (nothing overlaps) is priced
     * with the coefficients above and every r_chunks > 1 with these. */
    double alpha_in_beside, beta_in_beside;
    double alpha_e_beside, beta_e_beside;
    double alpha_out_beside, beta_out_beside;
} moe_ep_pipeline_model;

/* Least-squares fit of t = alpha + beta * x over n >= 2 samples (host arrays); *r2 (may be NULL)
 * receives the coefficient of determination.  MOE_EP_EINVAL if the x are all equal. */
int moe_ep_fit_linear(const double *x, const double *t, int32_t n, double *alpha, double *beta,
                      double *r2);

/* Finish time of one slice of n_tokens cut into r_chunks chunks on three serial resources:
 * t_in + t_e + t_out + (r - 1) * max(t_in, t_e, t_out), each at n_tokens / r_chunks tokens
 * (the paper's 2 t_a2e + t_e + (r_2 - 1) max(t_e, t_a2e) when both links are alike); with the
 * second set of coefficients present it prices r_chunks > 1.  Returns a negative value on bad
 * arguments. */
double moe_ep_pipeline_makespan(const moe_ep_pipeline_model *m, int32_t n_tokens, int32_t r_chunks);

/* The smallest r in 1..r_max that minimises moe_ep_pipeline_makespan: golden-section search over
 * 1/r (the objective is convex there) and a walk over the neighbouring integers; with the second
 * set of coefficients present the search covers r >= 2 and its result is compared with r = 1.
 * Returns r, or MOE_EP_EINVAL (negative) on bad arguments. */
int32_t moe_ep_choose_chunks(const moe_ep_pipeline_model *m, int32_t n_tokens, int32_t r_max);

/* Give a context its timing model: afterwards moe_ep_forward accepts r_chunks == 0 and picks
 * r = moe_ep_choose_chunks(model, n_tokens, max_chunks) itself.  m == NULL removes the model. */
int moe_ep_set_pipeline_model(moe_ep_ctx *ctx, const moe_ep_pipeline_model *m);

/* r_chunks the last forward ran with (the chosen value when 0 was passed); -1 before any forward. */
int32_t moe_ep_last_chunks(const moe_ep_ctx *ctx);

/*
 * Schedule model of disaggregated expert parallelism and the configuration search (host only, no
 * GPU call).  Notation of the paper: m_a samples per attention micro-batch, r_1 micro-batches,
 * m_e tokens per expert and chunk, r_2 chunks, T layers, ag / eg group sizes, S sequence length.
 * Task times are linear (Sec. 4.1): t_a(m_a), t_s(m_a), t_e(m_e), t_a2e(m_e) = t_e2a(m_e); m_e follows
 * from the conservation rule m_e * r_2 * E = m_a * ag * top_k * S (Sec. 3.2, Eq. limitation).
 */
typedef struct {
    double alpha_a, beta_a; /* attention of one micro-batch, argument m_a              */
    double alpha_s, beta_s; /* shared experts of one micro-batch, argument m_a         */
    double alpha_e, beta_e; /* routed experts of one chunk on one device, argument m_e */
    double alpha_c, beta_c; /* A2E (= E2A) transfer of one chunk, argument m_e         */
} moe_ep_dep_models;

typedef struct {
    int32_t ag;        /* attention-group size   */
    int32_t n_experts; /* E                      */
    int32_t top_k;
    int32_t seq_len;   /* S                      */
    int32_t n_layers;  /* T                      */
} moe_ep_dep_problem;

/* Order in which the attention group takes a layer's tasks (Sec. 4.2): a_0 s_0 a_1 s_1 ... or
 * a_0 a_1 ... s_0 s_1 ... */
typedef enum { MOE_EP_DEP_ASAS = 0, MOE_EP_DEP_AASS = 1 } moe_ep_dep_order;

/*
 * One MoE layer as the disaggregated schedule of Sec. 2.3 runs it, on one GPU (Fig. as, Eq.
 * limitation): the n_tokens are r_1 micro-batches of ceil(n_tokens / r_1) tokens, each cut into r_2
 * chunks of ceil(micro-batch / r_2) tokens.  The attention group is a stream of the context's own:
 * per micro-batch a stand-in for its attention - a kernel that occupies one wavefront for about
 * attn_us microseconds (0 = none) - and the micro-batch's shared experts, in the order
 * a_0 s_0 a_1 s_1 ... (MOE_EP_DEP_ASAS) or a_0 a_1 ... s_0 s_1 ... (MOE_EP_DEP_AASS).  A
 * micro-batch's chunks start after its attention (rule 6): in MOE_EP_IO_PINNED_HOST mode their
 * inbound copies (A2E), in device mode their gate; gate, partition and the routed experts of every
 * chunk run on `stream` (rules 7, 8), the aggregation of a chunk after the micro-batch's shared
 * experts have written its output rows, and in pinned-host mode the outbound copy (E2A) follows.
 * r_1 * r_2 <= max_chunks.  Everything else - arguments, layouts, ownership, errors, determinism -
 * is as for moe_ep_forward, and the output bits are the same as moe_ep_forward's for every r_1, r_2,
 * order and attn_us.  On one GPU the shared experts and the routed experts share the compute units,
 * which the paper's two groups of GPUs do not: the measured schedule (moe_ep_get_timeline) obeys the
 * rules, its makespan is not the paper's.  Not for stream capture (the first call creates the
 * attention-group stream).
 */
/*
 * Host only: the token range [*first, *first + *count) of chunk `chunk` = i * r_2 + j when n_tokens
 * are cut into r_1 micro-batches of ceil(n_tokens / r_1) tokens and each micro-batch into r_2 chunks
 * of ceil(micro-batch / r_2) tokens (Sec. 2.3; the last micro-batches and chunks may be short or
 * empty).  moe_ep_forward uses r_1 = 1, r_2 = r_chunks.  MOE_EP_EINVAL on arguments out of range.
 */
int moe_ep_chunk_range(int32_t n_tokens, int32_t r_1, int32_t r_2, int32_t chunk, int32_t *first,
                       int32_t *count);

/*
 * Host only: the tallest row tile (128 or 160 rows; 224- and 256-row shapes exist but are
 * never chosen) the library gives a routed projection
 * (Sec. 3.1, Eq. moe_detail) of a chunk of n_tokens tokens -- down == 0: gate/up projection, else
 * the down projection -- on a GPU of n_cu compute units.  An expert of the balanced load of Sec. 3.1
 * gets n_tokens * top_k / E rows; its row tiles are cut to equal heights below the tallest; the
 * choice compares expected rounds of tiles times the measured time of a tile of each shape.  It
 * changes no result bit.  MOE_EP_EINVAL (negative) on bad arguments.
 */
int32_t moe_ep_routed_tile_rows(const moe_ep_config *cfg, int32_t n_tokens, int32_t top_k, int32_t down,
                                int32_t n_cu);

/*
 * What the last forward launched for a projection: stage = index into ms[] of moe_ep_get_stage_ms
 * (2 routed gate/up, 3 routed down, 4 shared gate/up, 5 shared down; Sec. 3.1, Eq. moe_detail and
 * Eq. shared_detail), chunk = the chunk of that forward (ignored for the shared experts).  Receives
 * the kernel's tile shape -- tallest tile rows, weight rows per tile, K step, LDS ring slots,
 * wavefronts along rows and along columns --, whether it read the weights from a tile-order copy
 * (moe_ep_prepare_weights; 1 or 0), and the rows of the block its matrix instruction multiplies (16:
 * v_mfma_f32_16x16x32_bf16, 32: v_mfma_f32_32x32x16_bf16), so that a measurement can name the kernel it
 * timed.  Any pointer may be NULL.  MOE_EP_ESTATE before any forward or for a stage the layer does not have.
 */
int moe_ep_last_tile_shape(const moe_ep_ctx *ctx, int32_t chunk, int32_t stage, int32_t *rows,
                           int32_t *cols, int32_t *k_step, int32_t *ring_slots, int32_t *waves_m,
                           int32_t *waves_n, int32_t *tile_order, int32_t *mfma_rows);

int moe_ep_forward_dep(moe_ep_ctx *ctx, const void *tokens, const float *gate_logits,
                       const void *routed_w, const void *shared_w, int32_t top_k, int32_t r_1,
                       int32_t r_2, int32_t dep_order, double attn_us, int32_t n_tokens, void *out,
                       void *stream);

typedef struct {
    int32_t m_a, r_1, r_2, order;
    double m_e;        /* tokens per expert and chunk                         */
    double makespan;   /* of the T layers, in the unit of the models          */
    double throughput; /* r_1 * m_a * ag / makespan (Sec. 3.2, Eq. final-objective) */
} moe_ep_dep_config;

/* Primitives of Sec. 4.1: GEMM time alpha_gm + beta_gm * (m k n), attention time alpha_attn +
 * beta_attn * y, link time alpha_c + beta_c * z, and the layer's shape. */
typedef struct {
    double alpha_gm, beta_gm, alpha_attn, beta_attn, alpha_c, beta_c;
    int32_t seq_len, hidden, inter, n_heads, d_k, d_v, n_shared, n_experts, eg;
} moe_ep_dep_primitives;

/* Coefficients of the four task models from the primitives (Sec. 4.1, "Performance models of
 * different layers"; alpha_e includes the factor 3 of Eq. moe_detail). */
int moe_ep_dep_layer_models(const moe_ep_dep_primitives *q, moe_ep_dep_models *out);

/* m_e for (m_a, r_2); negative on bad arguments. */
double moe_ep_dep_tokens_per_expert(const moe_ep_dep_problem *p, int32_t m_a, int32_t r_2);

/*
 * Earliest-start replay of the timing rules of Eq. limitation: attention group, A2E link, expert
 * group and E2A link each run one task at a time in a fixed sequence (links and experts by layer,
 * micro-batch, chunk; the attention group by `order`), and a task starts when its resource is free
 * and what it depends on has finished.  *makespan = max(end of the last shared expert, end of the
 * last E2A).  The tau arrays (host, may be NULL) receive the start times, row-major
 * tau_a, tau_s [T][r_1];  tau_a2e, tau_e, tau_e2a [T][r_1][r_2].
 */
int moe_ep_dep_replay(const moe_ep_dep_models *m, const moe_ep_dep_problem *p, int32_t m_a, int32_t r_1,
                      int32_t r_2, int32_t order, double *makespan, double *tau_a, double *tau_s,
                      double *tau_a2e, double *tau_e, double *tau_e2a);

/*
 * The same replay for the stand-in in which both groups share one GPU (moe_ep_forward_dep): the rules
 * of Eq. limitation plus one the paper does not need -- a shared-expert task and an expert task do not
 * overlap, they run on the same compute units.  The rules then leave open which of two waiting tasks
 * goes first, so the schedule is the result of a procedure: of the next task of each of the four
 * sequences, those whose predecessors have been placed are candidates; the one that can start earliest
 * is placed at that time (ties: attention group, A2E, experts, E2A); repeat.  Arguments and outputs as
 * for moe_ep_dep_replay; the models' durations are those of the tasks running alone.
 */
int moe_ep_dep_replay_one_gpu(const moe_ep_dep_models *m, const moe_ep_dep_problem *p, int32_t m_a, int32_t r_1,
                      int32_t r_2, int32_t order, double *makespan, double *tau_a, double *tau_s,
                      double *tau_a2e, double *tau_e, double *tau_e2a);

/* Makespan model of the ASAS order over T layers (Sec. 4.2, denominator of Eq. simplify-objective):
 * (T-1) max(G, r_1 F) + max(X, G) + (r_1 - 1) F.  Negative on bad arguments. */
double moe_ep_dep_makespan(const moe_ep_dep_models *m, const moe_ep_dep_problem *p, int32_t m_a,
                           int32_t r_1, int32_t r_2);

/* The smallest r_2 in 1..r2_max with the smallest makespan for (m_a, r_1, order) (Sec. 4.2,
 * "Determine r_2 and m_e"; Theorem 4): ASAS by a convex search over 1 / r_2 on the model above,
 * AASS, for which the paper gives no closed form, by replaying every r_2. */
int moe_ep_dep_solve_r2(const moe_ep_dep_models *m, const moe_ep_dep_problem *p, int32_t m_a, int32_t r_1,
                        int32_t order, int32_t r2_max, int32_t *r_2, double *makespan);

/* Algorithm 1: m_a from m_a_max down to 1, r_1 = min(r1_cap, mem_cap / m_a) (the memory rule
 * r_1 * m_a <= mem_cap), pairs whose r_1 equals the previous one skipped, both orders, r_2 as above;
 * *best receives the configuration of highest throughput.  MOE_EP_ESTATE if no pair fits. */
int moe_ep_dep_search(const moe_ep_dep_models *m, const moe_ep_dep_problem *p, int32_t m_a_max,
                      int32_t mem_cap, int32_t r1_cap, int32_t r2_max, moe_ep_dep_config *best);

/* Last error text of this context (never NULL; valid until the next call on it). */
const char *moe_ep_last_error(const moe_ep_ctx *ctx);

/* Release everything the context owns.  NULL is allowed. */
int moe_ep_destroy(moe_ep_ctx *ctx);

/* Library version, "major.minor". */
const char *moe_ep_version(void);

#ifdef __cplusplus
}
#endif
#endif /* MOE_EP_H */
