// C ABI of the expert-group MoE layer: argument checks, workspaces, and the chunk pipeline
// that strings the kernels together (Sec. 2.3: the token range is cut into r_2 pieces whose
// transfers and expert compute overlap; Sec. 3.2, Eq. limitation: each of the three
// resources -- inbound transfer, expert compute, outbound transfer -- runs one task at a
// time, and a chunk's compute waits for its inbound transfer, its outbound transfer for its
// compute).  The resources are three HIP streams -- the caller's for compute, two of the context's
// for the link directions -- and the precedence rules are HIP events.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

#include "kernels.h"
#include "moe_ep.h"

using namespace moe_ep;

namespace {

enum Stage { ST_ROUTER = 0, ST_PARTITION, ST_GEMM1, ST_GEMM2, ST_SGEMM1, ST_SGEMM2, ST_COMBINE, ST_TOTAL, ST_COPY_IN, ST_COPY_OUT, ST_ATTN, ST_COUNT };

struct ProfSpan { hipEvent_t a, b; int stage; int forward; };

}  // namespace

struct moe_ep_ctx {
    moe_ep_config cfg;
    int n_cu = 0;
    int gemm_variant = -1;   // routed experts: tile variant, -1 = chosen per chunk (routed_variant)
    int up_variant = -1, down_variant = -1;  // the same for one projection only (tuning)
    int up_units = 0, down_units = 0;        // tallest row tile in units (0 = chosen / the variant's height)
    int shared_variant = 2;  // shared experts: dense rows, 256-row tiles
    // the shapes the library picks by itself multiply with v_mfma_f32_16x16x32_bf16 (MOE_EP_MFMA=32: with
    // v_mfma_f32_32x32x16_bf16); a shape named through a knob is taken as named
    bool mfma16 = true;
    bool shared_variant_named = false;
    bool fused_gather = true;  // the gate/up projection gathers the token rows itself (no grouped copy)
    int y_mode = 0;            // expert outputs: 0 bf16, 1 fp32, 2 bf16 scaled by the routing weight (expert_out_mode)
    // pinned-host mode, moe_ep_forward: the aggregation writes its rows straight into the caller's host
    // buffer and there is no outbound copy.  On this GPU a kernel that starts while another stream's
    // kernel streams writes to the host does not complete until that stream pauses, so an outbound copy
    // on a stream of its own overlaps with nothing and only adds a kernel; fused, every size and chunk
    // count measured 2-10 % faster.  MOE_EP_FUSED_OUT=0 restores the outbound link stream, which
    // moe_ep_forward_dep, whose point is the schedule of Sec. 2.3, always uses.
    bool fused_out = true;
    // a host-link copy kernel: 64 workgroups of one wavefront, two 16-byte loads per lane in flight
    // (128 KB over the link, enough to fill it).  A copy wavefront holds the vector memory path of its
    // compute unit with host-link latencies, and a GEMM tile that shares the unit runs at a fraction of
    // its rate; many thin copy workgroups slow 64 units a little instead of 8 units a lot (the launch
    // lasts as long as its slowest tile): 4096 decode tokens in 2 chunks 1.53 -> 1.44 ms
    int link_grid = 64;
    int link_threads = 64, link_unroll = 2;
    bool memcpy_in = false, memcpy_out = false;  // host-link copies through the runtime instead of kernels
    bool check_spans = true;   // every forward asks the runtime what its pointer arguments point at
    // Weights in tile order (moe_ep_prepare_weights): copies of the gate/up and of the down weights laid
    // out the way the GEMM's weight tiles read them, owned by the context, keyed by the caller's pointer
    struct Prepared { const void* key; uint16_t* up; uint16_t* down; };
    std::vector<Prepared> prepared_routed, prepared_shared;
    // device workspaces
    void* d_tokens = nullptr; float* d_logits = nullptr; void* d_out = nullptr;  // pinned-host mode staging
    int32_t* idx = nullptr; float* w = nullptr; int32_t* pos = nullptr; int32_t* perm = nullptr;
    unsigned long long* blk_mask = nullptr;
    int32_t* count = nullptr; int32_t* offset = nullptr;
    uint16_t* xp = nullptr; uint16_t* h = nullptr; uint16_t* y = nullptr;
    uint16_t* hs = nullptr;
    // streams and events
    hipStream_t s_in = nullptr, s_out = nullptr;  // the two link directions (pinned-host mode)
    hipEvent_t ev_start = nullptr, ev_done = nullptr, ev_comp_done = nullptr;
    std::vector<hipEvent_t> ev_in, ev_comp;
    // pinned-host mode: a chunk's gate scores have arrived (they travel first: gate and partition need
    // nothing else and run while the chunk's token rows are still on the link)
    std::vector<hipEvent_t> ev_scores;
    // attention-group side of moe_ep_forward_dep, created at its first call: the stream the attention
    // stand-ins and the shared experts run on, and per micro-batch "attention done" / "shared done"
    hipStream_t s_ag = nullptr;
    hipEvent_t ev_ag_done = nullptr;
    std::vector<hipEvent_t> ev_attn, ev_shared;
    // last forward (for moe_ep_get_routing): tokens, top_k, chunks = micro-batches x chunks of each
    int last_T = -1, last_k = 0, last_r = 0, last_r1 = 1;
    bool last_prepared_routed = false, last_prepared_shared = false;  // it read tile-order copies of the weights
    struct ChunkVariants { int up, down; };
    std::vector<ChunkVariants> last_variants;  // per chunk of the last forward: tile variants of the routed projections
    // stage profiling
    int prof_depth = 0, prof_recorded = 0;
    uint32_t prof_mask = ~0u;
    std::vector<hipEvent_t> prof_pool; size_t prof_next = 0;
    std::vector<ProfSpan> prof_spans;
    // timing model for r_chunks == 0
    bool has_model = false;
    moe_ep_pipeline_model model{};
    char err[256] = {0};
};

namespace {

const char* set_why(const char** why, const char* msg) { if (why) *why = msg; return msg; }

size_t align256(size_t b) { return (b + 255) & ~(size_t)255; }

struct WsLayout {
    size_t tokens, logits, out, idx, w, pos, perm, blk_mask, count, offset, xp, h, y, hs, total;
};

// MOE_EP_FUSED_GATHER=0 brings back the grouped copy of the token rows (for comparison)
bool fused_gather_enabled()
{
    const char* v = getenv("MOE_EP_FUSED_GATHER");
    return v == nullptr || atoi(v) != 0;
}

// MOE_EP_EXPERT_OUT = fp32 | scaled: how the routed experts' outputs travel from the down projection
// to the aggregation -- as fp32 (not rounded in between; twice the bytes) or as bf16 already
// multiplied by the routing weight (Sec. 2.1).  Unset: bf16, weighted by the aggregation.  Both
// change where the path rounds, hence the output bits; they exist to be measured against the default.
int expert_out_mode()
{
    const char* v = getenv("MOE_EP_EXPERT_OUT");
    if (!v) return 0;
    return v[0] == 'f' ? 1 : v[0] == 's' ? 2 : 0;
}

WsLayout ws_layout(const moe_ep_config& c)
{
    WsLayout L{};
    const size_t T = (size_t)c.max_tokens, k = (size_t)c.max_top_k, M = (size_t)c.hidden, H = (size_t)c.inter;
    const size_t A = T * k, El = (size_t)c.n_local, R = (size_t)c.max_chunks;
    const size_t nblk = (T + kTokPerBlock - 1) / kTokPerBlock + R;
    const bool pinned = c.io_mode == MOE_EP_IO_PINNED_HOST;
    size_t o = 0;
    auto take = [&](size_t bytes) { size_t at = o; o += align256(bytes ? bytes : 1); return at; };
    L.tokens = take(pinned ? T * M * 2 : 0);
    L.logits = take(pinned ? T * (size_t)c.n_experts * 4 : 0);
    L.out = take(pinned ? T * M * 2 : 0);
    L.idx = take(A * 4); L.w = take(A * 4); L.pos = take(A * 4); L.perm = take(A * 4);
    L.blk_mask = take(nblk * El * 8);
    L.count = take(R * El * 4); L.offset = take(R * (El + 1) * 4);
    // the grouped copy of the token rows exists only when the gate/up projection cannot gather them
    // itself: switched off, or a chunk of 4 GB and more (its lanes hold 32-bit byte offsets)
    const bool need_xp = !fused_gather_enabled() || T * M * 2 >= ((size_t)1 << 32);
    L.xp = take(need_xp ? A * M * 2 : 0); L.h = take(A * H * 2); L.y = take(A * M * (expert_out_mode() == 1 ? 4 : 2));
    L.hs = take(c.n_shared > 0 ? T * (size_t)c.n_shared * (size_t)c.shared_inter * 2 : 0);
    L.total = o;
    return L;
}

// every workspace pointer of a context, from the base of one block of device memory laid out by ws_layout
void bind_workspaces(moe_ep_ctx* ctx, char* slab, const WsLayout& L)
{
    ctx->d_tokens = slab + L.tokens;
    ctx->d_logits = reinterpret_cast<float*>(slab + L.logits);
    ctx->d_out = slab + L.out;
    ctx->idx = reinterpret_cast<int32_t*>(slab + L.idx);
    ctx->w = reinterpret_cast<float*>(slab + L.w);
    ctx->pos = reinterpret_cast<int32_t*>(slab + L.pos);
    ctx->perm = reinterpret_cast<int32_t*>(slab + L.perm);
    ctx->blk_mask = reinterpret_cast<unsigned long long*>(slab + L.blk_mask);
    ctx->count = reinterpret_cast<int32_t*>(slab + L.count);
    ctx->offset = reinterpret_cast<int32_t*>(slab + L.offset);
    ctx->xp = reinterpret_cast<uint16_t*>(slab + L.xp);
    ctx->h = reinterpret_cast<uint16_t*>(slab + L.h);
    ctx->y = reinterpret_cast<uint16_t*>(slab + L.y);
    ctx->hs = reinterpret_cast<uint16_t*>(slab + L.hs);
}

// the environment knobs of a context (tuning and comparison aids; none changes a result bit)
void read_knobs(moe_ep_ctx* ctx)
{
    // tile-shape overrides for tuning (indices into the variant table of grouped_gemm.hip)
    if (const char* v = getenv("MOE_EP_GEMM_VARIANT")) ctx->gemm_variant = atoi(v);
    if (const char* v = getenv("MOE_EP_SHARED_VARIANT")) { ctx->shared_variant = atoi(v); ctx->shared_variant_named = true; }
    if (const char* v = getenv("MOE_EP_MFMA")) ctx->mfma16 = atoi(v) != 32;
    if (!ctx->shared_variant_named && ctx->mfma16) ctx->shared_variant = grouped_gemm_variant_mfma16(ctx->shared_variant);
    if (const char* v = getenv("MOE_EP_UP_VARIANT")) ctx->up_variant = atoi(v);
    if (const char* v = getenv("MOE_EP_DOWN_VARIANT")) ctx->down_variant = atoi(v);
    if (const char* v = getenv("MOE_EP_UP_UNITS")) ctx->up_units = atoi(v);
    if (const char* v = getenv("MOE_EP_DOWN_UNITS")) ctx->down_units = atoi(v);
    // workgroups of a copy kernel: ~128 KB in flight fills the host link; more only queues up in the
    // memory fabric in front of the compute kernels
    if (const char* v = getenv("MOE_EP_LINK_GRID")) ctx->link_grid = atoi(v) > 0 ? atoi(v) : 64;
    if (const char* v = getenv("MOE_EP_LINK_THREADS")) ctx->link_threads = (atoi(v) >= 64 && atoi(v) <= 256 && atoi(v) % 64 == 0) ? atoi(v) : 64;
    if (const char* v = getenv("MOE_EP_LINK_UNROLL")) ctx->link_unroll = atoi(v) >= 1 ? atoi(v) : 2;
    // MOE_EP_LINK_MEMCPY = 1 | in | out: the runtime's asynchronous copies (DMA engines) instead of copy
    // kernels in both / one direction, kept for comparison: inbound they overlap cleanly with compute,
    // but each call costs the host thread 0.2-0.3 ms on this system
    if (const char* v = getenv("MOE_EP_LINK_MEMCPY")) {
        ctx->memcpy_in = v[0] == '1' || v[0] == 'i';
        ctx->memcpy_out = v[0] == '1' || v[0] == 'o';
    }
    ctx->fused_gather = fused_gather_enabled();
    ctx->y_mode = expert_out_mode();
    if (const char* v = getenv("MOE_EP_FUSED_OUT")) ctx->fused_out = atoi(v) != 0;
    // MOE_EP_CHECK_POINTERS=0 skips the per-forward pointer queries (a few microseconds of host time)
    if (const char* v = getenv("MOE_EP_CHECK_POINTERS")) ctx->check_spans = atoi(v) != 0;
}

int fail(moe_ep_ctx* ctx, int code, const char* what, hipError_t e = hipSuccess)
{
    if (ctx) {
        if (e != hipSuccess) snprintf(ctx->err, sizeof ctx->err, "%s: %s", what, hipGetErrorString(e));
        else snprintf(ctx->err, sizeof ctx->err, "%s", what);
    }
    return code;
}

#define HIP_TRY(ctx, call)                                                      \
    do {                                                                        \
        hipError_t e__ = (call);                                                \
        if (e__ != hipSuccess) return fail((ctx), MOE_EP_EHIP, #call, e__);     \
    } while (0)

// What the kernels are about to read or write through a caller's pointer: memory the GPU can
// address, of at least `bytes` bytes where the runtime knows the allocation's extent.  Turns a host
// pointer or an undersized buffer into an error before a kernel faults on it.  Returns nullptr when
// the span is usable, else what is wrong with it.  `want_host`: pinned host memory is required
// (the link stand-ins of MOE_EP_IO_PINNED_HOST); *dev_ptr receives the address kernels use.
const char* check_span(const void* p, size_t bytes, bool want_host, const void** dev_ptr)
{
    hipPointerAttribute_t attr;
    if (hipPointerGetAttributes(&attr, p) != hipSuccess) {
        (void)hipGetLastError();
        return want_host ? "must be pinned host memory in MOE_EP_IO_PINNED_HOST mode" : "is not memory the GPU can address";
    }
    if (want_host) {
        if (attr.type != hipMemoryTypeHost || attr.devicePointer == nullptr)
            return "must be pinned host memory in MOE_EP_IO_PINNED_HOST mode";
        if (dev_ptr) *dev_ptr = attr.devicePointer;
        return nullptr;
    }
    if (dev_ptr) *dev_ptr = p;
    if (attr.type == hipMemoryTypeHost) {  // pinned host memory works (at the host link's rate)
        if (attr.devicePointer == nullptr) return "is host memory the GPU cannot address";
        if (dev_ptr) *dev_ptr = attr.devicePointer;
        return nullptr;
    }
    if (attr.type != hipMemoryTypeDevice && attr.type != hipMemoryTypeManaged && attr.type != hipMemoryTypeUnified)
        return "is not memory the GPU can address";
    hipDeviceptr_t base = nullptr;
    size_t size = 0;
    if (hipMemGetAddressRange(&base, &size, const_cast<void*>(p)) != hipSuccess) {
        (void)hipGetLastError();  // mapped ranges without one owner: extent unknown, nothing to compare
        return nullptr;
    }
    const char* lo = static_cast<const char*>(base);
    const char* q = static_cast<const char*>(p);
    if (q < lo || (size_t)(lo + size - q) < bytes) return "points at an allocation smaller than the forward needs";
    return nullptr;
}

// Tile shape of a routed projection for a chunk of Tn tokens.  Row tiles are cut to fit each expert
// (units of unit_rows rows, at most max_units per tile, equal heights), so a shape is judged by how
// many tiles the experts need with it and what a tile of it costs.  A launch lasts as many tiles as
// its busiest workgroup works through: cost = rounds * time per tile, rounds = expected tiles of
// all experts and column tiles over the n_cu workgroups, rounded up, with an expert's row count
// taken as normal around the balanced share Tn * k / E of Sec. 3.1 with a Poisson spread (the host
// never learns the real counts).  Time per tile, relative to the 128-row shape, is a measurement
// (MI355X, DeepSeek-V2-shaped share, both projections; profiles/routed_tile_times_dsv2_eg.txt):
// a tile costs roughly what its rows cost, plus what loading its 256 weight rows costs.
// automatic: a candidate of the choice below.  The two tall shapes are not: a tile of them costs what its
// rows cost (1.74 = 7/4, 1.79 ~ 8/4 of a 128-row tile), so they only ever win by rounding the tile
// count in their favour, and on every workload measured here the launch they win on paper ran slower
// (Zipf-skewed Qwen3-30B-shaped layer, down projection: 372 us against 295 us); MOE_EP_GEMM_VARIANT /
// MOE_EP_UP_VARIANT / MOE_EP_DOWN_VARIANT select them.
struct RoutedShape { int variant, unit_rows, max_units; double rel_long_k, rel_short_k; bool automatic; };
constexpr RoutedShape kRoutedShapes[] = {
    {1, 64, 2, 1.000, 1.000, true},     // 128 x 256, 2 x 2 wavefronts, three ring slots
    {11, 32, 5, 1.141, 1.116, true},    // 160 x 256, 1 x 4, three slots (measured with the 16 x 16 x 32 instruction)
    {13, 32, 7, 1.744, 1.709, false},   // 224 x 256, 1 x 4, two slots
    {14, 32, 8, 1.794, 1.764, false},   // 256 x 256, 1 x 4, two slots
};
const RoutedShape* routed_shape(int Tn, int k, int E, int El, int col_tiles, int K, int n_cu)
{
    const double mean = (double)Tn * k / E, sd = sqrt(mean > 1.0 ? mean : 1.0);
    const RoutedShape* best = &kRoutedShapes[0];
    double best_cost = 0.0;
    for (const RoutedShape& sh : kRoutedShapes) {
        if (!sh.automatic) continue;
        // E[tiles] = sum over j >= 0 of P(rows > j * tile_rows): a group of n rows gets
        // ceil(ceil(n / unit_rows) / max_units) tiles, i.e. one more tile each time n passes a
        // multiple of unit_rows * max_units; 1 for every multiple more than 6 sd below the mean,
        // 0 beyond 6 sd above it, the normal tail in between
        const double bm = (double)sh.unit_rows * sh.max_units;
        const double lo = (mean - 6.0 * sd) / bm;
        const long long j0 = lo > 0.0 ? (long long)lo : 0;
        double tiles = (double)j0;
        for (long long j = j0; j * bm < mean + 6.0 * sd; ++j) tiles += 0.5 * erfc((j * bm - mean) / (sd * 1.4142135623730951));
        const double cost = ceil(tiles * El * col_tiles / n_cu - 0.02) * (K >= 2048 ? sh.rel_long_k : sh.rel_short_k);
        if (&sh == &kRoutedShapes[0] || cost < best_cost) { best = &sh; best_cost = cost; }
    }
    return best;
}
int routed_variant(int Tn, int k, int E, int El, int col_tiles, int K, int n_cu)
{
    return routed_shape(Tn, k, E, El, col_tiles, K, n_cu)->variant;
}

hipEvent_t prof_event(moe_ep_ctx* ctx)
{
    if (ctx->prof_next >= ctx->prof_pool.size()) return nullptr;
    return ctx->prof_pool[ctx->prof_next++];
}

// Marks the start of a timed stage on stream s; returns the span index or -1.
int prof_begin(moe_ep_ctx* ctx, bool on, int stage, hipStream_t s)
{
    if (!on || !((ctx->prof_mask >> stage) & 1u)) return -1;
    hipEvent_t a = prof_event(ctx), b = prof_event(ctx);
    if (!a || !b) return -1;
    if (hipEventRecord(a, s) != hipSuccess) return -1;
    ctx->prof_spans.push_back({a, b, stage, ctx->prof_recorded});
    return (int)ctx->prof_spans.size() - 1;
}
void prof_end(moe_ep_ctx* ctx, int span, hipStream_t s)
{
    if (span >= 0) (void)hipEventRecord(ctx->prof_spans[span].b, s);
}

}  // namespace

extern "C" {

const char* moe_ep_version(void) { return "0.3"; }

int moe_ep_validate_config(const moe_ep_config* c, const char** why)
{
    set_why(why, "ok");
    if (!c) { set_why(why, "cfg is NULL"); return MOE_EP_EINVAL; }
    if (c->hidden < 64 || c->hidden % 64) { set_why(why, "hidden must be a positive multiple of 64"); return MOE_EP_EINVAL; }
    if (c->inter < 64 || c->inter % 64) { set_why(why, "inter must be a positive multiple of 64"); return MOE_EP_EINVAL; }
    // the GEMM's lanes address one expert's W_gate | W_up pair with 32-bit byte offsets
    if ((long long)c->hidden * c->inter >= (1ll << 30)) { set_why(why, "hidden * inter must be below 2^30"); return MOE_EP_EINVAL; }
    if (c->n_experts < 1 || c->n_experts > 512) { set_why(why, "n_experts must be in 1..512"); return MOE_EP_EINVAL; }
    if (c->n_local < 1 || c->local_begin < 0 || (long long)c->local_begin + c->n_local > c->n_experts) {
        set_why(why, "local experts [local_begin, local_begin+n_local) must lie inside 0..n_experts"); return MOE_EP_EINVAL; }
    if (c->n_shared < 0 || c->n_shared > 64) { set_why(why, "n_shared must be in 0..64"); return MOE_EP_EINVAL; }
    if (c->n_shared > 0 && (c->shared_inter < 64 || c->shared_inter % 64)) {
        set_why(why, "shared_inter must be a positive multiple of 64 when n_shared > 0"); return MOE_EP_EINVAL; }
    if (c->n_shared > 0 && (long long)c->hidden * c->shared_inter >= (1ll << 30)) {
        set_why(why, "hidden * shared_inter must be below 2^30"); return MOE_EP_EINVAL; }
    if (c->max_tokens < 1 || c->max_tokens > (1 << 20)) { set_why(why, "max_tokens must be in 1..1048576"); return MOE_EP_EINVAL; }
    if (c->max_top_k < 1 || c->max_top_k > 64 || c->max_top_k > c->n_experts) {
        set_why(why, "max_top_k must be in 1..min(n_experts, 64)"); return MOE_EP_EINVAL; }
    if (c->max_chunks < 1 || c->max_chunks > 64) { set_why(why, "max_chunks must be in 1..64"); return MOE_EP_EINVAL; }
    if (c->io_mode != MOE_EP_IO_DEVICE && c->io_mode != MOE_EP_IO_PINNED_HOST) { set_why(why, "unknown io_mode"); return MOE_EP_EINVAL; }
    if (c->device < 0) { set_why(why, "device must be >= 0"); return MOE_EP_EINVAL; }
    if ((long long)c->max_tokens * c->max_top_k > (1ll << 30)) { set_why(why, "max_tokens * max_top_k too large"); return MOE_EP_EINVAL; }
    return MOE_EP_OK;
}

int moe_ep_validate_forward(const moe_ep_config* c, const void* tokens, const float* gate_logits,
                            const void* routed_w, const void* shared_w, int32_t top_k,
                            int32_t r_chunks, int32_t order, int32_t n_tokens, const void* out,
                            const char** why)
{
    int rc = moe_ep_validate_config(c, why);
    if (rc != MOE_EP_OK) return rc;
    if (n_tokens < 0 || n_tokens > c->max_tokens) { set_why(why, "n_tokens must be in 0..max_tokens"); return MOE_EP_EINVAL; }
    if (top_k < 1 || top_k > c->max_top_k || top_k > c->n_experts) { set_why(why, "top_k must be in 1..min(n_experts, max_top_k)"); return MOE_EP_EINVAL; }
    if (r_chunks < 0 || r_chunks > c->max_chunks) { set_why(why, "r_chunks must be in 0..max_chunks (0 = from the timing model)"); return MOE_EP_EINVAL; }
    if (c->n_shared > 0 && order != MOE_EP_ORDER_SHARED_FIRST && order != MOE_EP_ORDER_INTERLEAVED) {
        set_why(why, "unknown order"); return MOE_EP_EINVAL; }
    if (!routed_w) { set_why(why, "routed_w is NULL"); return MOE_EP_EINVAL; }
    if (c->n_shared > 0 && !shared_w) { set_why(why, "shared_w is NULL but n_shared > 0"); return MOE_EP_EINVAL; }
    if (c->n_shared == 0 && shared_w) { set_why(why, "shared_w given but n_shared == 0"); return MOE_EP_EINVAL; }
    if (n_tokens > 0 && (!tokens || !gate_logits || !out)) { set_why(why, "tokens, gate_logits and out must not be NULL"); return MOE_EP_EINVAL; }
    return MOE_EP_OK;
}

size_t moe_ep_workspace_bytes(const moe_ep_config* cfg)
{
    if (moe_ep_validate_config(cfg, nullptr) != MOE_EP_OK) return 0;
    return ws_layout(*cfg).total;
}

int moe_ep_destroy(moe_ep_ctx* ctx)
{
    if (!ctx) return MOE_EP_OK;
    (void)hipSetDevice(ctx->cfg.device);
    (void)hipDeviceSynchronize();  // forwards still in flight on the caller's streams use the workspaces
    for (hipEvent_t e : ctx->ev_in) (void)hipEventDestroy(e);
    for (hipEvent_t e : ctx->ev_scores) (void)hipEventDestroy(e);
    for (hipEvent_t e : ctx->ev_comp) (void)hipEventDestroy(e);
    for (hipEvent_t e : ctx->ev_attn) (void)hipEventDestroy(e);
    for (hipEvent_t e : ctx->ev_shared) (void)hipEventDestroy(e);
    if (ctx->ev_ag_done) (void)hipEventDestroy(ctx->ev_ag_done);
    if (ctx->s_ag) (void)hipStreamDestroy(ctx->s_ag);
    for (hipEvent_t e : ctx->prof_pool) (void)hipEventDestroy(e);
    if (ctx->ev_start) (void)hipEventDestroy(ctx->ev_start);
    if (ctx->ev_done) (void)hipEventDestroy(ctx->ev_done);
    if (ctx->ev_comp_done) (void)hipEventDestroy(ctx->ev_comp_done);
    if (ctx->s_in) (void)hipStreamDestroy(ctx->s_in);
    if (ctx->s_out) (void)hipStreamDestroy(ctx->s_out);
    if (ctx->d_tokens) (void)hipFree(ctx->d_tokens);  // one slab holds every workspace
    for (auto* v : {&ctx->prepared_routed, &ctx->prepared_shared})
        for (const moe_ep_ctx::Prepared& p : *v) { (void)hipFree(p.up); (void)hipFree(p.down); }
    delete ctx;
    return MOE_EP_OK;
}

int moe_ep_create(const moe_ep_config* cfg, moe_ep_ctx** out_ctx)
{
    if (!out_ctx) return MOE_EP_EINVAL;
    if (moe_ep_validate_config(cfg, nullptr) != MOE_EP_OK) return MOE_EP_EINVAL;
    int n_dev = 0;
    if (hipGetDeviceCount(&n_dev) != hipSuccess || cfg->device >= n_dev) return MOE_EP_EHIP;
    if (hipSetDevice(cfg->device) != hipSuccess) return MOE_EP_EHIP;
    moe_ep_ctx* ctx = new (std::nothrow) moe_ep_ctx();
    if (!ctx) return MOE_EP_ENOMEM;
    ctx->cfg = *cfg;
    hipDeviceProp_t prop;
    if (hipGetDeviceProperties(&prop, cfg->device) != hipSuccess) { delete ctx; return MOE_EP_EHIP; }
    ctx->n_cu = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;
    read_knobs(ctx);
    if (grouped_gemm_init() != hipSuccess) { delete ctx; return MOE_EP_EHIP; }

    const WsLayout L = ws_layout(*cfg);
    char* slab = nullptr;
    if (hipMalloc(reinterpret_cast<void**>(&slab), L.total) != hipSuccess) { delete ctx; return MOE_EP_ENOMEM; }
    bind_workspaces(ctx, slab, L);  // L.tokens == 0: d_tokens is the slab base, freed in destroy
    ctx->last_variants.assign((size_t)cfg->max_chunks, {-1, -1});

    // the chunk events order GPU work against GPU work only, so they skip the system-scope cache
    // write-back a default event record implies (it stalled the other streams' kernels)
    const unsigned ev_flags = hipEventDisableTiming | hipEventDisableSystemFence;
    bool ok = true;
    if (cfg->io_mode == MOE_EP_IO_PINNED_HOST) {
        ok = ok && hipStreamCreateWithFlags(&ctx->s_in, hipStreamNonBlocking) == hipSuccess;
        ok = ok && hipStreamCreateWithFlags(&ctx->s_out, hipStreamNonBlocking) == hipSuccess;
    }
    ok = ok && hipEventCreateWithFlags(&ctx->ev_start, ev_flags) == hipSuccess;
    ok = ok && hipEventCreateWithFlags(&ctx->ev_done, hipEventDisableTiming) == hipSuccess;
    ok = ok && hipEventCreateWithFlags(&ctx->ev_comp_done, ev_flags) == hipSuccess;
    for (int i = 0; ok && i < cfg->max_chunks; ++i) {
        hipEvent_t a = nullptr, b = nullptr;
        ok = ok && hipEventCreateWithFlags(&a, ev_flags) == hipSuccess;
        if (a) ctx->ev_in.push_back(a);
        if (cfg->io_mode == MOE_EP_IO_PINNED_HOST) {
            hipEvent_t c = nullptr;
            ok = ok && hipEventCreateWithFlags(&c, ev_flags) == hipSuccess;
            if (c) ctx->ev_scores.push_back(c);
        }
        ok = ok && hipEventCreateWithFlags(&b, ev_flags) == hipSuccess;
        if (b) ctx->ev_comp.push_back(b);
    }
    if (!ok) { moe_ep_destroy(ctx); return MOE_EP_EHIP; }
    *out_ctx = ctx;
    return MOE_EP_OK;
}

const char* moe_ep_last_error(const moe_ep_ctx* ctx) { return ctx ? ctx->err : "context is NULL"; }

int32_t moe_ep_last_chunks(const moe_ep_ctx* ctx) { return (ctx && ctx->last_T >= 0) ? ctx->last_r : -1; }

int moe_ep_set_pipeline_model(moe_ep_ctx* ctx, const moe_ep_pipeline_model* m)
{
    if (!ctx) return MOE_EP_EINVAL;
    ctx->has_model = m != nullptr;
    if (m) ctx->model = *m;
    return MOE_EP_OK;
}

int moe_ep_set_profiling(moe_ep_ctx* ctx, int32_t depth)
{
    if (!ctx || depth < 0 || depth > 256) return MOE_EP_EINVAL;
    HIP_TRY(ctx, hipSetDevice(ctx->cfg.device));
    HIP_TRY(ctx, hipDeviceSynchronize());
    const size_t per_forward = 2 * ((size_t)ctx->cfg.max_chunks * 12 + 4);
    const size_t want = (size_t)depth * per_forward;
    while (ctx->prof_pool.size() < want) {
        hipEvent_t e = nullptr;
        HIP_TRY(ctx, hipEventCreate(&e));
        ctx->prof_pool.push_back(e);
    }
    ctx->prof_depth = depth;
    ctx->prof_recorded = 0;
    ctx->prof_next = 0;
    ctx->prof_spans.clear();
    return MOE_EP_OK;
}

int moe_ep_set_profiling_stages(moe_ep_ctx* ctx, uint32_t mask)
{
    if (!ctx) return MOE_EP_EINVAL;
    ctx->prof_mask = mask;
    return MOE_EP_OK;
}

int moe_ep_get_timeline(moe_ep_ctx* ctx, int32_t* stage, int32_t* forward, float* begin_ms, float* end_ms,
                        int32_t max_spans, int32_t* n_spans)
{
    if (!ctx || !n_spans || max_spans < 0) return MOE_EP_EINVAL;
    if (ctx->prof_recorded == 0) return fail(ctx, MOE_EP_ESTATE, "no profiled forward recorded");
    HIP_TRY(ctx, hipSetDevice(ctx->cfg.device));
    HIP_TRY(ctx, hipDeviceSynchronize());
    // time zero of a forward = the start of its whole-forward span (or of its first span)
    std::vector<hipEvent_t> zero(ctx->prof_recorded, nullptr);
    for (const ProfSpan& sp : ctx->prof_spans)
        if (sp.forward < ctx->prof_recorded && (sp.stage == ST_TOTAL || !zero[sp.forward])) zero[sp.forward] = sp.a;
    int n = 0;
    for (const ProfSpan& sp : ctx->prof_spans) {
        if (sp.forward >= ctx->prof_recorded || n >= max_spans) continue;
        float t0 = 0.f, t1 = 0.f;
        HIP_TRY(ctx, hipEventElapsedTime(&t0, zero[sp.forward], sp.a));
        HIP_TRY(ctx, hipEventElapsedTime(&t1, zero[sp.forward], sp.b));
        if (stage) stage[n] = sp.stage;
        if (forward) forward[n] = sp.forward;
        if (begin_ms) begin_ms[n] = t0;
        if (end_ms) end_ms[n] = t1;
        ++n;
    }
    *n_spans = n;
    return MOE_EP_OK;
}

int moe_ep_get_stage_ms(moe_ep_ctx* ctx, float* ms, int32_t n)
{
    if (!ctx || !ms || n < 1) return MOE_EP_EINVAL;
    if (ctx->prof_recorded == 0) return fail(ctx, MOE_EP_ESTATE, "no profiled forward recorded");
    HIP_TRY(ctx, hipSetDevice(ctx->cfg.device));
    HIP_TRY(ctx, hipDeviceSynchronize());
    double acc[ST_COUNT] = {0};
    for (const ProfSpan& sp : ctx->prof_spans) {
        float t = 0.f;
        HIP_TRY(ctx, hipEventElapsedTime(&t, sp.a, sp.b));
        acc[sp.stage] += t;
    }
    for (int i = 0; i < n && i < ST_COUNT; ++i) ms[i] = (float)(acc[i] / ctx->prof_recorded);
    // start a fresh window
    ctx->prof_recorded = 0;
    ctx->prof_next = 0;
    ctx->prof_spans.clear();
    return MOE_EP_OK;
}

}  // extern "C"

namespace {

// The tokens of a forward are cut into r_1 micro-batches of ceil(T / r_1) tokens and every
// micro-batch into r_2 chunks of ceil(micro-batch / r_2) tokens (Sec. 2.3); chunk c = i * r_2 + j.
// the weight side of the four projections' launches: [0] routed gate/up, [1] routed down, [2] shared
// gate/up, [3] shared down (what a launch and the tile-order copy both need)
void weight_args(const moe_ep_config& c, const void* routed_w, const void* shared_w, GemmArgs g[4])
{
    const int M = c.hidden, H = c.inter, El = c.n_local, Ns = c.n_shared, Hs = c.shared_inter;
    const uint16_t* rw = static_cast<const uint16_t*>(routed_w);
    const uint16_t* sw = static_cast<const uint16_t*>(shared_w);
    for (int i = 0; i < 4; ++i) g[i] = GemmArgs{};
    g[0].W = rw; g[0].G = El; g[0].K = M; g[0].N = H; g[0].ldw = M;
    g[0].w_group_stride = (long long)3 * H * M; g[0].w_up_offset = (long long)H * M;
    g[0].kseg_len = M; g[0].w_kseg_stride = 0;
    g[1].W = rw ? rw + (size_t)2 * H * M : nullptr; g[1].G = El; g[1].K = H; g[1].N = M; g[1].ldw = H;
    g[1].w_group_stride = (long long)3 * H * M; g[1].w_up_offset = 0; g[1].kseg_len = H; g[1].w_kseg_stride = 0;
    g[2].W = sw; g[2].G = Ns; g[2].K = M; g[2].N = Hs; g[2].ldw = M;
    g[2].w_group_stride = (long long)3 * Hs * M; g[2].w_up_offset = (long long)Hs * M;
    g[2].kseg_len = M; g[2].w_kseg_stride = 0;
    g[3].W = sw ? sw + (size_t)2 * Hs * M : nullptr; g[3].G = 1; g[3].K = Ns * Hs; g[3].N = M; g[3].ldw = Hs;
    g[3].w_group_stride = 0; g[3].w_up_offset = 0; g[3].kseg_len = Hs > 0 ? Hs : 1; g[3].w_kseg_stride = (long long)3 * Hs * M;
}

const moe_ep_ctx::Prepared* find_prepared(const std::vector<moe_ep_ctx::Prepared>& v, const void* key)
{
    for (const moe_ep_ctx::Prepared& p : v) if (p.key == key) return &p;
    return nullptr;
}

void chunk_range(int T, int r_1, int r_2, int c, int* t0, int* Tn)
{
    const int Tm = (T + r_1 - 1) / r_1, i = c / r_2, j = c % r_2;
    const int mb0 = i * Tm, mb1 = mb0 + Tm < T ? mb0 + Tm : T;
    const int Tc = (Tm + r_2 - 1) / r_2;
    int a = mb0 + j * Tc, b = a + Tc;
    if (b > mb1) b = mb1;
    if (a > b) a = b;
    if (a < 0 || mb0 >= T) { a = T; b = T; }
    *t0 = a;
    *Tn = b - a;
}

// dep = false: moe_ep_forward (r_1 = 1, `order` is a moe_ep_order).  dep = true: moe_ep_forward_dep
// (`order` is a moe_ep_dep_order, attention stand-ins of attn_us microseconds per micro-batch).
int forward_impl(moe_ep_ctx* ctx, const void* tokens, const float* gate_logits, const void* routed_w,
                 const void* shared_w, int32_t top_k, int32_t r_1, int32_t r_2, int32_t order, bool dep,
                 double attn_us, int32_t n_tokens, void* out, void* stream)
{
    const moe_ep_config& c = ctx->cfg;
    const int T = n_tokens, k = top_k, r = r_1 * r_2;
    const int M = c.hidden, H = c.inter, E = c.n_experts, El = c.n_local, e0 = c.local_begin;
    const int Ns = c.n_shared, Hs = c.shared_inter;
    if (T == 0) {
        ctx->last_T = T; ctx->last_k = k; ctx->last_r = r; ctx->last_r1 = r_1;
        return MOE_EP_OK;
    }
    HIP_TRY(ctx, hipSetDevice(c.device));

    hipStream_t user = static_cast<hipStream_t>(stream);
    const bool pinned = c.io_mode == MOE_EP_IO_PINNED_HOST;
    hipStream_t s_in = pinned ? ctx->s_in : user;
    // compute always runs on the caller's stream; only the two link directions get streams of their own
    hipStream_t s_comp = user;
    const int n_cu = ctx->n_cu;
    hipStream_t s_out = pinned ? ctx->s_out : user;
    const bool prof = ctx->prof_depth > 0 && ctx->prof_recorded < ctx->prof_depth;
    const bool fused_out = pinned && ctx->fused_out && !dep;   // the aggregation's stores are the outbound transfer

    const uint16_t* tok_dev = static_cast<const uint16_t*>(pinned ? ctx->d_tokens : tokens);
    const float* log_dev = pinned ? ctx->d_logits : gate_logits;
    uint16_t* out_dev = static_cast<uint16_t*>(pinned ? ctx->d_out : out);
    const uint16_t* rw = static_cast<const uint16_t*>(routed_w);
    const uint16_t* sw = static_cast<const uint16_t*>(shared_w);

    // What every pointer argument points at is checked before anything is enqueued.  Pinned-host
    // mode: the copy kernels address the host buffers directly, so they must be pinned
    // (page-locked, device-visible) memory; that check is never skipped, it yields the device addresses.
    const char* h_tokens = nullptr; const char* h_logits = nullptr; char* h_out = nullptr;
    {
        struct Span { const void* p; size_t bytes; bool host; const char* name; };
        Span sp[5] = {
            {tokens, (size_t)T * M * 2, pinned, "tokens"},
            {gate_logits, (size_t)T * E * 4, pinned, "gate_logits"},
            {out, (size_t)T * M * 2, pinned, "out"},
            {routed_w, (size_t)El * 3 * H * M * 2, false, "routed_w"},
            {shared_w, (size_t)Ns * 3 * Hs * M * 2, false, "shared_w"},
        };
        for (const Span& x : sp) {
            if (!x.p || !(x.host || ctx->check_spans)) continue;
            const void* dev = nullptr;
            if (const char* bad = check_span(x.p, x.bytes, x.host, &dev)) {
                snprintf(ctx->err, sizeof ctx->err, "%s %s", x.name, bad);
                return MOE_EP_EINVAL;
            }
            if (&x == &sp[0]) h_tokens = static_cast<const char*>(dev);
            if (&x == &sp[1]) h_logits = static_cast<const char*>(dev);
            if (&x == &sp[2]) h_out = static_cast<char*>(const_cast<void*>(dev));
        }
    }
    ctx->last_T = T; ctx->last_k = k; ctx->last_r = r; ctx->last_r1 = r_1;
    auto link_copy = [&](void* dst, const void* src, size_t bytes, int grid, hipStream_t st) -> hipError_t {
        if (st == s_in ? ctx->memcpy_in : ctx->memcpy_out)
            return bytes ? hipMemcpyAsync(dst, src, bytes, hipMemcpyDefault, st) : hipSuccess;
        return launch_copy(dst, src, bytes, grid, st, ctx->link_threads, ctx->link_unroll);
    };
    const int link_grid = ctx->link_grid;
    const int span_total = prof_begin(ctx, prof, ST_TOTAL, user);
    hipStream_t s_ag = dep ? ctx->s_ag : user;  // attention stand-ins and, in dep mode, the shared experts
    if (pinned || dep) HIP_TRY(ctx, hipEventRecord(ctx->ev_start, user));
    if (pinned) {
        HIP_TRY(ctx, hipStreamWaitEvent(s_in, ctx->ev_start, 0));
        HIP_TRY(ctx, hipStreamWaitEvent(s_out, ctx->ev_start, 0));
    }
    if (dep) HIP_TRY(ctx, hipStreamWaitEvent(s_ag, ctx->ev_start, 0));
    const int bw_grid = n_cu * 8;  // bandwidth kernels: 8 workgroups of 4 wavefronts per CU

    GemmArgs w_args[4];   // the weight side of the four projections
    weight_args(c, routed_w, shared_w, w_args);
    auto shared_up_w = [&](GemmArgs& g) { g = w_args[2]; };
    auto shared_down_w = [&](GemmArgs& g) { g = w_args[3]; };
    auto routed_up_w = [&](GemmArgs& g) { g = w_args[0]; };
    auto routed_down_w = [&](GemmArgs& g) { g = w_args[1]; };
    // weights the caller has had laid out in tile order
    const moe_ep_ctx::Prepared* prep_r = find_prepared(ctx->prepared_routed, routed_w);
    const moe_ep_ctx::Prepared* prep_s = Ns > 0 ? find_prepared(ctx->prepared_shared, shared_w) : nullptr;
    ctx->last_prepared_routed = prep_r != nullptr;
    ctx->last_prepared_shared = prep_s != nullptr;

    // shared experts of token range [t0, t0+Tn) -> output rows [t0, t0+Tn); the aggregation adds to them
    auto run_shared = [&](int t0, int Tn, hipStream_t st) -> int {
        if (Tn <= 0) return MOE_EP_OK;
        GemmArgs g1{};
        shared_up_w(g1);
        g1.Wp = prep_s ? prep_s->up : nullptr;
        g1.A = tok_dev + (size_t)t0 * M; g1.C = ctx->hs + (size_t)t0 * Ns * Hs;
        g1.offset = nullptr; g1.dense_rows = Tn;
        g1.lda = M; g1.ldc = Ns * Hs; g1.c_group_col_stride = Hs;
        int sp = prof_begin(ctx, prof, ST_SGEMM1, st);
        HIP_TRY(ctx, launch_grouped_gemm(g1, true, ctx->shared_variant, n_cu, 0, st));
        prof_end(ctx, sp, st);
        GemmArgs g2{};
        shared_down_w(g2);
        g2.Wp = prep_s ? prep_s->down : nullptr;
        g2.A = ctx->hs + (size_t)t0 * Ns * Hs; g2.C = out_dev + (size_t)t0 * M;
        g2.offset = nullptr; g2.dense_rows = Tn;
        g2.lda = Ns * Hs; g2.ldc = M; g2.c_group_col_stride = 0;
        sp = prof_begin(ctx, prof, ST_SGEMM2, st);
        HIP_TRY(ctx, launch_grouped_gemm(g2, false, ctx->shared_variant, n_cu, 0, st));
        prof_end(ctx, sp, st);
        return MOE_EP_OK;
    };
    auto micro_batch_range = [&](int i, int* t0, int* Tn) {
        int a, n, b, m;
        chunk_range(T, r_1, r_2, i * r_2, &a, &n);
        chunk_range(T, r_1, r_2, i * r_2 + r_2 - 1, &b, &m);
        *t0 = a;
        *Tn = b + m - a;
    };

    // inbound transfer of chunk cidx on the inbound link stream
    auto enqueue_inbound = [&](int cidx) -> int {
        int t0, Tn;
        chunk_range(T, r_1, r_2, cidx, &t0, &Tn);
        // no timing events around the runtime's own copies (MOE_EP_LINK_MEMCPY): the one profiled run
        // that had them ended in a crash inside the profiler's exit handler; the copy kernels are timed
        const int sp_in = prof_begin(ctx, prof && Tn > 0 && !ctx->memcpy_in, ST_COPY_IN, s_in);
        if (Tn > 0)
            HIP_TRY(ctx, link_copy(ctx->d_logits + (size_t)t0 * E, h_logits + (size_t)t0 * E * 4,
                                     (size_t)Tn * E * 4, link_grid, s_in));
        HIP_TRY(ctx, hipEventRecord(ctx->ev_scores[cidx], s_in));
        if (Tn > 0)
            HIP_TRY(ctx, link_copy(static_cast<char*>(ctx->d_tokens) + (size_t)t0 * M * 2,
                                     h_tokens + (size_t)t0 * M * 2, (size_t)Tn * M * 2, link_grid, s_in));
        prof_end(ctx, sp_in, s_in);
        HIP_TRY(ctx, hipEventRecord(ctx->ev_in[cidx], s_in));
        return MOE_EP_OK;
    };
    if (dep) {
        // Attention-group side (Sec. 2.3, Fig. as): per micro-batch an attention stand-in, then its
        // tokens may leave for the experts (rule 6), and its shared experts run on the same stream
        // either right behind its attention (ASAS) or behind the last attention (AASS).  Every
        // event is recorded, in host order, before anything is told to wait for it.
        auto shared_of_micro_batch = [&](int i) -> int {
            if (Ns > 0) {
                int t0, Tn;
                micro_batch_range(i, &t0, &Tn);
                // in the stand-in the token rows reach the GPU through the inbound link
                if (pinned) HIP_TRY(ctx, hipStreamWaitEvent(s_ag, ctx->ev_in[i * r_2 + r_2 - 1], 0));
                const int rc = run_shared(t0, Tn, s_ag);
                if (rc != MOE_EP_OK) return rc;
            }
            HIP_TRY(ctx, hipEventRecord(ctx->ev_shared[i], s_ag));
            return MOE_EP_OK;
        };
        for (int i = 0; i < r_1; ++i) {
            const int sp_at = prof_begin(ctx, prof && attn_us > 0.0, ST_ATTN, s_ag);
            HIP_TRY(ctx, launch_busy(attn_us, s_ag));
            prof_end(ctx, sp_at, s_ag);
            HIP_TRY(ctx, hipEventRecord(ctx->ev_attn[i], s_ag));
            if (pinned) {
                HIP_TRY(ctx, hipStreamWaitEvent(s_in, ctx->ev_attn[i], 0));
                for (int j = 0; j < r_2; ++j) {
                    const int rc = enqueue_inbound(i * r_2 + j);
                    if (rc != MOE_EP_OK) return rc;
                }
            }
            if (order == MOE_EP_DEP_ASAS) {
                const int rc = shared_of_micro_batch(i);
                if (rc != MOE_EP_OK) return rc;
            }
        }
        if (order == MOE_EP_DEP_AASS)
            for (int i = 0; i < r_1; ++i) {
                const int rc = shared_of_micro_batch(i);
                if (rc != MOE_EP_OK) return rc;
            }
    } else if (pinned) {
        // all chunks are queued at once on their own stream
        for (int cidx = 0; cidx < r; ++cidx) {
            const int rc = enqueue_inbound(cidx);
            if (rc != MOE_EP_OK) return rc;
        }
    }
    if (!dep && Ns > 0 && order == MOE_EP_ORDER_SHARED_FIRST) {
        if (pinned) HIP_TRY(ctx, hipStreamWaitEvent(s_comp, ctx->ev_in[r - 1], 0));
        int rc = run_shared(0, T, s_comp);
        if (rc != MOE_EP_OK) return rc;
    }

    for (int cidx = 0; cidx < r; ++cidx) {
        int t0, Tn;
        chunk_range(T, r_1, r_2, cidx, &t0, &Tn);
        int32_t* count = ctx->count + (size_t)cidx * El;
        int32_t* offset = ctx->offset + (size_t)cidx * (El + 1);
        // gate and partition need the chunk's gate scores only, which travel first
        if (pinned) HIP_TRY(ctx, hipStreamWaitEvent(s_comp, ctx->ev_scores[cidx], 0));
        else if (dep && cidx % r_2 == 0) HIP_TRY(ctx, hipStreamWaitEvent(s_comp, ctx->ev_attn[cidx / r_2], 0));
        // tile shapes of the two routed projections: N = H in tiles of 128 activation columns, N = M in
        // tiles of 256 columns
        // a shape the library picks itself is taken in its 16 x 16 x 32 form, one named through a knob as named
        const auto picked = [&](int v) { return ctx->mfma16 ? grouped_gemm_variant_mfma16(v) : v; };
        int v_up = ctx->gemm_variant >= 0 ? ctx->gemm_variant : picked(routed_variant(Tn, k, E, El, (H + 127) / 128, M, n_cu));
        int v_down = ctx->gemm_variant >= 0 ? ctx->gemm_variant : picked(routed_variant(Tn, k, E, El, (M + 255) / 256, H, n_cu));
        if (ctx->up_variant >= 0) v_up = ctx->up_variant;
        if (ctx->down_variant >= 0) v_down = ctx->down_variant;
        if (cidx < (int)ctx->last_variants.size()) ctx->last_variants[cidx] = {v_up, v_down};
        int32_t* idx = ctx->idx + (size_t)t0 * k;
        float* w = ctx->w + (size_t)t0 * k;
        int32_t* pos = ctx->pos + (size_t)t0 * k;
        int32_t* perm = ctx->perm + (size_t)t0 * k;

        int sp = prof_begin(ctx, prof, ST_ROUTER, s_comp);
        HIP_TRY(ctx, launch_router(log_dev + (size_t)t0 * E, Tn, E, k, e0, El, idx, w, ctx->blk_mask, s_comp));
        prof_end(ctx, sp, s_comp);

        // the fused gather addresses a chunk's token rows with 32-bit byte offsets
        const bool fused = ctx->fused_gather && (unsigned long long)Tn * M * 2 < (1ull << 32);
        sp = prof_begin(ctx, prof, ST_PARTITION, s_comp);
        HIP_TRY(ctx, launch_dispatch(idx, ctx->blk_mask, Tn, k, e0, El, count, offset, pos, perm, s_comp));
        if (Tn > 0 && !fused) {   // the grouped copy reads the token rows
            if (pinned) HIP_TRY(ctx, hipStreamWaitEvent(s_comp, ctx->ev_in[cidx], 0));
            HIP_TRY(ctx, launch_gather_rows(tok_dev + (size_t)t0 * M, perm, offset + El, k, M, ctx->xp, bw_grid, s_comp));
        }
        prof_end(ctx, sp, s_comp);
        if (pinned) HIP_TRY(ctx, hipStreamWaitEvent(s_comp, ctx->ev_in[cidx], 0));   // the token rows
        if (Tn == 0) {
            if (pinned && !fused_out) HIP_TRY(ctx, hipEventRecord(ctx->ev_comp[cidx], s_comp));
            continue;
        }

        const long long a_max = (long long)Tn * k;  // the most rows the routing can keep

        GemmArgs g1{};
        routed_up_w(g1);
        g1.Wp = prep_r ? prep_r->up : nullptr;
        g1.A = ctx->xp; g1.C = ctx->h; g1.offset = offset;
        g1.dense_rows = 0; g1.lda = M; g1.ldc = H; g1.c_group_col_stride = 0;
        g1.max_units = ctx->up_units;
        if (fused) {  // the projection reads the token rows through the row -> assignment map
            g1.A = tok_dev + (size_t)t0 * M; g1.a_row_map = perm; g1.a_row_div = k; g1.a_src_rows = Tn;
        }
        sp = prof_begin(ctx, prof, ST_GEMM1, s_comp);
        HIP_TRY(ctx, launch_grouped_gemm(g1, true, v_up, n_cu, a_max, s_comp));
        prof_end(ctx, sp, s_comp);

        GemmArgs g2{};
        routed_down_w(g2);
        g2.Wp = prep_r ? prep_r->down : nullptr;
        g2.A = ctx->h; g2.C = ctx->y; g2.offset = offset;
        g2.dense_rows = 0; g2.lda = H; g2.ldc = M; g2.c_group_col_stride = 0;
        g2.max_units = ctx->down_units;
        g2.epi = ctx->y_mode; g2.row_weight = w; g2.row_assignment = perm;
        sp = prof_begin(ctx, prof, ST_GEMM2, s_comp);
        HIP_TRY(ctx, launch_grouped_gemm(g2, false, v_down, n_cu, a_max, s_comp));
        prof_end(ctx, sp, s_comp);

        if (!dep && Ns > 0 && order == MOE_EP_ORDER_INTERLEAVED) {
            int rc = run_shared(t0, Tn, s_comp);
            if (rc != MOE_EP_OK) return rc;
        }
        // the aggregation adds to what the micro-batch's shared experts have written (attention-group stream)
        if (dep && Ns > 0) HIP_TRY(ctx, hipStreamWaitEvent(s_comp, ctx->ev_shared[cidx / r_2], 0));

        // fused outbound transfer: the aggregation reads the shared experts' rows from the device
        // staging buffer and writes every row of the chunk into the caller's pinned buffer
        uint16_t* out_rows = out_dev + (size_t)t0 * M;
        sp = prof_begin(ctx, prof, ST_COMBINE, s_comp);
        HIP_TRY(ctx, launch_combine(ctx->y, pos, w, Tn, k, M, Ns > 0, ctx->y_mode, out_rows,
                                    fused_out ? reinterpret_cast<uint16_t*>(h_out) + (size_t)t0 * M : out_rows, bw_grid, s_comp));
        prof_end(ctx, sp, s_comp);

        if (pinned && !fused_out) {
            HIP_TRY(ctx, hipEventRecord(ctx->ev_comp[cidx], s_comp));
            HIP_TRY(ctx, hipStreamWaitEvent(s_out, ctx->ev_comp[cidx], 0));
            const int sp_out = prof_begin(ctx, prof && !ctx->memcpy_out, ST_COPY_OUT, s_out);
            HIP_TRY(ctx, link_copy(h_out + (size_t)t0 * M * 2,
                                   reinterpret_cast<const char*>(out_dev) + (size_t)t0 * M * 2,
                                   (size_t)Tn * M * 2, link_grid, s_out));
            prof_end(ctx, sp_out, s_out);
        }
    }
    if (pinned && !fused_out) {
        HIP_TRY(ctx, hipEventRecord(ctx->ev_comp_done, s_comp));
        HIP_TRY(ctx, hipStreamWaitEvent(s_out, ctx->ev_comp_done, 0));
        HIP_TRY(ctx, hipEventRecord(ctx->ev_done, s_out));
        HIP_TRY(ctx, hipStreamWaitEvent(user, ctx->ev_done, 0));
    }
    if (dep) {
        HIP_TRY(ctx, hipEventRecord(ctx->ev_ag_done, s_ag));
        HIP_TRY(ctx, hipStreamWaitEvent(user, ctx->ev_ag_done, 0));
    }
    prof_end(ctx, span_total, user);
    if (prof) ctx->prof_recorded++;
    return MOE_EP_OK;
}

}  // namespace

extern "C" {

int moe_ep_chunk_range(int32_t n_tokens, int32_t r_1, int32_t r_2, int32_t chunk, int32_t* first, int32_t* count)
{
    if (n_tokens < 0 || r_1 < 1 || r_2 < 1 || chunk < 0 || (long long)chunk >= (long long)r_1 * r_2 || !first || !count)
        return MOE_EP_EINVAL;
    int t0 = 0, Tn = 0;
    if (n_tokens > 0) chunk_range(n_tokens, r_1, r_2, chunk, &t0, &Tn);
    *first = t0;
    *count = Tn;
    return MOE_EP_OK;
}

int32_t moe_ep_routed_tile_rows(const moe_ep_config* cfg, int32_t n_tokens, int32_t top_k, int32_t down, int32_t n_cu)
{
    if (moe_ep_validate_config(cfg, nullptr) != MOE_EP_OK || n_tokens < 0 || top_k < 1 || n_cu < 1) return MOE_EP_EINVAL;
    const int col_tiles = down ? (cfg->hidden + 255) / 256 : (cfg->inter + 127) / 128;
    const RoutedShape* sh = routed_shape(n_tokens, top_k, cfg->n_experts, cfg->n_local, col_tiles,
                                         down ? cfg->inter : cfg->hidden, n_cu);
    return sh->unit_rows * sh->max_units;
}

int moe_ep_last_tile_shape(const moe_ep_ctx* ctx, int32_t chunk, int32_t stage, int32_t* rows, int32_t* cols,
                           int32_t* k_step, int32_t* ring_slots, int32_t* waves_m, int32_t* waves_n,
                           int32_t* tile_order, int32_t* mfma_rows)
{
    if (!ctx || stage < ST_GEMM1 || stage > ST_SGEMM2) return MOE_EP_EINVAL;
    if (ctx->last_T < 0) return MOE_EP_ESTATE;
    const bool shared = stage == ST_SGEMM1 || stage == ST_SGEMM2, up = stage == ST_GEMM1 || stage == ST_SGEMM1;
    if (shared && ctx->cfg.n_shared == 0) return MOE_EP_ESTATE;
    if (!shared && (chunk < 0 || chunk >= ctx->last_r || chunk >= (int)ctx->last_variants.size())) return MOE_EP_EINVAL;
    const moe_ep_config& c = ctx->cfg;
    const int variant = shared ? ctx->shared_variant : (up ? ctx->last_variants[chunk].up : ctx->last_variants[chunk].down);
    const int K = shared ? (up ? c.hidden : c.n_shared * c.shared_inter) : (up ? c.hidden : c.inter);
    int v[8];
    if (!grouped_gemm_variant_shape(variant, K, !shared, shared ? 1 : c.n_local, v)) return MOE_EP_ESTATE;
    if (mfma_rows) *mfma_rows = v[7];
    if (tile_order) *tile_order = v[6] && (shared ? ctx->last_prepared_shared : ctx->last_prepared_routed);
    if (rows) *rows = v[0];
    if (cols) *cols = v[1];
    if (k_step) *k_step = v[2];
    if (ring_slots) *ring_slots = v[3];
    if (waves_m) *waves_m = v[4];
    if (waves_n) *waves_n = v[5];
    return MOE_EP_OK;
}

int moe_ep_forward(moe_ep_ctx* ctx, const void* tokens, const float* gate_logits,
                   const void* routed_w, const void* shared_w, int32_t top_k, int32_t r_chunks,
                   int32_t order, int32_t n_tokens, void* out, void* stream)
{
    if (!ctx) return MOE_EP_EINVAL;
    const char* why = nullptr;
    if (moe_ep_validate_forward(&ctx->cfg, tokens, gate_logits, routed_w, shared_w, top_k, r_chunks,
                                order, n_tokens, out, &why) != MOE_EP_OK)
        return fail(ctx, MOE_EP_EINVAL, why);
    ctx->err[0] = 0;
    if (r_chunks == 0) {
        if (!ctx->has_model) return fail(ctx, MOE_EP_ESTATE, "r_chunks == 0 needs moe_ep_set_pipeline_model first");
        r_chunks = moe_ep_choose_chunks(&ctx->model, n_tokens, ctx->cfg.max_chunks);
    }
    return forward_impl(ctx, tokens, gate_logits, routed_w, shared_w, top_k, 1, r_chunks, order, false, 0.0,
                        n_tokens, out, stream);
}

size_t moe_ep_prepared_weight_bytes(const moe_ep_config* cfg, int32_t routed, int32_t shared)
{
    if (moe_ep_validate_config(cfg, nullptr) != MOE_EP_OK) return 0;
    if (cfg->hidden % kPackK || cfg->inter % kPackK || (cfg->n_shared > 0 && cfg->shared_inter % kPackK)) return 0;
    GemmArgs g[4];
    weight_args(*cfg, nullptr, nullptr, g);
    size_t bytes = 0;
    if (routed) bytes += align256(packed_weight_elems(g[0], true) * 2) + align256(packed_weight_elems(g[1], false) * 2);
    if (shared && cfg->n_shared > 0)
        bytes += align256(packed_weight_elems(g[2], true) * 2) + align256(packed_weight_elems(g[3], false) * 2);
    return bytes;
}

int moe_ep_prepare_weights(moe_ep_ctx* ctx, const void* routed_w, const void* shared_w, void* stream)
{
    if (!ctx) return MOE_EP_EINVAL;
    const moe_ep_config& c = ctx->cfg;
    if (!routed_w && !shared_w) return fail(ctx, MOE_EP_EINVAL, "moe_ep_prepare_weights: no weights given");
    if (shared_w && c.n_shared == 0) return fail(ctx, MOE_EP_EINVAL, "moe_ep_prepare_weights: shared_w without shared experts");
    if (c.hidden % kPackK || c.inter % kPackK || (c.n_shared > 0 && c.shared_inter % kPackK))
        return fail(ctx, MOE_EP_EINVAL, "moe_ep_prepare_weights: hidden, inter and shared_inter must be multiples of 64");
    HIP_TRY(ctx, hipSetDevice(c.device));
    if (ctx->check_spans) {
        const size_t rb = (size_t)c.n_local * 3 * c.inter * c.hidden * 2, sb = (size_t)c.n_shared * 3 * c.shared_inter * c.hidden * 2;
        const void* dev = nullptr;
        if (routed_w) if (const char* bad = check_span(routed_w, rb, false, &dev)) {
            snprintf(ctx->err, sizeof ctx->err, "routed_w %s", bad);
            return MOE_EP_EINVAL;
        }
        if (shared_w) if (const char* bad = check_span(shared_w, sb, false, &dev)) {
            snprintf(ctx->err, sizeof ctx->err, "shared_w %s", bad);
            return MOE_EP_EINVAL;
        }
    }
    GemmArgs g[4];
    weight_args(c, routed_w, shared_w, g);
    hipStream_t s = static_cast<hipStream_t>(stream);
    auto prepare = [&](std::vector<moe_ep_ctx::Prepared>& table, const void* key, const GemmArgs& up, const GemmArgs& down) -> int {
        moe_ep_ctx::Prepared* p = nullptr;
        for (moe_ep_ctx::Prepared& q : table) if (q.key == key) p = &q;
        if (!p) {
            moe_ep_ctx::Prepared n{key, nullptr, nullptr};
            if (hipMalloc(reinterpret_cast<void**>(&n.up), packed_weight_elems(up, true) * 2) != hipSuccess ||
                hipMalloc(reinterpret_cast<void**>(&n.down), packed_weight_elems(down, false) * 2) != hipSuccess) {
                (void)hipGetLastError();
                if (n.up) (void)hipFree(n.up);
                return fail(ctx, MOE_EP_ENOMEM, "moe_ep_prepare_weights: no device memory for the copy");
            }
            table.push_back(n);
            p = &table.back();
        }
        HIP_TRY(ctx, launch_pack_weights(up, true, p->up, ctx->n_cu * 8, s));
        HIP_TRY(ctx, launch_pack_weights(down, false, p->down, ctx->n_cu * 8, s));
        return MOE_EP_OK;
    };
    if (routed_w) { const int rc = prepare(ctx->prepared_routed, routed_w, g[0], g[1]); if (rc != MOE_EP_OK) return rc; }
    if (shared_w) { const int rc = prepare(ctx->prepared_shared, shared_w, g[2], g[3]); if (rc != MOE_EP_OK) return rc; }
    return MOE_EP_OK;
}

int moe_ep_forget_weights(moe_ep_ctx* ctx, const void* routed_w, const void* shared_w)
{
    if (!ctx) return MOE_EP_EINVAL;
    HIP_TRY(ctx, hipSetDevice(ctx->cfg.device));
    HIP_TRY(ctx, hipDeviceSynchronize());   // no kernel may still be reading a copy
    const bool all = !routed_w && !shared_w;
    auto drop = [&](std::vector<moe_ep_ctx::Prepared>& table, const void* key) {
        for (size_t i = 0; i < table.size();) {
            if (all || table[i].key == key) {
                (void)hipFree(table[i].up); (void)hipFree(table[i].down);
                table.erase(table.begin() + i);
            } else ++i;
        }
    };
    if (all || routed_w) drop(ctx->prepared_routed, routed_w);
    if (all || shared_w) drop(ctx->prepared_shared, shared_w);
    return MOE_EP_OK;
}

int moe_ep_forward_dep(moe_ep_ctx* ctx, const void* tokens, const float* gate_logits,
                       const void* routed_w, const void* shared_w, int32_t top_k, int32_t r_1, int32_t r_2,
                       int32_t dep_order, double attn_us, int32_t n_tokens, void* out, void* stream)
{
    if (!ctx) return MOE_EP_EINVAL;
    const char* why = nullptr;
    if (r_1 < 1 || r_2 < 1 || (long long)r_1 * r_2 > ctx->cfg.max_chunks)
        return fail(ctx, MOE_EP_EINVAL, "r_1 and r_2 must be at least 1 and r_1 * r_2 at most max_chunks");
    if (dep_order != MOE_EP_DEP_ASAS && dep_order != MOE_EP_DEP_AASS) return fail(ctx, MOE_EP_EINVAL, "dep_order must be MOE_EP_DEP_ASAS or MOE_EP_DEP_AASS");
    if (!(attn_us >= 0.0) || attn_us > 1e6) return fail(ctx, MOE_EP_EINVAL, "attn_us must be in 0..1e6");
    if (moe_ep_validate_forward(&ctx->cfg, tokens, gate_logits, routed_w, shared_w, top_k, r_1 * r_2,
                                MOE_EP_ORDER_INTERLEAVED, n_tokens, out, &why) != MOE_EP_OK)
        return fail(ctx, MOE_EP_EINVAL, why);
    ctx->err[0] = 0;
    HIP_TRY(ctx, hipSetDevice(ctx->cfg.device));
    if (!ctx->s_ag) {  // first call: the attention-group stream and its events
        const unsigned ev_flags = hipEventDisableTiming;
        HIP_TRY(ctx, hipStreamCreateWithFlags(&ctx->s_ag, hipStreamNonBlocking));
        HIP_TRY(ctx, hipEventCreateWithFlags(&ctx->ev_ag_done, ev_flags));
        for (int i = 0; i < ctx->cfg.max_chunks; ++i) {
            hipEvent_t a = nullptr, b = nullptr;
            HIP_TRY(ctx, hipEventCreateWithFlags(&a, ev_flags));
            ctx->ev_attn.push_back(a);
            HIP_TRY(ctx, hipEventCreateWithFlags(&b, ev_flags));
            ctx->ev_shared.push_back(b);
        }
    }
    return forward_impl(ctx, tokens, gate_logits, routed_w, shared_w, top_k, r_1, r_2, dep_order, true, attn_us,
                        n_tokens, out, stream);
}

int moe_ep_get_routing(moe_ep_ctx* ctx, int32_t chunk, int32_t* idx, float* w, int32_t* pos,
                       int32_t* count, int32_t* offset, int32_t* perm)
{
    if (!ctx) return MOE_EP_EINVAL;
    if (ctx->last_T < 0) return fail(ctx, MOE_EP_ESTATE, "no forward has run yet");
    if (chunk < 0 || chunk >= ctx->last_r) return fail(ctx, MOE_EP_EINVAL, "chunk out of range");
    const moe_ep_config& c = ctx->cfg;
    const int T = ctx->last_T, k = ctx->last_k, El = c.n_local;
    int t0 = 0, Tn = 0;
    if (T > 0) chunk_range(T, ctx->last_r1, ctx->last_r / ctx->last_r1, chunk, &t0, &Tn);
    HIP_TRY(ctx, hipSetDevice(c.device));
    HIP_TRY(ctx, hipDeviceSynchronize());
    if (T == 0) {
        if (count) memset(count, 0, sizeof(int32_t) * El);
        if (offset) memset(offset, 0, sizeof(int32_t) * (El + 1));
        return MOE_EP_OK;
    }
    std::vector<int32_t> off(El + 1);
    HIP_TRY(ctx, hipMemcpy(off.data(), ctx->offset + (size_t)chunk * (El + 1), sizeof(int32_t) * (El + 1), hipMemcpyDeviceToHost));
    if (offset) memcpy(offset, off.data(), sizeof(int32_t) * (El + 1));
    if (count) HIP_TRY(ctx, hipMemcpy(count, ctx->count + (size_t)chunk * El, sizeof(int32_t) * El, hipMemcpyDeviceToHost));
    const size_t na = (size_t)Tn * k;
    if (na > 0) {
        if (idx) HIP_TRY(ctx, hipMemcpy(idx, ctx->idx + (size_t)t0 * k, na * 4, hipMemcpyDeviceToHost));
        if (w) HIP_TRY(ctx, hipMemcpy(w, ctx->w + (size_t)t0 * k, na * 4, hipMemcpyDeviceToHost));
        if (pos) HIP_TRY(ctx, hipMemcpy(pos, ctx->pos + (size_t)t0 * k, na * 4, hipMemcpyDeviceToHost));
        if (perm && off[El] > 0) HIP_TRY(ctx, hipMemcpy(perm, ctx->perm + (size_t)t0 * k, (size_t)off[El] * 4, hipMemcpyDeviceToHost));
    }
    return MOE_EP_OK;
}

}  // extern "C"

// ---- the entry point that allocates nothing -------------------------------------------------------
// Workspaces of moe_ep_forward_noalloc: one array per GPU in the library's own device image, there from
// the moment the code object is loaded until the process ends.  In host code the name is only a handle
// for hipGetSymbolAddress; kernels and copies get the address that call returns on each device.
__device__ __align__(256) static unsigned char scratch[MOE_EP_NOALLOC_SCRATCH_BYTES];

namespace {

constexpr int kMaxStaticDevices = 16;
struct StaticSlot {
    bool ready = false;
    char* base = nullptr;   // this device's copy of `scratch`
    moe_ep_ctx ctx;         // no streams, no events, no owned memory: device mode needs none
};
StaticSlot g_static[kMaxStaticDevices];
std::mutex g_static_mutex;

}  // namespace

extern "C" int moe_ep_forward_noalloc(const moe_ep_config* cfg, const void* tokens, const float* gate_logits,
                                      const void* routed_w, const void* shared_w, int32_t top_k, int32_t r_chunks,
                                      int32_t order, int32_t n_tokens, void* out, void* stream, const char** why)
{
    set_why(why, "ok");
    if (moe_ep_validate_forward(cfg, tokens, gate_logits, routed_w, shared_w, top_k, r_chunks, order, n_tokens, out,
                                why) != MOE_EP_OK)
        return MOE_EP_EINVAL;
    if (r_chunks < 1) { set_why(why, "r_chunks must be at least 1 (there is no context to hold a timing model)"); return MOE_EP_EINVAL; }
    if (cfg->io_mode != MOE_EP_IO_DEVICE) { set_why(why, "moe_ep_forward_noalloc serves MOE_EP_IO_DEVICE only"); return MOE_EP_EINVAL; }
    if (cfg->device >= kMaxStaticDevices) { set_why(why, "device ordinal beyond what moe_ep_forward_noalloc serves"); return MOE_EP_EINVAL; }
    const WsLayout L = ws_layout(*cfg);
    if (L.total > (size_t)MOE_EP_NOALLOC_SCRATCH_BYTES) {
        set_why(why, "this configuration needs more workspace than MOE_EP_NOALLOC_SCRATCH_BYTES (see moe_ep_workspace_bytes)");
        return MOE_EP_EINVAL;
    }
    StaticSlot& slot = g_static[cfg->device];
    moe_ep_ctx* ctx = &slot.ctx;
    if (hipSetDevice(cfg->device) != hipSuccess) { set_why(why, "hipSetDevice failed"); return MOE_EP_EHIP; }
    {
        std::lock_guard<std::mutex> lock(g_static_mutex);
        if (!slot.ready) {  // once per device, with that device current
            void* p = nullptr;
            if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || p == nullptr) {
                (void)hipGetLastError();
                set_why(why, "hipGetSymbolAddress(scratch) failed");
                return MOE_EP_EHIP;
            }
            hipDeviceProp_t prop;
            if (hipGetDeviceProperties(&prop, cfg->device) != hipSuccess) { set_why(why, "hipGetDeviceProperties failed"); return MOE_EP_EHIP; }
            if (grouped_gemm_init() != hipSuccess) { set_why(why, "raising the kernels' LDS limit failed"); return MOE_EP_EHIP; }
            slot.base = static_cast<char*>(p);
            ctx->n_cu = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;
            read_knobs(ctx);
            slot.ready = true;
        }
    }
    ctx->cfg = *cfg;
    bind_workspaces(ctx, slot.base, L);
    ctx->err[0] = 0;
    const int rc = forward_impl(ctx, tokens, gate_logits, routed_w, shared_w, top_k, 1, r_chunks, order, false, 0.0,
                                n_tokens, out, stream);
    if (rc != MOE_EP_OK) set_why(why, ctx->err);
    return rc;
}
