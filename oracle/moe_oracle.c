/*
 * moe_oracle.c -- TEST INFRASTRUCTURE, not part of the product.
 *
 * A plain, slow CPU statement of what the expert-group side of one MoE layer
 * computes, written from the paper's definitions:
 *
 *   - gate: softmax over all E routing scores, top-k experts per token
 *           (Sec. 2.1, "MoE Layer")
 *   - the input is partitioned by expert and each expert sees only its own
 *           tokens; a device holds E/eg of the experts (Sec. 2.1; Sec. 3.1,
 *           "The MoE Part")
 *   - an expert is three projections W_gate, W_up in R^{H x M} and
 *           W_down in R^{M x H} around a Swish gate (Sec. 3.1, "The Shared
 *           Expert Part" and "The MoE Part")
 *   - the layer output is the sum of the selected experts' contributions and
 *           of the shared experts if present (Sec. 2.1)
 *   - the expert part is token-wise, so the token range may be cut into r_2
 *           pieces that are processed one after another (Sec. 2.3)
 *
 * Arithmetic is IEEE double throughout.  bf16 inputs are widened exactly.
 * There is no blocking, fusion or reordering: loops run in the order of the
 * definitions.  OpenMP only spreads independent rows over cores.
 *
 * Only tests, the smoke check and the benchmark's cpu_baseline leg may call
 * this file.  It shares no code with the HIP library.
 *
 * Readings of the paper taken here (the paper is silent or inconsistent):
 *   R1  routing weights are renormalised over the k selected experts;
 *   R2  selection order: larger score first, equal scores -> lower expert
 *       index first; selection is done on the raw fp32 scores (softmax is
 *       monotone, so this is the same set);
 *   R3  the activation is silu(z_gate) * z_up (SwiGLU).  The paper prints
 *       Swish applied to the product z_gate (x) z_up; that literal form is kept
 *       behind `literal_swish` for the record and is never used for parity;
 *   R4  several shared experts add up, each with weight 1;
 *   R5  a device keeps only assignments to its local experts and does not
 *       renormalise the weights after that filter; tokens with no local
 *       expert get the shared contribution only (zero if there is none);
 *   R6  r chunks are contiguous token ranges of ceil(T/r) tokens.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

static double bf16_to_double(uint16_t bits)
{
    uint32_t u = (uint32_t)bits << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

/* double -> bf16 bits, round to nearest even (via one exact-enough fp32 step) */
static uint16_t double_to_bf16(double v)
{
    float f = (float)v;
    uint32_t u;
    memcpy(&u, &f, sizeof u);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40u);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

int moe_oracle_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* ------------------------------------------------------------------------
 * Gate (Sec. 2.1): p = softmax(scores[t, 0:E]); the k experts with the largest
 * p are selected; weights are p restricted to the selection and renormalised
 * (R1).  Slots are ordered best first (R2).
 *   logits [T, E] fp32, idx [T, k] int32, w [T, k] double.
 * Returns 0, or -1 on bad arguments.
 * ---------------------------------------------------------------------- */
int moe_oracle_router(const float *logits, int T, int E, int k,
                      int32_t *idx, double *w)
{
    if (T < 0 || E < 1 || k < 1 || k > E) return -1;
    double *p = (double *)malloc(sizeof(double) * (size_t)E);
    char *taken = (char *)malloc((size_t)E);
    if (!p || !taken) { free(p); free(taken); return -1; }
    for (int t = 0; t < T; ++t) {
        const float *l = logits + (size_t)t * E;
        double mx = (double)l[0];
        for (int e = 1; e < E; ++e) if ((double)l[e] > mx) mx = (double)l[e];
        double z = 0.0;
        for (int e = 0; e < E; ++e) { p[e] = exp((double)l[e] - mx); z += p[e]; }
        for (int e = 0; e < E; ++e) p[e] /= z;
        memset(taken, 0, (size_t)E);
        double zsel = 0.0;
        for (int s = 0; s < k; ++s) {
            int best = -1;
            for (int e = 0; e < E; ++e) {
                if (taken[e]) continue;
                if (best < 0 || l[e] > l[best]) best = e;   /* strict: ties keep lower e */
            }
            taken[best] = 1;
            idx[(size_t)t * k + s] = best;
            zsel += p[best];
        }
        for (int s = 0; s < k; ++s)
            w[(size_t)t * k + s] = p[idx[(size_t)t * k + s]] / zsel;
    }
    free(p); free(taken);
    return 0;
}

/* ------------------------------------------------------------------------
 * Partition by expert (Sec. 2.1; Sec. 3.1 "The MoE Part"): of the T*k
 * assignments keep those whose expert lies in [e0, e0+El) (R5), count them per
 * expert, and lay them out grouped by expert, inside an expert by ascending
 * token (a stable counting sort of the assignments by expert).
 *   idx    [T, k]   global expert ids
 *   count  [El]     rows of each local expert
 *   offset [El+1]   exclusive prefix sum of count; offset[El] = rows kept
 *   perm   [T*k]    position -> assignment id (t*k + slot); first offset[El] valid
 *   pos    [T, k]   assignment -> position, or -1 if not kept
 * ---------------------------------------------------------------------- */
int moe_oracle_dispatch(const int32_t *idx, int T, int k, int e0, int El,
                        int32_t *count, int32_t *offset, int32_t *perm,
                        int32_t *pos)
{
    if (T < 0 || k < 1 || El < 1) return -1;
    for (int e = 0; e < El; ++e) count[e] = 0;
    for (int a = 0; a < T * k; ++a) {
        int e = idx[a] - e0;
        if (e >= 0 && e < El) count[e]++;
    }
    offset[0] = 0;
    for (int e = 0; e < El; ++e) offset[e + 1] = offset[e] + count[e];
    int32_t *fill = (int32_t *)calloc((size_t)El, sizeof(int32_t));
    if (!fill) return -1;
    for (int a = 0; a < T * k; ++a) {
        int e = idx[a] - e0;
        if (e >= 0 && e < El) {
            int p = offset[e] + fill[e]++;
            perm[p] = a;
            pos[a] = p;
        } else {
            pos[a] = -1;
        }
    }
    free(fill);
    return 0;
}

/* ------------------------------------------------------------------------
 * One expert on one token (Sec. 3.1): z_gate = W_gate x, z_up = W_up x,
 * y = W_down act, act = silu(z_gate) * z_up (R3), Swish(v) = v / (1 + e^-v).
 *   x [M] bf16 bits; wexp = W_gate[H,M] | W_up[H,M] | W_down[M,H] bf16 bits
 *   y [M] double (accumulated into when `accumulate` != 0, scaled by `scale`)
 * ---------------------------------------------------------------------- */
static double swish(double v) { return v / (1.0 + exp(-v)); }

static void expert_ffn_row(const uint16_t *x, const uint16_t *wexp, int M, int H,
                           int literal_swish, double scale, double *act,
                           double *y)
{
    const uint16_t *Wg = wexp;
    const uint16_t *Wu = wexp + (size_t)H * M;
    const uint16_t *Wd = wexp + (size_t)2 * H * M;
    for (int h = 0; h < H; ++h) {
        double g = 0.0, u = 0.0;
        for (int m = 0; m < M; ++m) {
            double xv = bf16_to_double(x[m]);
            g += bf16_to_double(Wg[(size_t)h * M + m]) * xv;
            u += bf16_to_double(Wu[(size_t)h * M + m]) * xv;
        }
        act[h] = literal_swish ? swish(g * u) : swish(g) * u;
    }
    for (int m = 0; m < M; ++m) {
        double d = 0.0;
        for (int h = 0; h < H; ++h)
            d += bf16_to_double(Wd[(size_t)m * H + h]) * act[h];
        y[m] += scale * d;
    }
}

/* Exposed for tests: y[M] = FFN(x) for a single expert. */
int moe_oracle_expert_ffn(const uint16_t *x, const uint16_t *wexp, int M, int H,
                          int literal_swish, double *y)
{
    if (M < 1 || H < 1) return -1;
    double *act = (double *)malloc(sizeof(double) * (size_t)H);
    if (!act) return -1;
    for (int m = 0; m < M; ++m) y[m] = 0.0;
    expert_ffn_row(x, wexp, M, H, literal_swish, 1.0, act, y);
    free(act);
    return 0;
}

/* ------------------------------------------------------------------------
 * The whole path on a token range, in the order router -> local filter ->
 * partition -> routed experts on their rows -> weighted aggregation -> shared
 * experts, repeated over r contiguous chunks (R6).
 *
 *   tokens   [T, M] bf16 bits        logits [T, E] fp32
 *   routed_w El experts, each W_gate|W_up|W_down;  shared_w Ns experts (or NULL)
 *   out      [T, M] double           out_bf16 [T, M] bf16 bits (may be NULL)
 * Optional per-chunk routing results (any may be NULL):
 *   idx [T,k], w [T,k] (chunk independent), pos [T,k] (chunk-local position),
 *   count [r, El], offset [r, El+1], perm [r, Tc*k] (chunk-local t*k+slot)
 * ---------------------------------------------------------------------- */
int moe_oracle_forward(const uint16_t *tokens, const float *logits,
                       const uint16_t *routed_w, const uint16_t *shared_w,
                       int T, int M, int H, int E, int e0, int El,
                       int Ns, int Hs, int k, int r, int literal_swish,
                       double *out, uint16_t *out_bf16,
                       int32_t *idx_out, double *w_out, int32_t *pos_out,
                       int32_t *count_out, int32_t *offset_out,
                       int32_t *perm_out)
{
    if (T < 0 || M < 1 || H < 1 || E < 1 || El < 1 || e0 < 0 || e0 + El > E ||
        k < 1 || k > E || r < 1 || Ns < 0 || (Ns > 0 && (!shared_w || Hs < 1)))
        return -1;
    const int Tc = (T + r - 1) / r;
    const size_t wsz = (size_t)3 * H * M, ssz = (size_t)3 * Hs * M;
    int rc = 0;
    for (int c = 0; c < r; ++c) {
        const int t0 = c * Tc;
        const int Tn = (t0 >= T) ? 0 : ((T - t0 < Tc) ? T - t0 : Tc);
        int32_t *count = (int32_t *)calloc((size_t)El, sizeof(int32_t));
        int32_t *offset = (int32_t *)calloc((size_t)El + 1, sizeof(int32_t));
        int32_t *idx = (int32_t *)malloc(sizeof(int32_t) * ((size_t)Tn * k + 1));
        int32_t *perm = (int32_t *)malloc(sizeof(int32_t) * ((size_t)Tn * k + 1));
        int32_t *pos = (int32_t *)malloc(sizeof(int32_t) * ((size_t)Tn * k + 1));
        double *w = (double *)malloc(sizeof(double) * ((size_t)Tn * k + 1));
        if (!count || !offset || !idx || !perm || !pos || !w) rc = -1;
        if (rc == 0 && Tn > 0) {
            /* gate */
            rc = moe_oracle_router(logits + (size_t)t0 * E, Tn, E, k, idx, w);
            /* local filter + partition */
            if (rc == 0)
                rc = moe_oracle_dispatch(idx, Tn, k, e0, El, count, offset, perm, pos);
        }
        if (rc == 0 && Tn > 0) {
            const int A = offset[El];
            /* the grouped input h' (one row per kept assignment) and its output */
            uint16_t *xp = (uint16_t *)malloc(sizeof(uint16_t) * ((size_t)A * M + 1));
            double *yp = (double *)calloc((size_t)A * M + 1, sizeof(double));
            int32_t *row_expert = (int32_t *)malloc(sizeof(int32_t) * ((size_t)A + 1));
            if (!xp || !yp || !row_expert) rc = -1;
            if (rc == 0) {
                for (int p = 0; p < A; ++p)
                    memcpy(xp + (size_t)p * M,
                           tokens + (size_t)(t0 + perm[p] / k) * M,
                           sizeof(uint16_t) * (size_t)M);
                for (int e = 0; e < El; ++e)
                    for (int p = offset[e]; p < offset[e + 1]; ++p) row_expert[p] = e;
                /* routed experts: each row through its expert */
                #pragma omp parallel
                {
                    double *act = (double *)malloc(sizeof(double) * (size_t)H);
                    #pragma omp for schedule(dynamic, 1)
                    for (int p = 0; p < A; ++p)
                        expert_ffn_row(xp + (size_t)p * M,
                                       routed_w + (size_t)row_expert[p] * wsz,
                                       M, H, literal_swish, 1.0, act,
                                       yp + (size_t)p * M);
                    free(act);
                }
                /* aggregation + shared experts, token by token */
                #pragma omp parallel
                {
                    double *act = (double *)malloc(sizeof(double) * (size_t)(Hs > 0 ? Hs : 1));
                    #pragma omp for schedule(dynamic, 1)
                    for (int t = 0; t < Tn; ++t) {
                        double *o = out + (size_t)(t0 + t) * M;
                        for (int m = 0; m < M; ++m) o[m] = 0.0;
                        for (int s = 0; s < k; ++s) {
                            int p = pos[(size_t)t * k + s];
                            if (p < 0) continue;
                            double ws = w[(size_t)t * k + s];
                            for (int m = 0; m < M; ++m)
                                o[m] += ws * yp[(size_t)p * M + m];
                        }
                        for (int i = 0; i < Ns; ++i)
                            expert_ffn_row(tokens + (size_t)(t0 + t) * M,
                                           shared_w + (size_t)i * ssz, M, Hs,
                                           literal_swish, 1.0, act, o);
                    }
                    free(act);
                }
            }
            free(xp); free(yp); free(row_expert);
        }
        if (rc == 0) {
            if (idx_out) memcpy(idx_out + (size_t)t0 * k, idx, sizeof(int32_t) * (size_t)Tn * k);
            if (w_out) memcpy(w_out + (size_t)t0 * k, w, sizeof(double) * (size_t)Tn * k);
            if (pos_out) memcpy(pos_out + (size_t)t0 * k, pos, sizeof(int32_t) * (size_t)Tn * k);
            if (count_out) memcpy(count_out + (size_t)c * El, count, sizeof(int32_t) * (size_t)El);
            if (offset_out) memcpy(offset_out + (size_t)c * (El + 1), offset, sizeof(int32_t) * ((size_t)El + 1));
            if (perm_out) memcpy(perm_out + (size_t)c * Tc * k, perm, sizeof(int32_t) * (size_t)offset[El]);
        }
        free(count); free(offset); free(idx); free(perm); free(pos); free(w);
        if (rc != 0) return rc;
    }
    if (out_bf16)
        for (size_t i = 0; i < (size_t)T * M; ++i) out_bf16[i] = double_to_bf16(out[i]);
    return 0;
}

/* ------------------------------------------------------------------------
 * The same definition evaluated for a chosen list of tokens only (tokens are
 * independent rows, Sec. 2.3): out[i, :] is the layer output of token ids[i].
 * Used where the full layer is too large to run on the CPU.
 * ---------------------------------------------------------------------- */
int moe_oracle_forward_tokens(const uint16_t *tokens, const float *logits,
                              const uint16_t *routed_w, const uint16_t *shared_w,
                              int T, int M, int H, int E, int e0, int El,
                              int Ns, int Hs, int k, int literal_swish,
                              const int32_t *ids, int n_ids, double *out)
{
    if (T < 0 || M < 1 || H < 1 || E < 1 || El < 1 || e0 < 0 || e0 + El > E ||
        k < 1 || k > E || n_ids < 0 || Ns < 0 || (Ns > 0 && (!shared_w || Hs < 1)))
        return -1;
    for (int i = 0; i < n_ids; ++i)
        if (ids[i] < 0 || ids[i] >= T) return -1;
    const size_t wsz = (size_t)3 * H * M, ssz = (size_t)3 * Hs * M;
    int rc = 0;
    #pragma omp parallel
    {
        int hmax = H > Hs ? H : Hs;
        double *act = (double *)malloc(sizeof(double) * (size_t)hmax);
        int32_t *idx = (int32_t *)malloc(sizeof(int32_t) * (size_t)k);
        double *w = (double *)malloc(sizeof(double) * (size_t)k);
        #pragma omp for schedule(dynamic, 1)
        for (int i = 0; i < n_ids; ++i) {
            const int t = ids[i];
            double *o = out + (size_t)i * M;
            for (int m = 0; m < M; ++m) o[m] = 0.0;
            if (moe_oracle_router(logits + (size_t)t * E, 1, E, k, idx, w) != 0) {
                #pragma omp atomic write
                rc = -1;
                continue;
            }
            for (int s = 0; s < k; ++s) {
                int e = idx[s] - e0;
                if (e < 0 || e >= El) continue;
                expert_ffn_row(tokens + (size_t)t * M, routed_w + (size_t)e * wsz,
                               M, H, literal_swish, w[s], act, o);
            }
            for (int j = 0; j < Ns; ++j)
                expert_ffn_row(tokens + (size_t)t * M, shared_w + (size_t)j * ssz,
                               M, Hs, literal_swish, 1.0, act, o);
        }
        free(act); free(idx); free(w);
    }
    return rc;
}
