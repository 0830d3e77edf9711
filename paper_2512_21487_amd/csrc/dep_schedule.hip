// Schedule model of disaggregated expert parallelism and the configuration search (host code).
//   * linear task models of the attention, shared-expert, expert and transfer tasks (Sec. 4.1,
//     "Performance models of different layers")
//   * earliest-start replay of the timing rules (Sec. 3.2, Eq. limitation) for T layers, r_1
//     attention micro-batches, r_2 expert chunks and the two attention-group orders of Sec. 4.2
//   * makespan model of the ASAS order (Sec. 4.2, denominator of Eq. simplify-objective)
//   * Algorithm 1: the (m_a, r_1) pairs on the memory frontier, both orders, r_2 by a search that
//     uses the convexity in 1 / r_2 (Theorem 4)
#include <cmath>
#include <vector>

#include "moe_ep.h"

namespace {

struct Durations { double a, s, e, c; };

bool problem_ok(const moe_ep_dep_problem* p)
{
    return p && p->ag >= 1 && p->n_experts >= 1 && p->top_k >= 1 && p->seq_len >= 1 && p->n_layers >= 1;
}

// m_e from the conservation rule (last line of Eq. limitation); r_2 may be fractional during the search
double m_e_of(const moe_ep_dep_problem& p, double m_a, double r_2)
{
    return m_a * p.ag * p.top_k * p.seq_len / (r_2 * p.n_experts);
}

Durations durations(const moe_ep_dep_models& m, const moe_ep_dep_problem& p, double m_a, double r_2)
{
    const double m_e = m_e_of(p, m_a, r_2);
    return {m.alpha_a + m.beta_a * m_a, m.alpha_s + m.beta_s * m_a, m.alpha_e + m.beta_e * m_e,
            m.alpha_c + m.beta_c * m_e};
}

// ASAS over T layers: (T-1) max(G, r_1 F) + max(X, G) + (r_1 - 1) F with X = t_a + t_s,
// Y = max(t_e, t_a2e), F = max(X, r_2 Y), G = t_a + 2 t_a2e + t_e + (r_2 - 1) Y.  The fine-grained
// term (r_2 - 1) Y is counted once, inside G.
double asas_span(const moe_ep_dep_models& m, const moe_ep_dep_problem& p, double m_a, double r_1, double r_2)
{
    const Durations d = durations(m, p, m_a, r_2);
    const double X = d.a + d.s;
    const double Y = d.e > d.c ? d.e : d.c;
    const double F = X > r_2 * Y ? X : r_2 * Y;
    const double G = d.a + 2.0 * d.c + d.e + (r_2 - 1.0) * Y;
    const double period = G > r_1 * F ? G : r_1 * F;
    return (p.n_layers - 1) * period + (X > G ? X : G) + (r_1 - 1.0) * F;
}

// The replay keeps one cursor per resource over that resource's fixed task sequence and starts the
// task under a cursor as soon as everything it waits for has been placed.
struct Replay {
    int T, r1, r2;
    Durations d;
    std::vector<double> a, s, a2e, e, e2a;  // start times; layouts [t][i] and [t][i][j]
    size_t ix(int t, int i) const { return (size_t)t * r1 + i; }
    size_t ix(int t, int i, int j) const { return ((size_t)t * r1 + i) * r2 + j; }

    double run(int order)
    {
        const size_t n2 = (size_t)T * r1, n3 = n2 * r2;
        a.assign(n2, -1.0); s.assign(n2, -1.0); a2e.assign(n3, -1.0); e.assign(n3, -1.0); e2a.assign(n3, -1.0);
        // attention-group sequence: per layer 2 r_1 entries, kind 0 = attention, 1 = shared expert
        std::vector<int> ag_kind, ag_mb;
        for (int i = 0; i < r1; ++i) {
            if (order == MOE_EP_DEP_ASAS) { ag_kind.push_back(0); ag_mb.push_back(i); ag_kind.push_back(1); ag_mb.push_back(i); }
        }
        if (order == MOE_EP_DEP_AASS) {
            for (int i = 0; i < r1; ++i) { ag_kind.push_back(0); ag_mb.push_back(i); }
            for (int i = 0; i < r1; ++i) { ag_kind.push_back(1); ag_mb.push_back(i); }
        }
        const size_t ag_len = (size_t)T * 2 * r1;
        size_t c_ag = 0, c_a2e = 0, c_e = 0, c_e2a = 0;
        double f_ag = 0, f_a2e = 0, f_e = 0, f_e2a = 0;  // when each resource falls free
        bool moved = true;
        while (moved) {
            moved = false;
            while (c_ag < ag_len) {
                const int t = (int)(c_ag / (2 * r1)), k = (int)(c_ag % (2 * r1));
                const int i = ag_mb[k];
                double ready;
                if (ag_kind[k] == 0) {
                    ready = 0.0;
                    if (t > 0) {  // the micro-batch's previous layer has come back and its shared expert is done
                        if (e2a[ix(t - 1, i, r2 - 1)] < 0 || s[ix(t - 1, i)] < 0) break;
                        ready = s[ix(t - 1, i)] + d.s;
                        for (int j = 0; j < r2; ++j) { const double x = e2a[ix(t - 1, i, j)] + d.c; if (x > ready) ready = x; }
                    }
                    a[ix(t, i)] = ready > f_ag ? ready : f_ag;
                    f_ag = a[ix(t, i)] + d.a;
                } else {
                    if (a[ix(t, i)] < 0) break;
                    ready = a[ix(t, i)] + d.a;
                    s[ix(t, i)] = ready > f_ag ? ready : f_ag;
                    f_ag = s[ix(t, i)] + d.s;
                }
                ++c_ag; moved = true;
            }
            while (c_a2e < n3) {
                const double att = a[c_a2e / r2];
                if (att < 0) break;
                const double ready = att + d.a;
                a2e[c_a2e] = ready > f_a2e ? ready : f_a2e;
                f_a2e = a2e[c_a2e] + d.c;
                ++c_a2e; moved = true;
            }
            while (c_e < n3 && a2e[c_e] >= 0) {
                const double ready = a2e[c_e] + d.c;
                e[c_e] = ready > f_e ? ready : f_e;
                f_e = e[c_e] + d.e;
                ++c_e; moved = true;
            }
            while (c_e2a < n3 && e[c_e2a] >= 0) {
                const double ready = e[c_e2a] + d.e;
                e2a[c_e2a] = ready > f_e2a ? ready : f_e2a;
                f_e2a = e2a[c_e2a] + d.c;
                ++c_e2a; moved = true;
            }
        }
        const double end_s = s[ix(T - 1, r1 - 1)] + d.s, end_x = e2a[ix(T - 1, r1 - 1, r2 - 1)] + d.c;
        return end_s > end_x ? end_s : end_x;
    }
};

// The same rules with one more: shared-expert and expert tasks run on one GPU's compute units and do not
// overlap (the stand-in of moe_ep_forward_dep; not a case the paper treats).  Which of two waiting tasks
// takes the compute units first is then a choice, so the schedule is defined by a procedure: among the
// next task of each of the four sequences whose predecessors are placed, the one that can start earliest
// is placed (ties: attention group, A2E, experts, E2A).  Kept as end times; a task not yet placed has
// end < 0.
struct OneGpuReplay {
    int T, r1, r2;
    Durations d;
    std::vector<double> a, s, a2e, e, e2a;   // start times, layouts as in Replay

    double run(int order)
    {
        const int n2 = T * r1, n3 = n2 * r2;
        a.assign(n2, -1.0); s.assign(n2, -1.0); a2e.assign(n3, -1.0); e.assign(n3, -1.0); e2a.assign(n3, -1.0);
        // position k of a layer's attention-group sequence -> (is shared expert, micro-batch)
        auto ag_task = [&](int k, bool* shared, int* i) {
            if (order == MOE_EP_DEP_ASAS) { *shared = (k & 1) != 0; *i = k >> 1; }
            else { *shared = k >= r1; *i = k % r1; }
        };
        const double never = -1.0;
        int c_ag = 0, c_a2e = 0, c_e = 0, c_e2a = 0;                  // next task of each sequence
        double f_ag = 0, f_a2e = 0, f_e = 0, f_e2a = 0, f_cu = 0;   // when each resource falls free
        // earliest start of the next task of each sequence, or `never`
        auto next_ag = [&]() -> double {
            if (c_ag == 2 * n2) return never;
            const int t = c_ag / (2 * r1);
            bool shared; int i;
            ag_task(c_ag % (2 * r1), &shared, &i);
            double at = f_ag;
            if (shared) {
                if (a[t * r1 + i] < 0) return never;
                at = std::fmax(at, a[t * r1 + i] + d.a);
                at = std::fmax(at, f_cu);
            } else if (t > 0) {
                const int q = (t - 1) * r1 + i;
                if (s[q] < 0 || e2a[q * r2 + r2 - 1] < 0) return never;
                at = std::fmax(at, s[q] + d.s);
                for (int j = 0; j < r2; ++j) at = std::fmax(at, e2a[q * r2 + j] + d.c);
            }
            return at;
        };
        auto next_a2e = [&]() -> double {
            if (c_a2e == n3 || a[c_a2e / r2] < 0) return never;
            return std::fmax(f_a2e, a[c_a2e / r2] + d.a);
        };
        auto next_e = [&]() -> double {
            if (c_e == n3 || a2e[c_e] < 0) return never;
            return std::fmax(std::fmax(f_e, f_cu), a2e[c_e] + d.c);
        };
        auto next_e2a = [&]() -> double {
            if (c_e2a == n3 || e[c_e2a] < 0) return never;
            return std::fmax(f_e2a, e[c_e2a] + d.e);
        };
        for (int placed = 0; placed < 2 * n2 + 3 * n3; ++placed) {
            const double at[4] = {next_ag(), next_a2e(), next_e(), next_e2a()};
            int pick = -1;
            for (int q = 0; q < 4; ++q)
                if (at[q] >= 0 && (pick < 0 || at[q] < at[pick])) pick = q;
            if (pick < 0) return -1.0;   // cannot happen: the first unplaced task of some sequence is always ready
            const double t0 = at[pick];
            if (pick == 0) {
                const int t = c_ag / (2 * r1);
                bool shared; int i;
                ag_task(c_ag % (2 * r1), &shared, &i);
                if (shared) { s[t * r1 + i] = t0; f_ag = f_cu = t0 + d.s; }
                else { a[t * r1 + i] = t0; f_ag = t0 + d.a; }
                ++c_ag;
            } else if (pick == 1) {
                a2e[c_a2e++] = t0; f_a2e = t0 + d.c;
            } else if (pick == 2) {
                e[c_e++] = t0; f_e = f_cu = t0 + d.e;
            } else {
                e2a[c_e2a++] = t0; f_e2a = t0 + d.c;
            }
        }
        return std::fmax(s[n2 - 1] + d.s, e2a[n3 - 1] + d.c);
    }
};

double replay_span(const moe_ep_dep_models& m, const moe_ep_dep_problem& p, int m_a, int r_1, int r_2, int order,
                   Replay* keep = nullptr)
{
    Replay local;
    Replay& R = keep ? *keep : local;
    R.T = p.n_layers; R.r1 = r_1; R.r2 = r_2;
    R.d = durations(m, p, m_a, r_2);
    return R.run(order);
}

// smallest integer minimiser on [1, r_max] of f, convex in 1 / r: golden section over u = 1 / r,
// then a walk over the neighbouring integers down to the first r of a flat bottom
template <class Fn>
int argmin_convex_in_reciprocal(Fn f, int r_max)
{
    if (r_max <= 1) return 1;
    const double g = 0.6180339887498949;
    double lo = 1.0 / r_max, hi = 1.0;
    double u1 = hi - g * (hi - lo), u2 = lo + g * (hi - lo);
    double f1 = f(1.0 / u1), f2 = f(1.0 / u2);
    for (int it = 0; it < 80; ++it) {
        if (f1 <= f2) { hi = u2; u2 = u1; f2 = f1; u1 = hi - g * (hi - lo); f1 = f(1.0 / u1); }
        else { lo = u1; u1 = u2; f1 = f2; u2 = lo + g * (hi - lo); f2 = f(1.0 / u2); }
    }
    int r = (int)std::floor(2.0 / (lo + hi) + 0.5);
    if (r < 1) r = 1;
    if (r > r_max) r = r_max;
    double fr = f((double)r);
    while (r < r_max && f((double)(r + 1)) < fr) { ++r; fr = f((double)r); }
    while (r > 1 && f((double)(r - 1)) <= fr) { --r; fr = f((double)r); }
    return r;
}

int solve_r2(const moe_ep_dep_models& m, const moe_ep_dep_problem& p, int m_a, int r_1, int order, int r2_max,
             double* span)
{
    int best;
    if (order == MOE_EP_DEP_ASAS) {
        best = argmin_convex_in_reciprocal([&](double r) { return asas_span(m, p, m_a, r_1, r); }, r2_max);
        *span = asas_span(m, p, m_a, r_1, best);
    } else {
        // no closed form is given for this order: every r_2 is replayed
        best = 1;
        *span = replay_span(m, p, m_a, r_1, 1, order);
        for (int r = 2; r <= r2_max; ++r) {
            const double t = replay_span(m, p, m_a, r_1, r, order);
            if (t < *span) { *span = t; best = r; }
        }
    }
    return best;
}

}  // namespace

extern "C" {

int moe_ep_dep_layer_models(const moe_ep_dep_primitives* q, moe_ep_dep_models* out)
{
    if (!q || !out || q->eg < 1 || q->n_experts < 1 || q->seq_len < 1 || q->hidden < 1 || q->inter < 1 || q->n_heads < 1 ||
        q->d_k < 1 || q->d_v < 1 || q->n_shared < 0) return MOE_EP_EINVAL;
    const double S = q->seq_len, M = q->hidden, H = q->inter, nh = q->n_heads, dk = q->d_k, dv = q->d_v;
    const double per_dev = (double)q->n_experts / q->eg;
    out->alpha_a = 4.0 * q->alpha_gm + q->alpha_attn;
    out->beta_a = q->beta_gm * (2.0 * S * M * nh * dk + 2.0 * S * M * nh * dv) + q->beta_attn * S * S * nh * (dk + dv);
    out->alpha_s = 3.0 * q->n_shared * q->alpha_gm;
    out->beta_s = 3.0 * q->n_shared * q->beta_gm * S * M * H;
    out->alpha_e = 3.0 * per_dev * q->alpha_gm;
    out->beta_e = 3.0 * per_dev * q->beta_gm * M * H;
    out->alpha_c = q->alpha_c;
    out->beta_c = q->beta_c * q->n_experts * M / q->eg;
    return MOE_EP_OK;
}

double moe_ep_dep_tokens_per_expert(const moe_ep_dep_problem* p, int32_t m_a, int32_t r_2)
{
    if (!problem_ok(p) || m_a < 1 || r_2 < 1) return -1.0;
    return m_e_of(*p, m_a, r_2);
}

int moe_ep_dep_replay(const moe_ep_dep_models* m, const moe_ep_dep_problem* p, int32_t m_a, int32_t r_1, int32_t r_2,
                      int32_t order, double* makespan, double* tau_a, double* tau_s, double* tau_a2e, double* tau_e,
                      double* tau_e2a)
{
    if (!m || !problem_ok(p) || m_a < 1 || r_1 < 1 || r_2 < 1 || (order != MOE_EP_DEP_ASAS && order != MOE_EP_DEP_AASS))
        return MOE_EP_EINVAL;
    if ((long long)p->n_layers * r_1 * r_2 > (1ll << 26)) return MOE_EP_EINVAL;
    Replay R;
    const double span = replay_span(*m, *p, m_a, r_1, r_2, order, &R);
    if (makespan) *makespan = span;
    auto put = [](double* dst, const std::vector<double>& v) { if (dst) for (size_t i = 0; i < v.size(); ++i) dst[i] = v[i]; };
    put(tau_a, R.a); put(tau_s, R.s); put(tau_a2e, R.a2e); put(tau_e, R.e); put(tau_e2a, R.e2a);
    return MOE_EP_OK;
}

int moe_ep_dep_replay_one_gpu(const moe_ep_dep_models* m, const moe_ep_dep_problem* p, int32_t m_a, int32_t r_1,
                              int32_t r_2, int32_t order, double* makespan, double* tau_a, double* tau_s,
                              double* tau_a2e, double* tau_e, double* tau_e2a)
{
    if (!m || !problem_ok(p) || m_a < 1 || r_1 < 1 || r_2 < 1 || (order != MOE_EP_DEP_ASAS && order != MOE_EP_DEP_AASS))
        return MOE_EP_EINVAL;
    if ((long long)p->n_layers * r_1 * r_2 > (1ll << 24)) return MOE_EP_EINVAL;
    OneGpuReplay R;
    R.T = p->n_layers; R.r1 = r_1; R.r2 = r_2;
    R.d = durations(*m, *p, m_a, r_2);
    const double span = R.run(order);
    if (span < 0) return MOE_EP_ESTATE;
    if (makespan) *makespan = span;
    auto put = [](double* dst, const std::vector<double>& v) { if (dst) for (size_t i = 0; i < v.size(); ++i) dst[i] = v[i]; };
    put(tau_a, R.a); put(tau_s, R.s); put(tau_a2e, R.a2e); put(tau_e, R.e); put(tau_e2a, R.e2a);
    return MOE_EP_OK;
}

double moe_ep_dep_makespan(const moe_ep_dep_models* m, const moe_ep_dep_problem* p, int32_t m_a, int32_t r_1, int32_t r_2)
{
    if (!m || !problem_ok(p) || m_a < 1 || r_1 < 1 || r_2 < 1) return -1.0;
    return asas_span(*m, *p, m_a, r_1, r_2);
}

int moe_ep_dep_solve_r2(const moe_ep_dep_models* m, const moe_ep_dep_problem* p, int32_t m_a, int32_t r_1, int32_t order,
                        int32_t r2_max, int32_t* r_2, double* makespan)
{
    if (!m || !problem_ok(p) || !r_2 || m_a < 1 || r_1 < 1 || r2_max < 1 || r2_max > 4096 ||
        (order != MOE_EP_DEP_ASAS && order != MOE_EP_DEP_AASS)) return MOE_EP_EINVAL;
    double span;
    *r_2 = solve_r2(*m, *p, m_a, r_1, order, r2_max, &span);
    if (makespan) *makespan = span;
    return MOE_EP_OK;
}

int moe_ep_dep_search(const moe_ep_dep_models* m, const moe_ep_dep_problem* p, int32_t m_a_max, int32_t mem_cap,
                      int32_t r1_cap, int32_t r2_max, moe_ep_dep_config* best)
{
    if (!m || !problem_ok(p) || !best || m_a_max < 1 || mem_cap < 0 || r1_cap < 1 || r2_max < 1 || r2_max > 4096)
        return MOE_EP_EINVAL;
    bool found = false;
    int prev_r1 = 0;
    for (int m_a = m_a_max; m_a >= 1; --m_a) {
        int r_1 = mem_cap / m_a;                     // memory rule r_1 * m_a <= mem_cap
        if (r_1 > r1_cap) r_1 = r1_cap;
        if (r_1 == 0 || r_1 == prev_r1) continue;    // not on the frontier: a larger m_a had the same r_1
        for (int order = MOE_EP_DEP_ASAS; order <= MOE_EP_DEP_AASS; ++order) {
            double span;
            const int r_2 = solve_r2(*m, *p, m_a, r_1, order, r2_max, &span);
            const double tps = (double)r_1 * m_a * p->ag / span;
            if (!found || tps > best->throughput) {
                found = true;
                best->m_a = m_a; best->r_1 = r_1; best->r_2 = r_2; best->order = order;
                best->m_e = m_e_of(*p, m_a, r_2); best->makespan = span; best->throughput = tps;
            }
        }
        prev_r1 = r_1;
    }
    return found ? MOE_EP_OK : MOE_EP_ESTATE;
}

}  // extern "C"
