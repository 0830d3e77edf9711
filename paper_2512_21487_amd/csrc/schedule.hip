// Choice of the fine-grained pipeline degree r_2 from fitted linear task models (host code).
//   * t = alpha + beta * x for every task (Sec. 4.1, Eq. gm and Eq. a_r); fitted by least squares
//   * finish time of one slice cut into r chunks, three serial resources (Sec. 4.2, layer 0):
//       t_in + t_e + t_out + (r - 1) * max(t_in, t_e, t_out),  each t evaluated at T / r tokens
//   * the objective is convex in u = 1 / r_2 (Theorem 4), so the minimiser is found by a
//     golden-section search over u followed by a walk over the neighbouring integers
//   * the paper's resources are separate hardware (Sec. 3.2); where they are not, a model may carry
//     a second set of coefficients, fitted while the other resources ran: r = 1 (nothing overlaps)
//     is priced with the first set, every r > 1 with the second, and the search runs over r >= 2
//     of the second set (convex there) before the two are compared
#include <cmath>

#include "moe_ep.h"

namespace {

bool has_beside(const moe_ep_pipeline_model& m)
{
    return m.alpha_in_beside != 0.0 || m.beta_in_beside != 0.0 || m.alpha_e_beside != 0.0 ||
           m.beta_e_beside != 0.0 || m.alpha_out_beside != 0.0 || m.beta_out_beside != 0.0;
}

// beside: the coefficients of tasks that run beside others (r > 1 of a model that has them)
double span_at(double r, double T, const moe_ep_pipeline_model& m, bool beside)
{
    const double x = T / r;
    const double t_in = beside ? m.alpha_in_beside + m.beta_in_beside * x : m.alpha_in + m.beta_in * x;
    const double t_e = beside ? m.alpha_e_beside + m.beta_e_beside * x : m.alpha_e + m.beta_e * x;
    const double t_out = beside ? m.alpha_out_beside + m.beta_out_beside * x : m.alpha_out + m.beta_out * x;
    double y = t_in > t_e ? t_in : t_e;
    if (t_out > y) y = t_out;
    return t_in + t_e + t_out + (r - 1.0) * y;
}

}  // namespace

extern "C" {

int moe_ep_fit_linear(const double* x, const double* t, int32_t n, double* alpha, double* beta, double* r2)
{
    if (!x || !t || !alpha || !beta || n < 2) return MOE_EP_EINVAL;
    double sx = 0, st = 0;
    for (int i = 0; i < n; ++i) { sx += x[i]; st += t[i]; }
    const double mx = sx / n, mt = st / n;
    double sxx = 0, sxt = 0, stt = 0;
    for (int i = 0; i < n; ++i) {
        const double dx = x[i] - mx, dt = t[i] - mt;
        sxx += dx * dx; sxt += dx * dt; stt += dt * dt;
    }
    if (sxx <= 0.0) return MOE_EP_EINVAL;  // all workloads equal: the slope is undetermined
    *beta = sxt / sxx;
    *alpha = mt - *beta * mx;
    if (r2) {
        double res = 0;
        for (int i = 0; i < n; ++i) { const double e = t[i] - (*alpha + *beta * x[i]); res += e * e; }
        *r2 = stt == 0.0 ? 1.0 : 1.0 - res / stt;
    }
    return MOE_EP_OK;
}

double moe_ep_pipeline_makespan(const moe_ep_pipeline_model* m, int32_t n_tokens, int32_t r_chunks)
{
    if (!m || n_tokens < 0 || r_chunks < 1) return -1.0;
    return span_at((double)r_chunks, (double)n_tokens, *m, r_chunks > 1 && has_beside(*m));
}

}  // extern "C"

namespace {

// the smallest r in r_min..r_max that minimises span_at(., T, m, beside): golden-section search for
// the minimiser of the convex f(u) = span(1/u) on [1/r_max, 1/r_min], then the integer neighbourhood
int32_t convex_argmin(const moe_ep_pipeline_model& m, double T, int32_t r_min, int32_t r_max, bool beside)
{
    if (r_max <= r_min) return r_min;
    const double g = 0.6180339887498949;
    double lo = 1.0 / r_max, hi = 1.0 / r_min;
    double a = hi - g * (hi - lo), b = lo + g * (hi - lo);
    double fa = span_at(1.0 / a, T, m, beside), fb = span_at(1.0 / b, T, m, beside);
    for (int it = 0; it < 80; ++it) {
        if (fa <= fb) { hi = b; b = a; fb = fa; a = hi - g * (hi - lo); fa = span_at(1.0 / a, T, m, beside); }
        else { lo = a; a = b; fa = fb; b = lo + g * (hi - lo); fb = span_at(1.0 / b, T, m, beside); }
    }
    int32_t r = (int32_t)std::floor(2.0 / (lo + hi) + 0.5);
    if (r < r_min) r = r_min;
    if (r > r_max) r = r_max;
    // the span over integer r is unimodal: walk downhill, then to the smallest r of a flat bottom
    double fr = span_at(r, T, m, beside);
    while (r < r_max && span_at(r + 1, T, m, beside) < fr) { ++r; fr = span_at(r, T, m, beside); }
    while (r > r_min && span_at(r - 1, T, m, beside) <= fr) { --r; fr = span_at(r, T, m, beside); }
    return r;
}

}  // namespace

extern "C" int32_t moe_ep_choose_chunks(const moe_ep_pipeline_model* m, int32_t n_tokens, int32_t r_max)
{
    if (!m || n_tokens < 0 || r_max < 1) return MOE_EP_EINVAL;
    if (r_max == 1 || n_tokens == 0) return 1;
    const double T = (double)n_tokens;
    if (!has_beside(*m)) return convex_argmin(*m, T, 1, r_max, false);
    const int32_t r = convex_argmin(*m, T, 2, r_max, true);
    return span_at(r, T, *m, true) < span_at(1.0, T, *m, false) ? r : 1;
}
