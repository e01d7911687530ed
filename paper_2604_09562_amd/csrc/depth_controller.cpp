// Speculation-depth controller: the closed-loop rule that picks each request's draft depth from the
// acceptance it just saw (acceptance gradient against a short history, its volatility, load and
// throughput factors).  Host code; the verify kernels only consume the resulting k.
#include <math.h>

#include "common.h"

extern "C" {

int32_t ss_depth_init(ss_depth_state *s)
{
    if (!s) return ss::fail(SS_ERR_INVALID_ARG, "state is NULL");
    s->h = 10;
    s->idx = 0;
    for (int j = 0; j < SS_FLOW_MAX; ++j) s->f[j] = 0.0;
    s->d_base = 5.0;
    s->gamma = 5.0;
    s->d_min = 2.0;
    s->d_max = 20.0;
    s->tau_target = 400.0;
    s->tau_recent = 0.0;
    return SS_OK;
}

int32_t ss_depth_update(ss_depth_state *s, double a, double load, double t, double *d_star, int32_t *b_micro,
                        double *t_proj, int32_t *k)
{
    if (!s || !d_star || !b_micro || !t_proj || !k) return ss::fail(SS_ERR_INVALID_ARG, "state or output pointer is NULL");
    if (s->h < 1 || s->h > SS_FLOW_MAX || s->idx < 0 || s->idx >= s->h)
        return ss::fail(SS_ERR_INVALID_ARG, "history length %d / index %d out of range", s->h, s->idx);
    if (a != a || load != load || t != t) return ss::fail(SS_ERR_INVALID_ARG, "NaN metric");
    const int h = s->h;
    double mean = 0.0;
    for (int j = 0; j < h; ++j) mean += s->f[j];
    const double delta = a - mean / h;                       // gradient against the history before the update
    s->f[s->idx] = delta;
    s->idx = (s->idx + 1) % h;
    double mag = 0.0;
    for (int j = 0; j < h; ++j) mag += fabs(s->f[j]);       // volatility, after the update
    mag /= h;
    const double scale = fmax(1.0, s->tau_target / fmax(t, 1.0));
    const double adj = 1.0 - fmin(load, 0.9);
    const double d = s->d_base + (a * mag * s->gamma) * adj * scale;
    const double dc = fmin(fmax(d, s->d_min), s->d_max);
    const double bm = floor(16.0 * 5.0 / dc);
    *d_star = dc;
    *b_micro = bm < 1.0 ? 1 : (bm > 2147483647.0 ? 2147483647 : (int32_t)bm);
    *t_proj = t * (1.0 + a * 0.5);
    s->tau_recent = 0.9 * s->tau_recent + 0.1 * *t_proj;
    const double kr = floor(dc + 0.5);
    *k = kr > (double)SS_MAX_DEPTH ? SS_MAX_DEPTH : (kr < 0.0 ? 0 : (int32_t)kr);
    return SS_OK;
}

}  // extern "C"
