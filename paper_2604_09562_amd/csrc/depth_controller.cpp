// Speculation-depth controller (paper Section 3.5): the closed-loop rule that picks each request's draft
// depth from the acceptance it just saw.  Host code; the verify kernels only consume the resulting k.
//
// Built from the section's equations, one helper per quantity:
//   flow state        the ring of the last h acceptance gradients, a_t minus the mean of the ring (Eq. 8, 9)
//   flow magnitude    mean absolute gradient over the ring, the volatility signal
//   throughput factor max(1, tau_target / max(throughput, 1))                                  (Eq. 10)
//   load factor       1 - min(load, 0.9)                                                       (Eq. 11)
//   depth             d_base + a_t * magnitude * gamma * load factor * throughput factor, clipped to
//                     [d_min, d_max]                                                           (Eq. 12, 13)
//   micro-batch       max(1, floor(80 / depth))                                                (Eq. 14)
//   projection        throughput * (1 + a_t / 2), smoothed into tau_recent with weight 0.1     (Eq. 15, 16)
// Reading where the section's equations and its algorithm box differ: the equations scale and project with
// the smoothed tau_recent, the algorithm with the throughput measured in the step just finished; the
// algorithm box (the complete procedure) is followed, tau_recent is the smoothed state only.  The gradient
// is taken against the ring BEFORE it receives the new entry, the magnitude over the ring AFTER it.
#include <math.h>

#include "common.h"

namespace {

struct FlowRing {
    ss_depth_state *s;
    double mean() const
    {
        double sum = 0.0;
        for (int j = 0; j < s->h; ++j) sum += s->f[j];
        return sum / s->h;
    }
    double mean_abs() const
    {
        double sum = 0.0;
        for (int j = 0; j < s->h; ++j) sum += fabs(s->f[j]);
        return sum / s->h;
    }
    void push(double v)
    {
        s->f[s->idx] = v;
        s->idx = s->idx + 1 == s->h ? 0 : s->idx + 1;
    }
};

inline double clip(double x, double lo, double hi) { return fmin(fmax(x, lo), hi); }
inline double throughput_factor(double target, double measured) { return fmax(1.0, target / fmax(measured, 1.0)); }
inline double load_factor(double load) { return 1.0 - fmin(load, 0.9); }

inline int32_t to_int32_floor(double x, int32_t lo, int32_t hi)
{
    const double f = floor(x);
    return f < (double)lo ? lo : (f > (double)hi ? hi : (int32_t)f);
}

}  // namespace

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

int32_t ss_depth_update(ss_depth_state *s, double accept_rate, double load, double throughput, double *d_star,
                        int32_t *b_micro, double *t_proj, int32_t *k)
{
    if (!s || !d_star || !b_micro || !t_proj || !k) return ss::fail(SS_ERR_INVALID_ARG, "state or output pointer is NULL");
    if (s->h < 1 || s->h > SS_FLOW_MAX || s->idx < 0 || s->idx >= s->h)
        return ss::fail(SS_ERR_INVALID_ARG, "history length %d / index %d out of range", s->h, s->idx);
    if (accept_rate != accept_rate || load != load || throughput != throughput)
        return ss::fail(SS_ERR_INVALID_ARG, "NaN metric");

    FlowRing ring{s};
    ring.push(accept_rate - ring.mean());
    const double boost = accept_rate * ring.mean_abs() * s->gamma;
    const double depth = clip(s->d_base + boost * load_factor(load) * throughput_factor(s->tau_target, throughput),
                              s->d_min, s->d_max);
    const double projected = throughput * (1.0 + accept_rate * 0.5);
    s->tau_recent = 0.9 * s->tau_recent + 0.1 * projected;

    *d_star = depth;
    *b_micro = to_int32_floor(16.0 * 5.0 / depth, 1, 2147483647);
    *t_proj = projected;
    *k = to_int32_floor(depth + 0.5, 0, SS_MAX_DEPTH);   // nearest integer depth, halves up
    return SS_OK;
}

}  // extern "C"
