// Metric-aware worker selection: score the lanes that are neither stale nor overloaded and take the
// best, else fall back to the shortest queue.  Host code; it decides where a request's verify steps run.
#include "common.h"

extern "C" int32_t ss_route_select(const ss_worker_metrics *workers, int32_t n, const double *alpha, double tau,
                                   double q_max, int32_t *chosen)
{
    if (!workers || !chosen || n <= 0) return ss::fail(SS_ERR_INVALID_ARG, "workers/chosen NULL or n <= 0");
    if (!(q_max > 0.0)) return ss::fail(SS_ERR_INVALID_ARG, "q_max must be positive");
    static const double kAlpha[4] = {0.4, 0.1, 0.3, 0.2};
    const double *al = alpha ? alpha : kAlpha;
    if (!(tau > 0.0)) tau = 0.85;
    int best = -1;
    double best_score = 0.0;
    for (int i = 0; i < n; ++i) {
        const ss_worker_metrics &m = workers[i];
        const double fill = (double)m.queue_depth / q_max;
        if (m.stale || m.mem + 2.0 * fill > tau) continue;
        const double q = fill < 1.0 ? fill : 1.0;
        const double s = al[0] * m.cache_hit + al[1] * (1.0 - m.mem) + al[2] * (1.0 - q) + al[3] * (1.0 - m.load);
        if (best < 0 || s > best_score) {
            best = i;
            best_score = s;
        }
    }
    if (best < 0) {   // every lane saturated or stale: the shortest queue
        best = 0;
        for (int i = 1; i < n; ++i)
            if (workers[i].queue_depth < workers[best].queue_depth) best = i;
    }
    *chosen = best;
    return SS_OK;
}
