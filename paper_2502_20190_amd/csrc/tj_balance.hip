// Production / consumption balance (Section 3.3 of the paper, Eq. 2-3; Appendix D.1), reduced
// to what one device-resident buffer can steer: the staleness gate of tj_sample.
//
// Serial execution with a buffer of N_s transitions and batches of B_s has the stable staleness
// ratio P = B_s / N_s (Eq. 2): a batch is 1/k of the pool, k = N_s / B_s (the Lag-k setting of
// Appendix D.1).  Asynchronously, the learner consumes TR_L transitions per second in batches of
// B, i.e. TR_L / B policy versions per second, while the actors add TR_A transitions per second:
// R = B * TR_A / TR_L transitions carry each version tag.  A gate of max_staleness keeps
// v = max_staleness + 1 versions eligible, a pool of N_s' = v * R transitions, and the constraint
// N_c / N_s' = P with N_c = B per step gives v = k * TR_L / TR_A, rounded to the nearest whole
// number of versions (at least one).  Host arithmetic only.
#include "tj_common.h"
#include <math.h>

extern "C" int tj_balance_plan(const tj_balance_in *in, tj_balance_out *out)
{
    if (!in || !out) return TJ_ERR_INVALID_ARG;
    if (!(in->tr_learner > 0.0) || !(in->tr_actor > 0.0) || !isfinite(in->tr_learner) || !isfinite(in->tr_actor))
        return TJ_ERR_INVALID_ARG;
    if (in->batch == 0 || in->serial_batch == 0 || in->serial_buffer < in->serial_batch || in->capacity == 0)
        return TJ_ERR_INVALID_ARG;
    const double k = (double)in->serial_buffer / (double)in->serial_batch;
    const double rows = (double)in->batch * in->tr_actor / in->tr_learner;
    double v = floor(k * in->tr_learner / in->tr_actor + 0.5);
    if (v < 1.0) v = 1.0;
    out->window_exceeds_capacity = 0;
    if (v * rows > (double)in->capacity) {   // the ring cannot hold that many versions
        out->window_exceeds_capacity = 1;
        v = floor((double)in->capacity / rows);
        if (v < 1.0) v = 1.0;
    }
    out->max_staleness = (int64_t)v - 1;
    out->rows_per_version = rows;
    out->window = v * rows;
    out->ratio = (double)in->batch / out->window;
    out->target_ratio = 1.0 / k;
    out->throughput = in->tr_learner < in->tr_actor ? in->tr_learner : in->tr_actor;
    const double rel = fabs(in->tr_learner - in->tr_actor) / (in->tr_learner > in->tr_actor ? in->tr_learner : in->tr_actor);
    out->bottleneck = rel <= 0.05 ? 0 : (in->tr_actor < in->tr_learner ? 1 : 2);
    return TJ_OK;
}
