// Host-side scheduling arithmetic around the training step: key-frame striding (Algorithm 2 of
// the paper) and the analytic traffic / throughput bounds of Section 4.4 (Eqs. 2-14).  No GPU
// work; plain double precision.
#include <math.h>

#include "../../include/shadowtutor_head.h"

extern "C" {

double st_next_stride(double stride, double metric, double threshold, double min_stride, double max_stride)
{
    if (!(threshold > 0.0 && threshold < 1.0) || !(min_stride <= max_stride) || isnan(stride) || isnan(metric))
        return NAN;
    // ratio of the next stride to this one: two straight lines meeting in (THRESHOLD, 1)
    const double below = metric / threshold;                                   // through (0, 0)
    const double above = 1.0 + (metric - threshold) / (1.0 - threshold);       // through (1, 2)
    const double next = stride * (metric < threshold ? below : above);
    return next < min_stride ? min_stride : (next > max_stride ? max_stride : next);
}

int st_schedule_bounds(const st_schedule_params* p, st_schedule_bounds_out* out)
{
    if (!p || !out) return ST_ERR_NULL;
    const double v[] = {p->t_si, p->t_sd, p->t_ti, p->t_net, p->s_net, p->min_stride, p->max_stride, p->max_updates};
    for (double x : v)
        if (!isfinite(x) || x < 0.0) return ST_ERR_ARG;
    if (p->min_stride <= 0.0 || p->max_stride < p->min_stride || p->t_si <= 0.0) return ST_ERR_ARG;
    const double infer_min = p->min_stride * p->t_si;      // client inference over the waiting window
    const double round_trip = p->t_net + p->t_ti;          // key frame up, teacher, update down
    out->t_c_lower = infer_min > round_trip ? infer_min : round_trip;          // Eq. 2, full overlap
    out->t_c_upper = infer_min + round_trip;                                   // Eq. 2, no overlap
    const double train_max = p->max_updates * p->t_sd;
    // rarest key frames, longest training, no overlap  /  most frequent key frames, no training, full overlap
    out->traffic_lower = p->s_net / (p->max_stride * p->t_si + train_max + round_trip);             // Eq. 8
    out->traffic_upper = p->s_net / out->t_c_lower;                                                 // Eq. 12
    out->throughput_lower = p->min_stride / (out->t_c_upper + train_max);                           // Eq. 13
    out->throughput_upper = p->max_stride / ((p->max_stride - p->min_stride) * p->t_si + out->t_c_lower);  // Eq. 14
    return ST_OK;
}

double st_schedule_total_time(const st_schedule_params* p, double n_frames, double n_distill_steps,
                              double n_key_frames, double t_c)
{
    if (!p) return NAN;
    // Eq. 3: frames outside the waiting windows, all distillation steps, one window per key frame
    return (n_frames - n_key_frames * p->min_stride) * p->t_si + n_distill_steps * p->t_sd + n_key_frames * t_c;
}

}  // extern "C"
