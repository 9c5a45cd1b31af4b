// Host-side granularity controller: the scalar decision formulas of the method,
// evaluated from measured stage throughput / latency.  No device code; it lives
// in the library so that the serving loop that calls fxp_stage_forward and
// fxp_kv_repartition can take its split / merge decisions through the same ABI.
//   Section 6    nu_t = sigma_t / mu_t of the request arrival intervals
//   Section 6.1  Eq. 4: score of every candidate granularity and its arg max
//                Eq. 5: parallel instances of a granularity
//   Section 6.2  multiplexing penalty gamma(CV)
//   Section 7    Eq. 11: scaling granularity from CV and queue length;
//                the SLO constraint on the chosen granularity
#include "../../include/flexstage.h"
#include <math.h>

namespace fxp { int ctl_fail(int code, const char *msg); }

extern "C" {

int fxp_ctl_cv(const double *intervals, int32_t n, double *cv_out)
{
    if (!intervals || !cv_out || n <= 0) return fxp::ctl_fail(FXP_EINVAL, "fxp_ctl_cv: null argument or no samples");
    double mean = 0.0;
    for (int32_t i = 0; i < n; ++i) mean += intervals[i];
    mean /= (double)n;
    if (!(mean > 0.0)) return fxp::ctl_fail(FXP_EINVAL, "fxp_ctl_cv: mean interval must be positive");
    double var = 0.0;
    for (int32_t i = 0; i < n; ++i) { const double d = intervals[i] - mean; var += d * d; }
    *cv_out = sqrt(var / (double)n) / mean;
    return FXP_OK;
}

int fxp_ctl_select_granularity(const fxp_granularity *cand, int32_t n_cand, double cv_now, double alpha, double sigma,
                               double *scores_out, int32_t *best_out)
{
    if (!cand || n_cand <= 0 || !best_out) return fxp::ctl_fail(FXP_EINVAL, "fxp_ctl_select_granularity: null argument or no candidates");
    if (!(alpha >= 0.0 && alpha <= 1.0) || !(sigma > 0.0)) return fxp::ctl_fail(FXP_EINVAL, "fxp_ctl_select_granularity: alpha must be in [0,1] and sigma positive");
    double t_max = 0.0, l_min = INFINITY;
    for (int32_t k = 0; k < n_cand; ++k) {
        if (!(cand[k].throughput > 0.0) || !(cand[k].latency > 0.0)) return fxp::ctl_fail(FXP_EINVAL, "fxp_ctl_select_granularity: throughput and latency must be positive");
        if (cand[k].throughput > t_max) t_max = cand[k].throughput;
        if (cand[k].latency < l_min) l_min = cand[k].latency;
    }
    int32_t best = 0;
    double best_score = -INFINITY;
    for (int32_t k = 0; k < n_cand; ++k) {
        const double bracket = alpha * cand[k].throughput / t_max + (1.0 - alpha) * l_min / cand[k].latency;
        const double score = bracket * exp(-fabs(cv_now - cand[k].cv_opt) / sigma);
        if (scores_out) scores_out[k] = score;
        if (score > best_score) { best_score = score; best = k; }      // ties: the lowest index stays
    }
    *best_out = best;
    return FXP_OK;
}

int64_t fxp_ctl_parallel_instances(double capacity_total, double throughput, double beta1, double beta2, int32_t n_stages)
{
    if (!(throughput > 0.0) || !(capacity_total >= 0.0) || n_stages <= 0 || !(beta1 + beta2 * n_stages > 0.0)) {
        fxp::ctl_fail(FXP_EINVAL, "fxp_ctl_parallel_instances: bad argument");
        return -1;
    }
    const double per_instance = throughput / (beta1 + beta2 * (double)n_stages);
    return (int64_t)floor(capacity_total / per_instance);
}

double fxp_ctl_multiplexing_penalty(double gamma0, double alpha, double cv) { return gamma0 * (1.0 + alpha * cv * cv); }

int32_t fxp_ctl_scaling_granularity(int32_t g_max, double beta, double gamma, double cv, double queue_len, double queue_cap)
{
    if (g_max <= 0 || !(queue_cap > 0.0) || !(queue_len >= 0.0) || !(beta >= 0.0)) {
        fxp::ctl_fail(FXP_EINVAL, "fxp_ctl_scaling_granularity: bad argument");
        return -1;
    }
    const double q_hat = queue_len / queue_cap < 1.0 ? queue_len / queue_cap : 1.0;
    return (int32_t)floor((double)g_max / (1.0 + beta * exp(-gamma * cv * q_hat)));
}

int fxp_ctl_slo_satisfied(double deadline, double init_time, const double *stage_throughput, int32_t n_stages,
                          double queue_len, double requests)
{
    if (!stage_throughput || n_stages <= 0 || !(queue_len > 0.0)) return fxp::ctl_fail(FXP_EINVAL, "fxp_ctl_slo_satisfied: bad argument");
    double sum = 0.0;
    for (int32_t k = 0; k < n_stages; ++k) sum += stage_throughput[k];
    return (deadline - init_time) * sum / queue_len >= requests ? 1 : 0;
}

}  // extern "C"
