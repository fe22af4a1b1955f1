// Automatic Graph Parallelism selection (paper Section 4.3, Algorithm 3; Eq. 7-8 for the runtime
// model).  Host arithmetic only: the coefficients beta_c(i) must be measured on a multi-GPU
// system and are passed in.
#include "gta_internal.h"

#include <math.h>

using namespace gta;

extern "C" GTA_API gta_status gta_agp_select(double t_iter1, int64_t n_nodes, const gta_agp_sample* samples,
                                             int n_samples, int max_gpus, int* strategy, int* gpus,
                                             double* est_t_iter) {
    if (!strategy || !gpus) return fail(GTA_ERR_INVALID_ARG, "null output pointer");
    if (!(t_iter1 > 0.0) || n_nodes <= 0) return fail(GTA_ERR_INVALID_ARG, "t_iter(1) and N must be positive");
    if (n_samples < 0 || (n_samples > 0 && !samples)) return fail(GTA_ERR_INVALID_ARG, "bad sample table");
    const double k = t_iter1 / (double)n_nodes;   // k = t_iter(1) / N
    *strategy = -1;                               // no admissible entry: stay on one GPU
    *gpus = 1;
    double best = INFINITY, best_beta = 0.0;
    for (int i = 0; i < n_samples; ++i) {
        const gta_agp_sample& s = samples[i];
        if (s.gpus < 2 || s.gpus > max_gpus) continue;
        if (!(s.beta >= 0.0)) return fail(GTA_ERR_INVALID_ARG, "beta must be non-negative (sample %d)", i);
        const double term = (double)s.gpus * s.beta / (double)(s.gpus - 1);   // s*beta_c(s)/(s-1)
        // smallest admissible term; ties go to fewer GPUs, then to the entry listed first
        if (term <= k && (term < best || (term == best && s.gpus < *gpus))) {
            best = term;
            best_beta = s.beta;
            *strategy = s.strategy;
            *gpus = s.gpus;
        }
    }
    if (est_t_iter)   // t_iter(s) = alpha(1) E / s + beta_c(s) N with alpha(1) E = t_iter(1)
        *est_t_iter = *gpus == 1 ? t_iter1 : t_iter1 / (double)*gpus + best_beta * (double)n_nodes;
    return GTA_OK;
}
