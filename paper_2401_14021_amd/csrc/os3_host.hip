// Optimal speculation stride scheduler (Section 4; parameter estimation in Appendix A.2).
// Host-only scalar code: the serving loop needs the stride on the host to size its next batch.
//
//   gamma estimate   maximum-likelihood estimate of the per-step speculation accuracy from
//                    the last w verification steps, truncated at gamma_max
//   objective        expected number of verified documents per unit time for a stride s,
//                    with synchronous or asynchronous verification
//   stride           the s in [1, s_max] that maximises the objective (smallest s on ties)
//   latency          a and b as the mean of the most recent measurements
//   next stride      the three combined: what the serving loop calls after each verification
#include "../../include/ralm.h"

#include <cmath>

extern "C" {

double ralm_os3_gamma(const int32_t *strides, const int32_t *matched, int32_t w, double gamma_max)
{
    if (!strides || !matched || w <= 0) return 0.0;
    double sum_m = 0.0, fails = 0.0;
    for (int32_t t = 0; t < w; ++t) {
        const int32_t s = strides[t] < 0 ? 0 : strides[t];
        int32_t m = matched[t] < 0 ? 0 : matched[t];
        if (m > s) m = s;
        sum_m += (double)m;
        if (m < s) fails += 1.0;
    }
    double g = sum_m + fails > 0.0 ? sum_m / (sum_m + fails) : 0.0;
    if (g > gamma_max) g = gamma_max;
    if (g < 0.0) g = 0.0;
    return g;
}

// expected verified documents sum_{i<s} gamma^i, accumulated term by term, and gamma^s
static void os3_expectation(double gamma, int32_t s, double *expected, double *gamma_s)
{
    double e = 0.0, gi = 1.0;
    for (int32_t i = 0; i < s; ++i) {
        e += gi;
        gi *= gamma;
    }
    *expected = e;
    *gamma_s = gi;
}

double ralm_os3_objective(double gamma, double a, double b, int32_t s, int32_t async)
{
    if (s < 1 || !(a >= 0.0) || !(b >= 0.0) || !(gamma >= 0.0) || !(gamma <= 1.0)) return std::nan("");
    double expected, gs;
    os3_expectation(gamma, s, &expected, &gs);
    const double sync_latency = (double)s * a + b;
    double latency = sync_latency;
    if (async) {
        const double overlapped = (double)(s - 1) * a + (a > b ? a : b);
        latency = gs * overlapped + (1.0 - gs) * sync_latency;
    }
    return expected / latency;
}

double ralm_os3_latency(const double *samples, int32_t n)
{
    if (!samples || n <= 0) return 0.0;
    double sum = 0.0;
    for (int32_t i = 0; i < n; ++i) sum += samples[i];
    return sum / (double)n;
}

int32_t ralm_os3_stride(double gamma, double a, double b, int32_t s_max, int32_t async)
{
    if (s_max < 1) return 1;
    int32_t best = 1;
    double best_v = ralm_os3_objective(gamma, a, b, 1, async);
    for (int32_t s = 2; s <= s_max; ++s) {
        const double v = ralm_os3_objective(gamma, a, b, s, async);
        if (v > best_v) {
            best_v = v;
            best = s;
        }
    }
    return best;
}

int32_t ralm_os3_next_stride(const int32_t *strides, const int32_t *matched, int32_t w, const double *a_samples,
                             int32_t n_a, const double *b_samples, int32_t n_b, double gamma_max, int32_t s_max,
                             int32_t async)
{
    if (w <= 0 || n_a <= 0 || n_b <= 0) return 1;   // no history yet: the paper starts with s = 1
    const double gamma = ralm_os3_gamma(strides, matched, w, gamma_max);
    return ralm_os3_stride(gamma, ralm_os3_latency(a_samples, n_a), ralm_os3_latency(b_samples, n_b), s_max, async);
}

}  // extern "C"
