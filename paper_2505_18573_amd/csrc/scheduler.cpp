// Host-side temperature scheduler of arXiv 2505.18573: Eq. 4 (closed-form update
// that scales the entropy by alpha) with the cosine-annealed entropy target of
// Eq. 5, and Appendix A's form of the same update with a measured logit gap.
// Pure double-precision scalar code, no GPU work.
#include <cmath>
#include <cstdint>

#include "../../include/e3.h"

namespace {

bool positive_finite(double x) { return std::isfinite(x) && x > 0.0; }

bool common_args_ok(double tau_t, double H_t, double H_init, double eta, double tau_min, double tau_max)
{
    return positive_finite(tau_t) && positive_finite(H_t) && positive_finite(H_init) &&
           eta >= 0.0 && eta <= 1.0 && tau_min >= 0.0 && tau_max >= tau_min;
}

// Entropy level the scheduler steers towards at step t (Eq. 5; constant H_init
// before t_anneal or when annealing is off).
double target_entropy(double H_init, int64_t t, int64_t t_anneal, int64_t t_max, double eta)
{
    if (t_anneal < 0 || t < t_anneal) return H_init;
    double progress = 1.0;
    if (t_max > t_anneal) {
        progress = static_cast<double>(t - t_anneal) / static_cast<double>(t_max - t_anneal);
        progress = std::fmin(std::fmax(progress, 0.0), 1.0);
    }
    const double cosine = 0.5 * (1.0 + std::cos(M_PI * progress));
    return H_init * (eta + (1.0 - eta) * cosine);
}

// tau' = tau (1 + tau ln(alpha) / gap), alpha = H_target / H_t, then the clamp.
int apply_update(double tau_t, double H_t, double H_target, double gap, double tau_min,
                 double tau_max, double* tau_next_out, double* H_target_out)
{
    if (!(H_target > 0.0)) return E3_ERR_VALUE;
    const double factor = 1.0 + tau_t * std::log(H_target / H_t) / gap;
    double tau_next = tau_t * factor;
    if (!(tau_next > 0.0) && !(tau_min > 0.0)) return E3_ERR_VALUE;
    tau_next = std::fmin(std::fmax(tau_next, tau_min), tau_max);
    *tau_next_out = tau_next;
    if (H_target_out != nullptr) *H_target_out = H_target;
    return E3_OK;
}

}  // namespace

extern "C" int e3_temperature_update(double tau_t, double H_t, double H_init, int64_t vocab,
                                     int64_t t, int64_t t_anneal, int64_t t_max, double eta,
                                     double tau_min, double tau_max,
                                     double* tau_next_out, double* H_target_out)
{
    if (tau_next_out == nullptr) return E3_ERR_NULL;
    if (!common_args_ok(tau_t, H_t, H_init, eta, tau_min, tau_max)) return E3_ERR_VALUE;
    if (vocab < 3) return E3_ERR_VALUE;                       // ln ln|V| must exist and be > 0
    const double ln_v = std::log(static_cast<double>(vocab));
    const double gap = ln_v + std::log(ln_v);                 // Appendix A: Delta ~ ln N + ln ln N
    return apply_update(tau_t, H_t, target_entropy(H_init, t, t_anneal, t_max, eta), gap,
                        tau_min, tau_max, tau_next_out, H_target_out);
}

extern "C" int e3_temperature_update_gap(double tau_t, double H_t, double H_init, double gap,
                                         int64_t t, int64_t t_anneal, int64_t t_max, double eta,
                                         double tau_min, double tau_max,
                                         double* tau_next_out, double* H_target_out)
{
    if (tau_next_out == nullptr) return E3_ERR_NULL;
    if (!common_args_ok(tau_t, H_t, H_init, eta, tau_min, tau_max) || !positive_finite(gap))
        return E3_ERR_VALUE;
    return apply_update(tau_t, H_t, target_entropy(H_init, t, t_anneal, t_max, eta), gap,
                        tau_min, tau_max, tau_next_out, H_target_out);
}
