// Dynamic dropout-ratio tuning (Section 5.3, Eq. 4-6): host-only scalar code.
//
// The prune possibility over the epochs follows a skew-normal curve
//   f_Y(y) = (2 / sigma) phi((y - mu) / sigma) Phi(lambda (y - mu) / sigma)              (Eq. 4)
// whose mu and sigma follow from the mean and the variance of the curve:
//   E(Y) = mu + mu0 sigma,  mu0 = sqrt(2/pi) lambda / sqrt(1 + lambda^2)                 (Eq. 5)
//   D(Y) = (1 - mu0^2) sigma^2                                                            (Eq. 6)
// Epoch e of n sits at the normalised time (e + 1/2) / n; its possibility is proportional to the
// curve there, scaled so that the average over the run is the total prune possibility, and
// clipped to [0, p_max].
#include <math.h>

#include "common.hpp"

using namespace ard;

static double skew_mu0(double lam) { return sqrt(2.0 / M_PI) * lam / sqrt(1.0 + lam * lam); }

extern "C" int32_t ard_skew_normal_params(double mean, double var, double lambda, double* mu, double* sigma) {
  if (!mu || !sigma) return fail(ARD_EINVAL, "null output pointer");
  if (!(var > 0.0) || !isfinite(mean) || !isfinite(lambda)) return fail(ARD_EINVAL, "variance must be positive, mean and lambda finite");
  const double m0 = skew_mu0(lambda);
  *sigma = sqrt(var / (1.0 - m0 * m0));
  *mu = mean - m0 * *sigma;
  return ARD_OK;
}

extern "C" double ard_skew_normal_pdf(double y, double mu, double sigma, double lambda) {
  const double z = (y - mu) / sigma;
  const double phi = exp(-0.5 * z * z) / sqrt(2.0 * M_PI);
  const double Phi = 0.5 * erfc(-lambda * z / sqrt(2.0));  // (erfc keeps the lower tail)
  return 2.0 / sigma * phi * Phi;
}

extern "C" int32_t ard_prune_schedule(int32_t n_epochs, double total, double mean, double var, double lambda, double p_max,
                                      double* p_out) {
  if (n_epochs < 1) return fail(ARD_ESHAPE, "n_epochs must be positive (got %d)", n_epochs);
  if (!p_out) return fail(ARD_EINVAL, "null output pointer");
  if (!(total >= 0.0 && total <= 1.0) || !(p_max >= 0.0 && p_max <= 1.0))
    return fail(ARD_EINVAL, "total and p_max must lie in [0, 1] (got %g, %g)", total, p_max);
  double mu, sigma;
  if (int32_t st = ard_skew_normal_params(mean, var, lambda, &mu, &sigma)) return st;
  double sum = 0.0;
  for (int e = 0; e < n_epochs; ++e) {
    p_out[e] = ard_skew_normal_pdf((e + 0.5) / n_epochs, mu, sigma, lambda);
    sum += p_out[e];
  }
  const double avg = sum / n_epochs;
  if (!(avg > 0.0)) return fail(ARD_EINVAL, "the curve vanishes on every epoch (mean %g, variance %g)", mean, var);
  for (int e = 0; e < n_epochs; ++e) {
    const double p = total * p_out[e] / avg;
    p_out[e] = p < 0.0 ? 0.0 : (p > p_max ? p_max : p);
  }
  return ARD_OK;
}
