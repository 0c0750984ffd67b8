// Host-only part of the library: the communication-time model of Section V ("Solution") and
// Algorithm 1, which picks schedule S1 or S2 from fitted alpha-beta constants.  No GPU work.
#include <math.h>
#include <stdint.h>

#include "parm_moe.h"

extern "C" int moe_alpha_beta_fit(const double* x, const double* t, int n, double* alpha, double* beta) {
  if (x == nullptr || t == nullptr || alpha == nullptr || beta == nullptr) return MOE_ENULL;
  if (n < 2) return MOE_EINVAL;
  // two passes: the sizes span many orders of magnitude, so the sums are taken about the means
  double mx = 0.0, mt = 0.0;
  for (int i = 0; i < n; ++i) { mx += x[i]; mt += t[i]; }
  mx /= n; mt /= n;
  double sxx = 0.0, sxt = 0.0;
  for (int i = 0; i < n; ++i) {
    const double dx = x[i] - mx;
    sxx += dx * dx;
    sxt += dx * (t[i] - mt);
  }
  if (!(sxx > 0.0) || !isfinite(sxx) || !isfinite(sxt)) return MOE_EINVAL;
  *beta = sxt / sxx;
  *alpha = mt - *beta * mx;
  return MOE_OK;
}

extern "C" int moe_choose_schedule(double alpha_ag_mp, double beta_ag_mp, double alpha_a2a, double beta_a2a,
                                   double alpha_o, double beta_o, int64_t B, int64_t L, int E, int M, int k, double f,
                                   int n_esp, int n_mp, double* t_d1, double* t_d2) {
  if (B < 1 || L < 1 || E < 1 || M < 1 || k < 1 || n_esp < 1 || n_mp < 1 || !(f > 0.0) || !isfinite(f)) return MOE_EINVAL;
  const double x = (double)B * (double)L * (double)M;        // MP-AllGather of the layer output (S1)
  const double T = (double)k * f * (double)B * (double)L / (double)E;
  const double y = (double)E * T * (double)M * (double)n_esp;
  const double d1 = 2.0 * (alpha_a2a + beta_a2a * y / n_mp) + alpha_ag_mp + beta_ag_mp * x;
  const double d2 = alpha_a2a + beta_a2a * y / n_mp + alpha_o + beta_o * y;
  if (t_d1) *t_d1 = d1;
  if (t_d2) *t_d2 = d2;
  return d1 <= d2 ? 1 : 2;
}
