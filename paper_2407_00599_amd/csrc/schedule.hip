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

namespace {

// alpha-beta model of one collective (Section V-A): start-up time plus time per element
struct Collective {
  double alpha, beta;
  double time(double elements) const { return alpha + beta * elements; }
};

}  // namespace

// Section V-B compares what the two schedules add on top of their common work.  Both move the
// dispatched tensor, E * T * M * N_ESP elements of which each MP rank carries 1 / N_MP, through the
// EP&ESP-AlltoAll.  S1 does so twice and then gathers the B * L * M layer output over the MP group;
// S2 does it once on its own and once overlapped with its MP-AllGather (the fitted "overlapped"
// collective, which sees the whole dispatched tensor).  Algorithm 1 picks the smaller total, S1 on a tie.
extern "C" int moe_choose_schedule(double alpha_ag_mp, double beta_ag_mp, double alpha_a2a, double beta_a2a,
                                   double alpha_o, double beta_o, int64_t B, int64_t L, int E, int M, int k, double f,
                                   int n_esp, int n_mp, double* t_d1, double* t_d2) {
  if (B < 1 || L < 1 || E < 1 || M < 1 || k < 1 || n_esp < 1 || n_mp < 1 || !(f > 0.0) || !isfinite(f)) return MOE_EINVAL;
  const Collective ag_mp{alpha_ag_mp, beta_ag_mp}, a2a{alpha_a2a, beta_a2a}, overlapped{alpha_o, beta_o};
  const double tokens = (double)B * (double)L;
  const double capacity = (double)k * f * tokens / (double)E;                  // T of Section II-A, not rounded
  const double dispatched = (double)E * capacity * (double)M * (double)n_esp;   // elements of the dispatched tensor
  const double a2a_once = a2a.time(dispatched / n_mp);
  const double s1 = 2.0 * a2a_once + ag_mp.time(tokens * (double)M);
  const double s2 = a2a_once + overlapped.time(dispatched);
  if (t_d1) *t_d1 = s1;
  if (t_d2) *t_d2 = s2;
  return s1 <= s2 ? 1 : 2;
}
