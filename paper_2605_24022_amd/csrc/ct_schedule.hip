// Hardware-aware choice of the recomputation ratio (Sec. 4.3): the per-layer latency model
// (Eq. 9), its crossover point (Eq. 11) and the warm-started golden-section search over measured
// latencies (Alg. 1).  Host code only; the latencies come from the caller's callback.
#include <math.h>

#include "ct_internal.h"

using namespace ct;

extern "C" {

double ct_layer_latency_model(double r, double n_tokens, double t_c, double t_i, double t_o) {
  const double compute = r * n_tokens * t_c;
  const double transfer = (1.0 - r) * n_tokens * t_i;
  return (compute > transfer ? compute : transfer) + t_o;
}

double ct_ratio_prior(double t_c, double t_i, double r_min, double r_max) {
  double r0 = (t_c + t_i) > 0.0 ? t_i / (t_c + t_i) : r_min;
  if (r0 < r_min) r0 = r_min;
  if (r0 > r_max) r0 = r_max;
  return r0;
}

ct_status ct_ratio_search(ct_ttft_fn eval, void* user, double r0, double r_min, double r_max, double eps,
                          int32_t max_evals, double* r_star, int32_t* n_evals) {
  if (eval == nullptr || r_star == nullptr) return fail(CT_ERR_NULL, "eval and r_star must be non-NULL");
  if (!(r_min <= r_max) || !(r_min >= 0.0) || !(r_max <= 1.0))
    return fail(CT_ERR_RATIO, "bounds [%g, %g] must satisfy 0 <= r_min <= r_max <= 1", r_min, r_max);
  if (!(eps > 0.0)) return fail(CT_ERR_SHAPE, "eps must be positive");
  if (max_evals < 2) return fail(CT_ERR_SHAPE, "max_evals %d: the search needs at least two evaluations", max_evals);
  if (r0 < r_min) r0 = r_min;
  if (r0 > r_max) r0 = r_max;
  double a = r_min, b = r_max;
  const double phi = (sqrt(5.0) - 1.0) / 2.0;
  int32_t evals = 0;
  if (b - a < eps) {   // nothing to search
    *r_star = 0.5 * (a + b);
    if (n_evals != nullptr) *n_evals = 0;
    return CT_OK;
  }
  // warm start: the roofline prior takes the place of the probe on its side of the interval; a
  // prior on a bound is moved inside by a hundredth of the interval (a probe on the bound would
  // say nothing about the interior)
  const double inset = 0.01 * (b - a);
  double x1, x2;
  if (r0 <= 0.5 * (a + b)) {
    x1 = r0 < a + inset ? a + inset : r0;
    x2 = a + phi * (b - a);
  } else {
    x1 = b - phi * (b - a);
    x2 = r0 > b - inset ? b - inset : r0;
  }
  double f1 = eval(x1, user), f2 = eval(x2, user);
  evals = 2;
  while (fabs(b - a) >= eps && evals < max_evals) {
    // shrink onto the side of the better probe; that probe survives as an interior point
    double xs, fs;
    if (f1 < f2) { b = x2; xs = x1; fs = f1; }
    else         { a = x1; xs = x2; fs = f2; }
    // the new probe is the golden-section point of the larger part next to the survivor: with
    // the survivor at a golden point of [a, b] this is the listing's b - phi (b - a) or
    // a + phi (b - a); after an off-golden warm start the listing's point can coincide with
    // the survivor or pass it, this one cannot
    if (xs - a > b - xs) {
      x2 = xs; f2 = fs;
      x1 = xs - (1.0 - phi) * (xs - a);
      f1 = eval(x1, user);
    } else {
      x1 = xs; f1 = fs;
      x2 = xs + (1.0 - phi) * (b - xs);
      f2 = eval(x2, user);
    }
    ++evals;
  }
  *r_star = 0.5 * (a + b);
  if (n_evals != nullptr) *n_evals = evals;
  return CT_OK;
}

}  // extern "C"
