// Reduction schedule from the appendix "Theoretical FLOPs Calculation": host arithmetic only.
// Layer cost 4 n D^2 + 2 n^2 D + 2 n D F over the tokens the layer sees, the method's own
// work N^2 + 2N + N^S (N^T + 2D + 1) + D (doubled first bracket for FiCoCo-L) in every reducing
// layer; the smallest uniform per-layer discard count within the budget is found by trying
// the counts in ascending order.
#include <cmath>

#include "../../include/ficoco.h"

namespace {

double layer_cost(double tokens, double D, double F) {
  return 4.0 * tokens * D * D + 2.0 * tokens * tokens * D + 2.0 * tokens * D * F;
}

double step_cost(bool L, double n, double s, double D) {
  const double first = n * n + 2.0 * n;
  return (L ? 2.0 * first : first) + s * ((n - s) + 2.0 * D + 1.0) + D;
}

// Cost of discarding `s` tokens per layer from start_layer on; fills n_discard when given.
double total_cost(const ficoco_schedule_problem& p, int s, int32_t* n_discard) {
  const bool L = p.variant == FICOCO_VARIANT_L;
  const double D = p.D, F = p.F, M = L ? p.M : 0;
  int n = p.N;
  double total = 0.0;
  for (int l = 0; l < p.layers; ++l) {
    int drop = 0;
    if (l >= p.start_layer) {
      drop = n - s >= p.min_keep ? s : n - p.min_keep;
      if (drop < 0) drop = 0;
    }
    if (drop > 0) total += step_cost(L, n, drop, D);
    n -= drop;
    total += layer_cost((double)n + M, D, F);
    if (n_discard) n_discard[l] = drop;
  }
  return total;
}

}  // namespace

extern "C" int ficoco_schedule(const ficoco_schedule_problem* p, int32_t* n_discard, double* total_flops) {
  if (!p || !n_discard) return FICOCO_EINVAL;
  if ((p->variant != FICOCO_VARIANT_V && p->variant != FICOCO_VARIANT_L) || p->layers < 1 || p->start_layer < 0 ||
      p->N < 1 || p->M < 0 || p->D < 1 || p->F < 1 || p->min_keep < 1 || p->min_keep > p->N ||
      !(p->budget_flops > 0.0))
    return FICOCO_EINVAL;
  const int hi = p->N - p->min_keep;          // the strongest per-layer count worth considering
  int lo = 0;
  while (lo <= hi && total_cost(*p, lo, nullptr) > p->budget_flops) ++lo;   // smallest count within the budget
  if (lo > hi) {
    const double t = total_cost(*p, hi, n_discard);
    if (total_flops) *total_flops = t;
    return FICOCO_EUNSUPPORTED;
  }
  const double t = total_cost(*p, lo, n_discard);
  if (total_flops) *total_flops = t;
  return FICOCO_OK;
}
