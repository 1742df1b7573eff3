// Adaptive control of the inexactness (paper section 3.2.3): a host-side policy over the residual
// norms that mgrit_forward / mgrit_adjoint export.  The convergence factor of iteration k is the
// ratio of consecutive fine-level residual norms; every `probe_every` batches the iteration
// count is doubled for one batch and the factor of its final iteration is looked at; a factor
// above the threshold (1 in the paper) means the iterations are no longer effective, and the
// policy either raises the iteration count or switches to serial propagation.  No GPU work here.
#include <math.h>
#include <string.h>

#include "../../include/mgrit.h"

extern "C" {

int mgrit_indicator_init(mgrit_indicator* s, int iters, int probe_every, int mitigation, int max_iters,
                         float threshold) {
  if (!s || iters < 1 || probe_every < 0 || max_iters < 0 || !isfinite(threshold) || threshold <= 0.f)
    return MGRIT_INVALID_ARG;
  if (mitigation != MGRIT_MITIGATE_SERIAL && mitigation != MGRIT_MITIGATE_MORE_ITERATIONS) return MGRIT_INVALID_ARG;
  memset(s, 0, sizeof(*s));
  s->iters = iters;
  s->probe_every = probe_every;
  s->mitigation = mitigation;
  s->max_iters = max_iters;
  s->threshold = threshold;
  s->last_factor = -1.f;
  return MGRIT_OK;
}

int mgrit_indicator_begin_batch(mgrit_indicator* s) {
  if (!s) return MGRIT_INVALID_ARG;
  s->probing = 0;
  if (s->serial) return 0;
  if (s->probe_every > 0 && (s->batch + 1) % s->probe_every == 0) {
    s->probing = 1;
    return 2 * s->iters;
  }
  return s->iters;
}

int mgrit_indicator_end_batch(mgrit_indicator* s, const float* resnorm, int n) {
  if (!s || n < 0 || (n > 0 && !resnorm)) return MGRIT_INVALID_ARG;
  s->batch += 1;
  const int was_probe = s->probing;
  s->probing = 0;
  if (!was_probe || s->serial) return 0;
  if (n < 2) return 0;                      // a factor needs two residuals
  const float prev = resnorm[n - 2], last = resnorm[n - 1];
  // a vanished or non-finite residual: converged (factor 0) or blown up (failing)
  float factor;
  if (!isfinite(last) || !isfinite(prev)) factor = INFINITY;
  else if (prev == 0.f) factor = last == 0.f ? 0.f : INFINITY;
  else factor = last / prev;
  s->last_factor = factor;
  if (!(factor > s->threshold)) return 0;
  s->failures += 1;
  if (s->mitigation == MGRIT_MITIGATE_MORE_ITERATIONS && 2 * (int64_t)s->iters <= s->max_iters) {
    s->iters *= 2;
    return 1;
  }
  s->serial = 1;
  return 1;
}

}  // extern "C"
