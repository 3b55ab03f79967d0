// Measured-time batch-size controller: procedure getBsz of Algorithm 1 with the stability kit
// of section "Control Stability for Dynamic-Batching" (exponential smoothing of the compute
// time, dead-band of equation omnibszdeadbandlimit, bounds, and the fixed-global-batch rule of
// equation dynbszGlobalBFixed in its multiplicative reading or as printed).
//
// The paper computes with real numbers.  Here every quantity is an IEEE double and every
// expression is a single operation per statement, in a fixed order, so that the results
// (which decide integers) repeat bit for bit on any conforming host; this file is compiled
// without floating-point contraction.  Integers are made by round-half-even (no global rule,
// or the printed rule) or by largest-remainder apportionment of floor(b* * 2^20) weights
// (global batch fixed).
#include <cmath>
#include <new>

#include "common.h"

struct omni_dyn {
  int32_t K, B, b_min, b_max, rule;
  double deadband, alpha;
  int32_t b[OMNI_MAX_WORKERS];
  double ewma[OMNI_MAX_WORKERS];
  int64_t nobs;
};

namespace {

inline double clampd(double x, double lo, double hi) { return x < lo ? lo : (x > hi ? hi : x); }

void write_out(const omni_dyn* c, int32_t* b_out, int32_t* off_out) {
  int64_t acc = 0;
  if (off_out) off_out[0] = 0;
  for (int k = 0; k < c->K; ++k) {
    if (b_out) b_out[k] = c->b[k];
    acc += c->b[k];
    if (off_out) off_out[k + 1] = (int32_t)acc;
  }
}

}  // namespace

extern "C" {

int omni_dyn_create(int32_t K, int32_t B, int32_t b_min, int32_t b_max, double deadband, double ewma_alpha,
                    int32_t global_rule, const int32_t* b_init, omni_dyn** out) {
  using omni::fail;
  if (!out) return fail(OMNI_EINVAL, "omni_dyn_create: out is NULL");
  *out = nullptr;
  if (K < 1 || B < K) return fail(OMNI_EINVAL, "omni_dyn_create: need 1 <= K <= B (K=%d B=%d)", K, B);
  if (K > OMNI_MAX_WORKERS) return fail(OMNI_ECAPACITY, "omni_dyn_create: K=%d exceeds %d", K, OMNI_MAX_WORKERS);
  if (b_max == 0) b_max = B;
  if (b_min < 1 || b_max < b_min) return fail(OMNI_EINVAL, "omni_dyn_create: bad bounds [%d,%d]", b_min, b_max);
  if (!(deadband >= 0.0 && deadband < 1.0)) return fail(OMNI_EINVAL, "omni_dyn_create: dead-band must lie in [0, 1)");
  if (!(ewma_alpha > 0.0 && ewma_alpha <= 1.0)) return fail(OMNI_EINVAL, "omni_dyn_create: alpha must lie in (0, 1]");
  if (global_rule < OMNI_RULE_NONE || global_rule > OMNI_RULE_ADDITIVE)
    return fail(OMNI_EINVAL, "omni_dyn_create: unknown global rule %d", global_rule);
  omni_dyn* c = new (std::nothrow) omni_dyn();
  if (!c) return fail(OMNI_EINVAL, "omni_dyn_create: out of host memory");
  c->K = K; c->B = B; c->b_min = b_min; c->b_max = b_max; c->rule = global_rule;
  c->deadband = deadband; c->alpha = ewma_alpha; c->nobs = 0;
  if (b_init) {
    for (int k = 0; k < K; ++k) {
      if (b_init[k] < 1) { delete c; return fail(OMNI_EINVAL, "omni_dyn_create: b_init[%d]=%d", k, b_init[k]); }
      c->b[k] = b_init[k];
    }
  } else {
    // Algorithm 1 starts every worker at B / K: equal weights, largest remainder
    uint64_t ones[OMNI_MAX_WORKERS];
    int64_t b[OMNI_MAX_WORKERS];
    for (int k = 0; k < K; ++k) ones[k] = 1;
    if (int rc = omni::apportion_bounded(ones, K, B, 1, B, b, "omni_dyn_create")) { delete c; return rc; }
    for (int k = 0; k < K; ++k) c->b[k] = (int32_t)b[k];
  }
  for (int k = 0; k < K; ++k) c->ewma[k] = 0.0;
  *out = c;
  return OMNI_OK;
}

int omni_dyn_observe(omni_dyn* c, const double* t) {
  using omni::fail;
  if (!c || !t) return fail(OMNI_EINVAL, "omni_dyn_observe: NULL argument");
  for (int k = 0; k < c->K; ++k)
    if (!(t[k] > 0.0) || std::isinf(t[k])) return fail(OMNI_EINVAL, "omni_dyn_observe: t[%d] must be positive and finite", k);
  for (int k = 0; k < c->K; ++k) {
    if (c->nobs == 0) {
      c->ewma[k] = t[k];
    } else {
      const double new_part = c->alpha * t[k];
      const double keep = 1.0 - c->alpha;
      const double old_part = keep * c->ewma[k];
      c->ewma[k] = new_part + old_part;
    }
  }
  c->nobs += 1;
  return OMNI_OK;
}

int omni_dyn_adjust(omni_dyn* c, int32_t* b_out, int32_t* off_out, int32_t* changed_out) {
  using omni::fail;
  if (!c) return fail(OMNI_EINVAL, "omni_dyn_adjust: NULL controller");
  if (c->nobs == 0) return fail(OMNI_EINVAL, "omni_dyn_adjust: no compute times observed since the last adjustment");
  const int K = c->K;
  double s = 0.0;
  for (int k = 0; k < K; ++k) s = s + c->ewma[k];
  const double t_avg = s / (double)K;
  double b_star[OMNI_MAX_WORKERS], ratio[OMNI_MAX_WORKERS];
  double max_ratio = 0.0;
  for (int k = 0; k < K; ++k) {
    const double bk = (double)c->b[k];
    const double T = bk / c->ewma[k];
    const double tau = c->ewma[k] - t_avg;
    const double delta = T * tau;
    const double bs = bk - delta;
    b_star[k] = bs;
    const double diff = bs - bk;
    const double q = diff / bs;
    ratio[k] = std::fabs(q);
    if (k == 0 || ratio[k] > max_ratio) max_ratio = ratio[k];
  }
  const double lo = (double)c->b_min, hi = (double)c->b_max;
  int32_t nb[OMNI_MAX_WORKERS];
  for (int k = 0; k < K; ++k) nb[k] = c->b[k];
  if (c->rule == OMNI_RULE_NONE) {
    for (int k = 0; k < K; ++k)
      if (ratio[k] >= c->deadband) nb[k] = (int32_t)std::nearbyint(clampd(b_star[k], lo, hi));
  } else if (max_ratio >= c->deadband) {
    if (c->rule == OMNI_RULE_MULTIPLICATIVE) {
      uint64_t w[OMNI_MAX_WORKERS];
      int64_t b[OMNI_MAX_WORKERS];
      for (int k = 0; k < K; ++k) {
        const double scaled = b_star[k] * 1048576.0;
        const int64_t fl = (int64_t)scaled;   // floor: the value is positive
        w[k] = fl < 1 ? 1u : (uint64_t)fl;
      }
      if (int rc = omni::apportion_bounded(w, K, c->B, c->b_min, c->b_max, b, "omni_dyn_adjust")) return rc;
      for (int k = 0; k < K; ++k) nb[k] = (int32_t)b[k];
    } else {
      double sum = 0.0;
      for (int k = 0; k < K; ++k) sum = sum + b_star[k];
      const double over = sum - (double)c->B;
      const double share = over / (double)K;
      for (int k = 0; k < K; ++k) {
        const double v = b_star[k] - share;
        nb[k] = (int32_t)std::nearbyint(clampd(v, lo, hi));
      }
    }
  }
  int32_t changed = 0;
  for (int k = 0; k < K; ++k) {
    if (nb[k] != c->b[k]) changed = 1;
    c->b[k] = nb[k];
  }
  c->nobs = 0;
  write_out(c, b_out, off_out);
  if (changed_out) *changed_out = changed;
  return OMNI_OK;
}

int omni_dyn_get(const omni_dyn* c, int32_t* b_out, int32_t* off_out) {
  if (!c) return omni::fail(OMNI_EINVAL, "omni_dyn_get: NULL controller");
  write_out(c, b_out, off_out);
  return OMNI_OK;
}

void omni_dyn_destroy(omni_dyn* c) { delete c; }

}  // extern "C"
