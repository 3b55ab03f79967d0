// Asynchronous training, Algorithm 2, host side: the order in which simulated workers of
// different speeds push to the parameter server (exact integer arithmetic), and the
// server's batch-size bookkeeping (procedure evalBsz with its wrkB / wrkTime maps, getBsz
// as in Algorithm 1).  Doubles are combined one operation per statement and this file is
// compiled without floating-point contraction, so the integers they decide repeat bit for
// bit on any conforming host.
#include <cmath>
#include <new>

#include "common.h"

struct omni_asp_ps {
  int32_t K, b_min, b_max;
  double deadband;
  int32_t reported;                       // how many distinct workers have reported so far
  bool has[OMNI_MAX_WORKERS];
  int32_t wrk_b[OMNI_MAX_WORKERS];
  double wrk_time[OMNI_MAX_WORKERS];
};

namespace {

typedef unsigned __int128 u128;

inline double clampd(double x, double lo, double hi) { return x < lo ? lo : (x > hi ? hi : x); }

// Procedure getBsz of Algorithm 1 for one worker.
int32_t get_bsz(int32_t b, double t, double t_avg, double deadband, int32_t b_min, int32_t b_max) {
  const double bk = (double)b;
  const double T = bk / t;
  const double tau = t - t_avg;
  const double delta = T * tau;
  const double bs = bk - delta;
  const double diff = bs - bk;
  const double q = diff / bs;
  if (std::fabs(q) >= deadband) return (int32_t)std::nearbyint(clampd(bs, (double)b_min, (double)b_max));
  return b;
}

}  // namespace

extern "C" {

int omni_asp_schedule(int32_t K, const uint64_t* T, const int32_t* b, int32_t n_events, int32_t* worker_out,
                      int32_t* pulled_version_out) {
  using omni::fail;
  if (!T || !b || n_events < 0 || (n_events > 0 && (!worker_out || !pulled_version_out)))
    return fail(OMNI_EINVAL, "omni_asp_schedule: bad argument");
  if (K < 1) return fail(OMNI_EINVAL, "omni_asp_schedule: K=%d", K);
  if (K > OMNI_MAX_WORKERS) return fail(OMNI_ECAPACITY, "omni_asp_schedule: K=%d exceeds %d", K, OMNI_MAX_WORKERS);
  for (int k = 0; k < K; ++k)
    if (T[k] < 1 || b[k] < 1) return fail(OMNI_EINVAL, "omni_asp_schedule: T[%d] and b[%d] must be at least 1", k, k);
  // worker k finishes its j-th iteration at j * b_k / T_k; (j * b_k) < 2^62 and T < 2^64, so
  // the cross products used to compare two such times fit 128 bits
  int64_t next[OMNI_MAX_WORKERS];          // j of the iteration each worker is computing
  int32_t pulled[OMNI_MAX_WORKERS];
  for (int k = 0; k < K; ++k) { next[k] = 1; pulled[k] = 0; }
  for (int32_t e = 0; e < n_events; ++e) {
    int best = 0;
    for (int k = 1; k < K; ++k) {
      const u128 lhs = (u128)((uint64_t)next[k] * (uint64_t)b[k]) * (u128)T[best];
      const u128 rhs = (u128)((uint64_t)next[best] * (uint64_t)b[best]) * (u128)T[k];
      if (lhs < rhs) best = k;             // strictly earlier: ties stay with the lower index
    }
    worker_out[e] = best;
    pulled_version_out[e] = pulled[best];
    next[best] += 1;
    pulled[best] = e + 1;                  // pulls again right after its own push
  }
  return OMNI_OK;
}

int omni_asp_ps_create(int32_t K, int32_t b_min, int32_t b_max, double deadband, omni_asp_ps** out) {
  using omni::fail;
  if (!out) return fail(OMNI_EINVAL, "omni_asp_ps_create: out is NULL");
  *out = nullptr;
  if (K < 1) return fail(OMNI_EINVAL, "omni_asp_ps_create: K=%d", K);
  if (K > OMNI_MAX_WORKERS) return fail(OMNI_ECAPACITY, "omni_asp_ps_create: K=%d exceeds %d", K, OMNI_MAX_WORKERS);
  if (b_min < 1 || b_max < b_min) return fail(OMNI_EINVAL, "omni_asp_ps_create: bad bounds [%d,%d]", b_min, b_max);
  if (!(deadband >= 0.0 && deadband < 1.0)) return fail(OMNI_EINVAL, "omni_asp_ps_create: dead-band must lie in [0, 1)");
  omni_asp_ps* p = new (std::nothrow) omni_asp_ps();
  if (!p) return fail(OMNI_EINVAL, "omni_asp_ps_create: out of host memory");
  p->K = K; p->b_min = b_min; p->b_max = b_max; p->deadband = deadband; p->reported = 0;
  for (int k = 0; k < K; ++k) { p->has[k] = false; p->wrk_b[k] = 0; p->wrk_time[k] = 0.0; }
  *out = p;
  return OMNI_OK;
}

int omni_asp_ps_eval_bsz(omni_asp_ps* ps, int32_t k, int32_t b, double t, int32_t* b_out) {
  using omni::fail;
  if (!ps || !b_out) return fail(OMNI_EINVAL, "omni_asp_ps_eval_bsz: NULL argument");
  if (k < 0 || k >= ps->K) return fail(OMNI_EINVAL, "omni_asp_ps_eval_bsz: worker %d out of range", k);
  if (b < 1) return fail(OMNI_EINVAL, "omni_asp_ps_eval_bsz: b=%d", b);
  if (!(t > 0.0) || std::isinf(t)) return fail(OMNI_EINVAL, "omni_asp_ps_eval_bsz: t must be positive and finite");
  if (!ps->has[k]) { ps->has[k] = true; ps->reported += 1; }
  ps->wrk_b[k] = b;
  ps->wrk_time[k] = t;
  if (ps->reported == ps->K) {
    double s = 0.0;
    for (int w = 0; w < ps->K; ++w) s = s + ps->wrk_time[w];
    const double t_avg = s / (double)ps->K;
    for (int w = 0; w < ps->K; ++w)
      ps->wrk_b[w] = get_bsz(ps->wrk_b[w], ps->wrk_time[w], t_avg, ps->deadband, ps->b_min, ps->b_max);
  }
  *b_out = ps->wrk_b[k];
  return OMNI_OK;
}

int omni_asp_ps_sizes(const omni_asp_ps* ps, int32_t* b_out) {
  if (!ps || !b_out) return omni::fail(OMNI_EINVAL, "omni_asp_ps_sizes: NULL argument");
  for (int k = 0; k < ps->K; ++k) b_out[k] = ps->has[k] ? ps->wrk_b[k] : 0;
  return OMNI_OK;
}

void omni_asp_ps_destroy(omni_asp_ps* ps) { delete ps; }

}  // extern "C"
