// Asynchronous training, Algorithm 2, host side: the order in which simulated workers of
// different speeds push to the parameter server (exact integer arithmetic), and the
// server's batch-size bookkeeping (what procedure evalBsz of Algorithm 2 keeps and decides).
// Doubles are combined one operation per statement and this file is compiled without
// floating-point contraction, so the integers they decide repeat bit for bit on any
// conforming host.
#include <cmath>
#include <new>

#include "common.h"

// The server's view of its workers as plain arrays: the latest batch size and iteration time each one
// reported, and which of them have reported at all.  Nothing is resized until every worker has been heard
// from; from then on EVERY report triggers a re-evaluation of all sizes against the mean of the latest times.
struct omni_asp_ps {
  int32_t K, b_min, b_max;
  double deadband;
  int32_t heard;                          // distinct workers heard from so far
  bool known[OMNI_MAX_WORKERS];
  int32_t size[OMNI_MAX_WORKERS];
  double seconds[OMNI_MAX_WORKERS];
};

namespace {

typedef unsigned __int128 u128;

// One pass over all workers (section "Dynamic-Batching", eqs itrtimeerror and dynbszadjust, with the bounds
// and the dead-band of procedure getBsz): a worker's throughput at its current size, times its distance from
// the mean iteration time, is how many samples it should hand over (or take on); the move is made only if it
// changes the size by at least the dead-band fraction of the proposed size, and lands inside [b_min, b_max].
// One floating-point operation per statement, no contraction: the integers repeat bit for bit elsewhere.
void resize_all(omni_asp_ps& ps) {
  double total = 0.0;
  for (int w = 0; w < ps.K; ++w) total = total + ps.seconds[w];
  const double mean = total / (double)ps.K;
  const double lo = (double)ps.b_min, hi = (double)ps.b_max;
  for (int w = 0; w < ps.K; ++w) {
    const double now = (double)ps.size[w];
    const double rate = now / ps.seconds[w];
    const double late = ps.seconds[w] - mean;
    const double surplus = rate * late;
    const double proposed = now - surplus;
    const double change = proposed - now;
    const double relative = change / proposed;
    if (!(std::fabs(relative) >= ps.deadband)) continue;   // inside the dead-band (or not a number): leave it
    const double bounded = proposed < lo ? lo : (proposed > hi ? hi : proposed);
    ps.size[w] = (int32_t)std::nearbyint(bounded);
  }
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
  p->K = K; p->b_min = b_min; p->b_max = b_max; p->deadband = deadband; p->heard = 0;
  for (int k = 0; k < K; ++k) { p->known[k] = false; p->size[k] = 0; p->seconds[k] = 0.0; }
  *out = p;
  return OMNI_OK;
}

int omni_asp_ps_eval_bsz(omni_asp_ps* ps, int32_t k, int32_t b, double t, int32_t* b_out) {
  using omni::fail;
  if (!ps || !b_out) return fail(OMNI_EINVAL, "omni_asp_ps_eval_bsz: NULL argument");
  if (k < 0 || k >= ps->K) return fail(OMNI_EINVAL, "omni_asp_ps_eval_bsz: worker %d out of range", k);
  if (b < 1) return fail(OMNI_EINVAL, "omni_asp_ps_eval_bsz: b=%d", b);
  if (!(t > 0.0) || std::isinf(t)) return fail(OMNI_EINVAL, "omni_asp_ps_eval_bsz: t must be positive and finite");
  if (!ps->known[k]) { ps->known[k] = true; ps->heard += 1; }
  ps->size[k] = b;
  ps->seconds[k] = t;
  if (ps->heard == ps->K) resize_all(*ps);
  *b_out = ps->size[k];
  return OMNI_OK;
}

int omni_asp_ps_sizes(const omni_asp_ps* ps, int32_t* b_out) {
  if (!ps || !b_out) return omni::fail(OMNI_EINVAL, "omni_asp_ps_sizes: NULL argument");
  for (int k = 0; k < ps->K; ++k) b_out[k] = ps->known[k] ? ps->size[k] : 0;
  return OMNI_OK;
}

void omni_asp_ps_destroy(omni_asp_ps* ps) { delete ps; }

}  // extern "C"
