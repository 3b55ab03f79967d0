// Host-side integer batch-size controller.
//
// Paper: section "Dynamic-Batching" (equations itrtimeerror, dynbszadjust), the
// fixed-global-batch rule (equation dynbszGlobalBFixed, applied
// multiplicatively as the accompanying text says) and the b_min/b_max bounds
// of procedure getBsz in Algorithm 1.  With throughput T_k the proportional
// update lands on T_k * mean(t); rescaling to sum B gives B*T_k/sum(T).  All of
// it is evaluated in exact integers: floor quotas plus largest remainders.
#include <algorithm>
#include <cstring>
#include <new>
#include <vector>

#include "common.h"

namespace omni {

static thread_local char g_err[512] = "";

int fail(int code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}

}  // namespace omni

struct omni_ctl {
  int32_t K, B, b_min, b_max;
  bool have_T;
  uint64_t T[OMNI_MAX_WORKERS];
};

typedef unsigned __int128 u128;

namespace {

// Hamilton apportionment of `total` units over the listed workers by weight T.
void largest_remainder(const uint64_t* T, const int* ids, int n, int64_t total, int64_t* share) {
  u128 W = 0;
  for (int i = 0; i < n; ++i) W += T[ids[i]];
  u128 rem[OMNI_MAX_WORKERS];
  int64_t given = 0;
  for (int i = 0; i < n; ++i) {
    u128 prod = (u128)(uint64_t)total * (u128)T[ids[i]];
    share[i] = (int64_t)(prod / W);
    rem[i] = prod % W;
    given += share[i];
  }
  int order[OMNI_MAX_WORKERS];
  for (int i = 0; i < n; ++i) order[i] = i;
  // larger remainder first; equal remainders keep ascending worker order
  std::stable_sort(order, order + n, [&](int a, int c) { return rem[a] > rem[c]; });
  int64_t left = total - given;
  for (int64_t i = 0; i < left; ++i) share[order[i]] += 1;
}

}  // namespace

namespace omni {

// Integer batch sizes proportional to the weights T with sum B inside [b_min, b_max]: largest
// remainder; if a share falls outside the bounds, the side with the larger total violation is
// clamped, those workers leave the pool with their units, and the rest is apportioned again.
int apportion_bounded(const uint64_t* T, int K, int64_t B, int64_t b_min, int64_t b_max, int64_t* b,
                      const char* who) {
  int ids[OMNI_MAX_WORKERS];
  int64_t share[OMNI_MAX_WORKERS];
  int n = K;
  for (int k = 0; k < K; ++k) ids[k] = k;
  int64_t remaining = B;
  for (;;) {
    if (n == 0) {
      if (remaining != 0) return fail(OMNI_EINFEASIBLE, "%s: clamping left %lld units", who, (long long)remaining);
      break;
    }
    if (remaining < 0) return fail(OMNI_EINFEASIBLE, "%s: clamping over-assigned", who);
    largest_remainder(T, ids, n, remaining, share);
    int64_t deficit = 0, excess = 0;
    int n_low = 0, n_high = 0;
    for (int i = 0; i < n; ++i) {
      if (share[i] < b_min) { deficit += b_min - share[i]; ++n_low; }
      if (share[i] > b_max) { excess += share[i] - b_max; ++n_high; }
    }
    if (!n_low && !n_high) {
      for (int i = 0; i < n; ++i) b[ids[i]] = share[i];
      break;
    }
    const bool clamp_high = n_high && excess >= deficit;
    int m = 0;
    for (int i = 0; i < n; ++i) {
      const bool hit = clamp_high ? share[i] > b_max : share[i] < b_min;
      if (hit) {
        b[ids[i]] = clamp_high ? b_max : b_min;
        remaining -= b[ids[i]];
      } else {
        ids[m++] = ids[i];
      }
    }
    n = m;
  }
  return OMNI_OK;
}

}  // namespace omni

extern "C" {

const char* omni_last_error(void) { return omni::g_err; }
const char* omni_version(void) { return "omnistep 0.1 (gfx950)"; }

int omni_ctl_create(int32_t K, int32_t B, int32_t b_min, int32_t b_max, omni_ctl** out) {
  if (!out) return omni::fail(OMNI_EINVAL, "omni_ctl_create: out is NULL");
  *out = nullptr;
  if (K < 1 || B < 1) return omni::fail(OMNI_EINVAL, "omni_ctl_create: K=%d B=%d must be positive", K, B);
  if (K > OMNI_MAX_WORKERS) return omni::fail(OMNI_ECAPACITY, "omni_ctl_create: K=%d exceeds %d", K, OMNI_MAX_WORKERS);
  if (b_max == 0) b_max = B;
  if (b_min < 1 || b_max < b_min) return omni::fail(OMNI_EINVAL, "omni_ctl_create: bad bounds [%d,%d]", b_min, b_max);
  if ((int64_t)K * b_min > B || (int64_t)K * b_max < B)
    return omni::fail(OMNI_EINFEASIBLE, "omni_ctl_create: K=%d workers in [%d,%d] cannot sum to B=%d", K, b_min, b_max, B);
  omni_ctl* c = new (std::nothrow) omni_ctl();
  if (!c) return omni::fail(OMNI_EINVAL, "omni_ctl_create: out of host memory");
  c->K = K; c->B = B; c->b_min = b_min; c->b_max = b_max; c->have_T = false;
  *out = c;
  return OMNI_OK;
}

int omni_ctl_set_throughputs(omni_ctl* ctl, const uint64_t* T) {
  if (!ctl || !T) return omni::fail(OMNI_EINVAL, "omni_ctl_set_throughputs: NULL argument");
  for (int k = 0; k < ctl->K; ++k)
    if (T[k] == 0) return omni::fail(OMNI_EINVAL, "omni_ctl_set_throughputs: T[%d] is zero", k);
  std::memcpy(ctl->T, T, sizeof(uint64_t) * ctl->K);
  ctl->have_T = true;
  return OMNI_OK;
}

int omni_ctl_run(omni_ctl* ctl, int32_t* b_out, int32_t* off_out) {
  if (!ctl || !b_out || !off_out) return omni::fail(OMNI_EINVAL, "omni_ctl_run: NULL argument");
  if (!ctl->have_T) return omni::fail(OMNI_EINVAL, "omni_ctl_run: throughputs not set");
  int64_t b[OMNI_MAX_WORKERS];
  if (int rc = omni::apportion_bounded(ctl->T, ctl->K, ctl->B, ctl->b_min, ctl->b_max, b, "omni_ctl_run")) return rc;
  int64_t acc = 0;
  off_out[0] = 0;
  for (int k = 0; k < ctl->K; ++k) {
    b_out[k] = (int32_t)b[k];
    acc += b[k];
    off_out[k + 1] = (int32_t)acc;
  }
  return OMNI_OK;
}

void omni_ctl_destroy(omni_ctl* ctl) { delete ctl; }

}  // extern "C"
