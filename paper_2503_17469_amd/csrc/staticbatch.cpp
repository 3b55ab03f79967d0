// Static variable batching and batch-size caps from memory, host side: equation varbszBSP
// (b_k = c_k / sum(c) * B from compute resources c_k), equation hlevel (heterogeneity level),
// and the memory model of section "Heterogeneous memory across workers" (equation hetmemeqn:
// model, gradient and optimiser memory fixed, activation and batch memory linear in the batch
// size, the batch term fitted by linear regression).  Doubles are combined one operation per
// statement and this file is compiled without floating-point contraction.
#include <cmath>

#include "common.h"

namespace {

typedef __int128 i128;

// Equation hetmemeqn for batch size b.
double mem_total(int64_t b, int64_t P, int32_t bytes_per_param, int32_t opt_copies, double act_per_sample,
                 double batch_slope, double batch_intercept) {
  const double model = (double)P * (double)bytes_per_param;
  const double copies = 2.0 + (double)opt_copies;
  const double fixed3 = copies * model;               // M_model + M_grad + M_opt
  const double act = act_per_sample * (double)b;
  const double batch_var = batch_slope * (double)b;
  const double batch = batch_var + batch_intercept;
  const double s1 = fixed3 + act;
  return s1 + batch;
}

int check_mem_args(const char* who, int64_t P, int32_t bytes_per_param, int32_t opt_copies, double act_per_sample,
                   double batch_slope, double batch_intercept) {
  using omni::fail;
  if (P < 1 || bytes_per_param < 1 || opt_copies < 0) return fail(OMNI_EINVAL, "%s: bad model size arguments", who);
  if (!(act_per_sample >= 0.0) || !(batch_slope >= 0.0) || !std::isfinite(act_per_sample) ||
      !std::isfinite(batch_slope) || !std::isfinite(batch_intercept))
    return fail(OMNI_EINVAL, "%s: per-sample terms must be finite and >= 0", who);
  return OMNI_OK;
}

}  // namespace

extern "C" {

int omni_static_batches(int32_t K, const uint64_t* c, int32_t B, int32_t b_min, int32_t b_max, int32_t* b_out,
                        int32_t* off_out) {
  using omni::fail;
  if (!c || !b_out) return fail(OMNI_EINVAL, "omni_static_batches: NULL argument");
  if (K < 1 || B < K) return fail(OMNI_EINVAL, "omni_static_batches: need 1 <= K <= B (K=%d B=%d)", K, B);
  if (K > OMNI_MAX_WORKERS) return fail(OMNI_ECAPACITY, "omni_static_batches: K=%d exceeds %d", K, OMNI_MAX_WORKERS);
  if (b_max == 0) b_max = B;
  if (b_min < 1 || b_max < b_min) return fail(OMNI_EINVAL, "omni_static_batches: bad bounds [%d,%d]", b_min, b_max);
  for (int k = 0; k < K; ++k)
    if (c[k] < 1) return fail(OMNI_EINVAL, "omni_static_batches: c[%d] must be at least 1", k);
  int64_t b[OMNI_MAX_WORKERS];
  if (int rc = omni::apportion_bounded(c, K, B, b_min, b_max, b, "omni_static_batches")) return rc;
  int64_t acc = 0;
  if (off_out) off_out[0] = 0;
  for (int k = 0; k < K; ++k) {
    b_out[k] = (int32_t)b[k];
    acc += b[k];
    if (off_out) off_out[k + 1] = (int32_t)acc;
  }
  return OMNI_OK;
}

int omni_heterogeneity_level(int32_t K, const uint64_t* c, uint64_t* max_out, uint64_t* min_out, double* hl_out) {
  using omni::fail;
  if (!c || K < 1) return fail(OMNI_EINVAL, "omni_heterogeneity_level: bad argument");
  uint64_t lo = c[0], hi = c[0];
  for (int k = 0; k < K; ++k) {
    if (c[k] < 1) return fail(OMNI_EINVAL, "omni_heterogeneity_level: c[%d] must be at least 1", k);
    if (c[k] < lo) lo = c[k];
    if (c[k] > hi) hi = c[k];
  }
  if (max_out) *max_out = hi;
  if (min_out) *min_out = lo;
  if (hl_out) *hl_out = (double)hi / (double)lo;
  return OMNI_OK;
}

int omni_mem_fit_linear(int32_t n, const int64_t* b, const int64_t* bytes, double* slope_out, double* intercept_out) {
  using omni::fail;
  if (!b || !bytes || !slope_out || !intercept_out) return fail(OMNI_EINVAL, "omni_mem_fit_linear: NULL argument");
  if (n < 2 || n > 4096) return fail(n < 2 ? OMNI_EINVAL : OMNI_ECAPACITY, "omni_mem_fit_linear: n=%d outside [2, 4096]", n);
  // the sums of the normal equations are integers: kept exact in 128 bits (b <= 2^24, bytes <= 2^48)
  i128 sb = 0, sm = 0, sbb = 0, sbm = 0;
  for (int i = 0; i < n; ++i) {
    if (b[i] < 0 || b[i] > (1 << 24) || bytes[i] < 0 || bytes[i] > ((int64_t)1 << 48))
      return fail(OMNI_ECAPACITY, "omni_mem_fit_linear: point %d outside b <= 2^24, bytes <= 2^48", i);
    sb += b[i];
    sm += bytes[i];
    sbb += (i128)b[i] * b[i];
    sbm += (i128)b[i] * bytes[i];
  }
  const i128 den = (i128)n * sbb - sb * sb;
  if (den == 0) return fail(OMNI_EINVAL, "omni_mem_fit_linear: need at least two distinct batch sizes");
  const i128 num_slope = (i128)n * sbm - sb * sm;
  const i128 num_icpt = sm * sbb - sb * sbm;
  *slope_out = (double)((long double)num_slope / (long double)den);
  *intercept_out = (double)((long double)num_icpt / (long double)den);
  return OMNI_OK;
}

int omni_mem_total(int64_t b, int64_t P, int32_t bytes_per_param, int32_t opt_copies, double act_per_sample,
                   double batch_slope, double batch_intercept, double* total_out) {
  if (!total_out || b < 0) return omni::fail(OMNI_EINVAL, "omni_mem_total: bad argument");
  if (int rc = check_mem_args("omni_mem_total", P, bytes_per_param, opt_copies, act_per_sample, batch_slope,
                              batch_intercept))
    return rc;
  *total_out = mem_total(b, P, bytes_per_param, opt_copies, act_per_sample, batch_slope, batch_intercept);
  return OMNI_OK;
}

int omni_mem_max_batch(double mem_avail, int64_t P, int32_t bytes_per_param, int32_t opt_copies,
                       double act_per_sample, double batch_slope, double batch_intercept, int64_t limit,
                       int64_t* b_max_out) {
  using omni::fail;
  if (!b_max_out || limit < 0 || !std::isfinite(mem_avail)) return fail(OMNI_EINVAL, "omni_mem_max_batch: bad argument");
  if (int rc = check_mem_args("omni_mem_max_batch", P, bytes_per_param, opt_copies, act_per_sample, batch_slope,
                              batch_intercept))
    return rc;
  auto fits = [&](int64_t b) {
    return mem_total(b, P, bytes_per_param, opt_copies, act_per_sample, batch_slope, batch_intercept) <= mem_avail;
  };
  if (!fits(0)) { *b_max_out = -1; return OMNI_OK; }
  int64_t lo = 0, hi = limit;
  if (fits(hi)) { *b_max_out = hi; return OMNI_OK; }
  while (hi - lo > 1) {              // fits(lo), not fits(hi); the prediction does not decrease with b
    const int64_t mid = lo + (hi - lo) / 2;
    if (fits(mid)) lo = mid; else hi = mid;
  }
  *b_max_out = lo;
  return OMNI_OK;
}

int omni_net_max_batch(const omni_layer_desc* layers, int32_t n_layers, int32_t in_h, int32_t in_w, int32_t in_c,
                       int32_t dtype, int32_t K_max, int32_t opt_copies, uint64_t budget_bytes, int32_t* B_max_out,
                       uint64_t* bytes_out) {
  using omni::fail;
  if (!B_max_out) return fail(OMNI_EINVAL, "omni_net_max_batch: B_max_out is NULL");
  if (opt_copies < 0 || opt_copies > 8) return fail(OMNI_EINVAL, "omni_net_max_batch: opt_copies=%d", opt_copies);
  *B_max_out = 0;
  // what a training state of this library holds on the device for batch capacity B:
  // the workspace (activations, their gradients, K_max gradient rows, scratch), the fp32
  // parameters and opt_copies buffers of the same size, the input batch and its labels
  auto need = [&](int32_t B, uint64_t* out) -> int {
    omni_net* net = nullptr;
    if (int rc = omni_net_create(layers, n_layers, in_h, in_w, in_c, dtype, K_max, B, &net)) return rc;
    const uint64_t P = omni_net_param_count(net);
    const uint64_t esize = dtype == OMNI_BF16 ? 2 : 4;
    uint64_t total = omni_net_workspace_bytes(net);
    total += (1 + (uint64_t)opt_copies) * 4 * P;
    total += (uint64_t)B * ((uint64_t)in_h * in_w * in_c * esize + 4);
    omni_net_destroy(net);
    *out = total;
    return OMNI_OK;
  };
  uint64_t bytes = 0;
  int rc = need(K_max, &bytes);           // also validates the layer list
  if (rc) return rc;
  if (bytes > budget_bytes)
    return fail(OMNI_EINFEASIBLE, "omni_net_max_batch: one sample per worker already needs %llu bytes",
                (unsigned long long)bytes);
  int32_t lo = K_max, hi = 1 << 24;
  uint64_t lo_bytes = bytes;
  while (hi - lo > 1) {                   // lo fits; hi does not (too large for the budget or for the library)
    const int32_t mid = lo + (hi - lo) / 2;
    rc = need(mid, &bytes);
    if (rc == OMNI_OK && bytes <= budget_bytes) { lo = mid; lo_bytes = bytes; }
    else if (rc == OMNI_OK || rc == OMNI_ECAPACITY) hi = mid;
    else return rc;
  }
  *B_max_out = lo;
  if (bytes_out) *bytes_out = lo_bytes;
  return OMNI_OK;
}

}  // extern "C"
