// Launch plan and step driver: turns a layer list into a fixed sequence of
// kernel launches over the ragged batch (Algorithm 1, procedure Train: the
// gradient line, the weighted AllReduce line and the update line).
//
// Forward and input-gradient kernels see all B rows at once: rows of different
// workers are independent there.  Only three things know about workers: the
// loss (1/b_k scaling), the parameter-gradient kernels (one output row of G per
// worker, reduction over that worker's rows) and per-worker batch norm.
#include <hip/hip_runtime_api.h>

#include <cmath>
#include <new>
#include <vector>

#include "common.h"
#include "kernels.h"

namespace {

constexpr size_t kAlign = 256;
inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

struct Tensor {
  int h = 0, w = 0, c = 0;
  size_t elems = 0;        // per row
  size_t act_off = 0;      // byte offsets into the workspace
  size_t grad_off = 0;
  bool relu = false;       // ReLU folded into the producer; grad buffer is w.r.t. the pre-ReLU value
  int consumers = 0;
};

struct Layer {
  omni_layer_desc d;
  int out = -1;            // tensor index
  int in0 = -1, in1 = -1;  // tensor indices (-1 = network input)
  size_t w_off = 0, b_off = 0;  // float offsets into params
  bool has_b = false;
  bool fused_away = false;      // ReLU merged into its producer
};

}  // namespace

struct omni_net {
  std::vector<Layer> layers;
  std::vector<Tensor> tensors;
  int in_h, in_w, in_c;
  int dtype, K_max, B_max;
  size_t P = 0, P_stride = 0;
  size_t ws_bytes = 0;
  size_t grads_off = 0, loss_rows_off = 0, status_off = 0, partial_off = 0, counters_off = 0;
  int classes = 0;
  const void* ws_ready = nullptr;   // workspace whose arrival counters are known to be zero
  // optional event timing of one kernel class
  int time_class = -1, time_layer = -1;
  std::vector<hipEvent_t> ev;   // pairs: start, stop
  size_t ev_used = 0;           // events recorded since the last read

  ~omni_net() {
    for (hipEvent_t e : ev) (void)hipEventDestroy(e);
  }
};

namespace {
// Records an event pair around the launches made while it is alive, if the
// network is timing this (class, layer) and has event pairs left.
struct TimedScope {
  omni_net* net;
  hipStream_t st;
  bool on;
  TimedScope(omni_net* n, hipStream_t s, int cls, int layer) : net(n), st(s) {
    on = n->time_class == cls && (n->time_layer < 0 || n->time_layer == layer) && n->ev_used + 2 <= n->ev.size();
    if (on) (void)hipEventRecord(net->ev[net->ev_used], st);
  }
  ~TimedScope() {
    if (on) {
      (void)hipEventRecord(net->ev[net->ev_used + 1], st);
      net->ev_used += 2;
    }
  }
};
}  // namespace

using omni::fail;

extern "C" {

int omni_net_create(const omni_layer_desc* descs, int32_t n, int32_t in_h, int32_t in_w, int32_t in_c,
                    int32_t dtype, int32_t K_max, int32_t B_max, omni_net** out) {
  if (!out) return fail(OMNI_EINVAL, "omni_net_create: out is NULL");
  *out = nullptr;
  if (!descs || n < 1) return fail(OMNI_EINVAL, "omni_net_create: empty layer list");
  if (in_h < 1 || in_w < 1 || in_c < 1) return fail(OMNI_EINVAL, "omni_net_create: bad input shape");
  if (K_max < 1 || B_max < K_max) return fail(OMNI_EINVAL, "omni_net_create: need 1 <= K_max <= B_max");
  if (K_max > OMNI_MAX_WORKERS) return fail(OMNI_ECAPACITY, "omni_net_create: K_max exceeds %d", OMNI_MAX_WORKERS);
  if (dtype != OMNI_F32) return fail(OMNI_EINVAL, "omni_net_create: dtype %d not supported", dtype);

  omni_net* net = new (std::nothrow) omni_net();
  if (!net) return fail(OMNI_EINVAL, "omni_net_create: out of host memory");
  net->in_h = in_h; net->in_w = in_w; net->in_c = in_c;
  net->dtype = dtype; net->K_max = K_max; net->B_max = B_max;

  auto bail = [&](int code) { delete net; return code; };
  auto shape_of = [&](int t, int& h, int& w, int& c) {
    if (t < 0) { h = in_h; w = in_w; c = in_c; }
    else { h = net->tensors[t].h; w = net->tensors[t].w; c = net->tensors[t].c; }
  };

  size_t ppos = 0;
  net->layers.resize(n);
  for (int i = 0; i < n; ++i) {
    Layer& L = net->layers[i];
    L.d = descs[i];
    if (L.d.src < -1 || L.d.src >= i) return bail(fail(OMNI_EINVAL, "layer %d: src %d out of range", i, L.d.src));
    L.in0 = L.d.src < 0 ? -1 : net->layers[L.d.src].out;
    if (L.d.src >= 0 && !net->layers[L.d.src].fused_away && net->tensors[L.in0].relu)
      return bail(fail(OMNI_EINVAL, "layer %d: reads layer %d before its ReLU, which was folded into it", i, L.d.src));
    int h, w, c;
    shape_of(L.in0, h, w, c);
    switch (L.d.op) {
      case OMNI_OP_LINEAR: {
        if (L.d.cin != h * w * c || L.d.cout < 1)
          return bail(fail(OMNI_EINVAL, "layer %d: linear cin=%d does not match input %dx%dx%d", i, L.d.cin, h, w, c));
        Tensor t; t.h = 1; t.w = 1; t.c = L.d.cout; t.elems = (size_t)L.d.cout;
        net->tensors.push_back(t);
        L.out = (int)net->tensors.size() - 1;
        L.w_off = ppos; ppos += (size_t)L.d.cout * L.d.cin;
        L.has_b = L.d.bias != 0;
        if (L.has_b) { L.b_off = ppos; ppos += (size_t)L.d.cout; }
        break;
      }
      case OMNI_OP_RELU: {
        if (L.in0 < 0) return bail(fail(OMNI_EINVAL, "layer %d: ReLU on the network input is not supported", i));
        const Layer& prod = net->layers[L.d.src];
        if (prod.d.op != OMNI_OP_LINEAR)
          return bail(fail(OMNI_EINVAL, "layer %d: ReLU after op %d is not supported for this dtype", i, prod.d.op));
        if (net->tensors[L.in0].consumers != 0 || net->tensors[L.in0].relu)
          return bail(fail(OMNI_EINVAL, "layer %d: ReLU input must have no other consumer", i));
        net->tensors[L.in0].relu = true;
        L.out = L.in0;
        L.fused_away = true;
        continue;  // not a consumer in its own right
      }
      default:
        return bail(fail(OMNI_EINVAL, "layer %d: op %d not supported for this dtype", i, L.d.op));
    }
    if (L.in0 >= 0) net->tensors[L.in0].consumers++;
  }
  net->P = ppos;
  net->P_stride = align_up(ppos, 64);
  const Tensor& last = net->tensors[net->layers[n - 1].out];
  if (last.h != 1 || last.w != 1) return bail(fail(OMNI_EINVAL, "last layer must produce [rows][classes]"));
  if (last.relu) return bail(fail(OMNI_EINVAL, "logits must not pass through ReLU"));
  net->classes = last.c;

  size_t pos = 0;
  net->grads_off = pos; pos += align_up((size_t)K_max * net->P_stride * sizeof(float), kAlign);
  net->loss_rows_off = pos; pos += align_up((size_t)B_max * sizeof(float), kAlign);
  net->status_off = pos; pos += kAlign;
  net->counters_off = pos; pos += align_up(omni::kSplitMaxTiles * sizeof(uint32_t), kAlign);
  net->partial_off = pos; pos += align_up(omni::kSplitPartialFloats * sizeof(float), kAlign);
  for (Tensor& t : net->tensors) {
    const size_t bytes = align_up((size_t)B_max * t.elems * sizeof(float), kAlign);
    t.act_off = pos; pos += bytes;
    t.grad_off = pos; pos += bytes;
  }
  net->ws_bytes = pos;
  *out = net;
  return OMNI_OK;
}

size_t omni_net_param_count(const omni_net* net) { return net ? net->P : 0; }
size_t omni_net_workspace_bytes(const omni_net* net) { return net ? net->ws_bytes : 0; }
size_t omni_net_grad_stride(const omni_net* net) { return net ? net->P_stride : 0; }

const float* omni_net_worker_grads(const omni_net* net, const void* ws) {
  if (!net || !ws) return nullptr;
  return reinterpret_cast<const float*>(static_cast<const char*>(ws) + net->grads_off);
}
const uint32_t* omni_net_status(const omni_net* net, const void* ws) {
  if (!net || !ws) return nullptr;
  return reinterpret_cast<const uint32_t*>(static_cast<const char*>(ws) + net->status_off);
}
int omni_net_activation(const omni_net* net, const void* ws, int32_t layer, const void** ptr, size_t* elems) {
  if (!net || !ws || !ptr || !elems) return fail(OMNI_EINVAL, "omni_net_activation: NULL argument");
  if (layer < 0 || layer >= (int)net->layers.size()) return fail(OMNI_EINVAL, "omni_net_activation: bad layer %d", layer);
  const Tensor& t = net->tensors[net->layers[layer].out];
  *ptr = static_cast<const char*>(ws) + t.act_off;
  *elems = t.elems;
  return OMNI_OK;
}

void omni_net_destroy(omni_net* net) { delete net; }

int omni_net_timing_enable(omni_net* net, int32_t kernel_class, int32_t layer, int32_t max_launches) {
  if (!net) return fail(OMNI_EINVAL, "omni_net_timing_enable: NULL net");
  if (kernel_class >= OMNI_KERNEL_CLASSES) return fail(OMNI_EINVAL, "omni_net_timing_enable: bad class %d", kernel_class);
  net->ev_used = 0;
  if (kernel_class < 0) { net->time_class = -1; return OMNI_OK; }
  if (max_launches < 1 || max_launches > (1 << 20)) return fail(OMNI_EINVAL, "omni_net_timing_enable: bad max_launches");
  while (net->ev.size() < (size_t)max_launches * 2) {
    hipEvent_t e;
    OMNI_HIP_CHECK(hipEventCreate(&e));
    net->ev.push_back(e);
  }
  net->time_class = kernel_class;
  net->time_layer = layer;
  return OMNI_OK;
}

int omni_net_timing_read(omni_net* net, double* total_ms, int64_t* launches) {
  if (!net || !total_ms || !launches) return fail(OMNI_EINVAL, "omni_net_timing_read: NULL argument");
  double tot = 0.0;
  for (size_t i = 0; i + 1 < net->ev_used; i += 2) {
    OMNI_HIP_CHECK(hipEventSynchronize(net->ev[i + 1]));
    float ms = 0.f;
    OMNI_HIP_CHECK(hipEventElapsedTime(&ms, net->ev[i], net->ev[i + 1]));
    tot += ms;
  }
  *total_ms = tot;
  *launches = (int64_t)(net->ev_used / 2);
  net->ev_used = 0;
  return OMNI_OK;
}

int omni_step(omni_net* net, void* stream, float* params, const void* x, const int32_t* labels,
              const int32_t* off, const int32_t* b, int32_t K, float lr, void* workspace,
              float* loss_per_worker, float* loss, uint32_t flags) {
  if (!net || !params || !x || !labels || !off || !b || !workspace || !loss_per_worker || !loss)
    return fail(OMNI_EINVAL, "omni_step: NULL argument");
  if (K < 1) return fail(OMNI_EINVAL, "omni_step: K=%d", K);
  if (K > net->K_max) return fail(OMNI_ECAPACITY, "omni_step: K=%d exceeds K_max=%d", K, net->K_max);
  if (off[0] != 0) return fail(OMNI_EINVAL, "omni_step: off[0] must be 0");
  for (int k = 0; k < K; ++k) {
    if (b[k] < 1) return fail(OMNI_EINVAL, "omni_step: b[%d]=%d must be at least 1", k, b[k]);
    if ((int64_t)off[k + 1] - off[k] != b[k]) return fail(OMNI_EINVAL, "omni_step: off and b disagree at worker %d", k);
  }
  if (off[K] > net->B_max) return fail(OMNI_ECAPACITY, "omni_step: %d rows exceed B_max=%d", off[K], net->B_max);
  if (!std::isfinite(lr)) return fail(OMNI_EINVAL, "omni_step: lr is not finite");
  if ((reinterpret_cast<uintptr_t>(params) & 15u) || (reinterpret_cast<uintptr_t>(workspace) & 255u) ||
      (reinterpret_cast<uintptr_t>(x) & 15u))
    return fail(OMNI_EINVAL, "omni_step: params/x must be 16-byte and workspace 256-byte aligned");

  hipStream_t st = static_cast<hipStream_t>(stream);
  char* ws = static_cast<char*>(workspace);
  const int rows = off[K];
  omni::Segments seg{};
  seg.K = K;
  for (int k = 0; k <= K; ++k) seg.off[k] = off[k];

  float* G = reinterpret_cast<float*>(ws + net->grads_off);
  float* loss_rows = reinterpret_cast<float*>(ws + net->loss_rows_off);
  uint32_t* status = reinterpret_cast<uint32_t*>(ws + net->status_off);
  auto act = [&](int t) -> const float* {
    return t < 0 ? static_cast<const float*>(x) : reinterpret_cast<const float*>(ws + net->tensors[t].act_off);
  };
  auto actw = [&](int t) { return reinterpret_cast<float*>(ws + net->tensors[t].act_off); };
  auto grad = [&](int t) { return reinterpret_cast<float*>(ws + net->tensors[t].grad_off); };

  // Arrival counters of the split reductions must start at zero; every launch
  // returns them to zero, so this runs once per workspace.
  omni::SplitWorkspace sw;
  sw.partial = reinterpret_cast<float*>(ws + net->partial_off);
  sw.counters = reinterpret_cast<uint32_t*>(ws + net->counters_off);
  if (net->ws_ready != workspace) {
    omni::fill_u32(st, sw.counters, omni::kSplitMaxTiles, 0u);
    net->ws_ready = workspace;
  }

  const int n_layers = (int)net->layers.size();
  const Layer& last = net->layers[n_layers - 1];
  const bool fused_head = last.d.op == OMNI_OP_LINEAR &&
                          omni::head_supported(last.d.cin, last.d.cout, act(last.in0), params + last.w_off);

  // ---- forward over the concatenated batch
  for (const Layer& L : net->layers) {
    if (L.fused_away) continue;
    if (fused_head && &L == &last) continue;
    switch (L.d.op) {
      case OMNI_OP_LINEAR: {
        TimedScope ts(net, st, OMNI_KERNEL_LINEAR_FWD, (int)(&L - net->layers.data()));
        omni::linear_fwd_f32(st, act(L.in0), params + L.w_off, L.has_b ? params + L.b_off : nullptr, actw(L.out),
                             rows, L.d.cin, L.d.cout, net->tensors[L.out].relu, sw);
        break;
      }
      default: break;
    }
  }

  // ---- loss: dz already carries 1/b_k, so everything downstream is a per-worker mean gradient
  const int logits = last.out;
  std::vector<char> written(net->tensors.size(), 0);
  if (fused_head) {
    TimedScope ts(net, st, OMNI_KERNEL_LOSS, n_layers - 1);
    const bool need_dx = last.in0 >= 0;
    omni::head_fwd_loss_dgrad_f32(st, act(last.in0), params + last.w_off, last.has_b ? params + last.b_off : nullptr,
                                  labels, last.d.cin, last.d.cout, seg, actw(logits), grad(logits), loss_rows,
                                  need_dx && net->tensors[last.in0].relu ? act(last.in0) : nullptr,
                                  need_dx ? grad(last.in0) : nullptr, false);
    if (need_dx) written[last.in0] = 1;
    omni::head_wgrad_loss_f32(st, grad(logits), act(last.in0), labels, last.d.cin, last.d.cout, seg, G + last.w_off,
                              last.has_b ? G + last.b_off : nullptr, net->P_stride, loss_rows, loss_per_worker, loss,
                              status);
  } else {
    TimedScope ts(net, st, OMNI_KERNEL_LOSS, n_layers - 1);
    omni::fill_u32(st, status, 1, 0u);
    omni::softmax_xent_f32(st, act(logits), labels, net->classes, seg, grad(logits), loss_rows, loss_per_worker,
                           loss, status);
  }

  // ---- backward: input gradients on all rows, parameter gradients per worker
  for (int i = n_layers - 1; i >= 0; --i) {
    const Layer& L = net->layers[i];
    if (L.fused_away) continue;
    if (fused_head && i == n_layers - 1) continue;
    switch (L.d.op) {
      case OMNI_OP_LINEAR: {
        {
          TimedScope ts(net, st, OMNI_KERNEL_LINEAR_WGRAD, i);
          omni::linear_wgrad_f32(st, grad(L.out), act(L.in0), G + L.w_off, L.has_b ? G + L.b_off : nullptr,
                                 net->P_stride, seg, L.d.cin, L.d.cout);
        }
        if (L.in0 >= 0) {
          const Tensor& ti = net->tensors[L.in0];
          TimedScope ts(net, st, OMNI_KERNEL_LINEAR_DGRAD, i);
          omni::linear_dgrad_f32(st, grad(L.out), params + L.w_off, ti.relu ? act(L.in0) : nullptr, grad(L.in0),
                                 rows, L.d.cin, L.d.cout, written[L.in0] != 0, sw);
          written[L.in0] = 1;
        }
        break;
      }
      default: break;
    }
  }

  // ---- weighted aggregation + update
  if (!(flags & OMNI_STEP_NO_UPDATE)) {
    TimedScope ts(net, st, OMNI_KERNEL_UPDATE, -1);
    omni::weighted_sgd_f32(st, params, G, net->P_stride, net->P, seg, lr, nullptr);
  }

  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(OMNI_EHIP, "omni_step: launch failed: %s", hipGetErrorString(e));
  return OMNI_OK;
}

int omni_weighted_sgd(void* stream, float* params, const float* grads, size_t stride, size_t P,
                      const int32_t* b, int32_t K, float lr, void* shadow_bf16) {
  if (!params || !grads || !b) return fail(OMNI_EINVAL, "omni_weighted_sgd: NULL argument");
  if (K < 1 || K > OMNI_MAX_WORKERS) return fail(K < 1 ? OMNI_EINVAL : OMNI_ECAPACITY, "omni_weighted_sgd: K=%d", K);
  if (P < 1 || stride < P || (stride & 3u)) return fail(OMNI_EINVAL, "omni_weighted_sgd: need P >= 1 and stride >= P, stride %% 4 == 0");
  if ((reinterpret_cast<uintptr_t>(params) & 15u) || (reinterpret_cast<uintptr_t>(grads) & 15u) ||
      (reinterpret_cast<uintptr_t>(shadow_bf16) & 7u))
    return fail(OMNI_EINVAL, "omni_weighted_sgd: params/grads must be 16-byte aligned");
  if (!std::isfinite(lr)) return fail(OMNI_EINVAL, "omni_weighted_sgd: lr is not finite");
  omni::Segments seg{};
  seg.K = K;
  int64_t acc = 0;
  for (int k = 0; k < K; ++k) {
    if (b[k] < 1) return fail(OMNI_EINVAL, "omni_weighted_sgd: b[%d]=%d must be at least 1", k, b[k]);
    acc += b[k];
    if (acc > INT32_MAX) return fail(OMNI_EOVERFLOW, "omni_weighted_sgd: sum of b overflows");
    seg.off[k + 1] = (int32_t)acc;
  }
  omni::weighted_sgd_f32(static_cast<hipStream_t>(stream), params, grads, stride, P, seg, lr,
                         static_cast<uint16_t*>(shadow_bf16));
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(OMNI_EHIP, "omni_weighted_sgd: launch failed: %s", hipGetErrorString(e));
  return OMNI_OK;
}

int omni_softmax_xent(void* stream, const float* z, const int32_t* labels, int32_t C, const int32_t* off,
                      int32_t K, float* dz, float* loss_rows, float* loss_per_worker, float* loss,
                      uint32_t* status) {
  if (!z || !labels || !off || !dz || !loss_rows || !loss_per_worker || !loss || !status)
    return fail(OMNI_EINVAL, "omni_softmax_xent: NULL argument");
  if (C < 1) return fail(OMNI_EINVAL, "omni_softmax_xent: C=%d", C);
  if (K < 1 || K > OMNI_MAX_WORKERS) return fail(K < 1 ? OMNI_EINVAL : OMNI_ECAPACITY, "omni_softmax_xent: K=%d", K);
  if (off[0] != 0) return fail(OMNI_EINVAL, "omni_softmax_xent: off[0] must be 0");
  omni::Segments seg{};
  seg.K = K;
  for (int k = 0; k < K; ++k) {
    if (off[k + 1] <= off[k]) return fail(OMNI_EINVAL, "omni_softmax_xent: worker %d has no rows", k);
    seg.off[k + 1] = off[k + 1];
  }
  omni::softmax_xent_f32(static_cast<hipStream_t>(stream), z, labels, C, seg, dz, loss_rows, loss_per_worker, loss,
                         status);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(OMNI_EHIP, "omni_softmax_xent: launch failed: %s", hipGetErrorString(e));
  return OMNI_OK;
}

}  // extern "C"
