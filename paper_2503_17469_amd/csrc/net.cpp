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
#include <algorithm>
#include <cstring>
#include <vector>

#include "common.h"
#include "kernels.h"

namespace {

constexpr size_t kAlign = 256;
constexpr size_t kNoGrad = ~(size_t)0;
inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

struct Tensor {
  int h = 0, w = 0, c = 0;
  size_t elems = 0;        // per row
  size_t esize = 4;        // bytes per element of the stored activation and its gradient
  size_t act_off = 0;      // byte offsets into the workspace
  size_t grad_off = 0;
  size_t bits_off = 0;     // bf16 tensors with a folded ReLU and a multiple of 64 channels: one bit per element (0: none)
  bool relu = false;       // ReLU folded into the producer; grad buffer is w.r.t. the pre-ReLU value
  int consumers = 0;
};

struct Layer {
  omni_layer_desc d;
  int out = -1;            // tensor index
  int in0 = -1, in1 = -1;  // tensor indices (-1 = network input)
  int ih = 0, iw = 0, ic = 0;   // input shape
  size_t w_off = 0, b_off = 0;  // float offsets into params
  bool has_b = false;
  bool fused_away = false;      // ReLU merged into its producer
  // bf16 path
  int cin_pad = 0;              // input channels as the kernels see them (multiple of 8)
  size_t wsh_off = 0;           // bf16 weight copy [cout][taps][cin_pad], element offset into the shadow area
  size_t wt_off = 0;            // transposed copy [cin_pad][taps][cout] for dgrad
  bool need_dgrad = false;
  size_t stat_off = 0;          // batch norm: float offset of [K_max][C][2] statistics (then as many for the backward means)
  size_t code_off = 0;          // max pooling: byte offset of one code per output element (where its gradient goes)
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
  size_t shadow_off = 0, shadow_elems = 0, xpad_off = 0, conv_partial_off = 0, conv_counters_off = 0;
  size_t conv_partial2_off = 0;     // chunk scratch of the second side stream
  size_t bn_off = 0, bn_floats = 0, bn_partial_off = 0;
  size_t reduced_off = 0;           // g = sum_k lambda_k g_k, written only on request
  int bn_cmax = 0;
  // Where the last step left each tensor's gradient (byte offset into the workspace; kNoGrad: that step
  // did not store it).  Two tensors may share a buffer: a residual add hands its output gradient on.
  std::vector<size_t> grad_view;
  int classes = 0;
  const void* ws_ready = nullptr;   // workspace of the last step
  // optimiser: velocity == nullptr is plain SGD
  float* velocity = nullptr;
  float momentum = 0.f, weight_decay = 0.f;
  // Side stream for parameter-gradient kernels: they only feed the final update,
  // so they run beside the input-gradient chain instead of in front of it.
  // (Two of them, each with a chunk scratch of its own, taking the layers' weight gradients in turn:
  // one stream ran them strictly one after the other although they do not depend on each other.)
  hipStream_t side = nullptr, side2 = nullptr;
  std::vector<hipEvent_t> sync_ev;  // fork / join points of one step (timing disabled)
  // Optional replay of a repeated step as a HIP graph (omni_net_graph_enable): the key is everything
  // the launches depend on; a step whose key was seen the call before is captured, later ones replay.
  bool graph_on = false;
  std::vector<uint64_t> graph_key, seen_key;
  hipGraphExec_t graph_exec = nullptr;
  long graph_matches = 0;        // launches of the timed class inside the captured step
  long step_matches = 0;         // ... inside the step being enqueued
  long last_matches = -1;        // ... inside the last step enqueued launch by launch (-1: none yet)
  long graph_replays = 0;
  bool capturing = false;        // between begin and end of a stream capture: no event is recorded
  // optional event timing of one kernel class
  int time_class = -1, time_layer = -1;
  int time_every = 1;            // bracket every time_every-th matching launch
  long time_seen = 0;
  std::vector<hipEvent_t> ev;   // pairs: start, stop
  size_t ev_used = 0;           // events recorded since the last read

  ~omni_net() {
    for (hipEvent_t e : ev) (void)hipEventDestroy(e);
    for (hipEvent_t e : sync_ev) (void)hipEventDestroy(e);
    if (side) (void)hipStreamDestroy(side);
    if (side2) (void)hipStreamDestroy(side2);
    if (graph_exec) (void)hipGraphExecDestroy(graph_exec);
  }
};

namespace {
// Records an event pair around the launches made while it is alive, if the
// network is timing this (class, layer) and has event pairs left.
// With `exact`, the scope records nothing itself: timer() hands the pair to a launcher that binds it
// to its kernel's own start and end time stamps.
struct TimedScope {
  omni_net* net;
  hipStream_t st;
  bool on, exact;
  omni::KernelTimer kt{nullptr, nullptr};
  TimedScope(omni_net* n, hipStream_t s, int cls, int layer, bool exact_ = false) : net(n), st(s), exact(exact_) {
    const bool match = n->time_class == cls && (n->time_layer < 0 || n->time_layer == layer);
    if (match) n->step_matches++;
    on = match && n->ev_used + 2 <= n->ev.size();
    if (on) on = (n->time_seen++ % n->time_every) == 0;     // every time_every-th matching launch is timed
    if (n->capturing) on = false;   // (a step in which a launch is due for timing is not captured in the first place)
    if (on) kt = omni::KernelTimer{net->ev[net->ev_used], net->ev[net->ev_used + 1]};
    if (on && !exact) (void)hipEventRecord(kt.start, st);
  }
  const omni::KernelTimer* timer() const { return on && exact ? &kt : nullptr; }
  ~TimedScope() {
    if (on) {
      if (!exact) (void)hipEventRecord(kt.stop, st);
      net->ev_used += 2;
    }
  }
};

bool is_param_op(int op) { return op == OMNI_OP_LINEAR || op == OMNI_OP_CONV; }
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
  if (dtype != OMNI_F32 && dtype != OMNI_BF16) return fail(OMNI_EINVAL, "omni_net_create: dtype %d not supported", dtype);
  const bool bf = dtype == OMNI_BF16;

  omni_net* net = new (std::nothrow) omni_net();
  if (!net) return fail(OMNI_EINVAL, "omni_net_create: out of host memory");
  net->in_h = in_h; net->in_w = in_w; net->in_c = in_c;
  net->dtype = dtype; net->K_max = K_max; net->B_max = B_max;

  auto bail = [&](int code) { delete net; return code; };
  auto shape_of = [&](int t, int& h, int& w, int& c) {
    if (t < 0) { h = in_h; w = in_w; c = in_c; }
    else { h = net->tensors[t].h; w = net->tensors[t].w; c = net->tensors[t].c; }
  };
  auto new_tensor = [&](int h, int w, int c) {
    Tensor t; t.h = h; t.w = w; t.c = c; t.elems = (size_t)h * w * c; t.esize = bf ? 2 : 4;
    net->tensors.push_back(t);
    return (int)net->tensors.size() - 1;
  };

  size_t ppos = 0, shpos = 0, bnpos = 0;
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
    L.ih = h; L.iw = w; L.ic = c;
    switch (L.d.op) {
      case OMNI_OP_LINEAR: {
        if (L.d.cin != h * w * c || L.d.cout < 1)
          return bail(fail(OMNI_EINVAL, "layer %d: linear cin=%d does not match input %dx%dx%d", i, L.d.cin, h, w, c));
        L.out = new_tensor(1, 1, L.d.cout);
        L.w_off = ppos; ppos += (size_t)L.d.cout * L.d.cin;
        L.has_b = L.d.bias != 0;
        if (L.has_b) { L.b_off = ppos; ppos += (size_t)L.d.cout; }
        if (bf) {
          if (L.d.cin % 8 != 0) return bail(fail(OMNI_EINVAL, "layer %d: bf16 linear needs cin %% 8 == 0", i));
          if (i != n - 1 && L.d.cout % 8 != 0)
            return bail(fail(OMNI_EINVAL, "layer %d: a hidden bf16 linear layer needs cout %% 8 == 0", i));
          L.cin_pad = L.d.cin;
        }
        break;
      }
      case OMNI_OP_CONV: {
        if (!bf) return bail(fail(OMNI_EINVAL, "layer %d: convolution is implemented for dtype bf16 only", i));
        const int k = L.d.ksize, s = L.d.stride, p = L.d.pad;
        if (L.d.cin != c || L.d.cout < 1 || k < 1 || k > 7 || s < 1 || s > 4 || p < 0 || p >= k)
          return bail(fail(OMNI_EINVAL, "layer %d: bad convolution (cin=%d on %d channels, k=%d s=%d p=%d)", i, L.d.cin, c, k, s, p));
        const int ho = (h + 2 * p - k) / s + 1, wo = (w + 2 * p - k) / s + 1;
        if (ho < 1 || wo < 1) return bail(fail(OMNI_EINVAL, "layer %d: convolution output is empty", i));
        if (L.d.cout % 8 != 0) return bail(fail(OMNI_EINVAL, "layer %d: bf16 convolution needs cout %% 8 == 0", i));
        L.cin_pad = (c + 7) / 8 * 8;
        if (L.cin_pad != c && L.in0 >= 0)
          return bail(fail(OMNI_EINVAL, "layer %d: only the network input may have a channel count off the multiples of 8", i));
        if ((long)k * k * L.cin_pad > 8192 || (long)k * k * L.d.cout > 8192)
          return bail(fail(OMNI_EINVAL, "layer %d: reduction length above 8192 is not supported", i));
        L.out = new_tensor(ho, wo, L.d.cout);
        L.w_off = ppos; ppos += (size_t)L.d.cout * k * k * c;
        L.has_b = L.d.bias != 0;
        if (L.has_b) { L.b_off = ppos; ppos += (size_t)L.d.cout; }
        break;
      }
      case OMNI_OP_RELU: {
        if (L.in0 < 0) return bail(fail(OMNI_EINVAL, "layer %d: ReLU on the network input is not supported", i));
        const Layer& prod = net->layers[L.d.src];
        const bool ok_prod = prod.d.op == OMNI_OP_LINEAR || prod.d.op == OMNI_OP_CONV || prod.d.op == OMNI_OP_BN ||
                             prod.d.op == OMNI_OP_ADD;
        if (!ok_prod || prod.fused_away)
          return bail(fail(OMNI_EINVAL, "layer %d: ReLU after op %d is not supported", i, prod.d.op));
        if (net->tensors[L.in0].consumers != 0 || net->tensors[L.in0].relu)
          return bail(fail(OMNI_EINVAL, "layer %d: ReLU input must have no other consumer", i));
        net->tensors[L.in0].relu = true;
        L.out = L.in0;
        L.fused_away = true;
        continue;  // not a consumer in its own right
      }
      case OMNI_OP_MAXPOOL2: {
        if (!bf) return bail(fail(OMNI_EINVAL, "layer %d: max pooling is implemented for dtype bf16 only", i));
        if (L.in0 < 0 || h % 2 || w % 2 || c % 8)
          return bail(fail(OMNI_EINVAL, "layer %d: max pooling needs even H, W, channels %% 8 == 0 and a layer input", i));
        L.out = new_tensor(h / 2, w / 2, c);
        break;
      }
      case OMNI_OP_BN: {
        if (!bf) return bail(fail(OMNI_EINVAL, "layer %d: batch norm is implemented for dtype bf16 only", i));
        if (L.in0 < 0 || !omni::bn_shape_supported(c) || L.d.cin != c)
          return bail(fail(OMNI_EINVAL, "layer %d: batch norm needs a layer input with channels %% 8 == 0, at most 2048 (got %d, declared %d)", i, c, L.d.cin));
        if (net->tensors[L.in0].relu)
          return bail(fail(OMNI_EINVAL, "layer %d: batch norm directly after a folded ReLU is not supported", i));
        L.out = new_tensor(h, w, c);
        L.w_off = ppos; ppos += (size_t)c;      // gamma
        L.b_off = ppos; ppos += (size_t)c;      // beta
        L.has_b = true;
        L.stat_off = bnpos; bnpos += (size_t)K_max * c * 4;
        if (c > net->bn_cmax) net->bn_cmax = c;
        break;
      }
      case OMNI_OP_ADD: {
        if (!bf) return bail(fail(OMNI_EINVAL, "layer %d: residual add is implemented for dtype bf16 only", i));
        if (L.d.src2 < 0 || L.d.src2 >= i || L.in0 < 0)
          return bail(fail(OMNI_EINVAL, "layer %d: add needs two layer inputs", i));
        L.in1 = net->layers[L.d.src2].out;
        if (!net->layers[L.d.src2].fused_away && net->tensors[L.in1].relu)
          return bail(fail(OMNI_EINVAL, "layer %d: reads layer %d before its ReLU, which was folded into it", i, L.d.src2));
        const Tensor& tb = net->tensors[L.in1];
        if (tb.h != h || tb.w != w || tb.c != c || c % 8)
          return bail(fail(OMNI_EINVAL, "layer %d: add operands differ in shape", i));
        L.out = new_tensor(h, w, c);
        net->tensors[L.in1].consumers++;
        break;
      }
      case OMNI_OP_GAP: {
        if (!bf) return bail(fail(OMNI_EINVAL, "layer %d: global average pooling is implemented for dtype bf16 only", i));
        if (L.in0 < 0 || c % 8) return bail(fail(OMNI_EINVAL, "layer %d: pooling needs a layer input with channels %% 8 == 0", i));
        L.out = new_tensor(1, 1, c);
        break;
      }
      default:
        return bail(fail(OMNI_EINVAL, "layer %d: op %d not supported", i, L.d.op));
    }
    if (L.in0 >= 0) net->tensors[L.in0].consumers++;
    if (bf && is_param_op(L.d.op)) {
      const size_t taps = L.d.op == OMNI_OP_CONV ? (size_t)L.d.ksize * L.d.ksize : 1;
      const size_t cnt = align_up((size_t)L.d.cout * taps * L.cin_pad, 64);
      L.wsh_off = shpos; shpos += cnt;
      L.need_dgrad = L.in0 >= 0 && i != n - 1;   // the head computes its own input gradient
      if (L.need_dgrad) { L.wt_off = shpos; shpos += cnt; }
    }
  }
  for (const Layer& L : net->layers)
    if ((L.d.op == OMNI_OP_MAXPOOL2 || L.d.op == OMNI_OP_BN) && net->tensors[L.in0].consumers != 1)
      return bail(fail(OMNI_EINVAL, "the input of a max pooling or batch norm layer must have no other consumer"));
  net->bn_floats = bnpos;
  net->P = ppos;
  net->P_stride = align_up(ppos, 64);
  net->shadow_elems = shpos;
  const Layer& lastL = net->layers[n - 1];
  const Tensor& last = net->tensors[lastL.out];
  if (last.h != 1 || last.w != 1) return bail(fail(OMNI_EINVAL, "last layer must produce [rows][classes]"));
  if (last.relu) return bail(fail(OMNI_EINVAL, "logits must not pass through ReLU"));
  net->classes = last.c;
  if (bf) {
    if (lastL.d.op != OMNI_OP_LINEAR || lastL.d.cin > 2048 || lastL.d.cout > 128)
      return bail(fail(OMNI_EINVAL, "bf16 networks must end in a linear layer with cin <= 2048 and at most 128 outputs"));
    if ((long)B_max * in_h * in_w >= (1L << 24))
      return bail(fail(OMNI_ECAPACITY, "B_max * H * W must stay below 2^24 positions"));
    net->tensors[lastL.out].esize = 4;   // logits and their gradient stay fp32
  }

  size_t pos = 0;
  auto take = [&](size_t bytes) { const size_t o = pos; pos += align_up(bytes, kAlign); return o; };
  net->grads_off = take((size_t)K_max * net->P_stride * sizeof(float));
  net->reduced_off = take(net->P_stride * sizeof(float));
  net->loss_rows_off = take((size_t)B_max * sizeof(float));
  net->status_off = take(kAlign);
  net->counters_off = take(omni::kSplitMaxTiles * sizeof(uint32_t));
  net->partial_off = take(omni::kSplitPartialFloats * sizeof(float));
  if (bf) {
    net->conv_counters_off = take(omni::kZeroPageWords * sizeof(uint32_t));
    net->conv_partial_off = take(omni::conv_wgrad_partial_floats() * sizeof(float));
    net->conv_partial2_off = take(omni::conv_wgrad_partial_floats() * sizeof(float));
    net->shadow_off = take(net->shadow_elems * 2);
    if (in_c % 8 != 0) net->xpad_off = take((size_t)B_max * in_h * in_w * ((in_c + 7) / 8 * 8) * 2);
    if (net->bn_floats) {
      net->bn_off = take(net->bn_floats * sizeof(float));
      net->bn_partial_off = take((size_t)K_max * omni::kBnMaxSplits * net->bn_cmax * 2 * sizeof(double));
    }
  }
  for (Tensor& t : net->tensors) {
    const size_t bytes = (size_t)B_max * t.elems * t.esize;
    t.act_off = take(bytes);
    t.grad_off = take(bytes);
  }
  for (Layer& L : net->layers)
    if (L.d.op == OMNI_OP_MAXPOOL2) L.code_off = take((size_t)B_max * net->tensors[L.out].elems);
  // where a batch norm writes a tensor with a folded ReLU, it also leaves "stored value > 0" at one bit per
  // element: all that the input-gradient kernels need of that tensor
  if (bf && net->bn_floats)
    for (Tensor& t : net->tensors)
      if (t.relu && t.esize == 2 && t.c % 64 == 0) t.bits_off = take((size_t)B_max * t.elems / 8);
  net->ws_bytes = pos;
  net->grad_view.assign(net->tensors.size(), kNoGrad);
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

const float* omni_net_reduced_grad(const omni_net* net, const void* ws) {
  if (!net || !ws) return nullptr;
  return reinterpret_cast<const float*>(static_cast<const char*>(ws) + net->reduced_off);
}
int omni_net_activation_grad(const omni_net* net, const void* ws, int32_t layer, const void** ptr, size_t* elems) {
  if (!net || !ws || !ptr || !elems) return fail(OMNI_EINVAL, "omni_net_activation_grad: NULL argument");
  if (layer < 0 || layer >= (int)net->layers.size())
    return fail(OMNI_EINVAL, "omni_net_activation_grad: bad layer %d", layer);
  const int t = net->layers[layer].out;
  if (net->grad_view[t] == kNoGrad)
    return fail(OMNI_EINVAL, "omni_net_activation_grad: the last step did not store the gradient of layer %d's output", layer);
  *ptr = static_cast<const char*>(ws) + net->grad_view[t];
  *elems = net->tensors[t].elems;
  return OMNI_OK;
}

void omni_net_destroy(omni_net* net) { delete net; }

int omni_net_timing_enable(omni_net* net, int32_t kernel_class, int32_t layer, int32_t max_launches) {
  if (!net) return fail(OMNI_EINVAL, "omni_net_timing_enable: NULL net");
  if (kernel_class >= OMNI_KERNEL_CLASSES) return fail(OMNI_EINVAL, "omni_net_timing_enable: bad class %d", kernel_class);
  net->ev_used = 0;
  // how many launches of the timed class a step has is learnt from the next step enqueued launch by
  // launch; a captured step counted them for the class of its day
  net->last_matches = -1;
  net->graph_matches = 0;
  if (net->graph_exec) { (void)hipGraphExecDestroy(net->graph_exec); net->graph_exec = nullptr; }
  net->graph_key.clear();
  net->seen_key.clear();
  if (kernel_class < 0) { net->time_class = -1; return OMNI_OK; }
  if (max_launches < 1 || max_launches > (1 << 20)) return fail(OMNI_EINVAL, "omni_net_timing_enable: bad max_launches");
  while (net->ev.size() < (size_t)max_launches * 2) {
    hipEvent_t e;
    OMNI_HIP_CHECK(hipEventCreate(&e));
    net->ev.push_back(e);
  }
  net->time_class = kernel_class;
  net->time_layer = layer;
  net->time_seen = 0;
  return OMNI_OK;
}

int omni_net_timing_sample(omni_net* net, int32_t every) {
  if (!net) return fail(OMNI_EINVAL, "omni_net_timing_sample: NULL net");
  if (every < 1) return fail(OMNI_EINVAL, "omni_net_timing_sample: every=%d", every);
  net->time_every = every;
  net->time_seen = 0;
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

}  // extern "C"

namespace {

struct StepCtx {
  omni_net* net;
  hipStream_t st;
  hipStream_t side;      // equals st when no side stream could be made
  hipStream_t side2;     // equals side when no second one could be made
  size_t sync_used = 0;
  // a side stream may start once everything enqueued on the main stream so far is done
  void fork(hipStream_t& to) {
    if (to == st) return;
    if (sync_used == net->sync_ev.size()) {
      hipEvent_t e;
      if (hipEventCreateWithFlags(&e, hipEventDisableTiming) != hipSuccess) { to = st; return; }
      net->sync_ev.push_back(e);
    }
    hipEvent_t e = net->sync_ev[sync_used++];
    (void)hipEventRecord(e, st);
    (void)hipStreamWaitEvent(to, e, 0);
  }
  void fork() { fork(side); }
  // The two halves of a fork, for when main-stream work is enqueued in between: the side stream
  // then waits only for what preceded the record, and the main stream's next kernel is not held up
  // by the host calls that set the side stream going.
  hipEvent_t fork_record() {
    if (side == st && side2 == st) return nullptr;   // one stream only: nothing to order
    if (sync_used == net->sync_ev.size()) {
      hipEvent_t e;
      if (hipEventCreateWithFlags(&e, hipEventDisableTiming) != hipSuccess) return nullptr;
      net->sync_ev.push_back(e);
    }
    hipEvent_t e = net->sync_ev[sync_used++];
    (void)hipEventRecord(e, st);
    return e;
  }
  void fork_wait(hipStream_t& to, hipEvent_t e) {
    if (to == st) return;
    if (!e) { to = st; return; }   // no event: fall back to the main stream (ordered by itself)
    (void)hipStreamWaitEvent(to, e, 0);
  }
  // the main stream waits for everything enqueued on the side streams so far
  void join_one(hipStream_t from) {
    if (from == st) return;
    if (sync_used == net->sync_ev.size()) {
      hipEvent_t e;
      if (hipEventCreateWithFlags(&e, hipEventDisableTiming) != hipSuccess) { (void)hipStreamSynchronize(from); return; }
      net->sync_ev.push_back(e);
    }
    hipEvent_t e = net->sync_ev[sync_used++];
    (void)hipEventRecord(e, from);
    (void)hipStreamWaitEvent(st, e, 0);
  }
  void join() {
    if (!forked) return;
    join_one(side);
    if (side2 != side && forked2) join_one(side2);
  }
  bool forked = false, forked2 = false;
  char* ws;
  float* params;
  const void* x;
  const int32_t* labels;
  int rows;
  omni::Segments seg;
  float* G;
  float* loss_rows;
  uint32_t* status;
  float* loss_per_worker;
  float* loss;
};

// ------------------------------------------------------------------ fp32 path
void step_f32(StepCtx& c) {
  omni_net* net = c.net;
  hipStream_t st = c.st;
  auto act = [&](int t) -> const float* {
    return t < 0 ? static_cast<const float*>(c.x) : reinterpret_cast<const float*>(c.ws + net->tensors[t].act_off);
  };
  auto actw = [&](int t) { return reinterpret_cast<float*>(c.ws + net->tensors[t].act_off); };
  auto grad = [&](int t) { return reinterpret_cast<float*>(c.ws + net->tensors[t].grad_off); };
  float* params = c.params;
  const int rows = c.rows;

  omni::SplitWorkspace sw;
  sw.partial = reinterpret_cast<float*>(c.ws + net->partial_off);
  sw.counters = reinterpret_cast<uint32_t*>(c.ws + net->counters_off);
  // The arrival counters of the split reductions must be zero when a launch that uses them starts.
  // Every such launch leaves them zero, but the workspace is the caller's memory (fresh, re-allocated at
  // the same address, shared with another network, written in between): the first launch of a step
  // that may split its reduction is therefore preceded by a fill.  A step whose products all take the
  // small-batch kernel never touches the counters and pays nothing.
  bool counters_clear = false;
  auto before_split_launch = [&]() {
    if (counters_clear) return;
    omni::fill_u32(st, sw.counters, omni::kSplitMaxTiles, 0u);
    counters_clear = true;
  };

  const int n_layers = (int)net->layers.size();
  const Layer& last = net->layers[n_layers - 1];
  const bool fused_head = last.d.op == OMNI_OP_LINEAR &&
                          omni::head_supported(last.d.cin, last.d.cout, act(last.in0), params + last.w_off, false);

  // ---- forward over the concatenated batch
  for (int i = 0; i < n_layers; ++i) {
    const Layer& L = net->layers[i];
    if (L.fused_away || (fused_head && i == n_layers - 1)) continue;
    if (!omni::linear_fwd_f32_direct_supported(act(L.in0), params + L.w_off, rows, L.d.cin, L.d.cout))
      before_split_launch();
    TimedScope ts(net, st, OMNI_KERNEL_LINEAR_FWD, i);
    omni::linear_fwd_f32(st, act(L.in0), params + L.w_off, L.has_b ? params + L.b_off : nullptr, actw(L.out), rows,
                         L.d.cin, L.d.cout, net->tensors[L.out].relu, sw);
  }

  // ---- loss: dz already carries 1/b_k, so everything downstream is a per-worker mean gradient
  const int logits = last.out;
  std::vector<char> written(net->tensors.size(), 0);
  int merge_layer = -1;
  omni::HeadWgradParams head_wgrad{};
  if (fused_head) {
    TimedScope ts(net, st, OMNI_KERNEL_LOSS, n_layers - 1);
    const bool need_dx = last.in0 >= 0;
    omni::head_fwd_loss_dgrad(st, false, act(last.in0), params + last.w_off,
                              last.has_b ? params + last.b_off : nullptr, c.labels, last.d.cin, last.d.cout, c.seg,
                              actw(logits), grad(logits), c.loss_rows, need_dx && net->tensors[last.in0].relu,
                              need_dx ? grad(last.in0) : nullptr, false);
    if (need_dx) written[last.in0] = 1;
    // The head's parameter gradients and the next layer's input gradient both wait for this kernel only:
    // where the latter takes the small-batch kernel the two share a launch (below), reported as that layer's dgrad.
    for (int i = n_layers - 2; i >= 0 && merge_layer < 0; --i) {
      const Layer& L = net->layers[i];
      if (L.fused_away) continue;
      if (L.in0 >= 0 && omni::linear_dgrad_f32_direct_supported(grad(L.out), params + L.w_off,
                                                                net->tensors[L.in0].relu ? act(L.in0) : nullptr,
                                                                grad(L.in0), rows, L.d.cin, L.d.cout))
        merge_layer = i;
      break;
    }
    head_wgrad = omni::HeadWgradParams{grad(logits), act(last.in0), c.labels, last.d.cin, last.d.cout,
                                       c.G + last.w_off, last.has_b ? c.G + last.b_off : nullptr, net->P_stride,
                                       c.loss_rows, c.loss_per_worker, c.loss, c.status};
    if (merge_layer < 0)
      omni::head_wgrad_loss(st, false, head_wgrad.dz, head_wgrad.x, head_wgrad.labels, head_wgrad.cin, head_wgrad.C,
                            c.seg, head_wgrad.gw, head_wgrad.gb, head_wgrad.worker_stride, head_wgrad.loss_rows,
                            head_wgrad.loss_per_worker, head_wgrad.loss, head_wgrad.status);
  } else {
    TimedScope ts(net, st, OMNI_KERNEL_LOSS, n_layers - 1);
    omni::fill_u32(st, c.status, 1, 0u);
    omni::softmax_xent_f32(st, act(logits), c.labels, net->classes, c.seg, grad(logits), c.loss_rows,
                           c.loss_per_worker, c.loss, c.status);
  }

  // ---- backward: input gradients on all rows first, then the parameter gradients of ALL layers per
  // worker in one launch (every layer's output gradient has a buffer of its own, so they can wait;
  // one launch has one start-up and one drain instead of one per layer).
  // (No side stream here: at this size a cross-stream fork and join each cost about 10 us of
  // idle GPU, more than the overlap returns; measured.)
  std::vector<omni::LinearWgradJob> jobs;
  int first_job_layer = -1;
  for (int i = n_layers - 1; i >= 0; --i) {
    const Layer& L = net->layers[i];
    if (L.fused_away || (fused_head && i == n_layers - 1)) continue;
    jobs.push_back({grad(L.out), act(L.in0), c.G + L.w_off, L.has_b ? c.G + L.b_off : nullptr, L.d.cin, L.d.cout});
    first_job_layer = i;
    if (L.in0 >= 0) {
      const Tensor& ti = net->tensors[L.in0];
      const float* mask = ti.relu ? act(L.in0) : nullptr;
      if (i != merge_layer &&
          !omni::linear_dgrad_f32_direct_supported(grad(L.out), params + L.w_off, mask, grad(L.in0), rows, L.d.cin,
                                                   L.d.cout))
        before_split_launch();
      TimedScope ts(net, st, OMNI_KERNEL_LINEAR_DGRAD, i);
      if (i == merge_layer)   // (chosen above by the very test the shared launcher requires)
        omni::linear_dgrad_f32_with_head_wgrad(st, grad(L.out), params + L.w_off, mask, grad(L.in0), rows, L.d.cin,
                                               L.d.cout, written[L.in0] != 0, head_wgrad, c.seg);
      else
        omni::linear_dgrad_f32(st, grad(L.out), params + L.w_off, mask, grad(L.in0), rows, L.d.cin, L.d.cout,
                               written[L.in0] != 0, sw);
      written[L.in0] = 1;
    }
  }
  if (!jobs.empty()) {
    // reported under the lowest layer it covers
    TimedScope ts(net, st, OMNI_KERNEL_LINEAR_WGRAD, first_job_layer, true);
    // (last layer's problem first in the launch: measured 47.1 us against 48.8 us the other way round)
    omni::linear_wgrad_f32_batch(st, jobs.data(), (int)jobs.size(), net->P_stride, c.seg, ts.timer());
  }
  for (size_t t = 0; t < net->tensors.size(); ++t)
    net->grad_view[t] = (written[t] || (int)t == logits) ? net->tensors[t].grad_off : kNoGrad;
}

// ------------------------------------------------------------------ bf16 path
void step_bf16(StepCtx& c) {
  using omni::bf16_t;
  omni_net* net = c.net;
  hipStream_t st = c.st;
  const int rows = c.rows;
  bf16_t* shadow = reinterpret_cast<bf16_t*>(c.ws + net->shadow_off);
  const int in_c_pad = (net->in_c + 7) / 8 * 8;
  const bf16_t* x_in = static_cast<const bf16_t*>(c.x);
  bool raw_input = false;   // the layers that read the network input take its 3 channels as they are
  auto act = [&](int t) -> const bf16_t* {
    return t < 0 ? x_in : reinterpret_cast<const bf16_t*>(c.ws + net->tensors[t].act_off);
  };
  auto actw = [&](int t) { return reinterpret_cast<bf16_t*>(c.ws + net->tensors[t].act_off); };
  // A tensor's gradient normally has a buffer of its own; where it would be a plain copy of another
  // tensor's gradient (a residual add passes its output gradient on unchanged to an input that has no
  // folded ReLU and no other consumer), it is that other buffer.
  std::vector<bf16_t*> grad_alias(net->tensors.size(), nullptr);
  auto grad = [&](int t) {
    return grad_alias[t] ? grad_alias[t] : reinterpret_cast<bf16_t*>(c.ws + net->tensors[t].grad_off);
  };
  float* bn_area = reinterpret_cast<float*>(c.ws + net->bn_off);
  double* bn_partial = reinterpret_cast<double*>(c.ws + net->bn_partial_off);
  float* conv_partial = reinterpret_cast<float*>(c.ws + net->conv_partial_off);
  uint32_t* conv_counters = reinterpret_cast<uint32_t*>(c.ws + net->conv_counters_off);

  const int n_layers = (int)net->layers.size();
  const Layer& last = net->layers[n_layers - 1];

  // geometry of a parameter layer's forward gather
  auto fwd_geom = [&](const Layer& L) {
    omni::ConvGeom g{};
    g.rows = rows;
    if (L.d.op == OMNI_OP_CONV) {
      const Tensor& to = net->tensors[L.out];
      g.Hs = L.ih; g.Ws = L.iw; g.Cs = L.cin_pad; g.Hp = to.h; g.Wp = to.w;
      g.ks = L.d.ksize; g.stride = L.d.stride; g.pad = L.d.pad;
    } else {
      g.Hs = 1; g.Ws = 1; g.Cs = L.cin_pad; g.Hp = 1; g.Wp = 1; g.ks = 1; g.stride = 1; g.pad = 0;
    }
    g.transposed = 0;
    g.K = g.ks * g.ks * g.Cs;
    g.zero = conv_counters;   // a few bytes of zeros, cleared by this step's first launch and not written otherwise
    g.raw3 = (raw_input && L.in0 < 0) ? 1 : 0;
    return g;
  };

  // ---- the network input: channel counts that are no multiple of 8 are padded into a copy, unless
  // every layer that reads the input is a first-layer convolution whose kernels read 3 channels directly
  if (in_c_pad != net->in_c) {
    raw_input = net->in_c == 3;
    for (int i = 0; i < n_layers && raw_input; ++i) {
      const Layer& L = net->layers[i];
      if (L.fused_away || L.in0 >= 0) continue;
      if (L.d.op != OMNI_OP_CONV) { raw_input = false; break; }
      const Tensor& to = net->tensors[L.out];
      raw_input = false;   // (fwd_geom reads the flag: ask with the padded layout's geometry)
      const omni::ConvGeom g = fwd_geom(L);
      raw_input = omni::conv_first_layer_raw_supported(L.d.cout, L.d.cin, g, (long)rows * to.h * to.w);
    }
    if (!raw_input) {
      bf16_t* xp = reinterpret_cast<bf16_t*>(c.ws + net->xpad_off);
      omni::pad_channels_bf16(st, x_in, xp, (long)rows * net->in_h * net->in_w, net->in_c, in_c_pad);
      x_in = xp;
    }
  }

  // ---- bf16 copies of the weights (forward layout, and transposed for dgrad)
  {
    std::vector<omni::CastEntry> casts;
    for (const Layer& L : net->layers) {
      if (!is_param_op(L.d.op)) continue;
      omni::CastEntry e{};
      e.src = (long)L.w_off; e.dst_fwd = (long)L.wsh_off; e.dst_t = L.need_dgrad ? (long)L.wt_off : -1;
      e.cout = L.d.cout;
      e.taps = L.d.op == OMNI_OP_CONV ? L.d.ksize * L.d.ksize : 1;
      e.cin_real = L.d.op == OMNI_OP_CONV ? L.d.cin : L.cin_pad;
      e.cin_pad = L.cin_pad;
      casts.push_back(e);
    }
    // (the same launch clears the few bytes of zeros that loads of absent pieces are pointed at: the workspace
    // is the caller's memory, so nothing in it is taken to have survived since the last step)
    omni::cast_weights_bf16(st, c.params, shadow, casts.data(), (int)casts.size(), conv_counters);
  }

  // ---- forward over the concatenated batch
  int pooled_layer = -1;   // a max pooling layer whose output the convolution before it has already written
  int added_layer = -1;    // a residual add that the batch norm before it has already done
  std::vector<char> bits_written(net->tensors.size(), 0);   // tensors whose sign bits this step's forward pass wrote
  auto sign_bits = [&](int t) {
    return net->tensors[t].bits_off ? reinterpret_cast<uint8_t*>(c.ws + net->tensors[t].bits_off) : nullptr;
  };
  int presummed_for = -1;  // a batch norm whose statistics' first pass the convolution before it has already done
  omni::ShareTable presummed{};
  std::vector<char> coded(n_layers, 0);   // ... together with the codes its backward pass then reads
  for (int i = 0; i < n_layers - 1; ++i) {
    const Layer& L = net->layers[i];
    if (L.fused_away) continue;
    if (is_param_op(L.d.op)) {
      TimedScope ts(net, st, L.d.op == OMNI_OP_CONV ? OMNI_KERNEL_CONV_FWD : OMNI_KERNEL_LINEAR_FWD, i);
      const omni::ConvGeom g = fwd_geom(L);
      const Tensor& to = net->tensors[L.out];
      // the next layer that runs, if it pools this layer's output (its only consumer then)
      int nx = i + 1;
      while (nx < n_layers - 1 && net->layers[nx].fused_away) ++nx;
      const bool pool_next = L.d.op == OMNI_OP_CONV && nx < n_layers - 1 &&
                             net->layers[nx].d.op == OMNI_OP_MAXPOOL2 && net->layers[nx].in0 == L.out;
      // ... or normalises it: the convolution is then offered the first pass of the statistics (the sums of
      // what it stores), which the kernels that hold a worker-pure group of positions take
      const bool bn_next = L.d.op == OMNI_OP_CONV && nx < n_layers - 1 && net->layers[nx].d.op == OMNI_OP_BN &&
                           net->layers[nx].in0 == L.out && !to.relu && !L.has_b;
      omni::BnStatRequest offer{bn_partial, &c.seg, {}, false};
      const bool pooled =
          omni::conv_gemm_bf16(st, act(L.in0), shadow + L.wsh_off, actw(L.out), rows * to.h * to.w, L.d.cout, g,
                               L.has_b ? c.params + L.b_off : nullptr, nullptr, to.relu, false,
                               pool_next ? actw(net->layers[nx].out) : nullptr,
                               pool_next ? reinterpret_cast<uint8_t*>(c.ws + net->layers[nx].code_off) : nullptr,
                               nullptr, bn_next ? &offer : nullptr);
      if (pooled) { pooled_layer = nx; coded[nx] = 1; }
      if (bn_next && offer.done) { presummed = offer.table; presummed_for = nx; }
    } else if (L.d.op == OMNI_OP_MAXPOOL2) {
      if (i != pooled_layer) omni::maxpool2_fwd_bf16(st, act(L.in0), actw(L.out), rows, L.ih, L.iw, L.ic);
    } else if (L.d.op == OMNI_OP_BN) {
      // a residual add that comes next and is this tensor's only consumer is done by the same kernel:
      // the normalised tensor itself is then never stored (nothing in the backward pass reads it)
      int nx = i + 1;
      while (nx < n_layers - 1 && net->layers[nx].fused_away) ++nx;
      const Layer& A = net->layers[nx];
      const bool add_next = nx < n_layers - 1 && A.d.op == OMNI_OP_ADD && (A.in0 == L.out) != (A.in1 == L.out) &&
                            net->tensors[L.out].consumers == 1 && !net->tensors[L.out].relu;
      if (add_next) {
        const int other = A.in0 == L.out ? A.in1 : A.in0;
        omni::bn_forward_bf16(st, act(L.in0), actw(A.out), c.params + L.w_off, c.params + L.b_off, L.ic, L.ih * L.iw,
                              c.seg, false, bn_area + L.stat_off, bn_partial, act(other), net->tensors[A.out].relu,
                              i == presummed_for ? &presummed : nullptr,
                              net->tensors[A.out].relu ? sign_bits(A.out) : nullptr);
        if (net->tensors[A.out].relu && sign_bits(A.out)) bits_written[A.out] = 1;
        added_layer = nx;
      } else {
        omni::bn_forward_bf16(st, act(L.in0), actw(L.out), c.params + L.w_off, c.params + L.b_off, L.ic, L.ih * L.iw,
                              c.seg, net->tensors[L.out].relu, bn_area + L.stat_off, bn_partial, nullptr, false,
                              i == presummed_for ? &presummed : nullptr,
                              net->tensors[L.out].relu ? sign_bits(L.out) : nullptr);
        if (net->tensors[L.out].relu && sign_bits(L.out)) bits_written[L.out] = 1;
      }
    } else if (L.d.op == OMNI_OP_ADD) {
      if (i != added_layer)
        omni::add_fwd_bf16(st, act(L.in0), act(L.in1), actw(L.out), (long)rows * L.ih * L.iw * L.ic,
                           net->tensors[L.out].relu);
    } else if (L.d.op == OMNI_OP_GAP) {
      omni::gap_fwd_bf16(st, act(L.in0), actw(L.out), rows, L.ih * L.iw, L.ic);
    }
  }

  // ---- classifier head: logits, loss, dz (with 1/b_k), first input gradient, head parameter gradients
  std::vector<char> written(net->tensors.size(), 0);
  {
    TimedScope ts(net, st, OMNI_KERNEL_LOSS, n_layers - 1);
    const int logits = last.out;
    float* z = reinterpret_cast<float*>(c.ws + net->tensors[logits].act_off);
    float* dz = reinterpret_cast<float*>(c.ws + net->tensors[logits].grad_off);
    const bool need_dx = last.in0 >= 0;
    omni::head_fwd_loss_dgrad(st, true, act(last.in0), shadow + last.wsh_off,
                              last.has_b ? c.params + last.b_off : nullptr, c.labels, last.d.cin, last.d.cout, c.seg,
                              z, dz, c.loss_rows, need_dx && net->tensors[last.in0].relu,
                              need_dx ? grad(last.in0) : nullptr, false);
    if (need_dx) written[last.in0] = 1;
    c.fork();
    c.forked = true;
    omni::head_wgrad_loss(c.side, true, dz, act(last.in0), c.labels, last.d.cin, last.d.cout, c.seg, c.G + last.w_off,
                          last.has_b ? c.G + last.b_off : nullptr, net->P_stride, c.loss_rows, c.loss_per_worker,
                          c.loss, c.status);
  }

  // ---- backward
  // A max pooling right after the FIRST layer (which needs no input gradient) does not write that
  // layer's output gradient out: the layer's weight-gradient kernel reads the pooled gradient and
  // the pooling's codes itself.  pooled_from[j] = that pooling layer, for conv layer j.
  std::vector<int> pooled_from(n_layers, -1);
  std::vector<char> not_stored(net->tensors.size(), 0);   // ... and such a gradient exists nowhere
  // A residual add's gradient for an input that a convolution also reads is not routed by a pass of
  // its own: that convolution's input-gradient kernel adds it before its ReLU mask.
  std::vector<const bf16_t*> pending_add(net->tensors.size(), nullptr);
  float* conv_partial2 = reinterpret_cast<float*>(c.ws + net->conv_partial2_off);
  bool second = false;   // which side stream (and scratch) takes the next weight gradient
  // The entry of a residual block: its input feeds a 3x3 / stride-2 convolution and the 1x1 / stride-2
  // projection of the shortcut, and nothing else.  The projection comes first in this backward walk: its
  // input gradient is not launched on its own but handed to the 3x3 convolution's, whose kernel writes
  // both contributions in one pass.  partner[m] = the projection layer whose gradient conv m takes along.
  std::vector<int> partner(n_layers, -1);
  auto entry_partner = [&](int sc) {   // the 3x3 / stride-2 convolution beside projection layer sc, or -1
    const Layer& S = net->layers[sc];
    if (S.d.op != OMNI_OP_CONV || S.d.ksize != 1 || S.d.stride != 2 || S.d.pad != 0 || S.in0 < 0) return -1;
    if (net->tensors[S.in0].consumers != 2 || written[S.in0] || pending_add[S.in0]) return -1;
    for (int m = sc - 1; m >= 0; --m) {
      const Layer& M = net->layers[m];
      if (M.fused_away || M.d.op != OMNI_OP_CONV || M.in0 != S.in0) continue;
      const bool shape = M.d.ksize == 3 && M.d.stride == 2 && M.d.pad == 1 && M.cin_pad == S.cin_pad &&
                         net->tensors[M.out].h == net->tensors[S.out].h && net->tensors[M.out].w == net->tensors[S.out].w;
      return shape && omni::conv3s2_dgrad_supported(rows, M.ih, M.iw, M.cin_pad, M.d.cout, S.d.cout) ? m : -1;
    }
    return -1;
  };
  for (int i = n_layers - 2; i >= 0; --i) {
    const Layer& L = net->layers[i];
    if (L.fused_away) continue;
    if (is_param_op(L.d.op)) {
      const omni::ConvGeom g = fwd_geom(L);
      const Tensor& to = net->tensors[L.out];
      const bool conv = L.d.op == OMNI_OP_CONV;
      // Parameter gradients run on the side streams beside the input-gradient chain.  ALL of
      // them do, the first layer's included.  The point they wait for is recorded first, then the
      // input gradient goes to the main stream, and only then are the side stream's wait and
      // launches issued: the main chain (the longer one) never waits for those host calls.
      hipEvent_t ready = c.fork_record();
      const int takes_me = conv && L.in0 >= 0 ? entry_partner(i) : -1;
      if (takes_me >= 0) partner[takes_me] = i;   // (this projection's input gradient rides with that convolution's)
      bool dgrad_done = takes_me >= 0;
      if (L.in0 >= 0 && !dgrad_done && conv && L.d.ksize == 3 && L.d.stride == 2 && L.d.pad == 1) {
        // a stride-2 3x3 convolution: the one-pass kernel, with the shortcut's projection if it waits for it
        TimedScope ts(net, st, OMNI_KERNEL_CONV_DGRAD, i);
        const Tensor& ti = net->tensors[L.in0];
        const int sc = partner[i];
        const bf16_t* addend = pending_add[L.in0];
        dgrad_done = omni::conv3s2_dgrad_bf16(
            st, grad(L.out), shadow + L.wt_off, L.d.cout, sc >= 0 ? grad(net->layers[sc].out) : nullptr,
            sc >= 0 ? shadow + net->layers[sc].wt_off : nullptr, sc >= 0 ? net->layers[sc].d.cout : 0, grad(L.in0), rows,
            L.ih, L.iw, L.cin_pad, ti.relu ? act(L.in0) : nullptr, written[L.in0] != 0, addend, conv_counters,
            (ti.relu && bits_written[L.in0]) ? sign_bits(L.in0) : nullptr);
        if (dgrad_done) { pending_add[L.in0] = nullptr; written[L.in0] = 1; }
        // (entry_partner asked conv3s2_dgrad_supported with these very shapes: a projection is never left behind)
      }
      if (L.in0 >= 0 && !dgrad_done) {
        TimedScope ts(net, st, conv ? OMNI_KERNEL_CONV_DGRAD : OMNI_KERNEL_LINEAR_DGRAD, i);
        omni::ConvGeom d = g;
        d.Hs = to.h; d.Ws = to.w; d.Cs = L.d.cout;      // gather from dY
        d.Hp = L.ih; d.Wp = L.iw;                        // one GEMM row per input position
        if (!conv) { d.Hp = 1; d.Wp = 1; }
        d.transposed = 1;
        d.K = d.ks * d.ks * d.Cs;
        const Tensor& ti = net->tensors[L.in0];
        const int m_rows = conv ? rows * L.ih * L.iw : rows;
        const bf16_t* addend = pending_add[L.in0];
        pending_add[L.in0] = nullptr;
        d.mask_bits = (ti.relu && bits_written[L.in0]) ? sign_bits(L.in0) : nullptr;
        omni::conv_gemm_bf16(st, grad(L.out), shadow + L.wt_off, grad(L.in0), m_rows, L.cin_pad, d, nullptr,
                             ti.relu ? act(L.in0) : nullptr, false, written[L.in0] != 0, nullptr, nullptr, addend);
        written[L.in0] = 1;
      }
      {
        const bool use2 = second && c.side2 != c.side;
        second = !second;
        c.fork_wait(use2 ? c.side2 : c.side, ready);
        c.forked = true;
        if (use2) c.forked2 = true;
        hipStream_t ws_ = use2 ? c.side2 : c.side;
        TimedScope ts(net, ws_, conv ? OMNI_KERNEL_CONV_WGRAD : OMNI_KERNEL_LINEAR_WGRAD, i);
        const int pl = pooled_from[i];
        omni::conv_wgrad_bf16(ws_, grad(L.out), act(L.in0), c.G + L.w_off, L.has_b ? c.G + L.b_off : nullptr,
                              net->P_stride, L.d.cout, L.d.cin, g, c.seg, use2 ? conv_partial2 : conv_partial,
                              conv_counters,
                              pl >= 0 ? grad(net->layers[pl].out) : nullptr,
                              pl >= 0 ? reinterpret_cast<const uint8_t*>(c.ws + net->layers[pl].code_off) : nullptr);
      }
    } else if (L.d.op == OMNI_OP_MAXPOOL2) {
      int prod = -1;   // the layer that produced the pooling's input
      for (int j = i - 1; j >= 0 && prod < 0; --j)
        if (!net->layers[j].fused_away && net->layers[j].out == L.in0) prod = j;
      if (coded[i] && prod >= 0 && net->layers[prod].d.op == OMNI_OP_CONV && net->layers[prod].in0 < 0 &&
          omni::conv_wgrad_pooled_supported(net->layers[prod].d.cout, net->layers[prod].d.cin,
                                            fwd_geom(net->layers[prod]))) {
        pooled_from[prod] = i;
        not_stored[L.in0] = 1;
      } else if (coded[i])
        omni::maxpool2_bwd_coded_bf16(st, reinterpret_cast<const uint8_t*>(c.ws + L.code_off), grad(L.out),
                                      grad(L.in0), rows, L.ih, L.iw, L.ic);
      else
        omni::maxpool2_bwd_bf16(st, act(L.in0), grad(L.out), grad(L.in0), rows, L.ih, L.iw, L.ic,
                                net->tensors[L.in0].relu);
      written[L.in0] = 1;
    } else if (L.d.op == OMNI_OP_BN) {
      float* stats = bn_area + L.stat_off;
      omni::bn_backward_bf16(st, act(L.in0), grad(L.out), grad(L.in0), c.params + L.w_off, L.ic, L.ih * L.iw, c.seg,
                             stats, stats + (size_t)net->K_max * L.ic * 2, bn_partial, c.G + L.w_off, c.G + L.b_off,
                             net->P_stride);
      written[L.in0] = 1;
    } else if (L.d.op == OMNI_OP_ADD) {
      const long elems = (long)rows * L.ih * L.iw * L.ic;
      for (int t : {L.in0, L.in1}) {
        if (!net->tensors[t].relu && net->tensors[t].consumers == 1 && !written[t]) {
          grad_alias[t] = grad(L.out);   // nothing to mask, nothing to add to: no copy
          written[t] = 1;
          continue;
        }
        if (net->tensors[t].consumers == 2 && !written[t] && !pending_add[t]) {
          // the other consumer: a convolution or fully connected layer further down whose input gradient is still to come
          bool taken = false;
          for (int j = i - 1; j >= 0 && !taken; --j) {
            const Layer& Lj = net->layers[j];
            taken = !Lj.fused_away && is_param_op(Lj.d.op) && Lj.in0 == t && Lj.d.op == OMNI_OP_CONV;
          }
          if (taken) { pending_add[t] = grad(L.out); continue; }
        }
        omni::route_grad_bf16(st, grad(L.out), net->tensors[t].relu ? act(t) : nullptr, grad(t), elems,
                              written[t] != 0);
        written[t] = 1;
      }
    } else if (L.d.op == OMNI_OP_GAP) {
      omni::gap_bwd_bf16(st, grad(L.out), net->tensors[L.in0].relu ? act(L.in0) : nullptr, grad(L.in0), rows,
                         L.ih * L.iw, L.ic, written[L.in0] != 0);
      written[L.in0] = 1;
    }
  }
  for (size_t t = 0; t < net->tensors.size(); ++t) {
    const bool have = (written[t] && !not_stored[t]) || (int)t == last.out;
    net->grad_view[t] = have ? (size_t)(reinterpret_cast<char*>(grad((int)t)) - c.ws) : kNoGrad;
  }
}

}  // namespace

extern "C" {

int omni_step(omni_net* net, void* stream, float* params, const void* x, const int32_t* labels,
              const int32_t* off, const int32_t* b, int32_t K, float lr, void* workspace,
              float* loss_per_worker, float* loss, uint32_t flags) {
  return omni::step_impl(net, stream, params, x, labels, off, b, K, lr, workspace, loss_per_worker, loss, flags, true);
}

}  // extern "C"

// may_create: the step may create the side streams it has not got yet (and with them, later, the events
// that order them); without it a network that has none runs the whole step on the caller's stream.
int omni::step_impl(omni_net* net, void* stream, float* params, const void* x, const int32_t* labels,
                    const int32_t* off, const int32_t* b, int32_t K, float lr, void* workspace,
                    float* loss_per_worker, float* loss, uint32_t flags, bool may_create) {
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
  if (flags & ~(uint32_t)(OMNI_STEP_NO_UPDATE | OMNI_STEP_KEEP_REDUCED_GRAD))
    return fail(OMNI_EINVAL, "omni_step: unknown flag bits 0x%x", flags);
  if ((reinterpret_cast<uintptr_t>(params) & 15u) || (reinterpret_cast<uintptr_t>(workspace) & 255u) ||
      (reinterpret_cast<uintptr_t>(x) & 15u))
    return fail(OMNI_EINVAL, "omni_step: params/x must be 16-byte and workspace 256-byte aligned");

  StepCtx c{};
  c.net = net;
  c.st = static_cast<hipStream_t>(stream);
  c.ws = static_cast<char*>(workspace);
  c.params = params;
  c.x = x;
  c.labels = labels;
  c.rows = off[K];
  c.seg.K = K;
  for (int k = 0; k <= K; ++k) c.seg.off[k] = off[k];
  c.G = reinterpret_cast<float*>(c.ws + net->grads_off);
  c.loss_rows = reinterpret_cast<float*>(c.ws + net->loss_rows_off);
  c.status = reinterpret_cast<uint32_t*>(c.ws + net->status_off);
  c.loss_per_worker = loss_per_worker;
  c.loss = loss;

  // ---- a repeated step as a graph: replay, capture, or enqueue launch by launch
  bool capture = false;
  if (net->graph_on) {
    std::vector<uint64_t> key;
    auto put = [&](const void* q) { key.push_back((uint64_t)reinterpret_cast<uintptr_t>(q)); };
    put(stream); put(params); put(x); put(labels); put(workspace); put(loss_per_worker); put(loss);
    put(net->velocity);
    uint32_t lr_bits, mo_bits, wd_bits;
    std::memcpy(&lr_bits, &lr, 4); std::memcpy(&mo_bits, &net->momentum, 4); std::memcpy(&wd_bits, &net->weight_decay, 4);
    key.push_back(((uint64_t)lr_bits << 32) | flags);
    key.push_back(((uint64_t)mo_bits << 32) | wd_bits);
    key.push_back((uint64_t)K);
    for (int k = 0; k <= K; ++k) key.push_back((uint64_t)off[k]);
    // Event timing records into events on the stream, which a replay cannot do: a step in which a
    // launch of the timed class is due for its event pair is enqueued launch by launch.
    bool timed_now = false;
    if (net->time_class >= 0) {
      if (net->last_matches < 0) timed_now = true;   // not known yet how many such launches a step has
      else if (net->ev_used + 2 <= net->ev.size())
        for (long j = 0; j < net->last_matches && !timed_now; ++j)
          timed_now = ((net->time_seen + j) % net->time_every) == 0;
    }
    if (!timed_now && stream != nullptr && net->ws_ready == workspace && net->side && net->side2) {
      if (net->graph_exec && key == net->graph_key) {
        if (hipGraphLaunch(net->graph_exec, static_cast<hipStream_t>(stream)) != hipSuccess)
          return fail(OMNI_EHIP, "omni_step: graph launch failed");
        net->time_seen += net->graph_matches;
        net->graph_replays++;
        return OMNI_OK;
      }
      capture = key == net->seen_key;    // the second call in a row with this key
    }
    net->seen_key = key;
    if (capture) {
      if (hipStreamBeginCapture(static_cast<hipStream_t>(stream), hipStreamCaptureModeThreadLocal) != hipSuccess) {
        (void)hipGetLastError();
        capture = false;
      }
    }
  }
  net->capturing = capture;
  net->step_matches = 0;

  net->ws_ready = workspace;   // (only tells the graph switch that this workspace has been stepped on before)

  if (may_create) {
    if (!net->side && hipStreamCreateWithFlags(&net->side, hipStreamNonBlocking) != hipSuccess) net->side = nullptr;
    if (!net->side2 && hipStreamCreateWithFlags(&net->side2, hipStreamNonBlocking) != hipSuccess) net->side2 = nullptr;
  }
  c.side = net->side ? net->side : c.st;
  c.side2 = (net->side && net->side2) ? net->side2 : c.side;

  if (net->dtype == OMNI_F32) step_f32(c);
  else step_bf16(c);
  c.join();

  // ---- weighted aggregation + update
  float* reduced = (flags & OMNI_STEP_KEEP_REDUCED_GRAD) ? reinterpret_cast<float*>(c.ws + net->reduced_off) : nullptr;
  if (!(flags & OMNI_STEP_NO_UPDATE)) {
    TimedScope ts(net, c.st, OMNI_KERNEL_UPDATE, -1, true);
    omni::weighted_sgd_f32(c.st, params, c.G, net->P_stride, net->P, c.seg, lr, nullptr, net->velocity,
                           net->momentum, net->weight_decay, ts.timer(), reduced);
  } else if (reduced) {
    omni::weighted_reduce_f32(c.st, c.G, net->P_stride, net->P, c.seg, reduced);
  }

  if (capture) {
    net->capturing = false;
    hipGraph_t graph = nullptr;
    hipGraphExec_t exec = nullptr;
    if (hipStreamEndCapture(c.st, &graph) != hipSuccess || !graph)
      return fail(OMNI_EHIP, "omni_step: stream capture failed");
    const hipError_t ie = hipGraphInstantiate(&exec, graph, nullptr, nullptr, 0);
    (void)hipGraphDestroy(graph);
    if (ie != hipSuccess) return fail(OMNI_EHIP, "omni_step: graph instantiation failed: %s", hipGetErrorString(ie));
    if (net->graph_exec) (void)hipGraphExecDestroy(net->graph_exec);
    net->graph_exec = exec;
    net->graph_key = net->seen_key;
    net->graph_matches = net->step_matches;
    if (hipGraphLaunch(exec, c.st) != hipSuccess) return fail(OMNI_EHIP, "omni_step: graph launch failed");
  }
  net->last_matches = net->step_matches;

  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(OMNI_EHIP, "omni_step: launch failed: %s", hipGetErrorString(e));
  return OMNI_OK;
}

extern "C" {

int omni_net_graph_enable(omni_net* net, int32_t on) {
  if (!net) return fail(OMNI_EINVAL, "omni_net_graph_enable: NULL net");
  net->graph_on = on != 0;
  if (!net->graph_on) {
    if (net->graph_exec) (void)hipGraphExecDestroy(net->graph_exec);
    net->graph_exec = nullptr;
    net->graph_key.clear();
    net->seen_key.clear();
  }
  return OMNI_OK;
}

int64_t omni_net_graph_replays(const omni_net* net) { return net ? net->graph_replays : 0; }

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

static int check_momentum(const char* who, float momentum, float weight_decay) {
  if (!std::isfinite(momentum) || momentum < 0.f || momentum >= 1.f)
    return fail(OMNI_EINVAL, "%s: momentum must lie in [0, 1)", who);
  if (!std::isfinite(weight_decay) || weight_decay < 0.f)
    return fail(OMNI_EINVAL, "%s: weight_decay must be finite and >= 0", who);
  return OMNI_OK;
}

int omni_weighted_sgd_momentum(void* stream, float* params, float* velocity, const float* grads, size_t stride,
                               size_t P, const int32_t* b, int32_t K, float lr, float momentum, float weight_decay,
                               void* shadow_bf16) {
  if (!params || !velocity || !grads || !b) return fail(OMNI_EINVAL, "omni_weighted_sgd_momentum: NULL argument");
  if (K < 1 || K > OMNI_MAX_WORKERS)
    return fail(K < 1 ? OMNI_EINVAL : OMNI_ECAPACITY, "omni_weighted_sgd_momentum: K=%d", K);
  if (P < 1 || stride < P || (stride & 3u))
    return fail(OMNI_EINVAL, "omni_weighted_sgd_momentum: need P >= 1 and stride >= P, stride %% 4 == 0");
  if ((reinterpret_cast<uintptr_t>(params) & 15u) || (reinterpret_cast<uintptr_t>(grads) & 15u) ||
      (reinterpret_cast<uintptr_t>(velocity) & 15u) || (reinterpret_cast<uintptr_t>(shadow_bf16) & 7u))
    return fail(OMNI_EINVAL, "omni_weighted_sgd_momentum: params/velocity/grads must be 16-byte aligned");
  if (!std::isfinite(lr)) return fail(OMNI_EINVAL, "omni_weighted_sgd_momentum: lr is not finite");
  if (int rc = check_momentum("omni_weighted_sgd_momentum", momentum, weight_decay)) return rc;
  omni::Segments seg{};
  seg.K = K;
  int64_t acc = 0;
  for (int k = 0; k < K; ++k) {
    if (b[k] < 1) return fail(OMNI_EINVAL, "omni_weighted_sgd_momentum: b[%d]=%d must be at least 1", k, b[k]);
    acc += b[k];
    if (acc > INT32_MAX) return fail(OMNI_EOVERFLOW, "omni_weighted_sgd_momentum: sum of b overflows");
    seg.off[k + 1] = (int32_t)acc;
  }
  omni::weighted_sgd_f32(static_cast<hipStream_t>(stream), params, grads, stride, P, seg, lr,
                         static_cast<uint16_t*>(shadow_bf16), velocity, momentum, weight_decay);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(OMNI_EHIP, "omni_weighted_sgd_momentum: launch failed: %s", hipGetErrorString(e));
  return OMNI_OK;
}

int omni_net_set_momentum(omni_net* net, float* velocity, float momentum, float weight_decay) {
  if (!net) return fail(OMNI_EINVAL, "omni_net_set_momentum: NULL net");
  if (!velocity) {
    net->velocity = nullptr; net->momentum = 0.f; net->weight_decay = 0.f;
    return OMNI_OK;
  }
  if (reinterpret_cast<uintptr_t>(velocity) & 15u)
    return fail(OMNI_EINVAL, "omni_net_set_momentum: velocity must be 16-byte aligned");
  if (int rc = check_momentum("omni_net_set_momentum", momentum, weight_decay)) return rc;
  net->velocity = velocity; net->momentum = momentum; net->weight_decay = weight_decay;
  return OMNI_OK;
}

int omni_lr_step_decay(double lr0, double gamma, const int32_t* milestones, int32_t n, int32_t epoch,
                       double* lr_out) {
  if (!lr_out || n < 0 || (n > 0 && !milestones)) return fail(OMNI_EINVAL, "omni_lr_step_decay: bad argument");
  if (!std::isfinite(lr0) || !std::isfinite(gamma)) return fail(OMNI_EINVAL, "omni_lr_step_decay: lr0/gamma not finite");
  double lr = lr0;
  for (int i = 0; i < n; ++i)
    if (epoch >= milestones[i]) lr *= gamma;
  *lr_out = lr;
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
  omni::fill_u32(static_cast<hipStream_t>(stream), status, 1, 0u);   // the kernel only ever sets bits
  omni::softmax_xent_f32(static_cast<hipStream_t>(stream), z, labels, C, seg, dz, loss_rows, loss_per_worker, loss,
                         status);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(OMNI_EHIP, "omni_softmax_xent: launch failed: %s", hipGetErrorString(e));
  return OMNI_OK;
}

}  // extern "C"
