/*
 * omnistep — one synchronous dynamic-batching SGD step for K simulated
 * heterogeneous workers on one MI355X (gfx950).
 *
 * The library follows OmniLearn (arXiv 2503.17469): a proportional controller
 * sizes each worker's mini-batch b_k from its throughput while the global batch
 * B = sum_k b_k stays fixed (section "Dynamic-Batching", equations
 * itrtimeerror / dynbszadjust / dynbszGlobalBFixed, procedure getBsz of
 * Algorithm 1); every worker computes the mean gradient over its own b_k
 * samples; the gradients are combined with weights lambda_k = b_k / sum_i b_i
 * (equation bspweightedgrads) and applied as theta <- theta - eta * sum_k
 * lambda_k g_k (equation bspvariableSGD; the AllReduce and update lines of
 * procedure Train in Algorithm 1).
 *
 * The K workers' samples arrive as ONE ragged batch: worker k owns rows
 * off[k] .. off[k+1]-1 of the concatenated input, off being the exclusive
 * prefix sum of b.  Re-sizing the b_k therefore costs O(K) host integers, not a
 * re-batching of data.
 *
 * Conventions for every call
 *   - returns OMNI_OK (0) or a negative error code; never throws, never aborts;
 *     omni_last_error() gives a thread-local message for the last failure;
 *   - "host" pointers are ordinary process memory, "dev" pointers are device
 *     memory of the current HIP device; the library never frees or keeps
 *     caller memory beyond what is stated;
 *   - GPU work is enqueued on the hipStream_t passed as `void* stream`
 *     (NULL = the default stream) and the call returns without synchronising;
 *     buffers must stay alive until the stream has passed the enqueued work;
 *   - host-side validation happens before anything is launched: on error no
 *     kernel has been enqueued.
 */
#ifndef OMNISTEP_H
#define OMNISTEP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
  OMNI_OK = 0,
  OMNI_EINVAL = -1,      /* malformed argument (NULL, non-positive size, b_k < 1, off/b mismatch, ...) */
  OMNI_EINFEASIBLE = -2, /* bounds cannot be met with sum b_k = B */
  OMNI_EOVERFLOW = -3,   /* an integer product would not fit */
  OMNI_ECAPACITY = -4,   /* K > K_max, B > B_max, or a compiled-in limit exceeded */
  OMNI_EHIP = -5         /* a HIP runtime call failed */
};

enum { OMNI_F32 = 0, OMNI_BF16 = 1 };

/* Largest K any call accepts (segment tables are passed to kernels by value). */
#define OMNI_MAX_WORKERS 64

const char* omni_last_error(void);
const char* omni_version(void);

/* ------------------------------------------------------------------ controller
 * Host only, integers only, no GPU needed.
 *
 * Given per-worker throughputs T_k (samples per unit time in any common
 * unit), the proportional controller of section "Dynamic-Batching" moves every
 * worker to the batch size that takes the cluster-average time, b_k - T_k *
 * tau_k = T_k * mean(t); the fixed-global-batch rule then rescales so that
 * sum_k b_k = B.  Together: b_k = B * T_k / sum_j T_j, which does not depend on
 * the previous batch sizes, so the controller is stateless.  The rescaling is
 * multiplicative (the paper's text) rather than the equal-share subtraction of
 * the printed equation.  Real values become integers by largest remainder,
 * ties to the lowest worker index.  Bounds b_min <= b_k <= b_max (procedure
 * getBsz) are enforced by clamping the violating side with the larger total
 * violation and re-apportioning the remaining workers, repeated until none
 * violates.
 */
typedef struct omni_ctl omni_ctl;

/* K in [1, OMNI_MAX_WORKERS], B >= K, 1 <= b_min <= b_max; b_max = 0 means B.
 * OMNI_EINFEASIBLE if K*b_min > B or K*b_max < B. *out is owned by the caller
 * and released with omni_ctl_destroy. */
int omni_ctl_create(int32_t K, int32_t B, int32_t b_min, int32_t b_max, omni_ctl** out);

/* T: host [K], every entry > 0 (else OMNI_EINVAL); copied. */
int omni_ctl_set_throughputs(omni_ctl* ctl, const uint64_t* T);

/* Writes b_out host [K] and off_out host [K+1] (off[0] = 0, off[K] = B).
 * OMNI_EINVAL if no throughputs were set; OMNI_EINFEASIBLE if clamping cannot
 * reach sum B.  Exact integer arithmetic (128-bit products): results are
 * reproducible bit for bit. */
int omni_ctl_run(omni_ctl* ctl, int32_t* b_out, int32_t* off_out);

void omni_ctl_destroy(omni_ctl* ctl);

/* ------------------------------------------------------------------ measured-time controller
 * Procedure getBsz of Algorithm 1 with the stability kit of section "Control Stability
 * for Dynamic-Batching": workers report the time one iteration took (omni_dyn_observe);
 * the controller smooths it (newest-sample weight alpha; the average restarts after
 * every adjustment) and, at the end of an epoch (omni_dyn_adjust), proposes
 * b* = b - T (t - t_avg), T = b / t (equations itrtimeerror, dynbszadjust), accepts it
 * only if |b* - b| / b* >= deadband (equation omnibszdeadbandlimit), and applies the
 * bounds and the global-batch rule:
 *   OMNI_RULE_NONE            each worker decides for itself; accepted b* is clamped to
 *                             [b_min, b_max] and rounded to nearest (ties to even); the
 *                             global batch may drift;
 *   OMNI_RULE_MULTIPLICATIVE  all workers move if any ratio reaches the dead-band; the
 *                             b* are rescaled to sum B ("proportionately", the text after
 *                             equation dynbszGlobalBFixed) and made integer inside the
 *                             bounds by largest remainder;
 *   OMNI_RULE_ADDITIVE        equation dynbszGlobalBFixed as printed: every b* loses
 *                             (sum b* - B) / K, is clamped and rounded (the sum is B only
 *                             up to rounding and while no clamp fires).
 * Host only, IEEE double arithmetic in a fixed operation order (results repeat bit for
 * bit).  b_init host [K] or NULL for Algorithm 1's uniform start B / K; b_max = 0 means
 * B; times host [K], positive and finite, any common unit.  b_out [K], off_out [K+1],
 * changed_out may each be NULL.  omni_dyn_adjust without an observation since the last
 * adjustment is OMNI_EINVAL; infeasible bounds are OMNI_EINFEASIBLE. */
typedef struct omni_dyn omni_dyn;
enum { OMNI_RULE_NONE = 0, OMNI_RULE_MULTIPLICATIVE = 1, OMNI_RULE_ADDITIVE = 2 };
int omni_dyn_create(int32_t K, int32_t B, int32_t b_min, int32_t b_max, double deadband,
                    double ewma_alpha, int32_t global_rule, const int32_t* b_init, omni_dyn** out);
int omni_dyn_observe(omni_dyn* ctl, const double* t);
int omni_dyn_adjust(omni_dyn* ctl, int32_t* b_out, int32_t* off_out, int32_t* changed_out);
int omni_dyn_get(const omni_dyn* ctl, int32_t* b_out, int32_t* off_out);
void omni_dyn_destroy(omni_dyn* ctl);

/* ------------------------------------------------------------------ network
 * A network is a list of layers over channels-last activations [rows, H, W, C].
 * `src` / `src2` name the producing layer (-1 = the network input); src2 is
 * used by OMNI_OP_ADD only.  The last layer's output is the logits [rows, C].
 *
 *   OMNI_OP_LINEAR   y = x W^T + bias     W [cout][cin], input flattened (h,w,c)
 *   OMNI_OP_CONV     ksize x ksize, stride, zero pad; W [cout][kh][kw][cin]
 *   OMNI_OP_RELU     max(x, 0); derivative 0 at 0
 *   OMNI_OP_MAXPOOL2 2x2 window, stride 2; gradient to the first maximum in
 *                    (dy, dx) scan order
 *   OMNI_OP_BN       batch norm with the statistics of EACH WORKER'S OWN ROWS
 *                    (biased variance, eps = 1e-5), channels = cin
 *   OMNI_OP_ADD      elementwise sum of two equal-shaped tensors
 *   OMNI_OP_GAP      mean over H and W
 *
 * Parameters are one flat fp32 vector in layer order: weight then bias (if
 * `bias` != 0) for LINEAR / CONV, gamma then beta for BN.
 */
enum {
  OMNI_OP_LINEAR = 0,
  OMNI_OP_CONV = 1,
  OMNI_OP_RELU = 2,
  OMNI_OP_MAXPOOL2 = 3,
  OMNI_OP_BN = 4,
  OMNI_OP_ADD = 5,
  OMNI_OP_GAP = 6
};

typedef struct omni_layer_desc {
  int32_t op;
  int32_t src;
  int32_t src2;
  int32_t cin;
  int32_t cout;
  int32_t ksize;
  int32_t stride;
  int32_t pad;
  int32_t bias;
} omni_layer_desc;

typedef struct omni_net omni_net;

/* Builds the launch plan for (layers, input shape, dtype, K_max, B_max).  Host
 * only: allocates no device memory and compiles nothing, now or later.
 * dtype OMNI_F32: fp32 operands and activations.  dtype OMNI_BF16: bf16
 * operands and stored activations, fp32 accumulation, fp32 master parameters,
 * gradients and loss.  OMNI_EINVAL on a malformed layer list or an unsupported
 * combination. */
int omni_net_create(const omni_layer_desc* layers, int32_t n_layers,
                    int32_t in_h, int32_t in_w, int32_t in_c,
                    int32_t dtype, int32_t K_max, int32_t B_max, omni_net** out);

/* Number of fp32 parameters P. */
size_t omni_net_param_count(const omni_net* net);

/* Bytes of device workspace omni_step needs (activations, activation
 * gradients, the K_max per-worker gradient rows, small tables).  The caller
 * allocates it (256-byte aligned) and may reuse it across steps, for other
 * networks or for anything else in between: a step relies on nothing that an
 * earlier step left in it (the few words that must be zero when a kernel
 * starts are cleared by the step itself), so fresh, recycled and overwritten
 * memory all do.  Steps that share one workspace must not overlap in time. */
size_t omni_net_workspace_bytes(const omni_net* net);

/* Row stride, in floats, of the per-worker gradient matrix (>= P, multiple of 64). */
size_t omni_net_grad_stride(const omni_net* net);

/* One training step (Algorithm 1, procedure Train: gradient, AllReduce, update).
 *
 *   params          dev [P] fp32, read and overwritten with theta - lr * g
 *   x               dev, off[K] rows of in_h*in_w*in_c values, fp32 or bf16 per dtype
 *   labels          dev [off[K]] int32 in [0, classes)
 *   off, b          host [K+1], [K]: off[0] = 0, off[k+1] - off[k] = b[k] >= 1,
 *                   off[K] <= B_max, K <= K_max           (else OMNI_EINVAL / OMNI_ECAPACITY)
 *   lr              finite
 *   workspace       dev, omni_net_workspace_bytes(net) bytes
 *   loss_per_worker dev [K] fp32: L_k = mean loss over worker k's rows
 *   loss            dev [1] fp32: sum_k lambda_k L_k
 *   flags           OMNI_STEP_NO_UPDATE leaves params untouched (gradients only);
 *                   OMNI_STEP_KEEP_REDUCED_GRAD also stores the aggregated gradient
 *                   g = sum_k lambda_k g_k of equation bspweightedgrads (the update
 *                   forms it in registers and otherwise never writes it) where
 *                   omni_net_reduced_grad points; other bits are OMNI_EINVAL
 *
 * The step allocates no device memory and never synchronises with the device.
 * The first steps of a network create what they need on the host side and keep
 * it until omni_net_destroy: two side streams (default priority) on which the
 * parameter gradients of a bf16 network run beside the input-gradient chain, a
 * few events that order them with the caller's stream, and the dynamic-LDS limit
 * of the kernels that need more than the default; later steps create nothing.
 * All work of a step has been ordered back onto `stream` when the call returns.
 *
 * After the step the workspace holds g_k (mean gradient of worker k) in row k
 * of the matrix returned by omni_net_worker_grads.  A label outside
 * [0, classes) sets bit 0 of the status word (omni_net_status) and contributes
 * zero loss and zero gradient. */
enum { OMNI_STEP_NO_UPDATE = 1u, OMNI_STEP_KEEP_REDUCED_GRAD = 2u };

int omni_step(omni_net* net, void* stream, float* params, const void* x,
              const int32_t* labels, const int32_t* off, const int32_t* b, int32_t K,
              float lr, void* workspace, float* loss_per_worker, float* loss,
              uint32_t flags);

/* omni_step for callers that cannot allocate device memory or have none to hand over as a workspace:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same step,
 * same kernels, same results bit for bit; the workspace is a fixed array of
 * OMNI_STATIC_WORKSPACE_BYTES inside the library's device image (each GPU the library runs on holds
 * its own copy until the process ends) instead of an argument.  The call allocates nothing and
 * creates nothing (no device memory, no stream, no event: a network that has not been stepped by
 * omni_step before runs entirely on `stream`).  OMNI_ECAPACITY, with nothing launched, if
 * omni_net_workspace_bytes(net) exceeds the array: in practice fp32 networks of a few layers at small
 * batch sizes (a bf16 network's weight-gradient scratch alone is larger).  The other arguments and
 * errors are omni_step's.  Every call on a GPU uses that GPU's one array: calls that overlap in time
 * on the same GPU (different streams, different networks, different threads) race; serialise them.
 * The per-worker gradients, activations and the status word stay inside the array and cannot be
 * viewed; params, loss_per_worker and loss are the outputs. */
#define OMNI_STATIC_WORKSPACE_BYTES (32u << 20)
int omni_step_static(omni_net* net, void* stream, float* params, const void* x,
                     const int32_t* labels, const int32_t* off, const int32_t* b, int32_t K,
                     float lr, float* loss_per_worker, float* loss, uint32_t flags);

/* Views into a workspace (device pointers; valid while the workspace is). */
const float* omni_net_worker_grads(const omni_net* net, const void* workspace);
const uint32_t* omni_net_status(const omni_net* net, const void* workspace);
/* Output of layer `layer` as stored by the last step: *ptr dev pointer (fp32 or
 * bf16 per dtype), *elems_per_row its row length.  Layers fused away into a
 * neighbour alias that neighbour's tensor.  One tensor is not stored at all: the
 * output of a batch norm whose only consumer is the residual add right after it
 * (the add's output is stored; the pointer returned for the batch norm layer then
 * points at memory no step writes).  OMNI_EINVAL on a bad index. */
int omni_net_activation(const omni_net* net, const void* workspace, int32_t layer,
                        const void** ptr, size_t* elems_per_row);

/* g = sum_k lambda_k g_k, dev [P] fp32, as the last step with OMNI_STEP_KEEP_REDUCED_GRAD left it
 * (the AllReduce line of procedure Train, Algorithm 1, before the update consumes it). */
const float* omni_net_reduced_grad(const omni_net* net, const void* workspace);
/* Gradient of worker k's mean loss L_k, on the rows of worker k (the 1/b_k of equation
 * bspweightedgrads is inside), with respect to the output of layer
 * `layer`, as the last step left it: *ptr dev pointer with the layout and type of omni_net_activation
 * (bf16, fp32 for the logits and for fp32 networks).  For a layer whose ReLU was folded into it the
 * gradient is the one with respect to the value BEFORE the ReLU (already zero where the stored output
 * is zero).  Layers fused away alias their neighbour as in omni_net_activation, and an input of a
 * residual add that nothing else reads shares the add's buffer.  OMNI_EINVAL on a bad index, and for a
 * tensor whose gradient that step did not store: a layer nothing differentiable depends on, and the
 * first convolution of a network when a 2 x 2 max pooling follows it (its weight-gradient kernel
 * rebuilds that gradient from the pooled one). */
int omni_net_activation_grad(const omni_net* net, const void* workspace, int32_t layer,
                             const void** ptr, size_t* elems_per_row);

/* Optional replay of repeated steps as a HIP graph.  A step is a chain of a few dozen short kernels
 * on up to three streams; launched one by one, the host calls and the waits between the streams cost
 * as much time as the kernels of a small network.  With the switch on, omni_step compares everything
 * its launches depend on (stream, all pointers, K, off, lr, flags, optimiser settings) with the call
 * before: the second call in a row with the same values is captured from the stream into a graph
 * (and run as one), later calls with these values launch that graph.  Different values, a step in
 * which a timed launch is due, the NULL stream, or a workspace used for the first time are enqueued
 * launch by launch as always; results are the same either way (same kernels, same order).  The
 * caller's stream must not be under capture itself.  Off by default; switching it off drops the
 * graph.  omni_net_graph_replays counts the steps that were replayed. */
int omni_net_graph_enable(omni_net* net, int32_t on);
int64_t omni_net_graph_replays(const omni_net* net);

/* Optional device-side timing of one kernel class inside omni_step, for
 * roofline reports.  After omni_net_timing_enable, every launch of that class
 * (for layer `layer`, or all layers if layer < 0) is bracketed by a pair of HIP
 * events recorded on the step's stream; at most `max_launches` launches are
 * recorded until the next read.  omni_net_timing_read waits for the recorded
 * events, returns their summed elapsed time and count, and clears the record.
 * kernel_class < 0 disables timing.  Events are created inside the enable call
 * (never inside omni_step).  Returns OMNI_EINVAL on a bad class.
 * Two classes are timed more exactly where they are a single kernel launch (the
 * fp32 weight gradients below, and OMNI_KERNEL_UPDATE): their event pair is bound
 * to the kernel's own start and end time stamps instead of bracketing it on the
 * stream, which leaves the 2-3 microseconds of the event packets out.
 * In an fp32 network the weight gradients of all fully connected layers before
 * the classifier head run as ONE launch; it counts as a launch of the lowest
 * layer index it covers (layer 0 of a multi-layer perceptron).  Likewise the
 * head's own parameter gradients (with the per-worker losses) share a launch
 * with the input gradient of the layer below it where that product takes the
 * small-batch kernel: the launch counts as that layer's OMNI_KERNEL_LINEAR_DGRAD,
 * and OMNI_KERNEL_LOSS then covers the head's forward / loss / dz kernel only. */
enum {
  OMNI_KERNEL_LINEAR_FWD = 0,
  OMNI_KERNEL_LINEAR_DGRAD = 1,
  OMNI_KERNEL_LINEAR_WGRAD = 2,
  OMNI_KERNEL_LOSS = 3,
  OMNI_KERNEL_UPDATE = 4,
  OMNI_KERNEL_CONV_FWD = 5,
  OMNI_KERNEL_CONV_DGRAD = 6,
  OMNI_KERNEL_CONV_WGRAD = 7,
  OMNI_KERNEL_CLASSES = 8
};
int omni_net_timing_enable(omni_net* net, int32_t kernel_class, int32_t layer, int32_t max_launches);
int omni_net_timing_read(omni_net* net, double* total_ms, int64_t* launches);
/* Bracket only every `every`-th matching launch (default 1: all of them).  An event pair
 * costs a few microseconds on the stream; sampling keeps a measurement that runs inside a
 * timed loop from stretching it.  Applies from the next omni_net_timing_enable on;
 * max_launches there counts bracketed launches. */
int omni_net_timing_sample(omni_net* net, int32_t every);

void omni_net_destroy(omni_net* net);

/* ------------------------------------------------------------------ single kernels
 * The aggregation + update of equations bspweightedgrads / bspvariableSGD on
 * its own: params[j] -= lr * sum_k (b[k] / sum_i b[i]) * grads[k*stride + j].
 *   params dev [P] in/out; grads dev [K][stride] fp32; b host [K], each >= 1;
 *   shadow_bf16: dev [P] uint16 receiving the updated params rounded to bf16
 *   (nearest even), or NULL. */
int omni_weighted_sgd(void* stream, float* params, const float* grads, size_t stride,
                      size_t P, const int32_t* b, int32_t K, float lr, void* shadow_bf16);

/* The optimiser of the paper's experiments (Section "Evaluation", model hyperparameters: momentum
 * SGD, coefficient 0.9, with an L2 weight decay of 5e-4 or 1e-4), fused with the aggregation of equation
 * bspweightedgrads.  The paper prints no formula; this is the update of the framework it
 * names (no dampening, no Nesterov look-ahead, L2 penalty folded into the gradient):
 *   g = sum_k (b[k] / sum_i b[i]) * grads[k*stride + j]
 *   d = g + weight_decay * params[j];  velocity[j] = momentum * velocity[j] + d
 *   params[j] -= lr * velocity[j]
 *   velocity dev [P] fp32 in/out, 16-byte aligned, owned by the caller, all zeros before
 *   the first step; the other arguments as omni_weighted_sgd.  momentum in [0, 1),
 *   weight_decay >= 0, all finite; anything else is OMNI_EINVAL and nothing is launched. */
int omni_weighted_sgd_momentum(void* stream, float* params, float* velocity, const float* grads,
                               size_t stride, size_t P, const int32_t* b, int32_t K, float lr,
                               float momentum, float weight_decay, void* shadow_bf16);

/* Make omni_step apply that update instead of plain SGD (velocity as above, P =
 * omni_net_param_count floats); velocity == NULL returns to plain SGD.  Host call, takes
 * effect from the next omni_step. */
int omni_net_set_momentum(omni_net* net, float* velocity, float momentum, float weight_decay);

/* Stepwise learning-rate schedule of the same hyperparameter list (for instance 0.1 at the start,
 * divided by ten once epochs 15, 30 and 45 are reached): *lr_out = lr0 * gamma^m with m
 * the number of milestones <= epoch (epochs counted from 0).  Host only, double
 * arithmetic; milestones host [n], may be NULL when n == 0. */
int omni_lr_step_decay(double lr0, double gamma, const int32_t* milestones, int32_t n,
                       int32_t epoch, double* lr_out);

/* ------------------------------------------------------------------ static variable batching
 * Equation varbszBSP (section "Variable Batching"): b_k = c_k / sum(c) * B from the compute
 * resource c_k of each worker (cores, FLOP/s, any common unit), made integer exactly like
 * omni_ctl_run (largest remainder, ties to the lowest index, bounds by clamping and
 * re-apportioning).  Host only.  c host [K] >= 1; b_out host [K]; off_out host [K+1] or NULL;
 * b_max = 0 means B.  Errors as omni_ctl_create / omni_ctl_run. */
int omni_static_batches(int32_t K, const uint64_t* c, int32_t B, int32_t b_min, int32_t b_max,
                        int32_t* b_out, int32_t* off_out);

/* Equation hlevel: heterogeneity level = largest / smallest resource.  Any of the outputs
 * may be NULL. */
int omni_heterogeneity_level(int32_t K, const uint64_t* c, uint64_t* max_out, uint64_t* min_out,
                             double* hl_out);

/* Memory model of section "Heterogeneous memory across workers", equation hetmemeqn:
 *   M_total(b) = (2 + opt_copies) * P * bytes_per_param            model, gradients, optimiser
 *              + act_per_sample * b                                activations
 *              + batch_slope * b + batch_intercept                 batch (data loader) memory
 * omni_mem_fit_linear: least-squares line through n measured (batch size, bytes) points
 * (the paper fits the batch term this way); integer sums are exact, 2 <= n <= 4096,
 * 0 <= b <= 2^24, 0 <= bytes <= 2^48, at least two distinct b.
 * omni_mem_total evaluates the model; omni_mem_max_batch returns the largest b in
 * [0, limit] whose total is <= mem_avail (0: only the fixed part fits, -1: not even that).
 * Host only, doubles, bit-reproducible. */
int omni_mem_fit_linear(int32_t n, const int64_t* b, const int64_t* bytes, double* slope_out,
                        double* intercept_out);
int omni_mem_total(int64_t b, int64_t P, int32_t bytes_per_param, int32_t opt_copies,
                   double act_per_sample, double batch_slope, double batch_intercept,
                   double* total_out);
int omni_mem_max_batch(double mem_avail, int64_t P, int32_t bytes_per_param, int32_t opt_copies,
                       double act_per_sample, double batch_slope, double batch_intercept,
                       int64_t limit, int64_t* b_max_out);

/* The same question for this library's own training state, answered exactly rather than
 * by a fitted model: the largest batch capacity B_max (>= K_max) for which
 *   omni_net_workspace_bytes + (1 + opt_copies) * 4 * P + B_max * (input row + label)
 * stays within budget_bytes of device memory (opt_copies = 1 with a velocity buffer).
 * Host only (plans are built and discarded; no device memory is touched).  bytes_out
 * (may be NULL) receives the total at B_max.  OMNI_EINFEASIBLE if even B_max = K_max does
 * not fit; layer-list errors as omni_net_create. */
int omni_net_max_batch(const omni_layer_desc* layers, int32_t n_layers, int32_t in_h, int32_t in_w,
                       int32_t in_c, int32_t dtype, int32_t K_max, int32_t opt_copies,
                       uint64_t budget_bytes, int32_t* B_max_out, uint64_t* bytes_out);

/* ------------------------------------------------------------------ asynchronous training
 * Algorithm 2 ("Asynchronous training in OmniLearn") and equations aspweightedgrads /
 * aspvariableSGD on simulated workers.  Worker k repeats: pull the server model, compute
 * the mean gradient g_k of its own b_k samples at the pulled model (omni_step with one
 * worker and OMNI_STEP_NO_UPDATE; the gradient stays in that call's workspace, so give
 * every simulated worker a workspace of its own), local SGD step with its own learning
 * rate eta_k = eta * b_k / B, push.
 *
 * omni_asp_schedule (host only, exact integers): an iteration of worker k takes b[k] / T[k]
 * time units; pushes are processed in order of their finishing time, simultaneous ones
 * lower worker index first, and a worker pulls again right after its own push.  Writes the
 * worker of each of the first n_events pushes and the server version (number of pushes
 * before the pull) its gradient was computed on; the staleness of push e is
 * e - pulled_version_out[e].  T host [K] >= 1, b host [K] >= 1, outputs host [n_events]. */
int omni_asp_schedule(int32_t K, const uint64_t* T, const int32_t* b, int32_t n_events,
                      int32_t* worker_out, int32_t* pulled_version_out);

/* What a push does to the server model: dst[j] = base[j] - eta_k * grad[j], with
 * eta_k = lr * b_k / B (lr_scaling != 0, the linear scaling rule of equation
 * aspvariableSGD) or lr.  dst == base == server model: the server adds the worker's local
 * change to its current model (an update computed on an older model lands on the newer
 * one).  base == the model the worker pulled, dst == server model: the server model is
 * replaced by the worker's local model, as pushToPS is printed.  dst, base, grad dev [P]
 * fp32, 16-byte aligned; dst and base equal or disjoint.  Enqueued on `stream`, no
 * synchronisation.  OMNI_EINVAL on NULL / misaligned / partially overlapping buffers,
 * b_k < 1, B < b_k or a non-finite lr. */
int omni_asp_update(void* stream, float* dst, const float* base, const float* grad, size_t P,
                    float lr, int32_t b_k, int32_t B, int32_t lr_scaling);

/* The server's batch-size bookkeeping, procedure evalBsz of Algorithm 2 (host only).  A
 * worker reports (k, the batch size it used, its smoothed compute time per iteration);
 * both are stored; once every worker has reported at least once, each report re-evaluates
 * getBsz (Algorithm 1: b* = b - (b / t)(t - mean t); accepted if |b* - b| / b* >= deadband;
 * clamped to [b_min, b_max]; rounded half to even) for all workers from the stored values,
 * and the caller gets its own new size; before that it keeps its size.  The global batch
 * is not re-normalised (Algorithm 2 has no such step).  Double arithmetic, bit-reproducible.
 * omni_asp_ps_sizes copies the stored sizes (0 for a worker that has not reported). */
typedef struct omni_asp_ps omni_asp_ps;
int omni_asp_ps_create(int32_t K, int32_t b_min, int32_t b_max, double deadband, omni_asp_ps** out);
int omni_asp_ps_eval_bsz(omni_asp_ps* ps, int32_t k, int32_t b, double t, int32_t* b_out);
int omni_asp_ps_sizes(const omni_asp_ps* ps, int32_t* b_out);
void omni_asp_ps_destroy(omni_asp_ps* ps);

/* Softmax cross-entropy over a ragged batch: for row s of worker k,
 * loss_rows[s] = -log softmax(z_s)[y_s] and dz_s = (softmax(z_s) - e_{y_s}) / b_k
 * (the 1/|b_k| of equation bspweightedgrads), then L_k and sum_k lambda_k L_k.
 *   z dev [off[K]][C] fp32, labels dev int32, dz dev like z, loss_rows dev [off[K]],
 *   loss_per_worker dev [K], loss dev [1], status dev [1] (cleared by the call, then bit 0 is set
 *   if a label lies outside [0, C)), off host [K+1]. */
int omni_softmax_xent(void* stream, const float* z, const int32_t* labels, int32_t C,
                      const int32_t* off, int32_t K, float* dz, float* loss_rows,
                      float* loss_per_worker, float* loss, uint32_t* status);

#ifdef __cplusplus
}
#endif
#endif /* OMNISTEP_H */
