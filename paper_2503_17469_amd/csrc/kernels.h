// Launchers of the HIP kernels (definitions in the .hip files of this directory).
// Every launcher only enqueues work on `st`; none synchronises or allocates.
#pragma once
#include <hip/hip_runtime_api.h>

#include <cstddef>
#include <cstdint>

#include "common.h"

namespace omni {

// Optional exact timing of ONE kernel launch: the two events receive the kernel's own start and end
// time stamps (hipExtLaunchKernelGGL) instead of bracketing the launch on the stream, where the
// event packets themselves add 2-3 microseconds.  A launcher that ends up making several launches
// records the events around them instead.
struct KernelTimer {
  hipEvent_t start;
  hipEvent_t stop;
};

// Scratch for split reductions: partial tiles plus one arrival counter per tile.
// Counters must be zero when a launch starts; every launch leaves them zero.
struct SplitWorkspace {
  float* partial = nullptr;      // kSplitPartialFloats floats
  uint32_t* counters = nullptr;  // kSplitMaxTiles words
};
constexpr int kSplitMaxTiles = 512;
constexpr size_t kSplitPartialFloats = (size_t)1024 * 16 * 256;  // tiles * splits <= 1024

// ---- fp32 fully connected layers (gemm_f32.hip) ----
// y[rows][cout] = x[rows][cin] * w[cout][cin]^T + bias, optional ReLU.
void linear_fwd_f32(hipStream_t st, const float* x, const float* w, const float* bias, float* y,
                    int rows, int cin, int cout, bool relu, const SplitWorkspace& sw);
// dx[rows][cin] (+)= dy[rows][cout] * w[cout][cin], zeroed where mask[rows][cin] <= 0 (mask may be null).
void linear_dgrad_f32(hipStream_t st, const float* dy, const float* w, const float* mask, float* dx,
                      int rows, int cin, int cout, bool accumulate, const SplitWorkspace& sw);
// Small-batch variants (gemm_f32_direct.hip): same results as the two above up to
// summation order; return false without launching when the shape does not qualify.
bool linear_fwd_f32_direct_supported(const float* x, const float* w, int rows, int cin, int cout);
bool linear_fwd_f32_direct(hipStream_t st, const float* x, const float* w, const float* bias, float* y,
                           int rows, int cin, int cout, bool relu);
bool linear_dgrad_f32_direct_supported(const float* dy, const float* w, const float* mask, const float* dx, int rows,
                                       int cin, int cout);
bool linear_dgrad_f32_direct(hipStream_t st, const float* dy, const float* w, const float* mask, float* dx,
                             int rows, int cin, int cout, bool accumulate);
// For every worker k: gw + k*worker_stride receives dy_k^T x_k ([cout][cin]) over rows
// seg.off[k]..seg.off[k+1]-1, and gb + k*worker_stride the column sums of dy_k (gb may be null).
void linear_wgrad_f32(hipStream_t st, const float* dy, const float* x, float* gw, float* gb,
                      size_t worker_stride, const Segments& seg, int cin, int cout);
// The same for several layers at once (same workers, same worker_stride): one launch where the
// shapes allow it, so that the start-up and drain of one layer's workgroups overlap the others' work.
struct LinearWgradJob {
  const float* dy;   // [rows][cout]
  const float* x;    // [rows][cin]
  float* gw;         // worker 0's [cout][cin]
  float* gb;         // worker 0's [cout], may be null
  int cin, cout;
};
void linear_wgrad_f32_batch(hipStream_t st, const LinearWgradJob* jobs, int n, size_t worker_stride,
                            const Segments& seg, const KernelTimer* timer = nullptr);

// ---- classifier head (head.hip): last fully connected layer with few outputs ----
// `bf16` selects the storage type of x, w and dx (bf16 words) versus fp32; the
// arithmetic, logits, dz and all gradients of parameters are fp32 either way.
// True if the fused head kernels can take this shape (else use the generic path).
bool head_supported(int cin, int classes, const void* x, const void* w, bool bf16);
// z = x w^T + bias; loss_rows, dz = (softmax(z) - onehot)/b_k; optionally
// dx (+)= dz w, zeroed where x <= 0 if use_mask (dx may be null when the input needs no gradient).
void head_fwd_loss_dgrad(hipStream_t st, bool bf16, const void* x, const void* w, const float* bias,
                         const int32_t* labels, int cin, int classes, const Segments& seg, float* z, float* dz,
                         float* loss_rows, bool use_mask, void* dx, bool accumulate);
// Per worker: gw_k = dz_k^T x_k, gb_k = column sums of dz_k; plus L_k, the total
// loss and the status word (bit 0: some label outside [0, classes)).
void head_wgrad_loss(hipStream_t st, bool bf16, const float* dz, const void* x, const int32_t* labels, int cin,
                     int classes, const Segments& seg, float* gw, float* gb, size_t worker_stride,
                     const float* loss_rows, float* loss_per_worker, float* loss, uint32_t* status);
// Arguments of the head's parameter-gradient kernel.  x has the storage type T of the body's
// instantiation (fp32, or bf16 words); everything else is fp32.
struct HeadWgradParams {
  const float* dz;            // [rows][classes], carries 1/b_k
  const void* x;              // [rows][cin]
  const int32_t* labels;      // [rows]
  int cin, C;
  float* gw;                  // worker k's [C][cin] at gw + k * worker_stride
  float* gb;                  // worker k's [C] at gb + k * worker_stride, may be null
  size_t worker_stride;
  const float* loss_rows;     // [rows]
  float* loss_per_worker;     // [K]
  float* loss;                // [1]
  uint32_t* status;           // [1]
};
// The input gradient of a fully connected fp32 layer (as linear_dgrad_f32) and the head's parameter
// gradients (as head_wgrad_loss with fp32 x) in ONE launch; the two must not depend on each other.
// Only for products that linear_dgrad_f32_direct_supported accepts (the caller asks first).
void linear_dgrad_f32_with_head_wgrad(hipStream_t st, const float* dy, const float* w, const float* mask, float* dx,
                                      int rows, int cin, int cout, bool accumulate, const HeadWgradParams& head,
                                      const Segments& seg);

// ---- bf16 convolutions / fully connected layers as implicit GEMMs (conv_bf16.hip) ----
typedef uint16_t bf16_t;   // raw bfloat16 bits
// How the left operand of an implicit GEMM is gathered from a channels-last tensor.
struct ConvGeom {
  int rows;             // samples
  int Hs, Ws, Cs;       // gathered tensor: height, width, channels (multiple of 8)
  int Hp, Wp;           // positions enumerated by the GEMM rows: m = (n*Hp + h)*Wp + w
  int ks, stride, pad;  // filter size, stride, zero padding of the forward convolution
  int transposed;       // 0: source = h*stride + u - pad.  1 (dgrad): t = h + pad - u, source = t/stride if divisible
  int K;                // ks*ks*Cs
  const void* zero;     // at least 16 bytes of zeros in device memory: where loads of absent pieces are pointed
  int raw3;             // 1: the source tensor holds 3 channels per pixel as given (6 bytes), not the Cs = 8 the
                        // kernels work on; only the first-layer kernels read it (conv_first_layer_raw_supported)
  const uint8_t* mask_bits;   // may be null; with a mask [M][N], N a multiple of 64: the same information at one bit
                              // per element ([M][N/8] bytes, bit e of byte c/8 set where mask[m][c - c%8 + e] > 0).
                              // Kernels that know how read it instead of the mask (a sixteenth of the bytes).
};
// True if both the forward and the weight-gradient pass of a first layer with this shape can read a
// 3-channel source as it is, so that no padded copy of the network input has to be made.
bool conv_first_layer_raw_supported(int Cout, int cin_real, const ConvGeom& g, long M);
constexpr int kConvMaxPartialTiles = 2048;   // (tile, chunk) slots of wgrad scratch
constexpr int kZeroPageWords = 64;           // 256 bytes of zeros that loads of absent pieces are pointed at (16 are read);
                                             // cast_weights_bf16 clears them at the start of every step
// Statistics of a per-worker batch norm are summed in two stages: partial records [record][C][2] (doubles: the
// sum of the values and of their squares over some positions of ONE worker), then, per worker, the records
// first[k] .. first[k+1]-1 in order.
struct ShareTable { int32_t first[OMNI_MAX_WORKERS + 1]; };
constexpr int kBnMaxSplits = 256;  // the statistics scratch holds K * kBnMaxSplits records in all
// A forward convolution whose output a batch norm normalises may write the first stage itself, from the
// values it stores, instead of the batch norm reading the tensor once more: the caller fills partial and seg;
// the kernel that takes the offer sets done and fills table (bn_forward_bf16 then skips its own first stage).
struct BnStatRequest {
  double* partial;       // [K * kBnMaxSplits][C][2]
  const Segments* seg;
  ShareTable table;
  bool done;
};
size_t conv_wgrad_partial_floats();
bool conv_shape_supported(const ConvGeom& g, long positions);
// out[M][N] = gather(src)[M][K] * wgt[N][K]^T (+bias) (ReLU) (masked where mask <= 0) (+= out)
// With pool_out and pool_code (forward of a layer that a 2 x 2 max pooling follows): the kernels that
// hold a whole unit of output rows in LDS also write [rows*(Hp/2)*(Wp/2)][N] = the pooling of `out`
// and, one byte per pooled element, which of the four inputs its gradient goes to (0-3 in scan
// order, first maximum; 4: none, the ReLU folded into `out` zeroed it); the call then returns true.
// False means `out` alone was written and the caller pools it itself.
// stats (may be null): see BnStatRequest.
bool conv_gemm_bf16(hipStream_t st, const bf16_t* src, const bf16_t* wgt, bf16_t* out, int M, int N,
                    const ConvGeom& g, const float* bias, const bf16_t* mask, bool relu, bool accumulate,
                    bf16_t* pool_out = nullptr, uint8_t* pool_code = nullptr, const bf16_t* addend = nullptr,
                    BnStatRequest* stats = nullptr);
// The wide-tile kernel for 3x3 / stride 1 / pad 1 layers (conv3_wide_bf16.hip): same arguments and result as
// conv_gemm_bf16 without pooling; false, with nothing launched, if the shape does not qualify.
bool conv3_wide_bf16(hipStream_t st, const bf16_t* src, const bf16_t* wgt, bf16_t* out, int M, int N,
                     const ConvGeom& g, const float* bias, const bf16_t* mask, bool relu, bool accumulate,
                     const bf16_t* addend, BnStatRequest* stats = nullptr);
// Input gradient of a residual block's entry (conv3s2_dgrad_bf16.hip): dx [rows][H][W][Cin] receives the gradient
// coming back through a 3x3 / stride-2 / pad-1 convolution (dy [rows][H/2][W/2][Cout], wt its transposed weights
// [Cin][9][Cout]) and, if dy_sc is not null, through the 1x1 / stride-2 projection beside it (dy_sc
// [rows][H/2][W/2][Cout_sc], wt_sc [Cin][Cout_sc]) in one pass; mask / accumulate / addend as conv_gemm_bf16.
// False, with nothing launched, for shapes it does not take (conv3s2_dgrad_supported tells beforehand).
bool conv3s2_dgrad_supported(int rows, int H, int W, int Cin, int Cout, int Cout_sc);
bool conv3s2_dgrad_bf16(hipStream_t st, const bf16_t* dy, const bf16_t* wt, int Cout, const bf16_t* dy_sc,
                        const bf16_t* wt_sc, int Cout_sc, bf16_t* dx, int rows, int H, int W, int Cin,
                        const bf16_t* mask, bool accumulate, const bf16_t* addend, const void* zero,
                        const uint8_t* mask_bits = nullptr);
// (mask_bits: as ConvGeom::mask_bits.)
// (addend, [M][N] or null, is added to the product before the mask: the input gradient of a layer
// whose input also feeds a residual add takes the add's share along instead of a separate pass.)
// Per worker k: gw_k[Cout][taps][cin_real] = dy_k^T gather(src)_k, gb_k = column sums of dy_k (gb may be null).
// With dpool and pool_code (only where conv_wgrad_pooled_supported says so: the first-layer kernel),
// dy is not read: the layer's output gradient is taken from the gradient of the 2 x 2 max pooling
// that follows the layer ([rows*(Hp/2)*(Wp/2)][Cout]) and the pooling's codes, so that it never has
// to be written out at full resolution.
void conv_wgrad_bf16(hipStream_t st, const bf16_t* dy, const bf16_t* src, float* gw, float* gb,
                     size_t worker_stride, int Cout, int cin_real, const ConvGeom& g, const Segments& seg,
                     float* partial, uint32_t* counters, const bf16_t* dpool = nullptr,
                     const uint8_t* pool_code = nullptr);
bool conv_wgrad_pooled_supported(int Cout, int cin_real, const ConvGeom& g);
// Weight gradient of a 3x3 / pad-1 convolution of stride 2 (or 1) without bias from operands left in their
// [position][channel] layout (conv3_wgrad_tr_bf16.hip); arguments as conv_wgrad_bf16.  False, with nothing
// launched, for shapes it does not take.
bool conv3_wgrad_tr_bf16(hipStream_t st, const bf16_t* dy, const bf16_t* src, float* gw, float* gb,
                         size_t worker_stride, int Cout, int cin_real, const ConvGeom& g, const Segments& seg,
                         float* partial);

// ---- bf16 pointwise kernels (pointwise_bf16.hip) ----
// fp32 weights [cout][taps][cin_real] -> bf16 [cout][taps][cin_pad] (zero padded) and,
// if w_t is not null, the transposed copy [cin_pad][taps][cout] used by dgrad.
// One layer's weight copy: fp32 [cout][taps][cin_real] at params + src -> bf16 [cout][taps][cin_pad] at
// shadow + dst_fwd and, if dst_t >= 0, the transposed [cin_pad][taps][cout] at shadow + dst_t (offsets in elements).
struct CastEntry {
  long src, dst_fwd, dst_t;
  int cout, taps, cin_real, cin_pad;
  int first_block;   // filled by the launcher
};
constexpr int kCastMaxEntries = 64;
struct CastTable {
  int n;
  CastEntry e[kCastMaxEntries];
};
// zero_page (may be null): kZeroPageWords words that the same launch sets to zero.
void cast_weights_bf16(hipStream_t st, const float* params, bf16_t* shadow, const CastEntry* entries, int n,
                       uint32_t* zero_page = nullptr);
void pad_channels_bf16(hipStream_t st, const bf16_t* x, bf16_t* xp, long pixels, int c_real, int c_pad);
void maxpool2_fwd_bf16(hipStream_t st, const bf16_t* in, bf16_t* out, int rows, int H, int W, int C);
// din = dout routed to the first maximum of each 2x2 window (scan order), zero elsewhere;
// with relu_mask also zero where the maximum is not positive.
// The same from the codes conv_gemm_bf16 wrote with the pooled tensor (8 bytes of codes per 16 of
// gradient instead of four 16-byte pieces of the pooling's input).
void maxpool2_bwd_coded_bf16(hipStream_t st, const uint8_t* code, const bf16_t* dout, bf16_t* din, int rows, int H,
                             int W, int C);
void maxpool2_bwd_bf16(hipStream_t st, const bf16_t* in, const bf16_t* dout, bf16_t* din, int rows, int H, int W,
                       int C, bool relu_mask);

// ---- per-worker batch norm, residual add, global average pool (bn.hip) ----
// stats: [K][C][2] (mean, 1/sqrt(var+eps)); partial: [K * kBnMaxSplits][C][2] doubles of scratch.
// Channel counts the batch-norm kernels handle: a multiple of 8, at most 2048.
bool bn_shape_supported(int C);
// With skip: y = bn(x) (rounded as it would have been stored) + skip, then ReLU if relu_add: the residual
// add that follows the normalisation, without writing and re-reading the normalised tensor.
// presummed (may be null): the partial records are already in `partial`, laid out by this table.
void bn_forward_bf16(hipStream_t st, const bf16_t* x, bf16_t* y, const float* gamma, const float* beta, int C, int hw,
                     const Segments& seg, bool relu, float* stats, double* partial, const bf16_t* skip = nullptr,
                     bool relu_add = false, const ShareTable* presummed = nullptr, uint8_t* sign_bits = nullptr);
// (sign_bits, [positions][C/8] bytes or null: one bit per element of y, set where the stored value is positive:
// what the input-gradient kernels need of a ReLU's output.)
// means: [K][C][2] scratch; g_gamma / g_beta: worker k's entries at + k*worker_stride.
void bn_backward_bf16(hipStream_t st, const bf16_t* x, const bf16_t* dy, bf16_t* dx, const float* gamma, int C, int hw,
                      const Segments& seg, const float* stats, float* means, double* partial, float* g_gamma,
                      float* g_beta, size_t worker_stride);
void add_fwd_bf16(hipStream_t st, const bf16_t* a, const bf16_t* b, bf16_t* out, long elems, bool relu);
// dst (+)= g, zeroed where mask <= 0 (mask may be null)
void route_grad_bf16(hipStream_t st, const bf16_t* g, const bf16_t* mask, bf16_t* dst, long elems, bool accumulate);
void gap_fwd_bf16(hipStream_t st, const bf16_t* in, bf16_t* out, int rows, int hw, int C);
void gap_bwd_bf16(hipStream_t st, const bf16_t* dout, const bf16_t* mask, bf16_t* din, int rows, int hw, int C,
                  bool accumulate);

// ---- loss and update (pointwise.hip) ----
void softmax_xent_f32(hipStream_t st, const float* z, const int32_t* labels, int C, const Segments& seg,
                      float* dz, float* loss_rows, float* loss_per_worker, float* loss, uint32_t* status);
// params[j] -= lr * sum_k lambda[k] * grads[k*stride + j]; optional bf16 copy of the result.
// velocity == nullptr: plain SGD.  Otherwise d = g + weight_decay*theta, velocity = momentum*velocity + d,
// theta -= lr*velocity (velocity [P], read and written).
void weighted_sgd_f32(hipStream_t st, float* params, const float* grads, size_t stride, size_t P,
                      const Segments& seg, float lr, uint16_t* shadow_bf16, float* velocity = nullptr,
                      float momentum = 0.f, float weight_decay = 0.f, const KernelTimer* timer = nullptr,
                      float* gout = nullptr);
// (gout, [P] or null, also receives the aggregated gradient sum_k lambda[k] * grads[k].)
// The aggregation alone: gout[j] = sum_k lambda[k] * grads[k*stride + j].
void weighted_reduce_f32(hipStream_t st, const float* grads, size_t stride, size_t P, const Segments& seg,
                         float* gout);
void fill_u32(hipStream_t st, uint32_t* p, size_t n, uint32_t v);

// The body of omni_step (net.cpp).  may_create = false: nothing is created on the way, not even the
// side streams of a network that has none yet (the step then runs on the caller's stream alone).
int step_impl(omni_net* net, void* stream, float* params, const void* x, const int32_t* labels, const int32_t* off,
              const int32_t* b, int32_t K, float lr, void* workspace, float* loss_per_worker, float* loss,
              uint32_t flags, bool may_create);

}  // namespace omni
