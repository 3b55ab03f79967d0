// Launchers of the HIP kernels (definitions in the .hip files of this directory).
// Every launcher only enqueues work on `st`; none synchronises or allocates.
#pragma once
#include <hip/hip_runtime_api.h>

#include <cstddef>
#include <cstdint>

#include "common.h"

namespace omni {

// Scratch for split reductions: partial tiles plus one arrival counter per tile.
// Counters must be zero before the first launch; every launch leaves them zero.
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
// For every worker k: gw + k*worker_stride receives dy_k^T x_k ([cout][cin]) over rows
// seg.off[k]..seg.off[k+1]-1, and gb + k*worker_stride the column sums of dy_k (gb may be null).
void linear_wgrad_f32(hipStream_t st, const float* dy, const float* x, float* gw, float* gb,
                      size_t worker_stride, const Segments& seg, int cin, int cout);

// ---- classifier head (head.hip): last fully connected layer with few outputs ----
// True if the fused head kernels can take this shape (else use the generic path).
bool head_supported(int cin, int classes, const void* x, const void* w);
// z = x w^T + bias; loss_rows, dz = (softmax(z) - onehot)/b_k; optionally
// dx (+)= dz w masked by mask > 0 (dx may be null when the input needs no gradient).
void head_fwd_loss_dgrad_f32(hipStream_t st, const float* x, const float* w, const float* bias,
                             const int32_t* labels, int cin, int classes, const Segments& seg, float* z,
                             float* dz, float* loss_rows, const float* mask, float* dx, bool accumulate);
// Per worker: gw_k = dz_k^T x_k, gb_k = column sums of dz_k; plus L_k, the total
// loss and the status word (bit 0: some label outside [0, classes)).
void head_wgrad_loss_f32(hipStream_t st, const float* dz, const float* x, const int32_t* labels, int cin,
                         int classes, const Segments& seg, float* gw, float* gb, size_t worker_stride,
                         const float* loss_rows, float* loss_per_worker, float* loss, uint32_t* status);

// ---- loss and update (pointwise.hip) ----
void softmax_xent_f32(hipStream_t st, const float* z, const int32_t* labels, int C, const Segments& seg,
                      float* dz, float* loss_rows, float* loss_per_worker, float* loss, uint32_t* status);
// params[j] -= lr * sum_k lambda[k] * grads[k*stride + j]; optional bf16 copy of the result.
void weighted_sgd_f32(hipStream_t st, float* params, const float* grads, size_t stride, size_t P,
                      const Segments& seg, float lr, uint16_t* shadow_bf16);
void fill_u32(hipStream_t st, uint32_t* p, size_t n, uint32_t v);

}  // namespace omni
