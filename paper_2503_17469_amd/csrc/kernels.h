// Launchers of the HIP kernels (definitions in the .hip files of this directory).
// Every launcher only enqueues work on `st`; none synchronises or allocates.
#pragma once
#include <hip/hip_runtime_api.h>

#include <cstddef>
#include <cstdint>

#include "common.h"

namespace omni {

// ---- fp32 fully connected layers (gemm_f32.hip) ----
// y[rows][cout] = x[rows][cin] * w[cout][cin]^T + bias, optional ReLU.
void linear_fwd_f32(hipStream_t st, const float* x, const float* w, const float* bias, float* y,
                    int rows, int cin, int cout, bool relu);
// dx[rows][cin] (+)= dy[rows][cout] * w[cout][cin], zeroed where mask[rows][cin] <= 0 (mask may be null).
void linear_dgrad_f32(hipStream_t st, const float* dy, const float* w, const float* mask, float* dx,
                      int rows, int cin, int cout, bool accumulate);
// For every worker k: gw + k*worker_stride receives dy_k^T x_k ([cout][cin]) over rows
// seg.off[k]..seg.off[k+1]-1, and gb + k*worker_stride the column sums of dy_k (gb may be null).
void linear_wgrad_f32(hipStream_t st, const float* dy, const float* x, float* gw, float* gb,
                      size_t worker_stride, const Segments& seg, int cin, int cout);

// ---- loss and update (pointwise.hip) ----
void softmax_xent_f32(hipStream_t st, const float* z, const int32_t* labels, int C, const Segments& seg,
                      float* dz, float* loss_rows, float* loss_per_worker, float* loss, uint32_t* status);
// params[j] -= lr * sum_k lambda[k] * grads[k*stride + j]; optional bf16 copy of the result.
void weighted_sgd_f32(hipStream_t st, float* params, const float* grads, size_t stride, size_t P,
                      const Segments& seg, float lr, uint16_t* shadow_bf16);
void fill_u32(hipStream_t st, uint32_t* p, size_t n, uint32_t v);

}  // namespace omni
