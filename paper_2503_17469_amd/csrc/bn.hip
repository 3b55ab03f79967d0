// Batch normalisation with PER-WORKER statistics, residual add and global
// average pooling for the bf16 path (channels-last, fp32 arithmetic).
//
// Each simulated worker normalises with the mean and biased variance of its own
// rows only (a worker in the paper's data-parallel setting sees nothing but its
// own mini-batch), so every reduction here is segmented by the worker row
// ranges.  All reductions use a fixed order: partial sums per (worker, split,
// channel), then a sequential sum over the splits.
//
// forward   y = gamma * (x - mu_k) * invstd_k + beta        (optionally ReLU)
// backward  dbeta_k = sum dy, dgamma_k = sum dy*xhat,
//           dx = gamma*invstd_k * (dy - mean_k(dy) - xhat * mean_k(dy*xhat))
#include <hip/hip_runtime.h>

#include "bf16.h"
#include "common.h"
#include "kernels.h"

namespace omni {

namespace {

constexpr float kBnEps = 1e-5f;

__device__ inline int owner_of_row(const Segments& seg, int n) {
  int lo = 0, hi = seg.K - 1;
  while (lo < hi) {
    const int mid = (lo + hi + 1) >> 1;
    if (n >= seg.off[mid]) lo = mid; else hi = mid - 1;
  }
  return lo;
}

// Partial sums of (a) x and x^2, or (b) dy and dy*xhat, over one split of one worker's positions.
// grid (splits, K, ceil(C/64)); block = 8 channel pieces x 32 position lanes.
template <bool BWD>
__global__ __launch_bounds__(256) void bn_partial_kernel(const bf16_t* __restrict__ x, const bf16_t* __restrict__ dy,
                                                         const float* __restrict__ stats, int C, int hw,
                                                         Segments seg, double* __restrict__ partial) {
  __shared__ double red[32][8][17];
  const int tid = threadIdx.x;
  const int c8 = tid & 7, pl = tid >> 3;
  const int wk = blockIdx.y, split = blockIdx.x, nsplit = gridDim.x;
  const int c0 = blockIdx.z * 64 + c8 * 8;
  const bool cok = c0 < C;
  const long pbeg = (long)seg.off[wk] * hw, pend = (long)seg.off[wk + 1] * hw;
  const long per = (pend - pbeg + nsplit - 1) / nsplit;
  const long sbeg = pbeg + split * per, send = min(pend, sbeg + per);
  // Sums run in double: this kernel waits on memory, and statistics good to fp32
  // rounding keep the normalised values from landing on the other side of a bf16
  // rounding boundary more often than the arithmetic forces.
  double s1[8], s2[8];
  float mu[8], is[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) { s1[e] = 0.0; s2[e] = 0.0; mu[e] = 0.f; is[e] = 1.f; }
  if (BWD && cok) {
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      mu[e] = stats[((size_t)wk * C + c0 + e) * 2];
      is[e] = stats[((size_t)wk * C + c0 + e) * 2 + 1];
    }
  }
  if (cok) {
    for (long p = sbeg + pl; p < send; p += 32) {
      float xv[8];
      Piece<bf16_t>::load(x + p * C + c0, xv);
      if (!BWD) {
#pragma unroll
        for (int e = 0; e < 8; ++e) { s1[e] += (double)xv[e]; s2[e] += (double)xv[e] * (double)xv[e]; }
      } else {
        float dv[8];
        Piece<bf16_t>::load(dy + p * C + c0, dv);
#pragma unroll
        for (int e = 0; e < 8; ++e) { s1[e] += (double)dv[e]; s2[e] += (double)(dv[e] * ((xv[e] - mu[e]) * is[e])); }
      }
    }
  }
#pragma unroll
  for (int e = 0; e < 8; ++e) { red[pl][c8][e] = s1[e]; red[pl][c8][8 + e] = s2[e]; }
  __syncthreads();
  if (tid < 128) {
    const int cc = tid & 63, which = tid >> 6;     // channel within the group, sum or second sum
    double t = 0.0;
#pragma unroll
    for (int r = 0; r < 32; ++r) t += red[r][cc >> 3][which * 8 + (cc & 7)];
    const int c = blockIdx.z * 64 + cc;
    if (c < C) partial[(((size_t)wk * nsplit + split) * C + c) * 2 + which] = t;
  }
}

// Forward: mean and 1/sqrt(var + eps) per (worker, channel).
__global__ __launch_bounds__(256) void bn_finalize_fwd_kernel(const double* __restrict__ partial, int C, int hw,
                                                              int nsplit, Segments seg, float* __restrict__ stats) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= seg.K * C) return;
  const int wk = i / C, c = i - wk * C;
  double a = 0.0, b = 0.0;
  for (int s = 0; s < nsplit; ++s) {
    a += partial[(((size_t)wk * nsplit + s) * C + c) * 2];
    b += partial[(((size_t)wk * nsplit + s) * C + c) * 2 + 1];
  }
  const double n = (double)(seg.off[wk + 1] - seg.off[wk]) * hw;
  const double mean = a / n;
  double var = b / n - mean * mean;
  var = var > 0.0 ? var : 0.0;
  stats[((size_t)wk * C + c) * 2] = (float)mean;
  stats[((size_t)wk * C + c) * 2 + 1] = (float)(1.0 / sqrt(var + (double)kBnEps));
}

// Backward: dbeta, dgamma into worker k's gradient row, and the two means used by dx.
__global__ __launch_bounds__(256) void bn_finalize_bwd_kernel(const double* __restrict__ partial, int C, int hw,
                                                              int nsplit, Segments seg, float* __restrict__ means,
                                                              float* __restrict__ g_gamma, float* __restrict__ g_beta,
                                                              size_t worker_stride) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= seg.K * C) return;
  const int wk = i / C, c = i - wk * C;
  double a = 0.0, b = 0.0;
  for (int s = 0; s < nsplit; ++s) {
    a += partial[(((size_t)wk * nsplit + s) * C + c) * 2];
    b += partial[(((size_t)wk * nsplit + s) * C + c) * 2 + 1];
  }
  const double n = (double)(seg.off[wk + 1] - seg.off[wk]) * hw;
  g_beta[(size_t)wk * worker_stride + c] = (float)a;
  g_gamma[(size_t)wk * worker_stride + c] = (float)b;
  means[((size_t)wk * C + c) * 2] = (float)(a / n);
  means[((size_t)wk * C + c) * 2 + 1] = (float)(b / n);
}

// One thread = 8 channels of one position.
template <bool BWD>
__global__ __launch_bounds__(256) void bn_apply_kernel(const bf16_t* __restrict__ x, const bf16_t* __restrict__ dy,
                                                       const float* __restrict__ stats, const float* __restrict__ means,
                                                       const float* __restrict__ gamma, const float* __restrict__ beta,
                                                       int C, int hw, long pieces, Segments seg, int relu,
                                                       bf16_t* __restrict__ out) {
  const long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= pieces) return;
  const int c8n = C / 8;
  const int c0 = (int)(i % c8n) * 8;
  const long p = i / c8n;
  const int wk = owner_of_row(seg, (int)(p / hw));
  float xv[8], o[8];
  Piece<bf16_t>::load(x + p * C + c0, xv);
  const float* st = stats + ((size_t)wk * C + c0) * 2;
  if (!BWD) {
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      float y = gamma[c0 + e] * ((xv[e] - st[2 * e]) * st[2 * e + 1]) + beta[c0 + e];
      if (relu) y = y > 0.f ? y : 0.f;
      o[e] = y;
    }
  } else {
    float dv[8];
    Piece<bf16_t>::load(dy + p * C + c0, dv);
    const float* mn = means + ((size_t)wk * C + c0) * 2;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const float xh = (xv[e] - st[2 * e]) * st[2 * e + 1];
      o[e] = gamma[c0 + e] * st[2 * e + 1] * (dv[e] - mn[2 * e] - xh * mn[2 * e + 1]);
    }
  }
  Piece<bf16_t>::store(out + p * C + c0, o);
}

// out = a + b (optionally ReLU)
__global__ __launch_bounds__(256) void add_fwd_kernel(const bf16_t* __restrict__ a, const bf16_t* __restrict__ b,
                                                      bf16_t* __restrict__ out, long pieces, int relu) {
  const long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= pieces) return;
  float av[8], bv[8];
  Piece<bf16_t>::load(a + i * 8, av);
  Piece<bf16_t>::load(b + i * 8, bv);
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    av[e] += bv[e];
    if (relu) av[e] = av[e] > 0.f ? av[e] : 0.f;
  }
  Piece<bf16_t>::store(out + i * 8, av);
}

// dst (+)= g, zeroed where mask <= 0 (mask may be null)
__global__ __launch_bounds__(256) void route_grad_kernel(const bf16_t* __restrict__ g, const bf16_t* __restrict__ mask,
                                                         bf16_t* __restrict__ dst, long pieces, int accumulate) {
  const long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= pieces) return;
  float gv[8];
  Piece<bf16_t>::load(g + i * 8, gv);
  if (mask) {
    float mv[8];
    Piece<bf16_t>::load(mask + i * 8, mv);
#pragma unroll
    for (int e = 0; e < 8; ++e) gv[e] = mv[e] > 0.f ? gv[e] : 0.f;
  }
  if (accumulate) {
    float ov[8];
    Piece<bf16_t>::load(dst + i * 8, ov);
#pragma unroll
    for (int e = 0; e < 8; ++e) gv[e] += ov[e];
  }
  Piece<bf16_t>::store(dst + i * 8, gv);
}

// global average pool: one thread = 8 channels of one sample
__global__ __launch_bounds__(256) void gap_fwd_kernel(const bf16_t* __restrict__ in, bf16_t* __restrict__ out, int C,
                                                      int hw, long pieces) {
  const long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= pieces) return;
  const int c8n = C / 8;
  const int c0 = (int)(i % c8n) * 8;
  const long n = i / c8n;
  float s[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) s[e] = 0.f;
  for (int q = 0; q < hw; ++q) {
    float v[8];
    Piece<bf16_t>::load(in + (n * hw + q) * C + c0, v);
#pragma unroll
    for (int e = 0; e < 8; ++e) s[e] += v[e];
  }
  const float inv = 1.0f / (float)hw;
#pragma unroll
  for (int e = 0; e < 8; ++e) s[e] *= inv;
  Piece<bf16_t>::store(out + n * C + c0, s);
}

// din[n][q][c] (+)= dout[n][c] / hw, zeroed where mask <= 0; one thread = 8 channels of one position
__global__ __launch_bounds__(256) void gap_bwd_kernel(const bf16_t* __restrict__ dout, const bf16_t* __restrict__ mask,
                                                      bf16_t* __restrict__ din, int C, int hw, long pieces,
                                                      int accumulate) {
  const long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= pieces) return;
  const int c8n = C / 8;
  const int c0 = (int)(i % c8n) * 8;
  const long p = i / c8n;
  const long n = p / hw;
  float g[8];
  Piece<bf16_t>::load(dout + n * C + c0, g);
  const float inv = 1.0f / (float)hw;
#pragma unroll
  for (int e = 0; e < 8; ++e) g[e] *= inv;
  if (mask) {
    float mv[8];
    Piece<bf16_t>::load(mask + p * C + c0, mv);
#pragma unroll
    for (int e = 0; e < 8; ++e) g[e] = mv[e] > 0.f ? g[e] : 0.f;
  }
  if (accumulate) {
    float ov[8];
    Piece<bf16_t>::load(din + p * C + c0, ov);
#pragma unroll
    for (int e = 0; e < 8; ++e) g[e] += ov[e];
  }
  Piece<bf16_t>::store(din + p * C + c0, g);
}

inline unsigned blocks_for(long n) { return (unsigned)((n + 255) / 256); }

int pick_bn_splits(const Segments& seg, int C) {
  const int groups = (C + 63) / 64;
  int s = 2048 / (seg.K * groups);
  s = s < 1 ? 1 : s;
  return s > kBnMaxSplits ? kBnMaxSplits : s;
}

}  // namespace

void bn_forward_bf16(hipStream_t st, const bf16_t* x, bf16_t* y, const float* gamma, const float* beta, int C, int hw,
                     const Segments& seg, bool relu, float* stats, double* partial) {
  const int ns = pick_bn_splits(seg, C);
  hipLaunchKernelGGL(bn_partial_kernel<false>, dim3(ns, seg.K, (C + 63) / 64), dim3(256), 0, st, x, nullptr, nullptr,
                     C, hw, seg, partial);
  hipLaunchKernelGGL(bn_finalize_fwd_kernel, dim3(blocks_for((long)seg.K * C)), dim3(256), 0, st, partial, C, hw, ns,
                     seg, stats);
  const long pieces = (long)seg.off[seg.K] * hw * (C / 8);
  hipLaunchKernelGGL(bn_apply_kernel<false>, dim3(blocks_for(pieces)), dim3(256), 0, st, x, nullptr, stats, nullptr,
                     gamma, beta, C, hw, pieces, seg, relu ? 1 : 0, y);
}

void bn_backward_bf16(hipStream_t st, const bf16_t* x, const bf16_t* dy, bf16_t* dx, const float* gamma, int C, int hw,
                      const Segments& seg, const float* stats, float* means, double* partial, float* g_gamma,
                      float* g_beta, size_t worker_stride) {
  const int ns = pick_bn_splits(seg, C);
  hipLaunchKernelGGL(bn_partial_kernel<true>, dim3(ns, seg.K, (C + 63) / 64), dim3(256), 0, st, x, dy, stats, C, hw,
                     seg, partial);
  hipLaunchKernelGGL(bn_finalize_bwd_kernel, dim3(blocks_for((long)seg.K * C)), dim3(256), 0, st, partial, C, hw, ns,
                     seg, means, g_gamma, g_beta, worker_stride);
  const long pieces = (long)seg.off[seg.K] * hw * (C / 8);
  hipLaunchKernelGGL(bn_apply_kernel<true>, dim3(blocks_for(pieces)), dim3(256), 0, st, x, dy, stats, means, gamma,
                     nullptr, C, hw, pieces, seg, 0, dx);
}

void add_fwd_bf16(hipStream_t st, const bf16_t* a, const bf16_t* b, bf16_t* out, long elems, bool relu) {
  hipLaunchKernelGGL(add_fwd_kernel, dim3(blocks_for(elems / 8)), dim3(256), 0, st, a, b, out, elems / 8, relu ? 1 : 0);
}

void route_grad_bf16(hipStream_t st, const bf16_t* g, const bf16_t* mask, bf16_t* dst, long elems, bool accumulate) {
  hipLaunchKernelGGL(route_grad_kernel, dim3(blocks_for(elems / 8)), dim3(256), 0, st, g, mask, dst, elems / 8,
                     accumulate ? 1 : 0);
}

void gap_fwd_bf16(hipStream_t st, const bf16_t* in, bf16_t* out, int rows, int hw, int C) {
  const long pieces = (long)rows * (C / 8);
  hipLaunchKernelGGL(gap_fwd_kernel, dim3(blocks_for(pieces)), dim3(256), 0, st, in, out, C, hw, pieces);
}

void gap_bwd_bf16(hipStream_t st, const bf16_t* dout, const bf16_t* mask, bf16_t* din, int rows, int hw, int C,
                  bool accumulate) {
  const long pieces = (long)rows * hw * (C / 8);
  hipLaunchKernelGGL(gap_bwd_kernel, dim3(blocks_for(pieces)), dim3(256), 0, st, dout, mask, din, C, hw, pieces,
                     accumulate ? 1 : 0);
}

}  // namespace omni
