// Bandwidth-bound kernels of the step: softmax cross-entropy over the ragged
// batch, and the fused weighted gradient aggregation + SGD update.
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>

#include "common.h"
#include "kernels.h"

namespace omni {

typedef float v4f __attribute__((ext_vector_type(4)));

namespace {

__device__ inline float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}
__device__ inline float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}

// Worker that owns row s (segments are few; a linear scan over kernel arguments).
__device__ inline int owner(const Segments& seg, int s) {
  int k = 0;
  while (k + 1 < seg.K && s >= seg.off[k + 1]) ++k;
  return k;
}

// One wavefront per row.  loss_row = logsumexp(z) - z[y]; dz = (softmax - onehot) / b_k:
// the 1/|b_k| of equation bspweightedgrads, so that the backward pass yields
// each worker's MEAN gradient.
__global__ __launch_bounds__(256) void softmax_xent_kernel(const float* __restrict__ z,
                                                           const int32_t* __restrict__ labels, int C,
                                                           Segments seg, float* __restrict__ dz,
                                                           float* __restrict__ loss_rows,
                                                           uint32_t* __restrict__ status) {
  const int lane = threadIdx.x & 63;
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
  const int rows = seg.off[seg.K];
  if (row >= rows) return;
  const int k = owner(seg, row);
  const float inv_b = 1.0f / (float)(seg.off[k + 1] - seg.off[k]);
  const float* zr = z + (size_t)row * C;
  float* dr = dz + (size_t)row * C;
  const int y = labels[row];
  if (y < 0 || y >= C) {
    if (lane == 0) {
      atomicOr(status, 1u);
      loss_rows[row] = 0.f;
    }
    for (int c = lane; c < C; c += 64) dr[c] = 0.f;
    return;
  }
  float m = -INFINITY;
  for (int c = lane; c < C; c += 64) m = fmaxf(m, zr[c]);
  m = wave_max(m);
  float s = 0.f;
  for (int c = lane; c < C; c += 64) s += expf(zr[c] - m);
  s = wave_sum(s);
  const float lse = logf(s);
  if (lane == 0) loss_rows[row] = lse - (zr[y] - m);
  for (int c = lane; c < C; c += 64) {
    float p = expf(zr[c] - m - lse);
    if (c == y) p -= 1.0f;
    dr[c] = p * inv_b;
  }
}

// One workgroup.  L_k = (1/b_k) sum of the worker's row losses (fixed-order tree,
// so results repeat bit for bit), loss = sum_k (b_k/B) L_k.
__global__ __launch_bounds__(256) void loss_reduce_kernel(const float* __restrict__ loss_rows, Segments seg,
                                                          float* __restrict__ loss_per_worker,
                                                          float* __restrict__ loss) {
  __shared__ float red[256];
  const int t = threadIdx.x;
  const float invB = 1.0f / (float)seg.off[seg.K];
  float total = 0.f;
  for (int k = 0; k < seg.K; ++k) {
    float a = 0.f;
    for (int s = seg.off[k] + t; s < seg.off[k + 1]; s += 256) a += loss_rows[s];
    red[t] = a;
    __syncthreads();
    for (int w = 128; w > 0; w >>= 1) {
      if (t < w) red[t] += red[t + w];
      __syncthreads();
    }
    if (t == 0) {
      const float bk = (float)(seg.off[k + 1] - seg.off[k]);
      const float Lk = red[0] / bk;
      loss_per_worker[k] = Lk;
      total += bk * invB * Lk;
    }
    __syncthreads();
  }
  if (t == 0) loss[0] = total;
}

struct Lambdas {
  float v[OMNI_MAX_WORKERS];
};

__device__ inline uint16_t bf16_rne(float f) {
  uint32_t u = __float_as_uint(f);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

// theta[j] -= lr * sum_k lambda_k G[k][j]  (equations bspweightedgrads and
// bspvariableSGD fused: the K gradient rows and theta are each read once, theta
// written once).  Rows of G are 256-byte aligned, so 16-byte loads throughout.
// The gradient rows are read exactly once (streaming, non-temporal loads); two
// 16-byte columns per thread are in flight together so that 2*(K+1) loads cover
// the HBM latency.
// MOM: the momentum / weight-decay update of the paper's experiments (velocity is read and
// written beside the parameters: (K+4)*4 bytes per parameter instead of (K+2)*4):
//   d = g + wd*theta;  v = mu*v + d;  theta -= lr*v.
struct Optim {
  float lr, momentum, weight_decay;
};

template <bool MOM>
__device__ inline void apply_update(v4f& th, v4f& v, const v4f& g, const Optim& o) {
  if (MOM) {
    const v4f d = g + o.weight_decay * th;
    v = o.momentum * v + d;
    th = th - o.lr * v;
  } else {
    th = th - o.lr * g;
  }
}

// KEEPG: the aggregated gradient g itself is also written to gout (4 more bytes per parameter; for
// callers that want to look at it: the update alone never stores it).
template <bool SHADOW, bool MOM, bool KEEPG>
__global__ __launch_bounds__(256) void weighted_sgd_kernel(float* __restrict__ params, float* __restrict__ velocity,
                                                           const float* __restrict__ grads, size_t stride,
                                                           size_t P, int K, Lambdas lam, Optim opt,
                                                           uint16_t* __restrict__ shadow, float* __restrict__ gout) {
  const size_t n4 = P / 4;
  const size_t nthreads = (size_t)gridDim.x * blockDim.x;
  const size_t t = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  for (size_t i0 = t; i0 < n4; i0 += 2 * nthreads) {
    const size_t i1 = i0 + nthreads;
    const bool has1 = i1 < n4;
    const size_t j1 = has1 ? i1 : i0;          // the second column re-reads the first when past the end
    v4f g0 = {0.f, 0.f, 0.f, 0.f}, g1 = {0.f, 0.f, 0.f, 0.f};
    v4f th0 = *reinterpret_cast<const v4f*>(params + 4 * i0);
    v4f th1 = *reinterpret_cast<const v4f*>(params + 4 * j1);
    v4f v0 = {0.f, 0.f, 0.f, 0.f}, v1 = {0.f, 0.f, 0.f, 0.f};
    if (MOM) {
      v0 = *reinterpret_cast<const v4f*>(velocity + 4 * i0);
      v1 = *reinterpret_cast<const v4f*>(velocity + 4 * j1);
    }
    int k = 0;
    for (; k + 4 <= K; k += 4) {
      v4f a[4], c[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        a[u] = __builtin_nontemporal_load(reinterpret_cast<const v4f*>(grads + (size_t)(k + u) * stride + 4 * i0));
        c[u] = __builtin_nontemporal_load(reinterpret_cast<const v4f*>(grads + (size_t)(k + u) * stride + 4 * j1));
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        g0 += lam.v[k + u] * a[u];
        g1 += lam.v[k + u] * c[u];
      }
    }
    for (; k < K; ++k) {
      g0 += lam.v[k] * __builtin_nontemporal_load(reinterpret_cast<const v4f*>(grads + (size_t)k * stride + 4 * i0));
      g1 += lam.v[k] * __builtin_nontemporal_load(reinterpret_cast<const v4f*>(grads + (size_t)k * stride + 4 * j1));
    }
    if (KEEPG) {
      *reinterpret_cast<v4f*>(gout + 4 * i0) = g0;
      if (has1) *reinterpret_cast<v4f*>(gout + 4 * i1) = g1;
    }
    apply_update<MOM>(th0, v0, g0, opt);
    apply_update<MOM>(th1, v1, g1, opt);
    *reinterpret_cast<v4f*>(params + 4 * i0) = th0;
    if (has1) *reinterpret_cast<v4f*>(params + 4 * i1) = th1;
    if (MOM) {
      *reinterpret_cast<v4f*>(velocity + 4 * i0) = v0;
      if (has1) *reinterpret_cast<v4f*>(velocity + 4 * i1) = v1;
    }
    if (SHADOW) {
      ushort4 s;
      s.x = bf16_rne(th0[0]); s.y = bf16_rne(th0[1]); s.z = bf16_rne(th0[2]); s.w = bf16_rne(th0[3]);
      *reinterpret_cast<ushort4*>(shadow + 4 * i0) = s;
      if (has1) {
        s.x = bf16_rne(th1[0]); s.y = bf16_rne(th1[1]); s.z = bf16_rne(th1[2]); s.w = bf16_rne(th1[3]);
        *reinterpret_cast<ushort4*>(shadow + 4 * i1) = s;
      }
    }
  }
  // tail (P not a multiple of 4)
  if (blockIdx.x == 0 && threadIdx.x < (P & 3)) {
    const size_t j = n4 * 4 + threadIdx.x;
    float g = 0.f;
    for (int k = 0; k < K; ++k) g += lam.v[k] * grads[(size_t)k * stride + j];
    if (KEEPG) gout[j] = g;
    float th = params[j];
    if (MOM) {
      const float d = g + opt.weight_decay * th;
      const float v = opt.momentum * velocity[j] + d;
      velocity[j] = v;
      th = th - opt.lr * v;
    } else {
      th = th - opt.lr * g;
    }
    params[j] = th;
    if (SHADOW) shadow[j] = bf16_rne(th);
  }
}

// g = sum_k lambda_k G[k] alone (equation bspweightedgrads without the update), same summation order.
__global__ __launch_bounds__(256) void weighted_reduce_kernel(const float* __restrict__ grads, size_t stride, size_t P,
                                                              int K, Lambdas lam, float* __restrict__ gout) {
  for (size_t j = (size_t)blockIdx.x * blockDim.x + threadIdx.x; j < P; j += (size_t)gridDim.x * blockDim.x) {
    float g = 0.f;
    for (int k = 0; k < K; ++k) g += lam.v[k] * grads[(size_t)k * stride + j];
    gout[j] = g;
  }
}

__global__ void fill_u32_kernel(uint32_t* p, size_t n, uint32_t v) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = v;
}

}  // namespace

void softmax_xent_f32(hipStream_t st, const float* z, const int32_t* labels, int C, const Segments& seg,
                      float* dz, float* loss_rows, float* loss_per_worker, float* loss, uint32_t* status) {
  const int rows = seg.off[seg.K];
  hipLaunchKernelGGL(softmax_xent_kernel, dim3((rows + 3) / 4), dim3(256), 0, st, z, labels, C, seg, dz,
                     loss_rows, status);
  hipLaunchKernelGGL(loss_reduce_kernel, dim3(1), dim3(256), 0, st, loss_rows, seg, loss_per_worker, loss);
}

static Lambdas lambdas_of(const Segments& seg) {
  Lambdas lam{};
  const double B = (double)seg.off[seg.K];
  for (int k = 0; k < seg.K; ++k) lam.v[k] = (float)((double)(seg.off[k + 1] - seg.off[k]) / B);
  return lam;
}

void weighted_sgd_f32(hipStream_t st, float* params, const float* grads, size_t stride, size_t P,
                      const Segments& seg, float lr, uint16_t* shadow_bf16, float* velocity, float momentum,
                      float weight_decay, const KernelTimer* timer, float* gout) {
  const Lambdas lam = lambdas_of(seg);
  const Optim opt{lr, momentum, weight_decay};
  const size_t n4 = P / 4;
  size_t blocks = (n4 + 511) / 512;          // two columns per thread per trip
  // Two workgroups per compute unit, each thread walking its columns: measured at P = 11.2 M, K = 8 (449 MB per
  // launch): 512 workgroups 71.8 us, 256: 73.8, 2048: 77.0, one trip per thread (5479): 74.7; counts that are no
  // multiple of the 256 compute units lose to the uneven last round (384: 78.5, 640: 80.6).
  if (blocks > 512) blocks = 512;
  if (blocks < 1) blocks = 1;
  const dim3 grid((unsigned)blocks), block(256);
#define OMNI_UPD(SH, MO, KG)                                                                                        \
  if (timer)                                                                                                        \
    hipExtLaunchKernelGGL((weighted_sgd_kernel<SH, MO, KG>), grid, block, 0, st, timer->start, timer->stop, 0,      \
                          params, velocity, grads, stride, P, seg.K, lam, opt, shadow_bf16, gout);                  \
  else                                                                                                              \
    hipLaunchKernelGGL((weighted_sgd_kernel<SH, MO, KG>), grid, block, 0, st, params, velocity, grads, stride, P,   \
                       seg.K, lam, opt, shadow_bf16, gout)
#define OMNI_UPD2(SH, MO)                                 \
  if (gout) { OMNI_UPD(SH, MO, true); } else { OMNI_UPD(SH, MO, false); }
  if (velocity) {
    if (shadow_bf16) { OMNI_UPD2(true, true) } else { OMNI_UPD2(false, true) }
  } else {
    if (shadow_bf16) { OMNI_UPD2(true, false) } else { OMNI_UPD2(false, false) }
  }
#undef OMNI_UPD2
#undef OMNI_UPD
}

void weighted_reduce_f32(hipStream_t st, const float* grads, size_t stride, size_t P, const Segments& seg,
                         float* gout) {
  size_t blocks = (P + 255) / 256;
  if (blocks > 4096) blocks = 4096;
  hipLaunchKernelGGL(weighted_reduce_kernel, dim3((unsigned)blocks), dim3(256), 0, st, grads, stride, P, seg.K,
                     lambdas_of(seg), gout);
}

void fill_u32(hipStream_t st, uint32_t* p, size_t n, uint32_t v) {
  if (n == 0) return;
  hipLaunchKernelGGL(fill_u32_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, p, n, v);
}

}  // namespace omni
