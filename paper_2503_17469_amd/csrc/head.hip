// Classifier head: the last fully connected layer (few outputs), the softmax
// cross-entropy loss over the ragged batch and the first backward step, fused.
//
// With 10 or 100 classes the last layer is far too thin for a matrix-core tile
// and far too small to fill the chip; what it costs is launches and round trips
// through HBM.  Two kernels replace six:
//   1. one wavefront per row: logits z = x w^T + bias, loss_row = logsumexp(z) -
//      z[y], dz = (softmax(z) - onehot(y)) / b_k  (the 1/|b_k| of equation
//      bspweightedgrads: everything downstream is worker k's MEAN gradient), and
//      the input gradient dx = dz w (masked by the folded ReLU);
//   2. per worker: gw_k = dz_k^T x_k and gb_k = sum of dz_k rows, plus (in one
//      extra workgroup) L_k, the lambda-weighted total loss and the label check.
#include <hip/hip_runtime.h>

#include "bf16.h"
#include "common.h"
#include "head_device.h"
#include "kernels.h"

namespace omni {

namespace {

constexpr int kMaxClasses = 128;

__device__ inline int owner(const Segments& seg, int s) {
  int k = 0;
  while (k + 1 < seg.K && s >= seg.off[k + 1]) ++k;
  return k;
}
__device__ inline float dot4(v4f a, v4f b) { return a[0] * b[0] + a[1] * b[1] + a[2] * b[2] + a[3] * b[3]; }

// T is the storage type of the input rows, the weights and the input gradient
// (fp32, or bf16 with fp32 arithmetic).  NV = 16-byte pieces of the input row
// each lane keeps in registers; one piece per lane covers 64 * EL consecutive
// inputs across the wavefront, so cin <= 64 * EL * NV.
// WLDS: the whole weight matrix (at most 48 KB) is copied into LDS once per workgroup, while
// the input rows are on their way, and both passes over it (logits, input gradient) read it
// there.  A wavefront then waits for memory once instead of once per group of classes in each
// pass; with one row per wavefront and two wavefronts per compute unit that chain of round
// trips, not bandwidth, is what the kernel's time consists of.
template <typename T, int NV, bool WLDS>
__global__ __launch_bounds__(256) void head_fwd_loss_dgrad_kernel(
    const T* __restrict__ x, const T* __restrict__ w, const float* __restrict__ bias,
    const int32_t* __restrict__ labels, int cin, int C, Segments seg, float* __restrict__ z,
    float* __restrict__ dz, float* __restrict__ loss_rows, int use_mask, T* __restrict__ dx, int accumulate) {
  constexpr int EL = Piece<T>::EL;
  constexpr int CH = NV * EL <= 16 ? 8 : 4;   // classes whose weight rows are in flight together
  __shared__ float zbuf[4][kMaxClasses];
  extern __shared__ __attribute__((aligned(16))) unsigned char wl_raw[];
  const T* wp = WLDS ? reinterpret_cast<const T*>(wl_raw) : w;
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  const int rows = seg.off[seg.K];
  const int row_raw = blockIdx.x * 4 + wv;
  const bool live = row_raw < rows;
  const int row = live ? row_raw : rows - 1;   // idle wavefronts shadow the last row and write nothing
  const T* xr = x + (size_t)row * cin;

  // ---- logits: the row stays in registers, weight rows stream past it.
  // Loads are unconditional (an out-of-range piece re-reads piece 0 and is zeroed
  // afterwards): guarded loads would serialise behind per-load waits.
  float a[NV][EL];
  int kk[NV];
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    const int k = (lane + 64 * i) * EL;
    kk[i] = k < cin ? k : 0;
    Piece<T>::load(xr + kk[i], a[i]);
  }
  if (WLDS) {
    const int npieces = C * cin / EL;          // 16-byte pieces; cin is a multiple of EL
    const u32x4* src = reinterpret_cast<const u32x4*>(w);
    u32x4* dst = reinterpret_cast<u32x4*>(wl_raw);
    // eight pieces per thread in flight at a time (a piece past the end re-reads the last one)
    for (int q0 = threadIdx.x; q0 < npieces; q0 += 256 * 8) {
      u32x4 t[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) t[u] = src[min(q0 + 256 * u, npieces - 1)];
#pragma unroll
      for (int u = 0; u < 8; ++u)
        if (q0 + 256 * u < npieces) dst[q0 + 256 * u] = t[u];
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < NV; ++i)
    if ((lane + 64 * i) * EL >= cin) {
#pragma unroll
      for (int e = 0; e < EL; ++e) a[i][e] = 0.f;
    }
  for (int c0 = 0; c0 < C; c0 += CH) {
    float acc[CH];
#pragma unroll
    for (int j = 0; j < CH; ++j) {
      acc[j] = 0.f;
      const int c = min(c0 + j, C - 1);
#pragma unroll
      for (int i = 0; i < NV; ++i) {
        float wv_[EL];
        Piece<T>::load(wp + (size_t)c * cin + kk[i], wv_);
#pragma unroll
        for (int e = 0; e < EL; ++e) acc[j] += a[i][e] * wv_[e];
      }
    }
#pragma unroll
    for (int j = 0; j < CH; ++j) {
      const float s = wave_sum(acc[j]);
      if (lane == j && c0 + j < C) zbuf[wv][c0 + j] = s + (bias ? bias[c0 + j] : 0.f);
    }
  }
  __syncthreads();

  // ---- loss and dz
  const int k_own = owner(seg, row);
  const float inv_b = 1.0f / (float)(seg.off[k_own + 1] - seg.off[k_own]);
  const int y = labels[row];
  const bool bad = (y < 0 || y >= C);
  float m = -INFINITY;
  for (int c = lane; c < C; c += 64) m = fmaxf(m, zbuf[wv][c]);
  m = wave_max(m);
  float s = 0.f;
  for (int c = lane; c < C; c += 64) s += expf(zbuf[wv][c] - m);
  s = wave_sum(s);
  const float lse = logf(s);
  if (live && lane == 0) loss_rows[row] = bad ? 0.f : lse - (zbuf[wv][bad ? 0 : y] - m);
  for (int c = lane; c < C; c += 64) {
    const float zc = zbuf[wv][c];
    float p = expf(zc - m - lse);
    if (c == y) p -= 1.0f;
    p = bad ? 0.f : p * inv_b;
    if (live) {
      z[(size_t)row * C + c] = zc;
      dz[(size_t)row * C + c] = p;
    }
    zbuf[wv][c] = p;        // the lane that read this slot overwrites it
  }
  __syncthreads();

  // ---- input gradient dx = dz w, masked by the folded ReLU (the input row itself)
  if (dx != nullptr && live) {
    float g[NV][EL];
#pragma unroll
    for (int i = 0; i < NV; ++i)
#pragma unroll
      for (int e = 0; e < EL; ++e) g[i][e] = 0.f;
#pragma unroll 4
    for (int c = 0; c < C; ++c) {
      const float d = zbuf[wv][c];
#pragma unroll
      for (int i = 0; i < NV; ++i) {
        float wv_[EL];
        Piece<T>::load(wp + (size_t)c * cin + kk[i], wv_);
#pragma unroll
        for (int e = 0; e < EL; ++e) g[i][e] += d * wv_[e];
      }
    }
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      const int k = (lane + 64 * i) * EL;
      if (k >= cin) continue;
      const size_t idx = (size_t)row * cin + k;
      if (use_mask) {
#pragma unroll
        for (int e = 0; e < EL; ++e) g[i][e] = a[i][e] > 0.f ? g[i][e] : 0.f;
      }
      if (accumulate) {
        float old[EL];
        Piece<T>::load(dx + idx, old);
#pragma unroll
        for (int e = 0; e < EL; ++e) g[i][e] += old[e];
      }
      Piece<T>::store(dx + idx, g[i]);
    }
  }
}

template <typename T>
__global__ __launch_bounds__(256) void head_wgrad_loss_kernel(HeadWgradParams h, Segments seg) {
  __shared__ __attribute__((aligned(16))) float smem[kHeadWgradLdsFloats];
  head_wgrad_loss_body<T>(h, seg, (int)blockIdx.x, (int)blockIdx.y, smem);
}

}  // namespace

bool head_supported(int cin, int classes, const void* x, const void* w, bool bf16) {
  const int el = bf16 ? 8 : 4;
  return classes >= 1 && classes <= kMaxClasses && cin % el == 0 && cin <= 2048 &&
         (reinterpret_cast<uintptr_t>(x) & 15u) == 0 && (reinterpret_cast<uintptr_t>(w) & 15u) == 0;
}

template <typename T>
static void launch_head_fwd(hipStream_t st, const T* x, const T* w, const float* bias, const int32_t* labels, int cin,
                            int classes, const Segments& seg, float* z, float* dz, float* loss_rows, bool use_mask,
                            T* dx, bool accumulate) {
  const int rows = seg.off[seg.K];
  const int nv = (cin + 64 * Piece<T>::EL - 1) / (64 * Piece<T>::EL);
  const dim3 grid((rows + 3) / 4), block(256);
  const int acc = accumulate ? 1 : 0, um = use_mask ? 1 : 0;
  const size_t wbytes = (size_t)classes * cin * sizeof(T);
  const bool wlds = wbytes <= 48 * 1024;
#define OMNI_HEAD(NV)                                                                                              \
  do {                                                                                                             \
    if (wlds)                                                                                                      \
      hipLaunchKernelGGL((head_fwd_loss_dgrad_kernel<T, NV, true>), grid, block, wbytes, st, x, w, bias, labels,   \
                         cin, classes, seg, z, dz, loss_rows, um, dx, acc);                                        \
    else                                                                                                           \
      hipLaunchKernelGGL((head_fwd_loss_dgrad_kernel<T, NV, false>), grid, block, 0, st, x, w, bias, labels, cin,  \
                         classes, seg, z, dz, loss_rows, um, dx, acc);                                             \
  } while (0)
  if (nv <= 1) OMNI_HEAD(1);
  else if (nv <= 2) OMNI_HEAD(2);
  else if (nv <= 4) OMNI_HEAD(4);
  else if constexpr (Piece<T>::EL == 4) OMNI_HEAD(8);
#undef OMNI_HEAD
}

void head_fwd_loss_dgrad(hipStream_t st, bool bf16, const void* x, const void* w, const float* bias,
                         const int32_t* labels, int cin, int classes, const Segments& seg, float* z, float* dz,
                         float* loss_rows, bool use_mask, void* dx, bool accumulate) {
  if (bf16)
    launch_head_fwd<bf16_t>(st, static_cast<const bf16_t*>(x), static_cast<const bf16_t*>(w), bias, labels, cin,
                            classes, seg, z, dz, loss_rows, use_mask, static_cast<bf16_t*>(dx), accumulate);
  else
    launch_head_fwd<float>(st, static_cast<const float*>(x), static_cast<const float*>(w), bias, labels, cin, classes,
                           seg, z, dz, loss_rows, use_mask, static_cast<float*>(dx), accumulate);
}

void head_wgrad_loss(hipStream_t st, bool bf16, const float* dz, const void* x, const int32_t* labels, int cin,
                     int classes, const Segments& seg, float* gw, float* gb, size_t worker_stride,
                     const float* loss_rows, float* loss_per_worker, float* loss, uint32_t* status) {
  const HeadWgradParams h{dz, x, labels, cin, classes, gw, gb, worker_stride, loss_rows, loss_per_worker, loss, status};
  const dim3 grid = head_wgrad_grid(cin, classes, seg.K);
  if (bf16)
    hipLaunchKernelGGL(head_wgrad_loss_kernel<bf16_t>, grid, dim3(256), 0, st, h, seg);
  else
    hipLaunchKernelGGL(head_wgrad_loss_kernel<float>, grid, dim3(256), 0, st, h, seg);
}

}  // namespace omni
