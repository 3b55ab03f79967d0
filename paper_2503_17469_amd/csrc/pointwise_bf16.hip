// Bandwidth-bound bf16 kernels of the convolutional path: weight casts, channel
// padding of the network input, 2x2 max pooling forward and backward.
#include <hip/hip_runtime.h>

#include "bf16.h"
#include "common.h"
#include "kernels.h"

namespace omni {

namespace {

__global__ __launch_bounds__(256) void cast_weights_kernel(const float* __restrict__ w, bf16_t* __restrict__ w_fwd,
                                                           bf16_t* __restrict__ w_t, int cout, int taps, int cin_real,
                                                           int cin_pad) {
  const long n = (long)cout * taps * cin_pad;
  const long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  const int ci = (int)(i % cin_pad);
  const long r = i / cin_pad;
  const int tap = (int)(r % taps), co = (int)(r / taps);
  const float v = ci < cin_real ? w[((long)co * taps + tap) * cin_real + ci] : 0.f;
  const bf16_t h = f32_to_bf16(v);
  w_fwd[i] = h;
  if (w_t) w_t[((long)ci * taps + tap) * cout + co] = h;
}

__global__ __launch_bounds__(256) void pad_channels_kernel(const bf16_t* __restrict__ x, bf16_t* __restrict__ xp,
                                                           long pixels, int c_real, int c_pad) {
  const long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= pixels * c_pad) return;
  const int c = (int)(i % c_pad);
  const long px = i / c_pad;
  xp[i] = c < c_real ? x[px * c_real + c] : (bf16_t)0;
}

// one thread = 8 channels of one output position
__global__ __launch_bounds__(256) void maxpool2_fwd_kernel(const bf16_t* __restrict__ in, bf16_t* __restrict__ out,
                                                           long n_out, int H, int W, int C) {
  const long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n_out) return;
  const int c8 = C / 8;
  const int cc = (int)(i % c8);
  long r = i / c8;
  const int wo = (int)(r % (W / 2)); r /= (W / 2);
  const int ho = (int)(r % (H / 2));
  const long n = r / (H / 2);
  const bf16_t* p = in + (((n * H + 2 * ho) * W + 2 * wo) * (long)C) + cc * 8;
  float a[8], b[8], c[8], d[8], m[8];
  Piece<bf16_t>::load(p, a);
  Piece<bf16_t>::load(p + C, b);
  Piece<bf16_t>::load(p + (long)W * C, c);
  Piece<bf16_t>::load(p + (long)W * C + C, d);
#pragma unroll
  for (int e = 0; e < 8; ++e) m[e] = fmaxf(fmaxf(a[e], b[e]), fmaxf(c[e], d[e]));
  Piece<bf16_t>::store(out + i * 8, m);
}

__global__ __launch_bounds__(256) void maxpool2_bwd_kernel(const bf16_t* __restrict__ in,
                                                           const bf16_t* __restrict__ dout, bf16_t* __restrict__ din,
                                                           long n_out, int H, int W, int C, int relu_mask) {
  const long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n_out) return;
  const int c8 = C / 8;
  const int cc = (int)(i % c8);
  long r = i / c8;
  const int wo = (int)(r % (W / 2)); r /= (W / 2);
  const int ho = (int)(r % (H / 2));
  const long n = r / (H / 2);
  const long o00 = (((n * H + 2 * ho) * W + 2 * wo) * (long)C) + cc * 8;
  const long offs[4] = {o00, o00 + C, o00 + (long)W * C, o00 + (long)W * C + C};   // (dy, dx) scan order
  float v[4][8], g[8], o[4][8];
#pragma unroll
  for (int q = 0; q < 4; ++q) Piece<bf16_t>::load(in + offs[q], v[q]);
  Piece<bf16_t>::load(dout + i * 8, g);
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    const float m = fmaxf(fmaxf(v[0][e], v[1][e]), fmaxf(v[2][e], v[3][e]));
    const bool pass = !relu_mask || m > 0.f;
    bool taken = false;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const bool hit = !taken && v[q][e] == m;
      o[q][e] = (hit && pass) ? g[e] : 0.f;
      taken = taken || hit;
    }
  }
#pragma unroll
  for (int q = 0; q < 4; ++q) Piece<bf16_t>::store(din + offs[q], o[q]);
}

inline unsigned blocks_for(long n) { return (unsigned)((n + 255) / 256); }

}  // namespace

void cast_weights_bf16(hipStream_t st, const float* w, bf16_t* w_fwd, bf16_t* w_t, int cout, int taps,
                       int cin_real, int cin_pad) {
  const long n = (long)cout * taps * cin_pad;
  hipLaunchKernelGGL(cast_weights_kernel, dim3(blocks_for(n)), dim3(256), 0, st, w, w_fwd, w_t, cout, taps, cin_real,
                     cin_pad);
}

void pad_channels_bf16(hipStream_t st, const bf16_t* x, bf16_t* xp, long pixels, int c_real, int c_pad) {
  hipLaunchKernelGGL(pad_channels_kernel, dim3(blocks_for(pixels * c_pad)), dim3(256), 0, st, x, xp, pixels, c_real,
                     c_pad);
}

void maxpool2_fwd_bf16(hipStream_t st, const bf16_t* in, bf16_t* out, int rows, int H, int W, int C) {
  const long n_out = (long)rows * (H / 2) * (W / 2) * (C / 8);
  hipLaunchKernelGGL(maxpool2_fwd_kernel, dim3(blocks_for(n_out)), dim3(256), 0, st, in, out, n_out, H, W, C);
}

void maxpool2_bwd_bf16(hipStream_t st, const bf16_t* in, const bf16_t* dout, bf16_t* din, int rows, int H, int W,
                       int C, bool relu_mask) {
  const long n_out = (long)rows * (H / 2) * (W / 2) * (C / 8);
  hipLaunchKernelGGL(maxpool2_bwd_kernel, dim3(blocks_for(n_out)), dim3(256), 0, st, in, dout, din, n_out, H, W, C,
                     relu_mask ? 1 : 0);
}

}  // namespace omni
