// Bandwidth-bound bf16 kernels of the convolutional path: weight casts, channel
// padding of the network input, 2x2 max pooling forward and backward.
#include <hip/hip_runtime.h>

#include <algorithm>

#include "bf16.h"
#include "common.h"
#include "kernels.h"

namespace omni {

namespace {

// All layers' weight copies in one launch: with a few thousand weights per layer a launch per
// layer is pure launch latency (4 x 4.6 us at the three-layer CNN).  The table travels in the
// kernel arguments.
__global__ __launch_bounds__(256) void cast_weights_kernel(CastTable tab, const float* __restrict__ params,
                                                           bf16_t* __restrict__ shadow, uint32_t* __restrict__ zero_page) {
  if (zero_page && blockIdx.x == 0 && threadIdx.x < kZeroPageWords) zero_page[threadIdx.x] = 0u;
  int e = 0;
  while (e + 1 < tab.n && (int)blockIdx.x >= tab.e[e + 1].first_block) ++e;
  const CastEntry t = tab.e[e];
  const long n = (long)t.cout * t.taps * t.cin_pad;
  const long i = (long)(blockIdx.x - t.first_block) * blockDim.x + threadIdx.x;
  if (i >= n) return;
  const int ci = (int)(i % t.cin_pad);
  const long r = i / t.cin_pad;
  const int tap = (int)(r % t.taps), co = (int)(r / t.taps);
  const float v = ci < t.cin_real ? params[t.src + ((long)co * t.taps + tap) * t.cin_real + ci] : 0.f;
  const bf16_t h = f32_to_bf16(v);
  shadow[t.dst_fwd + i] = h;
  if (t.dst_t >= 0) shadow[t.dst_t + ((long)ci * t.taps + tap) * t.cout + co] = h;
}

__global__ __launch_bounds__(256) void pad_channels_kernel(const bf16_t* __restrict__ x, bf16_t* __restrict__ xp,
                                                           long pixels, int c_real, int c_pad) {
  const long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= pixels * c_pad) return;
  const int c = (int)(i % c_pad);
  const long px = i / c_pad;
  xp[i] = c < c_real ? x[px * c_real + c] : (bf16_t)0;
}

// 3 -> 8 channels, four pixels per thread: 24 bytes in (three 8-byte loads), four 16-byte pieces out
__global__ __launch_bounds__(256) void pad_3to8_kernel(const bf16_t* __restrict__ x, bf16_t* __restrict__ xp,
                                                       long quads) {
  const long q = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (q >= quads) return;
  const u32x2* src = reinterpret_cast<const u32x2*>(x + q * 12);
  const u32x2 a = src[0], b = src[1], c = src[2];        // 12 values: a0 a1 | a2 b0 || b1 b2 | c0 c1 || c2 d0 | d1 d2
  u32x4* dst = reinterpret_cast<u32x4*>(xp + q * 32);
  dst[0] = u32x4{a[0], a[1] & 0xFFFFu, 0u, 0u};
  dst[1] = u32x4{(a[1] >> 16) | (b[0] << 16), b[0] >> 16, 0u, 0u};
  dst[2] = u32x4{b[1], c[0] & 0xFFFFu, 0u, 0u};
  dst[3] = u32x4{(c[0] >> 16) | (c[1] << 16), c[1] >> 16, 0u, 0u};
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

// one thread = 8 channels of one pooled position; the codes say where each gradient goes
__global__ __launch_bounds__(256) void maxpool2_bwd_coded_kernel(const uint8_t* __restrict__ code,
                                                                 const bf16_t* __restrict__ dout,
                                                                 bf16_t* __restrict__ din, long n_out, int H, int W,
                                                                 int C) {
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
  const u32x2 k = *reinterpret_cast<const u32x2*>(code + i * 8);
  float g[8], o[4][8];
  Piece<bf16_t>::load(dout + i * 8, g);
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    const uint32_t ke = (k[e >> 2] >> (8 * (e & 3))) & 0xFFu;
#pragma unroll
    for (int q = 0; q < 4; ++q) o[q][e] = ke == (uint32_t)q ? g[e] : 0.f;
  }
#pragma unroll
  for (int q = 0; q < 4; ++q) Piece<bf16_t>::store(din + offs[q], o[q]);
}

inline unsigned blocks_for(long n) { return (unsigned)((n + 255) / 256); }

}  // namespace

void cast_weights_bf16(hipStream_t st, const float* params, bf16_t* shadow, const CastEntry* entries, int n,
                       uint32_t* zero_page) {
  for (int base = 0; base < n; base += kCastMaxEntries) {
    CastTable tab{};
    tab.n = std::min(n - base, kCastMaxEntries);
    int blocks = 0;
    for (int i = 0; i < tab.n; ++i) {
      tab.e[i] = entries[base + i];
      tab.e[i].first_block = blocks;
      blocks += (int)blocks_for((long)tab.e[i].cout * tab.e[i].taps * tab.e[i].cin_pad);
    }
    if (blocks > 0)
      hipLaunchKernelGGL(cast_weights_kernel, dim3(blocks), dim3(256), 0, st, tab, params, shadow,
                         base == 0 ? zero_page : nullptr);
  }
}

void pad_channels_bf16(hipStream_t st, const bf16_t* x, bf16_t* xp, long pixels, int c_real, int c_pad) {
  if (c_real == 3 && c_pad == 8 && pixels % 4 == 0 && (reinterpret_cast<uintptr_t>(x) & 7u) == 0 &&
      (reinterpret_cast<uintptr_t>(xp) & 15u) == 0) {
    hipLaunchKernelGGL(pad_3to8_kernel, dim3(blocks_for(pixels / 4)), dim3(256), 0, st, x, xp, pixels / 4);
    return;
  }
  hipLaunchKernelGGL(pad_channels_kernel, dim3(blocks_for(pixels * c_pad)), dim3(256), 0, st, x, xp, pixels, c_real,
                     c_pad);
}

void maxpool2_fwd_bf16(hipStream_t st, const bf16_t* in, bf16_t* out, int rows, int H, int W, int C) {
  const long n_out = (long)rows * (H / 2) * (W / 2) * (C / 8);
  hipLaunchKernelGGL(maxpool2_fwd_kernel, dim3(blocks_for(n_out)), dim3(256), 0, st, in, out, n_out, H, W, C);
}

void maxpool2_bwd_coded_bf16(hipStream_t st, const uint8_t* code, const bf16_t* dout, bf16_t* din, int rows, int H,
                             int W, int C) {
  const long n_out = (long)rows * (H / 2) * (W / 2) * (C / 8);
  hipLaunchKernelGGL(maxpool2_bwd_coded_kernel, dim3(blocks_for(n_out)), dim3(256), 0, st, code, dout, din, n_out, H,
                     W, C);
}

void maxpool2_bwd_bf16(hipStream_t st, const bf16_t* in, const bf16_t* dout, bf16_t* din, int rows, int H, int W,
                       int C, bool relu_mask) {
  const long n_out = (long)rows * (H / 2) * (W / 2) * (C / 8);
  hipLaunchKernelGGL(maxpool2_bwd_kernel, dim3(blocks_for(n_out)), dim3(256), 0, st, in, dout, din, n_out, H, W, C,
                     relu_mask ? 1 : 0);
}

}  // namespace omni
