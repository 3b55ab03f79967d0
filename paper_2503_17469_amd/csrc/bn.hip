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

#include <algorithm>

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

// Work is dealt to workgroups in proportion to the workers' sizes: worker k owns the
// splits / chunks first[k] .. first[k+1]-1 of a ShareTable, each covering an equal share of ITS
// positions, so ragged b_k do not leave most of the chip waiting for the largest worker.

__device__ inline int share_owner(const ShareTable& tb, int K, int id) {
  int lo = 0, hi = K - 1;
  while (lo < hi) {
    const int mid = (lo + hi + 1) >> 1;
    if (id >= tb.first[mid]) lo = mid; else hi = mid - 1;
  }
  return lo;
}

// Partial sums of (a) x and x^2, or (b) dy and dy*xhat, over one split of one worker's positions.
// grid (total splits, ceil(C/64)); block = 8 channel pieces x 32 position lanes; four
// positions per lane in flight.
template <bool BWD>
__global__ __launch_bounds__(256) void bn_partial_kernel(const bf16_t* __restrict__ x, const bf16_t* __restrict__ dy,
                                                         const float* __restrict__ stats, int C, int hw,
                                                         Segments seg, ShareTable tb, double* __restrict__ partial) {
  __shared__ double red[32][8][17];
  const int tid = threadIdx.x;
  const int c8 = tid & 7, pl = tid >> 3;
  const int wk = share_owner(tb, seg.K, blockIdx.x);
  const int split = blockIdx.x - tb.first[wk], nsplit = tb.first[wk + 1] - tb.first[wk];
  const int c0 = blockIdx.y * 64 + c8 * 8;
  const bool cok = c0 < C;
  const int cl = cok ? c0 : 0;   // a piece past the last channel shadows piece 0 and is not stored
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
  if (BWD) {
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      mu[e] = stats[((size_t)wk * C + cl + e) * 2];
      is[e] = stats[((size_t)wk * C + cl + e) * 2 + 1];
    }
  }
  for (long p = sbeg + pl; p < send; p += 128) {
    // loads are unconditional (a position past the end re-reads the last one and adds zero)
    float xv[4][8], dv[4][8];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const long q = min(p + 32 * u, send - 1);
      Piece<bf16_t>::load(x + q * C + cl, xv[u]);
      if (BWD) Piece<bf16_t>::load(dy + q * C + cl, dv[u]);
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const float live = p + 32 * u < send ? 1.f : 0.f;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        if (!BWD) {
          const float v = xv[u][e] * live;
          s1[e] += (double)v;
          s2[e] += (double)v * (double)v;
        } else {
          const float d = dv[u][e] * live;
          s1[e] += (double)d;
          s2[e] += (double)(d * ((xv[u][e] - mu[e]) * is[e]));
        }
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
    const int c = blockIdx.y * 64 + cc;
    if (c < C) partial[((size_t)blockIdx.x * C + c) * 2 + which] = t;
  }
}

// Sum of worker wk's split partials for 64 channels: 4 lanes per channel walk the splits
// (stride 4, fixed order), then the 4 lane sums are added in lane order.
__device__ inline void bn_sum_splits(const double* __restrict__ partial, int C, const ShareTable& tb, int wk,
                                     int c, int sg, double (*red)[64][2], double& a, double& b) {
  a = 0.0; b = 0.0;
  if (c < C) {
    int s = tb.first[wk] + sg;
    const int s_end = tb.first[wk + 1];
    for (; s + 28 < s_end; s += 32) {   // eight loads in flight; the additions keep their order
      double2 v[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) v[u] = *reinterpret_cast<const double2*>(partial + ((size_t)(s + 4 * u) * C + c) * 2);
#pragma unroll
      for (int u = 0; u < 8; ++u) { a += v[u].x; b += v[u].y; }
    }
    for (; s < s_end; s += 4) {
      const double2 v = *reinterpret_cast<const double2*>(partial + ((size_t)s * C + c) * 2);
      a += v.x; b += v.y;
    }
  }
  red[sg][threadIdx.x & 63][0] = a;
  red[sg][threadIdx.x & 63][1] = b;
  __syncthreads();
  const int cc = threadIdx.x & 63;
  a = (red[0][cc][0] + red[1][cc][0]) + (red[2][cc][0] + red[3][cc][0]);
  b = (red[0][cc][1] + red[1][cc][1]) + (red[2][cc][1] + red[3][cc][1]);
}

// Forward: mean and 1/sqrt(var + eps) per (worker, channel).  grid (K, ceil(C/64)).
__global__ __launch_bounds__(256) void bn_finalize_fwd_kernel(const double* __restrict__ partial, int C, int hw,
                                                              Segments seg, ShareTable tb, float* __restrict__ stats) {
  __shared__ double red[4][64][2];
  const int wk = blockIdx.x, c = blockIdx.y * 64 + (threadIdx.x & 63), sg = threadIdx.x >> 6;
  double a, b;
  bn_sum_splits(partial, C, tb, wk, c, sg, red, a, b);
  if (sg != 0 || c >= C) return;
  const double n = (double)(seg.off[wk + 1] - seg.off[wk]) * hw;
  const double mean = a / n;
  double var = b / n - mean * mean;
  var = var > 0.0 ? var : 0.0;
  stats[((size_t)wk * C + c) * 2] = (float)mean;
  stats[((size_t)wk * C + c) * 2 + 1] = (float)(1.0 / sqrt(var + (double)kBnEps));
}

// Backward: dbeta, dgamma into worker k's gradient row, and the two means used by dx.
__global__ __launch_bounds__(256) void bn_finalize_bwd_kernel(const double* __restrict__ partial, int C, int hw,
                                                              Segments seg, ShareTable tb, float* __restrict__ means,
                                                              float* __restrict__ g_gamma, float* __restrict__ g_beta,
                                                              size_t worker_stride) {
  __shared__ double red[4][64][2];
  const int wk = blockIdx.x, c = blockIdx.y * 64 + (threadIdx.x & 63), sg = threadIdx.x >> 6;
  double a, b;
  bn_sum_splits(partial, C, tb, wk, c, sg, red, a, b);
  if (sg != 0 || c >= C) return;
  const double n = (double)(seg.off[wk + 1] - seg.off[wk]) * hw;
  g_beta[(size_t)wk * worker_stride + c] = (float)a;
  g_gamma[(size_t)wk * worker_stride + c] = (float)b;
  means[((size_t)wk * C + c) * 2] = (float)(a / n);
  means[((size_t)wk * C + c) * 2 + 1] = (float)(b / n);
}

// Normalise (forward) or input gradient (backward).  grid (total chunks); a workgroup
// walks one chunk of ONE worker's positions, so each thread keeps the statistics and
// the affine parameters of its 8 channels in registers; C/8 threads cover a position,
// floor(256 / (C/8)) positions are in flight per trip, four trips unrolled.
template <bool BWD>
__global__ __launch_bounds__(256) void bn_apply_kernel(const bf16_t* __restrict__ x, const bf16_t* __restrict__ dy,
                                                       const float* __restrict__ stats, const float* __restrict__ means,
                                                       const float* __restrict__ gamma, const float* __restrict__ beta,
                                                       int C, int hw, Segments seg, ShareTable tb, int relu,
                                                       bf16_t* __restrict__ out, const bf16_t* __restrict__ skip,
                                                       int relu_add, uint8_t* __restrict__ sign_bits) {
  const int c8n = C / 8;
  const int ppar = 256 / c8n;                   // positions per trip
  const int tid = threadIdx.x;
  const int pc = tid % c8n, lp = tid / c8n;
  if (lp >= ppar) return;
  const int wk = share_owner(tb, seg.K, blockIdx.x);
  const int chunk = blockIdx.x - tb.first[wk], nchunk = tb.first[wk + 1] - tb.first[wk];
  const long pbeg = (long)seg.off[wk] * hw, pend = (long)seg.off[wk + 1] * hw;
  const long per = (pend - pbeg + nchunk - 1) / nchunk;
  const long cbeg = pbeg + chunk * per, cend = min(pend, cbeg + per);
  const int c0 = pc * 8;
  float mu[8], is[8], gm[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    mu[e] = stats[((size_t)wk * C + c0 + e) * 2];
    is[e] = stats[((size_t)wk * C + c0 + e) * 2 + 1];
    gm[e] = gamma[c0 + e];
  }
  float bt[8], mn1[8], mn2[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    bt[e] = BWD ? 0.f : beta[c0 + e];
    mn1[e] = BWD ? means[((size_t)wk * C + c0 + e) * 2] : 0.f;
    mn2[e] = BWD ? means[((size_t)wk * C + c0 + e) * 2 + 1] : 0.f;
  }
  for (long p = cbeg + lp; p < cend; p += 4 * ppar) {
    float xv[4][8], dv[4][8];   // dv: the output gradient (backward) or the residual input (forward, with skip)
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const long q = min(p + (long)u * ppar, cend - 1);
      Piece<bf16_t>::load(x + q * C + c0, xv[u]);
      if (BWD) Piece<bf16_t>::load(dy + q * C + c0, dv[u]);
      else if (skip) Piece<bf16_t>::load(skip + q * C + c0, dv[u]);
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const long q = p + (long)u * ppar;
      if (q >= cend) break;
      float o[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const float xh = (xv[u][e] - mu[e]) * is[e];
        if (!BWD) {
          float y = gm[e] * xh + bt[e];
          if (relu) y = y > 0.f ? y : 0.f;
          if (skip) {
            // the residual add that follows, on the normalised value as it would have been stored
            y = bf16_to_f32(f32_to_bf16(y)) + dv[u][e];
            if (relu_add) y = y > 0.f ? y : 0.f;
          }
          o[e] = y;
        } else {
          o[e] = gm[e] * is[e] * (dv[u][e] - mn1[e] - xh * mn2[e]);
        }
      }
      if (!BWD && sign_bits) {
        // (the piece is packed here rather than in Piece::store: the bits are those of the values as stored)
        u32x4 t;
#pragma unroll
        for (int d = 0; d < 4; ++d) t[d] = pack_bf16(o[2 * d], o[2 * d + 1]);
        *reinterpret_cast<u32x4*>(out + q * C + c0) = t;
        uint32_t bits = 0;
#pragma unroll
        for (int d = 0; d < 4; ++d) {
          const uint32_t lo = t[d] & 0xFFFFu, hi = t[d] >> 16;
          bits |= ((lo != 0u && lo < 0x8000u) ? 1u : 0u) << (2 * d);
          bits |= ((hi != 0u && hi < 0x8000u) ? 1u : 0u) << (2 * d + 1);
        }
        sign_bits[q * c8n + pc] = (uint8_t)bits;
      } else {
        Piece<bf16_t>::store(out + q * C + c0, o);
      }
    }
  }
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

// Deal `total` shares to the workers in proportion to their rows (at least one each).
ShareTable deal_shares(const Segments& seg, long total) {
  ShareTable tb{};
  const long B = std::max(1, seg.off[seg.K]);
  int acc = 0;
  for (int k = 0; k < seg.K; ++k) {
    tb.first[k] = acc;
    const long bk = seg.off[k + 1] - seg.off[k];
    acc += (int)std::max<long>(1, (total * bk + B / 2) / B);
  }
  tb.first[seg.K] = acc;
  return tb;
}

ShareTable bn_splits(const Segments& seg, int C) {
  const int groups = (C + 63) / 64;
  // about 2048 workgroups, never more splits than the scratch holds (K * kBnMaxSplits in all)
  long total = std::max<long>(seg.K, 2048 / groups);
  total = std::min<long>(total, (long)seg.K * (kBnMaxSplits - 2));
  return deal_shares(seg, total);
}

ShareTable bn_chunks(const Segments& seg, int C, int hw) {
  const long positions = (long)seg.off[seg.K] * hw;
  const int ppar = 256 / (C / 8);
  // about 4096 workgroups, at least 8 trips each
  long total = std::min<long>(4096, std::max<long>(seg.K, positions / (32L * ppar)));
  return deal_shares(seg, total);
}

}  // namespace

bool bn_shape_supported(int C) { return C % 8 == 0 && C >= 8 && C <= 2048; }

void bn_forward_bf16(hipStream_t st, const bf16_t* x, bf16_t* y, const float* gamma, const float* beta, int C, int hw,
                     const Segments& seg, bool relu, float* stats, double* partial, const bf16_t* skip,
                     bool relu_add, const ShareTable* presummed, uint8_t* sign_bits) {
  const ShareTable sp = presummed ? *presummed : bn_splits(seg, C);
  const int groups = (C + 63) / 64;
  if (!presummed)
    hipLaunchKernelGGL(bn_partial_kernel<false>, dim3(sp.first[seg.K], groups), dim3(256), 0, st, x, nullptr,
                       nullptr, C, hw, seg, sp, partial);
  hipLaunchKernelGGL(bn_finalize_fwd_kernel, dim3(seg.K, groups), dim3(256), 0, st, partial, C, hw, seg, sp, stats);
  const ShareTable ch = bn_chunks(seg, C, hw);
  hipLaunchKernelGGL(bn_apply_kernel<false>, dim3(ch.first[seg.K]), dim3(256), 0, st, x, nullptr, stats, nullptr,
                     gamma, beta, C, hw, seg, ch, relu ? 1 : 0, y, skip, relu_add ? 1 : 0, sign_bits);
}

void bn_backward_bf16(hipStream_t st, const bf16_t* x, const bf16_t* dy, bf16_t* dx, const float* gamma, int C, int hw,
                      const Segments& seg, const float* stats, float* means, double* partial, float* g_gamma,
                      float* g_beta, size_t worker_stride) {
  const ShareTable sp = bn_splits(seg, C);
  const int groups = (C + 63) / 64;
  hipLaunchKernelGGL(bn_partial_kernel<true>, dim3(sp.first[seg.K], groups), dim3(256), 0, st, x, dy, stats, C, hw,
                     seg, sp, partial);
  hipLaunchKernelGGL(bn_finalize_bwd_kernel, dim3(seg.K, groups), dim3(256), 0, st, partial, C, hw, seg, sp, means,
                     g_gamma, g_beta, worker_stride);
  const ShareTable ch = bn_chunks(seg, C, hw);
  hipLaunchKernelGGL(bn_apply_kernel<true>, dim3(ch.first[seg.K]), dim3(256), 0, st, x, dy, stats, means, gamma,
                     nullptr, C, hw, seg, ch, 0, dx, nullptr, 0, nullptr);
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
