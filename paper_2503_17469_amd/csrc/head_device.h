// Device code of the classifier head that more than one kernel uses: the wavefront
// reductions and the body of the head's parameter-gradient kernel (a kernel of its own
// in head.hip; one role of a merged launch in gemm_f32_direct.hip).
#pragma once
#include <hip/hip_runtime.h>

#include "bf16.h"
#include "common.h"
#include "kernels.h"

namespace omni {

// Wavefront-wide reductions on the vector ALU's data-parallel primitives: two quad
// permutes and two row mirrors leave every lane with the result of its row of 16, four
// lane reads combine the rows.  (A butterfly of __shfl_xor goes through the LDS crossbar:
// six dependent round trips of ~170 cycles each per reduction; with one wavefront per SIMD
// nothing hides them, and the ten per-class sums of the classifier were most of this
// kernel's time.)
template <int CTRL>
__device__ inline float dpp_move(float v) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xF, 0xF, false));
}
__device__ inline float lane_value(float v, int lane) {
  return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), lane));
}
__device__ inline float wave_sum(float v) {
  v += dpp_move<0xB1>(v);    // quad_perm [1,0,3,2]
  v += dpp_move<0x4E>(v);    // quad_perm [2,3,0,1]
  v += dpp_move<0x141>(v);   // row_half_mirror
  v += dpp_move<0x140>(v);   // row_mirror
  return (lane_value(v, 0) + lane_value(v, 16)) + (lane_value(v, 32) + lane_value(v, 48));
}
__device__ inline float wave_max(float v) {
  v = fmaxf(v, dpp_move<0xB1>(v));
  v = fmaxf(v, dpp_move<0x4E>(v));
  v = fmaxf(v, dpp_move<0x141>(v));
  v = fmaxf(v, dpp_move<0x140>(v));
  return fmaxf(fmaxf(lane_value(v, 0), lane_value(v, 16)), fmaxf(lane_value(v, 32), lane_value(v, 48)));
}
constexpr int kHeadWgradLdsFloats = 16 * 16 * 17 + 256 * 16;
inline dim3 head_wgrad_grid(int cin, int classes, int K) {
  return dim3(K * ((cin + 15) / 16) + 1, (classes + 15) / 16, 1);
}

// Workgroup (bx, by) of a K * ceil(cin/16) + 1 by ceil(C/16) grid (head_wgrad_grid), 256 threads,
// kHeadWgradLdsFloats floats of LDS at smem (16-byte aligned).  A workgroup is 16 input
// columns x 16 row groups; each thread walks its share of the worker's rows.
// The worker's dz rows (16 classes of them) are staged in LDS 256 rows at a time:
// fetched per thread they would be 16 global loads per row, and the vector cache,
// not the arithmetic, would set the pace.
template <typename T>
__device__ __forceinline__ void head_wgrad_loss_body(const HeadWgradParams& h, const Segments& seg, int bx, int by,
                                                     float* smem) {
  float (*red)[16][17] = reinterpret_cast<float (*)[16][17]>(smem);
  float (*dzs)[16] = reinterpret_cast<float (*)[16]>(smem + 16 * 16 * 17);
  const float* __restrict__ dz = h.dz;
  const T* __restrict__ x = static_cast<const T*>(h.x);
  const int32_t* __restrict__ labels = h.labels;
  const int cin = h.cin, C = h.C;
  float* __restrict__ gw = h.gw;
  float* __restrict__ gb = h.gb;
  const size_t worker_stride = h.worker_stride;
  const float* __restrict__ loss_rows = h.loss_rows;
  float* __restrict__ loss_per_worker = h.loss_per_worker;
  float* __restrict__ loss = h.loss;
  uint32_t* __restrict__ status = h.status;
  const int tid = threadIdx.x;
  const int jchunks = (cin + 15) / 16;

  if (bx == seg.K * jchunks) {
    // ---- the extra workgroup: losses and label check; one wavefront per worker
    if (by != 0) return;
    float* part = &red[0][0][0];
    const int lane = tid & 63, wv = tid >> 6;
    const int rows = seg.off[seg.K];
    const float invB = 1.0f / (float)rows;
    for (int k = wv; k < seg.K; k += 4) {
      float a = 0.f;
      for (int s = seg.off[k] + lane; s < seg.off[k + 1]; s += 64) a += loss_rows[s];
      a = wave_sum(a);
      if (lane == 0) {
        const float bk = (float)(seg.off[k + 1] - seg.off[k]);
        const float Lk = a / bk;
        loss_per_worker[k] = Lk;
        part[k] = bk * invB * Lk;   // lambda_k L_k
      }
    }
    int badl = 0;
    for (int s = tid; s < rows; s += 256) badl |= (labels[s] < 0 || labels[s] >= C) ? 1 : 0;
    const int anybad = __syncthreads_or(badl);
    if (tid == 0) {
      float total = 0.f;
      for (int k = 0; k < seg.K; ++k) total += part[k];
      loss[0] = total;
      status[0] = anybad ? 1u : 0u;
    }
    return;
  }

  const int wk = bx / jchunks, jc = bx % jchunks;
  const int jl = tid & 15, rs = tid >> 4;
  const int j = min(jc * 16 + jl, cin - 1);   // a column past the end shadows the last one and is not stored
  const int c0 = by * 16;
  const int nc = min(16, C - c0);
  const int s_end = seg.off[wk + 1];
  const bool want_bias = jc == 0 && gb != nullptr;
  float acc[16];
#pragma unroll
  for (int c = 0; c < 16; ++c) acc[c] = 0.f;
  float bsum = 0.f;   // class jl, rows rs, rs+16, ...

  for (int base = seg.off[wk]; base < s_end; base += 256) {
    const int n = min(256, s_end - base);
    __syncthreads();   // the previous 256 rows have been consumed
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int f = tid + 256 * i, rr = f >> 4, c = f & 15;
      const bool ok = rr < n && c < nc;
      const float v = dz[(size_t)(base + (ok ? rr : 0)) * C + c0 + (ok ? c : 0)];
      dzs[rr][c] = ok ? v : 0.f;
    }
    __syncthreads();
    const T* xb = x + (size_t)base * cin + j;
    int sl = rs;
    for (; sl + 112 < n; sl += 128) {        // eight rows per trip: their loads overlap
      float av[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) av[u] = Piece<T>::get(xb + (size_t)(sl + 16 * u) * cin);
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const v4f* d = reinterpret_cast<const v4f*>(&dzs[sl + 16 * u][0]);
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const v4f dv = d[q];
#pragma unroll
          for (int e = 0; e < 4; ++e) acc[4 * q + e] += dv[e] * av[u];
        }
      }
    }
    for (; sl < n; sl += 16) {
      const float a = Piece<T>::get(xb + (size_t)sl * cin);
      const v4f* d = reinterpret_cast<const v4f*>(&dzs[sl][0]);
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const v4f dv = d[q];
#pragma unroll
        for (int e = 0; e < 4; ++e) acc[4 * q + e] += dv[e] * a;
      }
    }
    if (want_bias)
      for (int r2 = rs; r2 < n; r2 += 16) bsum += dzs[r2][jl];
  }

#pragma unroll
  for (int c = 0; c < 16; ++c) red[rs][c][jl] = acc[c];
  __syncthreads();
  {
    const int c = tid >> 4, jj = tid & 15;
    float t = 0.f;
#pragma unroll
    for (int r = 0; r < 16; ++r) t += red[r][c][jj];
    if (c < nc && jc * 16 + jj < cin)
      gw[(size_t)wk * worker_stride + (size_t)(c0 + c) * cin + jc * 16 + jj] = t;
  }
  if (want_bias) {
    // bias gradient: column sums of dz over the worker's rows, 16 row groups x 16 classes
    __syncthreads();
    float* r2 = &red[0][0][0];
    r2[rs * 16 + jl] = bsum;
    __syncthreads();
    if (tid < 16 && tid < nc) {
      float u = 0.f;
      for (int r = 0; r < 16; ++r) u += r2[r * 16 + tid];
      gb[(size_t)wk * worker_stride + c0 + tid] = u;
    }
  }
}


}  // namespace omni
