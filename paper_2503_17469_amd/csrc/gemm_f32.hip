// fp32 matrix products on the CDNA4 matrix cores (v_mfma_f32_32x32x2_f32).
//
// These are the dense contractions inside the per-worker gradient of
// Algorithm 1 (procedure Train, gradient line) for fully connected layers:
//   forward   Y  = X W^T + bias            (rows of all workers in one launch)
//   dgrad     dX = dY W                     (rows of all workers in one launch)
//   wgrad     G_k = dY_k^T X_k              (one output per worker, reduction
//                                            over that worker's rows only)
//
// One kernel template serves all three.  It computes C[i][j] = sum_kk A(i,kk) *
// B(j,kk) where each operand is either "k-contiguous" (element (r,kk) at
// base[r*ld + kk]) or "row-contiguous" (element (r,kk) at base[kk*ld + r]).
// A workgroup is 4 wavefronts in a 2x2 grid; each wavefront owns TM x TN
// accumulator blocks of 32x32.  Operand slabs of BK reduction steps are staged
// through LDS with register prefetch of the next slab (double-buffered LDS,
// one barrier per slab).
#include <hip/hip_runtime.h>

#include "common.h"
#include "kernels.h"

namespace omni {

typedef float v4f __attribute__((ext_vector_type(4)));
typedef float v16f __attribute__((ext_vector_type(16)));

namespace {

constexpr int kThreads = 256;

// Staging of one operand slab: R rows x BK reduction steps.
template <int R, int BK, bool MC>
struct Slab {
  static constexpr int kChunks = R * BK / 4;
  static constexpr int kPerThread = kChunks / kThreads;
  static_assert(kChunks % kThreads == 0 && kPerThread >= 1, "slab must divide over the workgroup");
  // k-contiguous slabs sit in LDS as [row][BK+4] (16-byte reads along kk, rows
  // land 4 banks apart); row-contiguous slabs as [kk][R+8].
  static constexpr int kStride = MC ? (R + 8) : (BK + 4);
  static constexpr int kFloats = MC ? BK * (R + 8) : R * (BK + 4);

  template <bool VEC>
  __device__ static inline void load(v4f (&reg)[kPerThread], const float* __restrict__ base, int ld,
                                     int row0, int rows, int k0, int kend, int tid) {
#pragma unroll
    for (int i = 0; i < kPerThread; ++i) {
      const int c = tid + kThreads * i;
      if (!MC) {
        const int r = c / (BK / 4), kc = (c % (BK / 4)) * 4;
        const int gr = row0 + r, gk = k0 + kc;
        const float* p = base + (size_t)gr * ld + gk;
        if (VEC && gr < rows && gk + 3 < kend) {
          reg[i] = *reinterpret_cast<const v4f*>(p);
        } else {
          v4f v;
#pragma unroll
          for (int e = 0; e < 4; ++e) v[e] = (gr < rows && gk + e < kend) ? p[e] : 0.f;
          reg[i] = v;
        }
      } else {
        const int kk = c / (R / 4), rc = (c % (R / 4)) * 4;
        const int gk = k0 + kk, gr = row0 + rc;
        const float* p = base + (size_t)gk * ld + gr;
        if (VEC && gk < kend && gr + 3 < rows) {
          reg[i] = *reinterpret_cast<const v4f*>(p);
        } else {
          v4f v;
#pragma unroll
          for (int e = 0; e < 4; ++e) v[e] = (gk < kend && gr + e < rows) ? p[e] : 0.f;
          reg[i] = v;
        }
      }
    }
  }

  __device__ static inline void store(const v4f (&reg)[kPerThread], float* lds, int tid) {
#pragma unroll
    for (int i = 0; i < kPerThread; ++i) {
      const int c = tid + kThreads * i;
      if (!MC) {
        const int r = c / (BK / 4), kc = (c % (BK / 4)) * 4;
        *reinterpret_cast<v4f*>(lds + r * kStride + kc) = reg[i];
      } else {
        const int kk = c / (R / 4), rc = (c % (R / 4)) * 4;
        *reinterpret_cast<v4f*>(lds + kk * kStride + rc) = reg[i];
      }
    }
  }

  // Operand registers for the 4 MFMA steps covering kk = ks*8 .. ks*8+7 of the
  // slab, for the 32-row block starting at `row`.  Lane l supplies row l%32 and
  // reduction index ks*8 + (l/32)*4 + q in step q; both operands use the same
  // map, which is all the instruction needs.
  __device__ static inline v4f frag(const float* lds, int row, int ks, int lane) {
    const int r = row + (lane & 31), kb = ks * 8 + (lane >> 5) * 4;
    if (!MC) {
      return *reinterpret_cast<const v4f*>(lds + r * kStride + kb);
    } else {
      v4f v;
#pragma unroll
      for (int q = 0; q < 4; ++q) v[q] = lds[(kb + q) * kStride + r];
      return v;
    }
  }
};

enum { MODE_FWD = 0, MODE_DGRAD = 1, MODE_WGRAD = 2 };

struct GemmParams {
  const float* A;
  const float* B;
  float* C;
  int M, N;  // rows of A / rows of B = rows / cols of C
  int lda, ldb, ldc;
  int kred;            // reduction length (FWD / DGRAD)
  const float* bias;   // FWD: added per output column, may be null
  const float* mask;   // DGRAD: [M][ldc]; the value passes where mask > 0, may be null
  int relu;            // FWD
  int accumulate;      // DGRAD: C += result
  size_t c_worker_stride;  // WGRAD: floats between consecutive workers' outputs
  float* bias_grad;        // WGRAD: per worker column sums of A (at + worker*c_worker_stride), may be null
};

template <int TM, int TN, int BK, bool A_MC, bool B_MC, int MODE, bool VEC>
__global__ __launch_bounds__(kThreads) void gemm_f32_kernel(GemmParams p, Segments seg) {
  constexpr int BM = 64 * TM, BN = 64 * TN;
  using SA = Slab<BM, BK, A_MC>;
  using SB = Slab<BN, BK, B_MC>;
  __shared__ __attribute__((aligned(16))) float lds[2 * (SA::kFloats + SB::kFloats)];
  constexpr int kStage = SA::kFloats + SB::kFloats;
  auto sA = [&](int stage) { return lds + stage * kStage; };
  auto sB = [&](int stage) { return lds + stage * kStage + SA::kFloats; };

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int tiles_n = (p.N + BN - 1) / BN;
  const int tile_m = blockIdx.x / tiles_n, tile_n = blockIdx.x % tiles_n;
  const int row0 = tile_m * BM, col0 = tile_n * BN;
  const int wrow = (wave >> 1) * 32 * TM, wcol = (wave & 1) * 32 * TN;

  int kbeg = 0, kend = p.kred;
  float* C = p.C;
  if (MODE == MODE_WGRAD) {
    const int w = blockIdx.y;
    kbeg = seg.off[w];
    kend = seg.off[w + 1];
    C += (size_t)w * p.c_worker_stride;
  }

  v16f acc[TM][TN];
#pragma unroll
  for (int a = 0; a < TM; ++a)
#pragma unroll
    for (int b = 0; b < TN; ++b)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.f;

  const bool want_bias_grad = (MODE == MODE_WGRAD) && p.bias_grad != nullptr && tile_n == 0;
  float bsum = 0.f;

  v4f ra[SA::kPerThread], rb[SB::kPerThread];
  const int nslab = (kend - kbeg + BK - 1) / BK;
  if (nslab > 0) {
    SA::template load<VEC>(ra, p.A, p.lda, row0, p.M, kbeg, kend, tid);
    SB::template load<VEC>(rb, p.B, p.ldb, col0, p.N, kbeg, kend, tid);
    SA::store(ra, sA(0), tid);
    SB::store(rb, sB(0), tid);
  }
  __syncthreads();

  for (int s = 0; s < nslab; ++s) {
    const int cur = s & 1;
    if (s + 1 < nslab) {
      const int k0 = kbeg + (s + 1) * BK;
      SA::template load<VEC>(ra, p.A, p.lda, row0, p.M, k0, kend, tid);
      SB::template load<VEC>(rb, p.B, p.ldb, col0, p.N, k0, kend, tid);
    }
#pragma unroll
    for (int ks = 0; ks < BK / 8; ++ks) {
      v4f fa[TM], fb[TN];
#pragma unroll
      for (int a = 0; a < TM; ++a) fa[a] = SA::frag(sA(cur), wrow + a * 32, ks, lane);
#pragma unroll
      for (int b = 0; b < TN; ++b) fb[b] = SB::frag(sB(cur), wcol + b * 32, ks, lane);
#pragma unroll
      for (int q = 0; q < 4; ++q)
#pragma unroll
        for (int a = 0; a < TM; ++a)
#pragma unroll
          for (int b = 0; b < TN; ++b)
            acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[a][q], fb[b][q], acc[a][b], 0, 0, 0);
    }
    if (want_bias_grad && tid < BM) {
      // A is the output-gradient slab [kk][row]: its column sums are the bias gradient.
#pragma unroll 8
      for (int kk = 0; kk < BK; ++kk) bsum += sA(cur)[kk * SA::kStride + tid];
    }
    if (s + 1 < nslab) {
      SA::store(ra, sA(cur ^ 1), tid);
      SB::store(rb, sB(cur ^ 1), tid);
    }
    __syncthreads();
  }

  if (want_bias_grad && tid < BM && row0 + tid < p.M)
    p.bias_grad[(size_t)blockIdx.y * p.c_worker_stride + row0 + tid] = bsum;

  // Accumulator layout of the 32x32 block: register v of lane l holds
  // row 8*(v/4) + 4*(l/32) + v%4, column l%32.
#pragma unroll
  for (int a = 0; a < TM; ++a)
#pragma unroll
    for (int b = 0; b < TN; ++b) {
      const int j = col0 + wcol + b * 32 + (lane & 31);
      if (j >= p.N) continue;
      float bj = 0.f;
      if (MODE == MODE_FWD && p.bias) bj = p.bias[j];
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int i = row0 + wrow + a * 32 + 8 * (v / 4) + 4 * (lane >> 5) + (v % 4);
        if (i >= p.M) continue;
        float val = acc[a][b][v];
        const size_t idx = (size_t)i * p.ldc + j;
        if (MODE == MODE_FWD) {
          val += bj;
          if (p.relu) val = val > 0.f ? val : 0.f;
        } else if (MODE == MODE_DGRAD) {
          if (p.mask) val = p.mask[idx] > 0.f ? val : 0.f;
          if (p.accumulate) val += C[idx];
        }
        C[idx] = val;
      }
    }
}

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

template <int TM, int TN, int BK, bool A_MC, bool B_MC, int MODE>
void launch(hipStream_t st, const GemmParams& p, const Segments& seg, int workers, bool vec) {
  constexpr int BM = 64 * TM, BN = 64 * TN;
  dim3 grid(((p.M + BM - 1) / BM) * ((p.N + BN - 1) / BN), workers, 1);
  if (vec)
    hipLaunchKernelGGL((gemm_f32_kernel<TM, TN, BK, A_MC, B_MC, MODE, true>), grid, dim3(kThreads), 0, st, p, seg);
  else
    hipLaunchKernelGGL((gemm_f32_kernel<TM, TN, BK, A_MC, B_MC, MODE, false>), grid, dim3(kThreads), 0, st, p, seg);
}

}  // namespace

void linear_fwd_f32(hipStream_t st, const float* x, const float* w, const float* bias, float* y,
                    int rows, int cin, int cout, bool relu) {
  GemmParams p{};
  p.A = x; p.B = w; p.C = y; p.M = rows; p.N = cout; p.lda = cin; p.ldb = cin; p.ldc = cout;
  p.kred = cin; p.bias = bias; p.relu = relu ? 1 : 0;
  Segments seg{};
  const bool vec = aligned16(x) && aligned16(w) && (cin % 4 == 0);
  launch<1, 1, 32, false, false, MODE_FWD>(st, p, seg, 1, vec);
}

void linear_dgrad_f32(hipStream_t st, const float* dy, const float* w, const float* mask, float* dx,
                      int rows, int cin, int cout, bool accumulate) {
  GemmParams p{};
  p.A = dy; p.B = w; p.C = dx; p.M = rows; p.N = cin; p.lda = cout; p.ldb = cin; p.ldc = cin;
  p.kred = cout; p.mask = mask; p.accumulate = accumulate ? 1 : 0;
  Segments seg{};
  const bool vec = aligned16(dy) && aligned16(w) && (cout % 4 == 0) && (cin % 4 == 0);
  launch<1, 1, 32, false, true, MODE_DGRAD>(st, p, seg, 1, vec);
}

void linear_wgrad_f32(hipStream_t st, const float* dy, const float* x, float* gw, float* gb,
                      size_t worker_stride, const Segments& seg, int cin, int cout) {
  GemmParams p{};
  p.A = dy; p.B = x; p.C = gw; p.M = cout; p.N = cin; p.lda = cout; p.ldb = cin; p.ldc = cin;
  p.c_worker_stride = worker_stride; p.bias_grad = gb;
  const bool vec = aligned16(dy) && aligned16(x) && (cout % 4 == 0) && (cin % 4 == 0);
  const long tiles128 = (long)((cout + 127) / 128) * ((cin + 127) / 128) * seg.K;
  if (tiles128 >= 512)
    launch<2, 2, 16, true, true, MODE_WGRAD>(st, p, seg, seg.K, vec);
  else
    launch<1, 1, 32, true, true, MODE_WGRAD>(st, p, seg, seg.K, vec);
}

}  // namespace omni
