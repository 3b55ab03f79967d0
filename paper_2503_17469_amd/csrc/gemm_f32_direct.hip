// fp32 forward / dgrad products for SMALL batches (v_mfma_f32_32x32x2_f32).
//
// Same contractions as the tiled kernel of gemm_f32.hip (Algorithm 1, procedure
// Train, the gradient line, fully connected layers):
//   forward   Y  = X W^T + bias, optional ReLU
//   dgrad     dX = dY W, optional ReLU mask, optional accumulate
// but for the case where the output has far fewer 32x32 blocks than the chip has
// matrix pipes (a few hundred rows): the reduction has to be split to fill the
// chip, and splitting it across workgroups costs a round trip through memory
// plus a cross-XCD release per tile.  Here the split stays INSIDE a workgroup:
//
//   * a workgroup owns a 32 x 64 output tile; its four wavefronts each own a
//     quarter of the reduction and the whole tile (two 32x32 accumulator blocks);
//   * wavefronts of one workgroup therefore share no operand data: each stages
//     its own operands (wavefront-private LDS blocks, used only to turn coalesced
//     loads into the MFMA lane layout), so the main loop has no barrier; a lane
//     supplies 16 consecutive reduction elements of its row per step, and the
//     order in which reduction elements meet the MFMAs is permuted the same way
//     for both operands (any order gives the same sum up to rounding; the order
//     is fixed, so results repeat bit for bit);
//   * the next steps' loads are in flight while the current step's 32 MFMAs run;
//   * at the end the four partial tiles are added in wavefront order through LDS
//     and the epilogue writes the tile.
#include <hip/hip_runtime.h>

#include <type_traits>

#include "common.h"
#include "head_device.h"
#include "kernels.h"

namespace omni {

typedef float v2f __attribute__((ext_vector_type(2)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef float v16f __attribute__((ext_vector_type(16)));

namespace {

constexpr int kStep = 32;   // reduction elements per step: 16 per lane half

struct DirectParams {
  const float* A;      // [M][lda], reduction index contiguous
  const float* B;      // forward: [N][ldb], reduction contiguous; dgrad: [K][ldb], output column contiguous
  float* C;            // [M][ldc]
  int M, N, K;
  int lda, ldb, ldc;
  const float* bias;   // forward, may be null
  const float* mask;   // dgrad, [M][ldc], may be null
  int relu, accumulate;
  int xcd_remap;
};

// A k-contiguous 32 x 32 operand block (32 rows, 128 bytes of each) is fetched
// with 8 lanes per row (whole 128-byte lines per quad of lanes: one lane per row
// would cost the vector cache one access per LANE, four times as many) and turned
// into the MFMA layout (lane = row) through a wavefront-private LDS block with
// 36-float rows (both the 16-byte writes and the 16-byte reads are conflict-free).
// No barrier is needed: LDS operations of one wavefront complete in order.
constexpr int kBlk = 32 * 36;
struct Staged { v4f a[4], b0[4], b1[4]; };   // b0/b1 unused by dgrad (row-contiguous B is loaded directly)

// LDS of one workgroup, in floats: the wavefronts' staging blocks, then their partial tiles.
template <bool DGRAD, int NW>
constexpr int direct_lds_floats() { return NW * (DGRAD ? 1 : 3) * kBlk + NW * 32 * 64; }

// Workgroup `tile_index` of `n_tiles` (64 * NW threads); smem holds direct_lds_floats() floats, 16-byte aligned.
template <bool DGRAD, int NW>
__device__ __forceinline__ void gemm_f32_direct_body(const DirectParams& p, int tile_index, int n_tiles, float* smem) {
  constexpr int kWave = (DGRAD ? 1 : 3) * kBlk;
  float* stage = smem;
  float (*red)[32 * 64] = reinterpret_cast<float (*)[32 * 64]>(smem + NW * kWave);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int r = lane & 31, h = lane >> 5;
  const int lrow = lane >> 3, lpiece = lane & 7;
  const int tiles_m = (p.M + 31) / 32;
  int t = tile_index;
  // Workgroups are dealt to the 8 XCDs round-robin by index; re-order them so an
  // XCD owns a contiguous run of tiles (row tiles fastest): its L2 then holds a
  // few column panels of B once.
  if (p.xcd_remap) t = (t & 7) * (n_tiles >> 3) + (t >> 3);
  const int tile_n = t / tiles_m, tile_m = t - tile_n * tiles_m;
  const int row0 = tile_m * 32, col0 = tile_n * 64;
  const int nsteps = p.K / kStep;
  const int sbeg = wave * nsteps / NW, send = (wave + 1) * nsteps / NW;

  // Rows / columns beyond the matrix are read from the last valid one: they only
  // feed outputs that are never stored.
  int aoff[4], b0off[4], b1off[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    aoff[i] = min(row0 + lrow + 8 * i, p.M - 1) * p.lda + lpiece * 4;
    b0off[i] = DGRAD ? 0 : min(col0 + lrow + 8 * i, p.N - 1) * p.ldb + lpiece * 4;
    b1off[i] = DGRAD ? 0 : min(col0 + 32 + lrow + 8 * i, p.N - 1) * p.ldb + lpiece * 4;
  }
  const float* bcol = DGRAD ? p.B + (size_t)(16 * h) * p.ldb + min(col0 + 2 * r, p.N - 2) : nullptr;
  float* wl = stage + wave * kWave;
  float* wl_w = wl + lrow * 36 + lpiece * 4;   // where this lane writes row lrow (+8i) of a block
  const float* wl_r = wl + r * 36 + h * 16;    // where this lane reads its 16 reduction elements of row r

  v16f acc0, acc1;
#pragma unroll
  for (int v = 0; v < 16; ++v) { acc0[v] = 0.f; acc1[v] = 0.f; }

  Staged G, F0, F1;
  v2f B0[16], B1[16];   // dgrad: columns (2r, 2r+1) of the lane's 16 reduction rows

  // One memory operation of the pipeline, selected by a compile-time index, so
  // that they can be dealt out between the MFMAs of a step (the wavefront issues
  // in order: a burst of 36 memory instructions between two steps would leave
  // the matrix pipe idle while the LDS and the vector cache work through it).
#define OMNI_GLOAD1(G, j, k0)                                                                      \
  {                                                                                             \
    if constexpr (DGRAD) {                                                                      \
      G.a[(j)] = *reinterpret_cast<const v4f*>(p.A + aoff[(j)] + (k0));                         \
    } else {                                                                                    \
      if ((j) < 4) G.a[(j) & 3] = *reinterpret_cast<const v4f*>(p.A + aoff[(j) & 3] + (k0));    \
      else if ((j) < 8) G.b0[(j) & 3] = *reinterpret_cast<const v4f*>(p.B + b0off[(j) & 3] + (k0)); \
      else G.b1[(j) & 3] = *reinterpret_cast<const v4f*>(p.B + b1off[(j) & 3] + (k0));          \
    }                                                                                           \
  }
#define OMNI_LWRITE1(G, j)                                                                         \
  {                                                                                             \
    if ((j) < 4) *reinterpret_cast<v4f*>(wl_w + 8 * ((j) & 3) * 36) = G.a[(j) & 3];             \
    else if ((j) < 8) *reinterpret_cast<v4f*>(wl_w + kBlk + 8 * ((j) & 3) * 36) = G.b0[(j) & 3]; \
    else *reinterpret_cast<v4f*>(wl_w + 2 * kBlk + 8 * ((j) & 3) * 36) = G.b1[(j) & 3];         \
  }
#define OMNI_LREAD1(F, j)                                                                       \
  {                                                                                             \
    if ((j) < 4) F.a[(j) & 3] = *reinterpret_cast<const v4f*>(wl_r + 4 * ((j) & 3));            \
    else if ((j) < 8) F.b0[(j) & 3] = *reinterpret_cast<const v4f*>(wl_r + kBlk + 4 * ((j) & 3)); \
    else F.b1[(j) & 3] = *reinterpret_cast<const v4f*>(wl_r + 2 * kBlk + 4 * ((j) & 3));        \
  }
#define OMNI_MMA1(F, BV, e)                                                                     \
  {                                                                                             \
    const float av = F.a[(e) >> 2][(e) & 3];                                                    \
    float bv0, bv1;                                                                             \
    if constexpr (DGRAD) { bv0 = BV[(e)][0]; bv1 = BV[(e)][1]; }                                \
    else { bv0 = F.b0[(e) >> 2][(e) & 3]; bv1 = F.b1[(e) >> 2][(e) & 3]; }                      \
    acc0 = __builtin_amdgcn_mfma_f32_32x32x2f32(av, bv0, acc0, 0, 0, 0);                        \
    acc1 = __builtin_amdgcn_mfma_f32_32x32x2f32(av, bv1, acc1, 0, 0, 0);                        \
  }
  // One step: multiply (FC, BC) while the data of the next step (in G) goes
  // through LDS into (FN), G is refilled from step `gstep`, and (dgrad) BN is
  // loaded for step `bstep`.  (A second G set, giving loads two steps to arrive,
  // measured no faster.)  Forward: 12 writes, 12 reads, 12 loads over 16
  // slots; dgrad: 4 + 4 + 4 and one B load per slot.
#define OMNI_STEP(FC, BC, FN, BN, G, gstep, bstep)                                                 \
  {                                                                                             \
    const int gk0 = min((gstep), nsteps - 1) * kStep;                                           \
    const float* bp = DGRAD ? bcol + (size_t)(min((bstep), nsteps - 1) * kStep) * p.ldb : nullptr; \
    _Pragma("unroll") for (int e = 0; e < 16; ++e) {                                            \
      OMNI_MMA1(FC, BC, e)                                                                      \
      if constexpr (DGRAD) {                                                                    \
        BN[e] = *reinterpret_cast<const v2f*>(bp + (size_t)e * p.ldb);                          \
        if (e < 4) OMNI_LWRITE1(G, e)                                                              \
        else if (e < 8) OMNI_GLOAD1(G, e - 4, gk0)                                                 \
        else if (e >= 10 && e < 14) OMNI_LREAD1(FN, e - 10)                                     \
      } else {                                                                                  \
        /* reads in the order the next step's MFMAs need them: (a, b0, b1) of elements 0-3, then 4-7, ... */ \
        if (e < 4) { OMNI_LWRITE1(G, 3 * e) OMNI_LWRITE1(G, 3 * e + 1) OMNI_LWRITE1(G, 3 * e + 2) }      \
        else if (e < 10) { OMNI_GLOAD1(G, 2 * (e - 4), gk0) OMNI_GLOAD1(G, 2 * (e - 4) + 1, gk0) }    \
        else {                                                                                  \
          OMNI_LREAD1(FN, ((2 * (e - 10)) % 3) * 4 + (2 * (e - 10)) / 3)                        \
          OMNI_LREAD1(FN, ((2 * (e - 10) + 1) % 3) * 4 + (2 * (e - 10) + 1) / 3)                \
        }                                                                                       \
      }                                                                                         \
      __builtin_amdgcn_sched_barrier(0);                                                        \
    }                                                                                           \
  }

  // Prologue: step sbeg into F0 (and B0), step sbeg+1 into G.
  {
    constexpr int kOps = DGRAD ? 4 : 12;
    const int k0 = min(sbeg, nsteps - 1) * kStep;
#pragma unroll
    for (int j = 0; j < kOps; ++j) OMNI_GLOAD1(G, j, k0)
    if constexpr (DGRAD) {
      const float* bp = bcol + (size_t)k0 * p.ldb;
#pragma unroll
      for (int e = 0; e < 16; ++e) B0[e] = *reinterpret_cast<const v2f*>(bp + (size_t)e * p.ldb);
    }
#pragma unroll
    for (int j = 0; j < kOps; ++j) OMNI_LWRITE1(G, j)
    const int k1 = min(sbeg + 1, nsteps - 1) * kStep;
#pragma unroll
    for (int j = 0; j < kOps; ++j) OMNI_GLOAD1(G, j, k1)
#pragma unroll
    for (int j = 0; j < kOps; ++j) OMNI_LREAD1(F0, j)
  }
  int s = sbeg;
  for (; s + 1 < send; s += 2) {
    OMNI_STEP(F0, B0, F1, B1, G, s + 2, s + 1)
    OMNI_STEP(F1, B1, F0, B0, G, s + 3, s + 2)
  }
  if (s < send) {
#pragma unroll
    for (int e = 0; e < 16; ++e) OMNI_MMA1(F0, B0, e)
  }
#undef OMNI_GLOAD1
#undef OMNI_LWRITE1
#undef OMNI_LREAD1
#undef OMNI_MMA1
#undef OMNI_STEP

  // ---- add the four partial tiles in wavefront order
#pragma unroll
  for (int v = 0; v < 16; ++v) {
    red[wave][v * 64 + lane] = acc0[v];
    red[wave][(16 + v) * 64 + lane] = acc1[v];
  }
  __syncthreads();
  auto total = [&](int slot) {
    const int i = slot * 64 + lane;
    float sum = red[0][i];
#pragma unroll
    for (int w = 1; w < NW; ++w) sum += red[w][i];
    return sum;
  };
  // accumulator register v of lane (r, h) is row 8*(v/4) + 4*h + v%4, column r of its block
  if (DGRAD) {
    // block 0 holds even output columns, block 1 odd ones: one 8-byte store per pair
    const int col = col0 + 2 * r;
#pragma unroll
    for (int u = 0; u < 16 / NW; ++u) {
      const int v = wave * (16 / NW) + u;
      const int row = row0 + 8 * (v >> 2) + 4 * h + (v & 3);
      v2f y = {total(v), total(16 + v)};
      if (row < p.M && col < p.N) {
        const size_t idx = (size_t)row * p.ldc + col;
        if (p.mask) {
          const v2f m = *reinterpret_cast<const v2f*>(p.mask + idx);
          y[0] = m[0] > 0.f ? y[0] : 0.f;
          y[1] = m[1] > 0.f ? y[1] : 0.f;
        }
        if (p.accumulate) y += *reinterpret_cast<const v2f*>(p.C + idx);
        *reinterpret_cast<v2f*>(p.C + idx) = y;
      }
    }
  } else {
#pragma unroll
    for (int u = 0; u < 32 / NW; ++u) {
      const int slot = wave * (32 / NW) + u;
      const int b = slot >> 4, v = slot & 15;
      const int row = row0 + 8 * (v >> 2) + 4 * h + (v & 3);
      const int col = col0 + 32 * b + r;
      float y = total(slot);
      if (row < p.M && col < p.N) {
        if (p.bias) y += p.bias[col];
        if (p.relu) y = fmaxf(y, 0.f);
        p.C[(size_t)row * p.ldc + col] = y;
      }
    }
  }
}

template <bool DGRAD, int NW>
__global__ __launch_bounds__(64 * NW) void gemm_f32_direct_kernel(DirectParams p) {
  __shared__ __attribute__((aligned(16))) float smem[direct_lds_floats<DGRAD, NW>()];
  gemm_f32_direct_body<DGRAD, NW>(p, (int)blockIdx.x, (int)gridDim.x, smem);
}

// Two independent kernels of the fp32 backward pass in one launch: the input gradient of the layer
// below the classifier, and the classifier's own parameter gradients with the losses (both need
// only the head's output gradient).  The first dgrad_tiles workgroups are the product's tiles,
// the rest the head's grid flattened row by row.  Launched one after the other, the second
// starts when the first has drained; the product has fewer tiles than the chip has room for,
// and the head's short workgroups run beside them.
__global__ __launch_bounds__(256) void dgrad_and_head_wgrad_kernel(DirectParams p, int dgrad_tiles, HeadWgradParams h,
                                                                   int head_gx, Segments seg) {
  constexpr int kFloats = direct_lds_floats<true, 4>() > kHeadWgradLdsFloats ? direct_lds_floats<true, 4>()
                                                                              : kHeadWgradLdsFloats;
  __shared__ __attribute__((aligned(16))) float smem[kFloats];
  const int b = blockIdx.x;
  if (b < dgrad_tiles) {
    gemm_f32_direct_body<true, 4>(p, b, dgrad_tiles, smem);
  } else {
    const int hb = b - dgrad_tiles;
    head_wgrad_loss_body<float>(h, seg, hb % head_gx, hb / head_gx, smem);
  }
}

inline bool aligned16(const void* q) { return (reinterpret_cast<uintptr_t>(q) & 15u) == 0; }

template <bool DGRAD>
void launch_direct(hipStream_t st, DirectParams& p) {
  const int tiles = ((p.M + 31) / 32) * ((p.N + 63) / 64);
  p.xcd_remap = tiles % 8 == 0 ? 1 : 0;
  // (eight wavefronts with an eighth of the reduction each measured slower: more streams in flight than the vector cache holds)
  hipLaunchKernelGGL((gemm_f32_direct_kernel<DGRAD, 4>), dim3(tiles), dim3(256), 0, st, p);
}

// Worth it while the output has too few 64x64 tiles to fill the chip without a
// split, and every wavefront gets at least two steps.
bool small_batch_shape(int rows, int cols, int kred) {
  const long tiles64 = (long)((rows + 63) / 64) * ((cols + 63) / 64);
  // with fewer than ~100 of this kernel's 32 x 64 tiles most compute units would sit idle while a
  // few walk a quarter of the reduction each: the split-K kernel spreads such a product better
  const long tiles32 = (long)((rows + 31) / 32) * ((cols + 63) / 64);
  if (tiles32 < 100) return false;
  return rows >= 1 && tiles64 < 256 && kred % kStep == 0 && kred / kStep >= 8 &&
         (long)rows * kred < (1L << 30) && (long)cols * kred < (1L << 30);   // 32-bit element offsets
}

}  // namespace

bool linear_fwd_f32_direct_supported(const float* x, const float* w, int rows, int cin, int cout) {
  return small_batch_shape(rows, cout, cin) && aligned16(x) && aligned16(w);
}

bool linear_fwd_f32_direct(hipStream_t st, const float* x, const float* w, const float* bias, float* y,
                           int rows, int cin, int cout, bool relu) {
  if (!linear_fwd_f32_direct_supported(x, w, rows, cin, cout)) return false;
  DirectParams p{};
  p.A = x; p.B = w; p.C = y; p.M = rows; p.N = cout; p.K = cin; p.lda = cin; p.ldb = cin; p.ldc = cout;
  p.bias = bias; p.relu = relu ? 1 : 0;
  launch_direct<false>(st, p);
  return true;
}

bool linear_dgrad_f32_direct_supported(const float* dy, const float* w, const float* mask, const float* dx, int rows,
                                       int cin, int cout) {
  return small_batch_shape(rows, cin, cout) && cin % 2 == 0 && aligned16(dy) && aligned16(w) && aligned16(dx) &&
         (!mask || aligned16(mask));
}

bool linear_dgrad_f32_direct(hipStream_t st, const float* dy, const float* w, const float* mask, float* dx,
                             int rows, int cin, int cout, bool accumulate) {
  if (!linear_dgrad_f32_direct_supported(dy, w, mask, dx, rows, cin, cout)) return false;
  DirectParams p{};
  p.A = dy; p.B = w; p.C = dx; p.M = rows; p.N = cin; p.K = cout; p.lda = cout; p.ldb = cin; p.ldc = cin;
  p.mask = mask; p.accumulate = accumulate ? 1 : 0;
  launch_direct<true>(st, p);
  return true;
}

void linear_dgrad_f32_with_head_wgrad(hipStream_t st, const float* dy, const float* w, const float* mask, float* dx,
                                      int rows, int cin, int cout, bool accumulate, const HeadWgradParams& head,
                                      const Segments& seg) {
  DirectParams p{};
  p.A = dy; p.B = w; p.C = dx; p.M = rows; p.N = cin; p.K = cout; p.lda = cout; p.ldb = cin; p.ldc = cin;
  p.mask = mask; p.accumulate = accumulate ? 1 : 0;
  const int tiles = ((p.M + 31) / 32) * ((p.N + 63) / 64);
  p.xcd_remap = tiles % 8 == 0 ? 1 : 0;
  const dim3 hg = head_wgrad_grid(head.cin, head.C, seg.K);
  hipLaunchKernelGGL(dgrad_and_head_wgrad_kernel, dim3(tiles + hg.x * hg.y), dim3(256), 0, st, p, tiles, head,
                     (int)hg.x, seg);
}

}  // namespace omni
