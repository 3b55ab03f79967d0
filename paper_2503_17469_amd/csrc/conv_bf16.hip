// bf16 convolutions and fully connected layers as implicit GEMMs on the CDNA4
// matrix cores (v_mfma_f32_32x32x16_bf16, fp32 accumulation).
//
// These are the contractions inside the per-worker gradient of Algorithm 1
// (procedure Train, gradient line) for the convolutional networks:
//   forward  Y[m][co]  = sum_{u,v,ci} X[n, h*s+u-p, w*s+v-p, ci] * W[co][u][v][ci]
//   dgrad    dX[m][ci] = sum_{u,v,co} dY[n, (h+p-u)/s, (w+p-v)/s, co] * Wt[ci][u][v][co]
//   wgrad    G_k[co][u][v][ci] = sum over worker k's rows and all positions of
//                                dY[m][co] * X[n, h*s+u-p, w*s+v-p, ci]
// with channels-last activations, m = (n, h, w).  Forward and dgrad see all
// workers' rows in one launch; wgrad writes one output per worker.
//
// Kernel A (forward / dgrad): 128 x (64*TN) output tile per workgroup, 4
// wavefronts in a 2x2 grid, each 64 x (32*TN).  The left operand is gathered
// on the fly (no im2col buffer): a 16-byte piece holds 8 consecutive channels of
// one filter tap, so it is contiguous in memory.  Slabs of 64 reduction
// elements go through LDS (double buffered, next slab prefetched to registers).
// The output width must be a multiple of 8 (16-byte output pieces).
//
// Kernel B (wgrad): the reduction runs over positions m, which is the SLOW index
// of both operands, while the matrix instruction wants 8 consecutive reduction
// elements per lane.  Each thread therefore loads 4 consecutive positions of
// one 8-channel piece and transposes them in registers into 8 four-position
// words before writing LDS.  Each worker's position range is cut into equal
// chunks, one workgroup per (tile, chunk): every workgroup does the same amount
// of work however ragged the b_k are.  Chunks of one worker park partial tiles;
// a second kernel adds them in chunk order (bit-reproducible, no atomics).
//
// 3x3 / pad-1 / stride-1 layers (most of a residual net) have kernels of their own
// that keep the input patch of a block of positions resident in LDS, so the nine
// taps cost no extra global loads, transposes or LDS stores:
//   kernel C (wgrad, 32 channels and more): 64 x 64 channels x all nine taps per
//     workgroup; column shifts of the patch are made in registers;
//   kernel D (forward and dgrad, channels a multiple of 64): 256 positions x 64
//     channels per workgroup; taps are row offsets into the patch.
// Kernel A also has a mode for the dgrad of stride-2 layers that multiplies only
// the filter taps an input position can meet (a quarter of a 3x3 filter).
// The first layer (3 input channels stored as 8) has two more: kernel F (forward, the
// filter bank in registers) and kernel G (weight gradient, (tap, channel) pairs as the
// columns of the product).
#include <hip/hip_runtime.h>

#include <algorithm>

#include "bf16.h"
#include "common.h"
#include "kernels.h"

namespace omni {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float v16f __attribute__((ext_vector_type(16)));

namespace {

constexpr int kThreads = 256;
constexpr int BM = 128;
constexpr int BK = 32;
constexpr int kMaxPieces = 1024;   // reduction pieces (8 channels of one tap) a kernel can index: K <= 8192

__device__ inline bf16x8 as_bf16x8(u32x4 v) { return __builtin_bit_cast(bf16x8, v); }

// q-th 8-channel piece of the reduction -> (filter row u, filter column v, first channel)
__device__ inline void build_tap_table(int* tab, const ConvGeom& g, int tid) {
  for (int q = tid; q * 8 < g.K && q < kMaxPieces; q += kThreads) {
    const int k = q * 8;
    const int tap = k / g.Cs, ci = k - tap * g.Cs;
    const int u = tap / g.ks, v = tap - u * g.ks;
    tab[q] = u | (v << 4) | (ci << 8);
  }
}

// Source element offset of (sample n, position h,w, tap u,v, channel ci); -1 if it falls in the padding.
__device__ inline long gather_offset(const ConvGeom& g, int n, int h, int w, int u, int v, int ci) {
  // written without early exits: the callers' loads must not sit behind divergent branches
  const int th = g.transposed ? h + g.pad - u : h * g.stride + u - g.pad;
  const int tw = g.transposed ? w + g.pad - v : w * g.stride + v - g.pad;
  const bool strided = g.transposed && g.stride > 1;
  const int hs = strided ? th / g.stride : th, ws = strided ? tw / g.stride : tw;
  bool ok = th >= 0 && tw >= 0 && hs < g.Hs && ws < g.Ws;
  ok = ok && (!strided || (hs * g.stride == th && ws * g.stride == tw));
  const long o = (((long)n * g.Hs + hs) * g.Ws + ws) * g.Cs + ci;
  return ok ? o : -1;
}

// position index m -> (n, h, w); m < 2^24 so the float quotient is exact after one correction
__device__ inline void decode_pos(const ConvGeom& g, int m, int& n, int& h, int& w) {
  const int hw = g.Hp * g.Wp;
  n = (int)((float)m * (1.0f / (float)hw));
  if (n * hw > m) --n;
  if ((n + 1) * hw <= m) ++n;
  const int r = m - n * hw;
  h = (int)((float)r * (1.0f / (float)g.Wp));
  if (h * g.Wp > r) --h;
  if ((h + 1) * g.Wp <= r) ++h;
  w = r - h * g.Wp;
}

// the same with explicit extents: m -> (n, h, w) over planes of hw positions, rows of wd
__device__ inline void decode_pos2(int hw, int wd, int m, int& n, int& h, int& w) {
  n = (int)((float)m * (1.0f / (float)hw));
  if (n * hw > m) --n;
  if ((n + 1) * hw <= m) ++n;
  const int r = m - n * hw;
  h = (int)((float)r * (1.0f / (float)wd));
  if (h * wd > r) --h;
  if ((h + 1) * wd <= r) ++h;
  w = r - h * wd;
}

// ------------------------------------------------------------------ kernel A
struct ConvParams {
  const bf16_t* src;   // gathered tensor [rows][Hs][Ws][Cs]
  const bf16_t* wgt;   // [N][K]
  bf16_t* out;         // [M][N]
  int M, N;
  ConvGeom g;
  const float* bias;   // [N] or null
  const bf16_t* mask;  // [M][N] or null: the value passes where mask > 0
  int relu, accumulate;
  const bf16_t* addend;   // [M][N] or null: added to the product before the mask (a second gradient contribution)
};

// Balance of kernel A: the vector ALU shares issue slots with the matrix pipe, and
// a first version (32-element slabs, per-piece gather arithmetic, 2-byte stores)
// spent three quarters of them away from the matrix pipe.  Hence
//   * a slab is 64 reduction elements (16 MFMAs per wavefront per barrier);
//   * FAST (channels a multiple of 64, filter <= 3x3, dgrad only for stride 1): a
//     slab lies inside one filter tap, so the tap is wavefront-uniform; each
//     thread keeps the pixel offset of its four rows and a 9-bit "tap inside the
//     image" mask, and a piece address is two adds;
//   * the output tile is staged through LDS as fp32 and leaves as 16-byte pieces
//     (bias, ReLU, mask, accumulate applied there).
//   * PHASED (dgrad of a stride-2 convolution, channels a multiple of 64): an input
//     position (h, w) only meets the filter taps whose parity matches (h+pad-u and
//     w+pad-v even), a quarter of a 3x3 filter on average.  Rows are enumerated
//     parity class by parity class (each class padded to whole tiles), so the set
//     of live taps is uniform over a workgroup and dead taps are never multiplied.
constexpr int BK2 = 64;
enum { GEN = 0, FASTM = 1, PHASED = 2 };

// (Launch bounds cap the kernels at 256 registers: the compiler then issues the MFMAs on ordinary
// registers; with accumulation registers it copied every accumulator in around the MFMAs of each slab.)
template <int TN, int MODE>
__global__ __launch_bounds__(kThreads, 2) void conv_gemm2_kernel(ConvParams p) {
  constexpr bool FAST = MODE != GEN;
  constexpr int BN = 64 * TN;
  constexpr int NB = 2 * TN;                 // right-operand pieces per thread per slab
  constexpr int kRow = BK2 + 8;              // 144-byte rows: 16-byte reads, rows 4 banks apart
  constexpr int kA = BM * kRow, kB = BN * kRow;
  constexpr int kOutPitch = BN + 4;          // fp32 staging of the output tile
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  bf16_t* lds = reinterpret_cast<bf16_t*>(smem);
  int* tab = reinterpret_cast<int*>(smem + (size_t)2 * (kA + kB) * sizeof(bf16_t));
  auto sA = [&](int s) { return lds + s * (kA + kB); };
  auto sB = [&](int s) { return lds + s * (kA + kB) + kA; };

  __shared__ int outrow[BM];   // PHASED: output row of every tile row (-1: none)
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int tiles_n = (p.N + BN - 1) / BN;
  const int tile_m = blockIdx.x / tiles_n, tile_n = blockIdx.x % tiles_n;
  const int col0 = tile_n * BN;
  const int wrow = (wave >> 1) * 64, wcol = (wave & 1) * 32 * TN;
  const ConvGeom g = p.g;
  const int kc = tid & 7, rbase = tid >> 3;   // piece within a slab; rows rbase + 32*i

  // PHASED: this tile's parity class, its rows within the class, its live taps
  int row0 = tile_m * BM;
  int cls_size = 0, ph = 0, pw = 0, H2 = 1, W2 = 1;
  int u0 = 0, v0 = 0, nv = 1, nlive = 0;   // live taps: u = u0 + 2i, v = v0 + 2j, enumerated i-major
  if (MODE == PHASED) {
    H2 = g.Hp >> 1; W2 = g.Wp >> 1;
    cls_size = g.rows * H2 * W2;
    const int tiles_per_class = (cls_size + BM - 1) / BM;
    const int cls = tile_m / tiles_per_class;
    row0 = (tile_m - cls * tiles_per_class) * BM;   // first row within the class
    ph = cls >> 1; pw = cls & 1;
    u0 = (ph + g.pad) & 1; v0 = (pw + g.pad) & 1;
    const int nu = u0 < g.ks ? (g.ks - u0 + 1) >> 1 : 0;
    nv = v0 < g.ks ? (g.ks - v0 + 1) >> 1 : 0;
    nlive = nu * nv;
    if (nv == 0) nv = 1;
  }
  // t-th live tap -> filter tap (u, v) and source displacement (du, dv) in the half-resolution grid
  auto live_tap = [&](int t, int& u, int& v, int& du, int& dv) {
    const int i = t / nv, j = t - i * nv;
    u = u0 + 2 * i; v = v0 + 2 * j;
    du = (ph + g.pad - u) >> 1;   // arithmetic shift: -2 -> -1
    dv = (pw + g.pad - v) >> 1;
  };

  if (!FAST) build_tap_table(tab, g, tid);

  // ---- per-thread invariants of the left operand
  long rowbase[4];
  uint32_t tapmask[4];
  int an[4], ah[4], aw[4];
  uint32_t arow_ok = 0;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int m = row0 + rbase + 32 * i;
    const bool ok = MODE == PHASED ? m < cls_size : m < p.M;
    arow_ok |= (ok ? 1u : 0u) << i;
    int n, h, w;
    if (MODE == PHASED) decode_pos2(H2 * W2, W2, ok ? m : 0, n, h, w);
    else decode_pos(g, ok ? m : 0, n, h, w);
    an[i] = n; ah[i] = h; aw[i] = w;
    rowbase[i] = 0;
    tapmask[i] = 0;
    if (MODE == PHASED) {
      // (h, w) are the half-resolution coordinates: the output position is (2h+ph, 2w+pw)
      rowbase[i] = (((long)n * g.Hs + h) * g.Ws + w) * g.Cs + kc * 8;
      for (int t = 0; t < nlive; ++t) {
        int u, v, du, dv;
        live_tap(t, u, v, du, dv);
        const int hs = h + du, ws = w + dv;
        const bool in = ok && hs >= 0 && hs < g.Hs && ws >= 0 && ws < g.Ws;
        tapmask[i] |= (in ? 1u : 0u) << t;
      }
    } else if (MODE == GEN) {
      // (unless the source is strided: then ah/aw stay the position and gather_offset divides)
      if (!(g.transposed && g.stride > 1)) {
        ah[i] = g.transposed ? h + g.pad : h * g.stride - g.pad;
        aw[i] = g.transposed ? w + g.pad : w * g.stride - g.pad;
        rowbase[i] = (((long)n * g.Hs + ah[i]) * g.Ws + aw[i]) * g.Cs;
      }
    } else if (FAST) {
      const int hb = g.transposed ? h + g.pad : h * g.stride - g.pad;
      const int wb = g.transposed ? w + g.pad : w * g.stride - g.pad;
      rowbase[i] = (((long)n * g.Hs + hb) * g.Ws + wb) * g.Cs + kc * 8;
      for (int u = 0; u < g.ks; ++u)
        for (int v = 0; v < g.ks; ++v) {
          const int hs = g.transposed ? hb - u : hb + u, ws = g.transposed ? wb - v : wb + v;
          const bool in = ok && hs >= 0 && hs < g.Hs && ws >= 0 && ws < g.Ws;
          tapmask[i] |= (in ? 1u : 0u) << (u * g.ks + v);
        }
    }
  }
  // ---- and of the right operand
  long brow[NB];
  uint32_t brow_ok = 0;
#pragma unroll
  for (int i = 0; i < NB; ++i) {
    const int r = col0 + rbase + 32 * i;
    brow[i] = (long)r * g.K + kc * 8;
    brow_ok |= (r < p.N ? 1u : 0u) << i;
  }
  if (MODE == PHASED && tid < BM) {
    const int m = row0 + tid;
    int n, h, w;
    decode_pos2(H2 * W2, W2, m < cls_size ? m : 0, n, h, w);
    outrow[tid] = m < cls_size ? (n * g.Hp + 2 * h + ph) * g.Wp + 2 * w + pw : -1;
  }
  if (!FAST || MODE == PHASED) __syncthreads();   // tap table / row map ready

  v16f acc[2][TN];
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int b = 0; b < TN; ++b)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.f;

  u32x4 ra[4], rb[NB];
  // Loads of absent pieces (padding, ragged tile edges) are pointed at a page of zeros: one pointer
  // select instead of a select per loaded register, and the load itself stays unconditional.
  const bf16_t* const zp = static_cast<const bf16_t*>(g.zero);
  // FAST: (tap, channel base) of the slab advance uniformly
  int tap = 0, cb = 0;
  auto load_slab = [&](int k0, int tap_, int cb_) {
    if (FAST) {
      long tapoff;
      if (MODE == PHASED) {
        int u, v, du, dv;
        live_tap(tap_, u, v, du, dv);   // tap_ counts the live taps
        tapoff = ((long)du * g.Ws + dv) * g.Cs + cb_;
      } else {
        const int u = tap_ / g.ks, v = tap_ - u * g.ks;
        tapoff = (g.transposed ? -1L : 1L) * ((long)u * g.Ws + v) * g.Cs + cb_;
      }
      const bool kin = k0 < g.K;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const bool in = kin && ((tapmask[i] >> tap_) & 1u);
        ra[i] = *reinterpret_cast<const u32x4*>(in ? p.src + (rowbase[i] + tapoff) : zp);
      }
    } else {
      const int q = (k0 >> 3) + kc;
      const bool kin = q * 8 < g.K;
      const int t = tab[kin ? q : 0];
      const int u = t & 15, v = (t >> 4) & 15, ci = t >> 8;
      if (g.transposed && g.stride > 1) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const long o = gather_offset(g, an[i], ah[i], aw[i], u, v, ci);
          const bool in = kin && ((arow_ok >> i) & 1u) && o >= 0;
          ra[i] = *reinterpret_cast<const u32x4*>(in ? p.src + o : zp);
        }
      } else {
        // ah/aw hold the source coordinates of tap (0, 0); a tap is a displacement
        const int su = g.transposed ? -u : u, sv = g.transposed ? -v : v;
        const long tapoff = ((long)su * g.Ws + sv) * g.Cs + ci;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const bool in = kin && ((arow_ok >> i) & 1u) && (unsigned)(ah[i] + su) < (unsigned)g.Hs &&
                          (unsigned)(aw[i] + sv) < (unsigned)g.Ws;
          ra[i] = *reinterpret_cast<const u32x4*>(in ? p.src + (rowbase[i] + tapoff) : zp);
        }
      }
    }
    const bool bkin = k0 + kc * 8 < g.K;
#pragma unroll
    for (int i = 0; i < NB; ++i) {
      const bool in = bkin && ((brow_ok >> i) & 1u);
      rb[i] = *reinterpret_cast<const u32x4*>(in ? p.wgt + (brow[i] + k0) : zp);
    }
  };
  auto store_a = [&](int s, int i) {
    *reinterpret_cast<u32x4*>(sA(s) + (rbase + 32 * i) * kRow + kc * 8) = ra[i];
  };
  auto store_b = [&](int s, int i) {
    *reinterpret_cast<u32x4*>(sB(s) + (rbase + 32 * i) * kRow + kc * 8) = rb[i];
  };
  auto advance = [&]() {
    cb += BK2;
    if (cb >= g.Cs) { cb = 0; ++tap; }
  };

  const int nslab = MODE == PHASED ? nlive * (g.Cs / BK2) : (g.K + BK2 - 1) / BK2;
  // first reduction element of a slab (the right operand's column); g.K = none
  auto slab_k0 = [&](int s_, int tap_, int cb_) {
    if (s_ >= nslab) return g.K;
    if (MODE != PHASED) return s_ * BK2;
    int u, v, du, dv;
    live_tap(tap_, u, v, du, dv);
    return (u * g.ks + v) * g.Cs + cb_;
  };
  load_slab(slab_k0(0, 0, 0), 0, 0);
#pragma unroll
  for (int i = 0; i < 4; ++i) store_a(0, i);
#pragma unroll
  for (int i = 0; i < NB; ++i) store_b(0, i);
  __syncthreads();
  for (int s = 0; s < nslab; ++s) {
    const int cur = s & 1;
    if (FAST) advance();
    // always issued (past the end it re-reads element 0 and is dropped): a load
    // issued on one path only would make every later wait drain the queue
    load_slab(slab_k0(s + 1, tap, cb), s + 1 < nslab ? tap : 0, cb);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int ks = 0; ks < BK2 / 16; ++ks) {
      bf16x8 fa[2], fb[TN];
      const int ko = ks * 16 + (lane >> 5) * 8;
#pragma unroll
      for (int a = 0; a < 2; ++a)
        fa[a] = as_bf16x8(*reinterpret_cast<const u32x4*>(sA(cur) + (wrow + a * 32 + (lane & 31)) * kRow + ko));
#pragma unroll
      for (int b = 0; b < TN; ++b)
        fb[b] = as_bf16x8(*reinterpret_cast<const u32x4*>(sB(cur) + (wcol + b * 32 + (lane & 31)) * kRow + ko));
#pragma unroll
      for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < TN; ++b)
          acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[a], fb[b], acc[a][b], 0, 0, 0);
    }
    if (s + 1 < nslab) {
#pragma unroll
      for (int i = 0; i < 4; ++i) store_a(cur ^ 1, i);
#pragma unroll
      for (int i = 0; i < NB; ++i) store_b(cur ^ 1, i);
    }
    __syncthreads();
  }

  // ---- output tile -> LDS (fp32) -> 16-byte pieces.  Accumulator layout of a 32x32
  // block: register v of lane l holds row 8*(v/4) + 4*(l/32) + v%4, column l%32.
  float* so = reinterpret_cast<float*>(smem);
#pragma unroll
  for (int b = 0; b < TN; ++b) {
    const int jl = wcol + b * 32 + (lane & 31);
    const int j = col0 + jl;
    const float bj = (p.bias && j < p.N) ? p.bias[j] : 0.f;
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int il = wrow + a * 32 + 8 * (v / 4) + 4 * (lane >> 5) + (v % 4);
        float val = acc[a][b][v] + bj;
        if (p.relu) val = val > 0.f ? val : 0.f;
        so[il * kOutPitch + jl] = val;
      }
  }
  __syncthreads();
  constexpr int kPiecesPerRow = BN / 8;
#pragma unroll
  for (int it = 0; it < BM * kPiecesPerRow / kThreads; ++it) {
    const int c = tid + kThreads * it;
    const int il = c / kPiecesPerRow, jl = (c % kPiecesPerRow) * 8;
    const int i = MODE == PHASED ? outrow[il] : row0 + il, j = col0 + jl;
    if (i < 0 || i >= p.M || j >= p.N) continue;   // N is a multiple of 8: a piece is wholly inside or outside
    float v[8];
    const v4f lo = *reinterpret_cast<const v4f*>(so + il * kOutPitch + jl);
    const v4f hi = *reinterpret_cast<const v4f*>(so + il * kOutPitch + jl + 4);
#pragma unroll
    for (int e = 0; e < 4; ++e) { v[e] = lo[e]; v[4 + e] = hi[e]; }
    const size_t idx = (size_t)i * p.N + j;
    if (p.addend) {
      float av[8];
      Piece<bf16_t>::load(p.addend + idx, av);
#pragma unroll
      for (int e = 0; e < 8; ++e) v[e] += av[e];
    }
    if (p.mask) {
      float mv[8];
      Piece<bf16_t>::load(p.mask + idx, mv);
#pragma unroll
      for (int e = 0; e < 8; ++e) v[e] = mv[e] > 0.f ? v[e] : 0.f;
    }
    if (p.accumulate) {
      float ov[8];
      Piece<bf16_t>::load(p.out + idx, ov);
#pragma unroll
      for (int e = 0; e < 8; ++e) v[e] += ov[e];
    }
    Piece<bf16_t>::store(p.out + idx, v);
  }
}

// ------------------------------------------------------------------ kernel D
// Forward and stride-1 dgrad of 3x3 / pad-1 convolutions with a channel count that
// is a multiple of 64 (most of a residual net).  Kernel A gathers the left operand
// once per filter tap: nine global loads, nine LDS stores of every input element.
// Here a workgroup owns 256 output positions (a strip of rows of one image, or a few
// whole small images) x 64 output channels:
//   * the input patch of those positions, halo included, is staged in LDS once per
//     64-channel slice ([patch position][64 channels], 144-byte rows);
//   * the left operand of tap (u, v) is that patch read at a row offset: no data
//     moves between taps, only the 8 KB weight slab of the tap streams through LDS
//     (double buffered, prefetched to registers);
//   * each wavefront owns 64 positions x 64 channels (2 x 2 accumulator blocks).
// For dgrad the gathered tensor is dY, the weights are the transposed copy and the
// taps are mirrored (dX(p) meets tap (u, v) at p + (1-u, 1-v)).
struct Conv3Params {
  const bf16_t* src;   // [rows][H][W][Cs]
  const bf16_t* wgt;   // [N][9][Cs]
  bf16_t* out;         // [rows*H*W][N]
  int rows, H, W, Cs, N;
  int R, nimg;         // a unit is nimg images x R rows; nimg * R * W = 256
  int units, upw;      // units in all, units per workgroup
  int flip;            // 1: dgrad (mirrored taps)
  const void* zero;    // page of zeros for absent pieces
  const float* bias;
  const bf16_t* mask;
  int relu, accumulate;
  bf16_t* pool;        // forward only, may be null: [rows*(H/2)*(W/2)][N], the 2 x 2 max pooling of `out`
  uint8_t* pool_code;  // with pool: one byte per pooled element, which of the four inputs the gradient goes to
  const bf16_t* addend;   // may be null: [rows*H*W][N] added to the product before the mask
};
constexpr int kUnitD = 256;

// Where the gradient of a 2 x 2 max pooling goes: the first of the four inputs (scan order (0,0),
// (0,1), (1,0), (1,1)) that holds the maximum, or nowhere (4) when a ReLU folded into the pooled
// tensor has zeroed the maximum.  The comparison is on the values as stored (bf16).
__device__ inline uint32_t pool_code_of(float a, float b, float c, float d, bool relu, float& m) {
  m = a;
  uint32_t k = 0;
  if (b > m) { m = b; k = 1; }
  if (c > m) { m = c; k = 2; }
  if (d > m) { m = d; k = 3; }
  return (relu && !(m > 0.f)) ? 4u : k;
}
__device__ inline float as_stored(float v) { return bf16_to_f32(f32_to_bf16(v)); }
constexpr int kRowD = 64 + 8;   // elements per LDS row (144 bytes): 16-byte reads land 4 banks apart
constexpr int kMaxPatchPieces = 13;   // 16-byte pieces of the patch per thread (up to 416 patch positions)

// A workgroup walks `upw` consecutive units of one channel tile: the next unit's patch
// and first weight slab travel to registers during the last taps of the current one,
// so only the first unit of a workgroup waits for memory before it can multiply.
// NB: 32-channel blocks of output per workgroup (2: a 64-channel tile; 1: layers with at most 32
// output channels, which would leave half of every fragment read and MFMA of the wide tile empty).
// KC: channels of the reduction staged at a time (64; 32 for layers with 32, 96, ... input channels, whose
// patch rows are then 80 bytes: sixteen lanes still cover all 64 banks).
// W8: maps 8 wide with units of whole groups of 8 map rows (see the fragment addresses below).
template <int NP, int NB, int KC, bool W8>   // NP: 16-byte patch pieces per thread
__global__ __launch_bounds__(kThreads, 2) void conv3_gemm_kernel(Conv3Params p) {
  constexpr int TN = 32 * NB;   // output channels per workgroup
  constexpr int OC = KC / 8;    // 16-byte pieces per patch position and per weight row
  constexpr int kRow = KC + 8;  // elements per LDS row
  constexpr int RP = kThreads / OC;               // weight rows staged per pass
  constexpr int WP = (TN + RP - 1) / RP;          // passes
  extern __shared__ __attribute__((aligned(16))) unsigned char smemD[];
  const int W = p.W, H = p.H, R = p.R;
  const int PW = W + 2, PR = R + 2;
  const int npatch = p.nimg * PR * PW;                    // patch positions
  bf16_t* sP = reinterpret_cast<bf16_t*>(smemD);          // [npatch][kRow]
  bf16_t* sW = sP + (size_t)npatch * kRow;                // 2 x [TN][kRow]
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int j = lane & 31, h = lane >> 5;
  const int tiles_n = (p.N + TN - 1) / TN;
  const int group = blockIdx.x / tiles_n, tile_n = blockIdx.x - group * tiles_n;
  const int col0 = tile_n * TN;
  const int K = 9 * p.Cs;
  const int ubeg = group * p.upw, uend = min(p.units, ubeg + p.upw);

  // ---- patch staging tasks: piece x = tid + 256 t -> patch position x / OC, channel octet x % OC.
  // Relative to the unit's first image and row; which pieces exist depends on the unit.
  int prel[NP];                // element offset relative to the unit (the host checks the tensor has fewer than 2^31)
  uint32_t col_ok = 0, top = 0, bottom = 0;   // piece t: inside the image's columns / in the first / last patch row
  uint64_t img4 = 0;                           // piece t: image within the unit, 4 bits each
  const int npieces = npatch * OC;
#pragma unroll
  for (int t = 0; t < NP; ++t) {
    const int x = tid + t * kThreads;
    const int pp = min(x, npieces - 1) / OC, oct = x % OC;
    const int il = pp / (PR * PW), rem = pp - il * (PR * PW);
    const int pr = rem / PW, pc = rem - pr * PW;
    prel[t] = ((il * H + pr - 1) * W + pc - 1) * p.Cs + oct * 8;
    col_ok |= (x < npieces && pc >= 1 && pc <= W ? 1u : 0u) << t;
    top |= (pr == 0 ? 1u : 0u) << t;
    bottom |= (pr == PR - 1 ? 1u : 0u) << t;
    img4 |= (uint64_t)il << (4 * t);
  }
  // ---- weight staging: rows tid/OC (+ RP per pass) of the channel tile, octet tid % OC
  const int wr = tid / OC, woct = tid % OC;
  long woff[WP];
  uint32_t wvalid = 0;
#pragma unroll
  for (int i = 0; i < WP; ++i) {
    const int r = col0 + wr + RP * i;
    const bool in = r < p.N && wr + RP * i < TN;
    woff[i] = in ? (long)r * K + woct * 8 : 0;
    wvalid |= (in ? 1u : 0u) << i;
  }
  // ---- fragment addresses: this wavefront's positions wave*64 + a*32 + j
  // On maps 8 wide, sixteen consecutive lanes of a fragment read would cover two consecutive map
  // rows, whose patch rows (10 positions apart) share two of the sixteen bank groups (measured: 40 %
  // of this kernel's LDS cycles were conflicts there, against 15 % on wider maps).  Map rows 4 apart
  // are exactly complementary, so the wavefront takes the 8 map rows of its 64 positions in the order
  // 0 4 1 5 2 6 3 7; the epilogue puts every result back in its place.
  constexpr bool w8 = W8;
  auto row_order = [](int t) { return (t >> 1) + 4 * (t & 1); };   // t: 0..7
  int pbase[2];
#pragma unroll
  for (int a = 0; a < 2; ++a) {
    int pos = wave * 64 + a * 32 + j;
    if (w8) pos = wave * 64 + row_order(a * 4 + (j >> 3)) * 8 + (j & 7);
    const int rr = pos / W, w = pos - rr * W;
    const int il = rr / R, r = rr - il * R;
    pbase[a] = ((il * PR + r) * PW + w) * kRow + h * 8;   // patch origin is (-1, -1): tap (u, v) adds u*PW + v
  }
  const int bfrag = j * kRow + h * 8;

  const bf16_t* const zp = static_cast<const bf16_t*>(p.zero);   // absent pieces are read from a page of zeros
  u32x4 rp[NP], rw[WP];
  uint32_t pvalid = 0;
  // unit -> first image, first row, images present
  auto unit_geom = [&](int unit, int& n0, int& r0, int& nvalid) {
    if (p.nimg == 1) {
      const int upi = H / R, img = unit / upi;
      n0 = img; r0 = (unit - img * upi) * R; nvalid = 1;
    } else {
      n0 = unit * p.nimg; r0 = 0; nvalid = min(p.nimg, p.rows - n0);
    }
  };
  // loads are unconditional
  auto load_patch = [&](int unit, int cs) {
    int n0, r0, nvalid;
    unit_geom(unit, n0, r0, nvalid);
    const int ubase = (n0 * H + r0) * W * p.Cs + cs * KC;
    // the first / last patch row lies outside the image when the unit touches its top / bottom edge
    pvalid = col_ok & ~(r0 == 0 ? top : 0u) & ~(r0 + R == H ? bottom : 0u);
#pragma unroll
    for (int t = 0; t < NP; ++t) {
      const int il = (int)(img4 >> (4 * t)) & 15;
      if (il >= nvalid) pvalid &= ~(1u << t);
      rp[t] = *reinterpret_cast<const u32x4*>(((pvalid >> t) & 1u) ? p.src + (ubase + prel[t]) : zp);
    }
  };
  auto store_patch = [&]() {
#pragma unroll
    for (int t = 0; t < NP; ++t) {
      const int x = tid + t * kThreads;
      if (x < npieces)
        *reinterpret_cast<u32x4*>(sP + (x / OC) * kRow + (x % OC) * 8) = rp[t];
    }
  };
  auto load_w = [&](int k0) {
#pragma unroll
    for (int i = 0; i < WP; ++i) {
      rw[i] = *reinterpret_cast<const u32x4*>(((wvalid >> i) & 1u) ? p.wgt + (woff[i] + k0) : zp);
    }
  };
  auto store_w = [&](int buf) {
#pragma unroll
    for (int i = 0; i < WP; ++i)
      if (wr + RP * i < TN)   // (a pass may cover more rows than the tile has)
        *reinterpret_cast<u32x4*>(sW + buf * TN * kRow + (wr + RP * i) * kRow + woct * 8) = rw[i];
  };

  const int nslice = p.Cs / KC;   // the patch is re-staged per KC-channel slice
  load_patch(min(ubeg, p.units - 1), 0);
  load_w(0);
  for (int unit = ubeg; unit < uend; ++unit) {
    // the unit's first patch slice and first weight slab are in registers
    store_patch();
    store_w(0);
    __syncthreads();
    v16f acc[2][NB];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
      for (int b = 0; b < NB; ++b)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.f;

    for (int cs = 0; cs < nslice; ++cs) {
      const bool last_slice = cs + 1 == nslice;
#pragma unroll
      for (int tap = 0; tap < 9; ++tap) {
        const int cur = tap & 1 ? 1 - (cs & 1) : (cs & 1);   // step cs*9 + tap, odd/even (9 taps per slice)
        const int u = tap / 3, v = tap - u * 3;
        // next step's weights (always issued): next tap, next slice, or the next unit's first slab
        if (tap < 8) load_w((tap + 1) * p.Cs + cs * KC);
        else load_w(last_slice ? 0 : (cs + 1) * KC);
        // the next slice's patch (or the next unit's first) starts its way to registers a few taps early
        if (tap == 4) load_patch(last_slice ? min(unit + 1, uend - 1) : unit, last_slice ? 0 : cs + 1);
        __builtin_amdgcn_sched_barrier(0);   // the loads stay here, a whole tap ahead of their use
        const int toff = (p.flip ? (2 - u) * PW + (2 - v) : u * PW + v) * kRow;
        const bf16_t* wb = sW + cur * TN * kRow + bfrag;
#pragma unroll
        for (int kk = 0; kk < KC / 16; ++kk) {
          bf16x8 fa[2], fb[NB];
#pragma unroll
          for (int a = 0; a < 2; ++a)
            fa[a] = as_bf16x8(*reinterpret_cast<const u32x4*>(sP + pbase[a] + toff + kk * 16));
#pragma unroll
          for (int b = 0; b < NB; ++b)
            fb[b] = as_bf16x8(*reinterpret_cast<const u32x4*>(wb + b * 32 * kRow + kk * 16));
#pragma unroll
          for (int a = 0; a < 2; ++a)
#pragma unroll
            for (int b = 0; b < NB; ++b)
              acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[a], fb[b], acc[a][b], 0, 0, 0);
        }
        __builtin_amdgcn_sched_barrier(0);   // nothing that touches the loaded registers moves above the MFMAs
        if (tap < 8 || !last_slice) store_w(cur ^ 1);
        __syncthreads();
        if (tap == 8 && !last_slice) {
          store_patch();       // every wavefront is past its last read of the old slice
          __syncthreads();
        }
      }
    }

    // ---- output tile -> LDS (fp32) -> 16-byte pieces (the staging area is free: the taps ended with a barrier)
    int n0, r0, nvalid;
    unit_geom(unit, n0, r0, nvalid);
    const long out_base = ((long)n0 * H + r0) * W;   // the unit's positions are contiguous rows of `out`
    const int npos = nvalid * R * W;                 // live positions of this unit
    constexpr int kOutPitch = TN + 4;
    float* so = reinterpret_cast<float*>(smemD);
#pragma unroll
    for (int b = 0; b < NB; ++b) {
      const int jl = b * 32 + j;
      const int c = col0 + jl;
      const float bj = (p.bias && c < p.N) ? p.bias[c] : 0.f;
#pragma unroll
      for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          // accumulator register v of lane (j, h) is row 8 (v/4) + 4 h + v%4 of the block: map row a*4 + v/4 of the wavefront's eight
          const int il = wave * 64 + (w8 ? row_order(a * 4 + v / 4) * 8 : a * 32 + 8 * (v / 4)) + 4 * h + (v % 4);
          float val = acc[a][b][v] + bj;
          if (p.relu) val = val > 0.f ? val : 0.f;
          so[il * kOutPitch + jl] = val;
        }
    }
    __syncthreads();
#pragma unroll
    for (int it = 0; it < kUnitD * (TN / 8) / kThreads; ++it) {
      const int c = tid + kThreads * it;
      const int il = c / (TN / 8), jl = (c % (TN / 8)) * 8;
      const int jg = col0 + jl;
      if (il >= npos || jg >= p.N) continue;   // N is a multiple of 8: a piece is wholly inside or outside
      float v[8];
      const v4f lo = *reinterpret_cast<const v4f*>(so + il * kOutPitch + jl);
      const v4f hi = *reinterpret_cast<const v4f*>(so + il * kOutPitch + jl + 4);
#pragma unroll
      for (int e = 0; e < 4; ++e) { v[e] = lo[e]; v[4 + e] = hi[e]; }
      const size_t idx = (size_t)(out_base + il) * p.N + jg;
      if (p.addend) {
        float av[8];
        Piece<bf16_t>::load(p.addend + idx, av);
#pragma unroll
        for (int e = 0; e < 8; ++e) v[e] += av[e];
      }
      if (p.mask) {
        float mv[8];
        Piece<bf16_t>::load(p.mask + idx, mv);
#pragma unroll
        for (int e = 0; e < 8; ++e) v[e] = mv[e] > 0.f ? v[e] : 0.f;
      }
      if (p.accumulate) {
        float ov[8];
        Piece<bf16_t>::load(p.out + idx, ov);
#pragma unroll
        for (int e = 0; e < 8; ++e) v[e] += ov[e];
      }
      Piece<bf16_t>::store(p.out + idx, v);
    }
    if (p.pool) {
      // 2 x 2 max pooling of the unit straight from the staged tile (rounding to bf16 is monotonic:
      // the maximum of the rounded values is the rounded maximum).  A unit is whole rows of whole
      // images, so its pooled positions are a contiguous run of the pooled tensor too.
      const int Wh = W >> 1, Rh = R >> 1;
      const long pool_base = ((long)n0 * (H >> 1) + (r0 >> 1)) * Wh;
      const int npool = nvalid * Rh * Wh;
#pragma unroll
      for (int it = 0; it < (kUnitD / 4) * (TN / 8) / kThreads; ++it) {
        const int c = tid + kThreads * it;
        const int q = c / (TN / 8), jl = (c % (TN / 8)) * 8;
        const int jg = col0 + jl;
        if (q >= npool || jg >= p.N) continue;
        const int img = q / (Rh * Wh), rem = q - img * (Rh * Wh);
        const int pr = rem / Wh, pw = rem - pr * Wh;
        const float* s0 = so + ((img * R + 2 * pr) * W + 2 * pw) * kOutPitch + jl;
        float m[8];
        u32x2 code = {0u, 0u};
#pragma unroll
        for (int half = 0; half < 2; ++half) {
          const v4f a = *reinterpret_cast<const v4f*>(s0 + 4 * half);
          const v4f b = *reinterpret_cast<const v4f*>(s0 + kOutPitch + 4 * half);
          const v4f cc = *reinterpret_cast<const v4f*>(s0 + W * kOutPitch + 4 * half);
          const v4f d = *reinterpret_cast<const v4f*>(s0 + (W + 1) * kOutPitch + 4 * half);
#pragma unroll
          for (int e = 0; e < 4; ++e)
            code[half] |= pool_code_of(as_stored(a[e]), as_stored(b[e]), as_stored(cc[e]), as_stored(d[e]),
                                       p.relu != 0, m[4 * half + e]) << (8 * e);
        }
        Piece<bf16_t>::store(p.pool + (size_t)(pool_base + q) * p.N + jg, m);
        *reinterpret_cast<u32x2*>(p.pool_code + (size_t)(pool_base + q) * p.N + jg) = code;
      }
    }
    __syncthreads();   // the staging area is about to be refilled
  }
}

// ------------------------------------------------------------------ kernel F
// Forward of the FIRST layer: 3x3 / pad 1 / stride 1 on 8 stored channels (3 real ones), at most
// 64 output channels.  The reduction is 9 taps x 8 channels = 72: one 16-byte piece per tap, so a
// k-step of 16 is two taps, and the lane halves of an MFMA operand simply read the patch at two
// different tap offsets.  All weights (at most 64 x 80 values) live in registers for the whole
// kernel; per unit of 256 positions the patch is 5 KB of LDS and the work is 10-20 MFMAs per
// wavefront: the kernel is bound by reading the input and writing the output once.
struct Conv1Params {
  const bf16_t* src;   // [rows][H][W][8]
  const bf16_t* wgt;   // [N][9][8]
  bf16_t* out;         // [rows*H*W][N]
  int rows, H, W, N;
  int R, nimg;         // a unit is nimg images x R rows; nimg * R * W = 256
  int units, upw;
  const float* bias;
  int relu;
  const void* zero;
  bf16_t* pool;        // may be null: [rows*(H/2)*(W/2)][N], the 2 x 2 max pooling of `out`
  uint8_t* pool_code;  // with pool: one byte per pooled element (see pool_code_of)
  int raw3;            // src is [rows][H][W][3]: a pixel is three 2-byte loads, channels 3-7 are zero
};

template <int NBLK>   // 32-channel blocks of output channels: 1 or 2
__global__ __launch_bounds__(kThreads, 2) void conv1_fwd_kernel(Conv1Params p) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smemF[];
  constexpr int NT = 32 * NBLK;
  constexpr int kPitch = NT + 8;   // bf16 elements per staged output row
  const int W = p.W, H = p.H, R = p.R;
  const int PW = W + 2, PR = R + 2;
  const int npatch = p.nimg * PR * PW;
  u32x4* sP = reinterpret_cast<u32x4*>(smemF);                                  // [npatch] pieces of 8 channels
  bf16_t* so = reinterpret_cast<bf16_t*>(smemF + (size_t)((npatch + 3) & ~3) * 16);   // [256][kPitch]
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int j = lane & 31, h = lane >> 5;
  const bf16_t* const zp = static_cast<const bf16_t*>(p.zero);

  // ---- weights: B fragment of k-step ks = taps 2ks (lanes 0-31) and 2ks+1 (lanes 32-63) of channel j
  bf16x8 wf[NBLK][5];
#pragma unroll
  for (int b = 0; b < NBLK; ++b)
#pragma unroll
    for (int ks = 0; ks < 5; ++ks) {
      const int tap = 2 * ks + h, co = 32 * b + j;
      const bool in = tap < 9 && co < p.N;
      wf[b][ks] = as_bf16x8(*reinterpret_cast<const u32x4*>(in ? p.wgt + ((size_t)co * 9 + tap) * 8 : zp));
    }
  float bj[NBLK];
#pragma unroll
  for (int b = 0; b < NBLK; ++b) bj[b] = (p.bias && 32 * b + j < p.N) ? p.bias[32 * b + j] : 0.f;

  // ---- patch staging: piece x = tid + 256 t is patch position x (two per thread)
  int prel[2], pil[2], ppr[2];
  bool pcol[2];
#pragma unroll
  for (int t = 0; t < 2; ++t) {
    const int x = min(tid + t * kThreads, npatch - 1);
    const int il = x / (PR * PW), rem = x - il * (PR * PW);
    const int pr = rem / PW, pc = rem - pr * PW;
    pil[t] = il; ppr[t] = pr;
    pcol[t] = tid + t * kThreads < npatch && pc >= 1 && pc <= W;
    prel[t] = ((il * H + pr - 1) * W + pc - 1) * (p.raw3 ? 3 : 8);
  }
  // ---- fragment addresses: positions wave*64 + a*32 + j, tap offset by lane half
  int pbase[2];
#pragma unroll
  for (int a = 0; a < 2; ++a) {
    const int pos = wave * 64 + a * 32 + j;
    const int rr = pos / W, w = pos - rr * W;
    const int il = rr / R, r = rr - il * R;
    pbase[a] = (il * PR + r) * PW + w;
  }
  int toff[5];
#pragma unroll
  for (int ks = 0; ks < 5; ++ks) {
    const int tap = min(2 * ks + h, 8);   // the tenth "tap" does not exist: its weights are zero, its data are zeroed below
    toff[ks] = (tap / 3) * PW + tap % 3;
  }

  auto unit_geom = [&](int unit, int& n0, int& r0, int& nvalid) {
    if (p.nimg == 1) {
      const int upi = H / R, img = unit / upi;
      n0 = img; r0 = (unit - img * upi) * R; nvalid = 1;
    } else {
      n0 = unit * p.nimg; r0 = 0; nvalid = min(p.nimg, p.rows - n0);
    }
  };
  u32x4 rp[2];
  auto load_patch = [&](int unit) {
    int n0, r0, nvalid;
    unit_geom(unit, n0, r0, nvalid);
    const long ubase = ((long)n0 * H + r0) * W * (p.raw3 ? 3 : 8);
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      const int row = r0 + ppr[t] - 1;
      const bool in = pcol[t] && pil[t] < nvalid && row >= 0 && row < H;
      const bf16_t* q = in ? p.src + (ubase + prel[t]) : zp;
      if (p.raw3) rp[t] = u32x4{(uint32_t)q[0] | ((uint32_t)q[1] << 16), (uint32_t)q[2], 0u, 0u};
      else rp[t] = *reinterpret_cast<const u32x4*>(q);
    }
  };

  const int ubeg = blockIdx.x * p.upw, uend = min(p.units, ubeg + p.upw);
  load_patch(min(ubeg, p.units - 1));
  for (int unit = ubeg; unit < uend; ++unit) {
#pragma unroll
    for (int t = 0; t < 2; ++t)
      if (tid + t * kThreads < npatch) sP[tid + t * kThreads] = rp[t];
    __syncthreads();
    load_patch(min(unit + 1, uend - 1));
    __builtin_amdgcn_sched_barrier(0);

    v16f acc[2][NBLK];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
      for (int b = 0; b < NBLK; ++b)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.f;
#pragma unroll
    for (int ks = 0; ks < 5; ++ks) {
#pragma unroll
      for (int a = 0; a < 2; ++a) {
        u32x4 q = sP[pbase[a] + toff[ks]];
        if (ks == 4 && h == 1) q = u32x4{0u, 0u, 0u, 0u};
        const bf16x8 fa = as_bf16x8(q);
#pragma unroll
        for (int b = 0; b < NBLK; ++b)
          acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa, wf[b][ks], acc[a][b], 0, 0, 0);
      }
    }
    // bias, ReLU, round to bf16, stage so that rows leave as 16-byte pieces
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
      for (int b = 0; b < NBLK; ++b)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int il = wave * 64 + a * 32 + 8 * (v / 4) + 4 * h + (v % 4);
          float val = acc[a][b][v] + bj[b];
          if (p.relu) val = val > 0.f ? val : 0.f;
          so[il * kPitch + 32 * b + j] = f32_to_bf16(val);
        }
    __syncthreads();
    int n0, r0, nvalid;
    unit_geom(unit, n0, r0, nvalid);
    const long out_base = ((long)n0 * H + r0) * W;
    const int npos = nvalid * R * W;
    constexpr int kPieces = NT / 8;
#pragma unroll
    for (int it = 0; it < kUnitD * kPieces / kThreads; ++it) {
      const int c = tid + kThreads * it;
      const int il = c / kPieces, jl = (c % kPieces) * 8;
      if (il < npos && jl < p.N)   // N is a multiple of 8
        *reinterpret_cast<u32x4*>(p.out + (size_t)(out_base + il) * p.N + jl) =
            *reinterpret_cast<const u32x4*>(so + il * kPitch + jl);
    }
    if (p.pool) {
      // 2 x 2 max pooling of the unit from the staged rows (a unit is whole rows of whole images: its
      // pooled positions are a contiguous run of the pooled tensor)
      const int Wh = W >> 1, Rh = R >> 1;
      const long pool_base = ((long)n0 * (H >> 1) + (r0 >> 1)) * Wh;
      const int npool = nvalid * Rh * Wh;
#pragma unroll
      for (int it = 0; it < ((kUnitD / 4) * kPieces + kThreads - 1) / kThreads; ++it) {
        const int c = tid + kThreads * it;
        const int q = c / kPieces, jl = (c % kPieces) * 8;
        if (q >= npool || jl >= p.N) continue;
        const int img = q / (Rh * Wh), rem = q - img * (Rh * Wh);
        const int pr = rem / Wh, pw = rem - pr * Wh;
        const bf16_t* s0 = so + ((img * R + 2 * pr) * W + 2 * pw) * kPitch + jl;
        float a[8], b[8], cc[8], d[8], m[8];
        Piece<bf16_t>::load(s0, a);
        Piece<bf16_t>::load(s0 + kPitch, b);
        Piece<bf16_t>::load(s0 + W * kPitch, cc);
        Piece<bf16_t>::load(s0 + (W + 1) * kPitch, d);
        u32x2 code = {0u, 0u};
#pragma unroll
        for (int e = 0; e < 8; ++e)
          code[e >> 2] |= pool_code_of(a[e], b[e], cc[e], d[e], p.relu != 0, m[e]) << (8 * (e & 3));
        Piece<bf16_t>::store(p.pool + (size_t)(pool_base + q) * p.N + jl, m);
        *reinterpret_cast<u32x2*>(p.pool_code + (size_t)(pool_base + q) * p.N + jl) = code;
      }
    }
    // (the next iteration's patch store touches sP only; `so` is rewritten after the next barrier)
  }
}

// ------------------------------------------------------------------ kernel B
struct WgradParams {
  const bf16_t* dy;    // [positions][Cout]
  const bf16_t* src;   // layer input [rows][Hs][Ws][Cs]
  float* gw;           // worker w: gw + w*worker_stride, [Cout][taps][cin_real]
  float* gb;           // worker w: gb + w*worker_stride, [Cout]; may be null
  size_t worker_stride;
  int Cout, cin_real;
  ConvGeom g;          // Hp, Wp: output positions; gather as in the forward pass
  int chunk;           // positions per workgroup (multiple of BK)
  float* partial;      // [(tile * total_chunks + chunk index)][TM*TN*16][256] (+ bias tail)
  uint32_t* counters;  // [tile * K + worker], zero between launches
};
struct ChunkTable {
  int32_t first[OMNI_MAX_WORKERS + 1];   // first chunk index of every worker; first[K] = total
};

template <int TM, int TN>
__global__ __launch_bounds__(kThreads, 2) void conv_wgrad_kernel(WgradParams p, Segments seg, ChunkTable ct) {
  constexpr int BM = 64 * TM, BN = 64 * TN;   // output tile: BM output channels x BN reduction columns
  // 80-byte rows: a fragment is one aligned 16-byte read, and the 16 consecutive rows that sixteen
  // lanes read spread evenly over the 64 read banks.  Rows 8 apart would land in the same banks, and
  // the channel pieces that the lanes of one transposing write cover are 8 rows apart: every group of
  // 16 rows is moved by another 32 bytes, so that the pieces of a write spread over the four quarters
  // of the 32 write banks while no fragment read is disturbed.  (72-byte rows with 8-byte fragment
  // reads measured 70 % of their LDS cycles as bank conflicts.)
  constexpr int kRow = BK + 8;
  auto roff = [](int row) { return row * kRow + (row >> 4) * 16; };
  constexpr int kA = BM * kRow + BM, kB = BN * kRow + BN;
  constexpr int kTileFloats = TM * TN * 16 * kThreads;
  __shared__ __attribute__((aligned(16))) bf16_t lds[2 * (kA + kB)];
  __shared__ int tab[kMaxPieces];
  auto sA = [&](int s) { return lds + s * (kA + kB); };
  auto sB = [&](int s) { return lds + s * (kA + kB) + kA; };

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const ConvGeom g = p.g;
  const int N = g.K;
  const int tiles_n = (N + BN - 1) / BN;
  const int tile = blockIdx.x;
  const int tile_m = tile / tiles_n, tile_n = tile % tiles_n;
  const int row0 = tile_m * BM, col0 = tile_n * BN;
  const int wrow = (wave >> 1) * 32 * TM, wcol = (wave & 1) * 32 * TN;

  // which worker and which chunk of its positions
  int wk = 0;
  while (wk + 1 < seg.K && (int)blockIdx.y >= ct.first[wk + 1]) ++wk;
  const int chunk_idx = blockIdx.y - ct.first[wk];
  const int nchunks = ct.first[wk + 1] - ct.first[wk];
  const int hw = g.Hp * g.Wp;
  const int mbeg = seg.off[wk] * hw + chunk_idx * p.chunk;
  const int mend = min(seg.off[wk + 1] * hw, mbeg + p.chunk);

  build_tap_table(tab, g, tid);
  __syncthreads();

  // Staging tasks.  The first BM threads: (BM/8) output-channel pieces x 8
  // groups of 4 positions of dY.  The next BN threads: (BN/8) reduction pieces x
  // 8 groups of the gathered input.
  const bool is_a = tid < BM;
  const int t2 = is_a ? tid : tid - BM;
  const int npiece = is_a ? BM / 8 : BN / 8;
  // consecutive lanes: 8 pieces (128 contiguous bytes of one position), then 2 position groups, then
  // the second 8 pieces if there are 16, then the remaining position groups
  const int piece = npiece == 8 ? (t2 & 7) : ((t2 & 7) | ((t2 >> 1) & 8));
  const int mg = npiece == 8 ? (t2 >> 3) : (((t2 >> 3) & 1) | ((t2 >> 4) & 6));
  const bool task = tid < BM + BN;   // (mg < 8 follows)
  int bu = 0, bv = 0, bci = 0;
  bool piece_ok;
  if (is_a) {
    piece_ok = row0 + piece * 8 < p.Cout;
  } else {
    const int q = (col0 >> 3) + piece;
    piece_ok = q * 8 < g.K;
    const int t = tab[piece_ok ? q : 0];
    bu = t & 15; bv = (t >> 4) & 15; bci = t >> 8;
  }

  v16f acc[TM][TN];
#pragma unroll
  for (int a = 0; a < TM; ++a)
#pragma unroll
    for (int b = 0; b < TN; ++b)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.f;
  const bool want_bias = p.gb != nullptr && tile_n == 0;
  float bsum = 0.f;

  u32x4 r[4];
  // Loads never branch and their base pointer is chosen once (a guarded load, or a pointer
  // re-selected per load, makes the compiler wait for every load before issuing the next):
  // an absent piece is read from a page of zeros.
  const bf16_t* const base = is_a ? p.dy : p.src;
  const bf16_t* const zp = static_cast<const bf16_t*>(g.zero);
  auto load_slab = [&](int m0) {
    const int mfirst = m0 + mg * 4;
    int n = 0, h = 0, w = 0;
    decode_pos(g, min(mfirst, max(mend - 1, 0)), n, h, w);
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int m = mfirst + q;
      const long oa = (long)m * p.Cout + row0 + piece * 8;
      const long ob = gather_offset(g, n, h, w, bu, bv, bci);
      const long o = is_a ? oa : ob;
      const bool in = task && piece_ok && m < mend && o >= 0;
      if (++w == g.Wp) { w = 0; if (++h == g.Hp) { h = 0; ++n; } }
      r[q] = *reinterpret_cast<const u32x4*>(in ? base + o : zp);
    }
  };
  auto store_slab = [&](int s) {
    if (!task) return;
    const u32x4* c = r;
    bf16_t* dst = (is_a ? sA(s) : sB(s)) + roff(piece * 8) + mg * 4;
    // word d of piece q holds channels 2d (low half) and 2d+1 (high half) of position q
#pragma unroll
    for (int d = 0; d < 4; ++d) {
      u32x2 lo, hi;
      lo[0] = (c[0][d] & 0xFFFFu) | (c[1][d] << 16);
      lo[1] = (c[2][d] & 0xFFFFu) | (c[3][d] << 16);
      hi[0] = (c[0][d] >> 16) | (c[1][d] & 0xFFFF0000u);
      hi[1] = (c[2][d] >> 16) | (c[3][d] & 0xFFFF0000u);
      *reinterpret_cast<u32x2*>(dst + (2 * d) * kRow) = lo;
      *reinterpret_cast<u32x2*>(dst + (2 * d + 1) * kRow) = hi;
    }
  };
  auto frag = [&](const bf16_t* base, int row, int ko) {
    return as_bf16x8(*reinterpret_cast<const u32x4*>(base + roff(row) + ko));
  };

  const int nslab = (mend - mbeg + BK - 1) / BK;
  load_slab(mbeg);
  store_slab(0);
  __syncthreads();
  for (int s = 0; s < nslab; ++s) {
    const int cur = s & 1;
    load_slab(s + 1 < nslab ? mbeg + (s + 1) * BK : mend);
#pragma unroll
    for (int ks = 0; ks < BK / 16; ++ks) {
      bf16x8 fa[TM], fb[TN];
      const int ko = ks * 16 + (lane >> 5) * 8;
#pragma unroll
      for (int a = 0; a < TM; ++a) fa[a] = frag(sA(cur), wrow + a * 32 + (lane & 31), ko);
#pragma unroll
      for (int b = 0; b < TN; ++b) fb[b] = frag(sB(cur), wcol + b * 32 + (lane & 31), ko);
#pragma unroll
      for (int a = 0; a < TM; ++a)
#pragma unroll
        for (int b = 0; b < TN; ++b)
          acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[a], fb[b], acc[a][b], 0, 0, 0);
    }
    if (want_bias && tid < BM) {
      // rows of the dY slab are output channels: their sums over positions are the bias gradient
      const u32x4* rowp = reinterpret_cast<const u32x4*>(sA(cur) + roff(tid));
#pragma unroll
      for (int d = 0; d < BK / 8; ++d) {
        const u32x4 q = rowp[d];
#pragma unroll
        for (int e = 0; e < 4; ++e) bsum += bf16_lo(q[e]) + bf16_hi(q[e]);
      }
    }
    if (s + 1 < nslab) {
      store_slab(cur ^ 1);
      __syncthreads();
    }
  }

  // ---- a worker cut into several chunks: park the partial tile, a second kernel adds them up
  if (nchunks > 1) {
    float* mine = p.partial + ((size_t)tile * ct.first[seg.K] + blockIdx.y) * (kTileFloats + BM);
#pragma unroll
    for (int a = 0; a < TM; ++a)
#pragma unroll
      for (int b = 0; b < TN; ++b)
#pragma unroll
        for (int v = 0; v < 16; ++v) mine[((a * TN + b) * 16 + v) * kThreads + tid] = acc[a][b][v];
    if (tid < BM) mine[kTileFloats + tid] = bsum;
    return;
  }

  const int taps = g.ks * g.ks;
  float* gw = p.gw + (size_t)wk * p.worker_stride;
#pragma unroll
  for (int b = 0; b < TN; ++b) {
    const int kcol = col0 + wcol + b * 32 + (lane & 31);
    if (kcol >= g.K) continue;
    const int tap = kcol / g.Cs, ci = kcol - tap * g.Cs;
    if (ci >= p.cin_real) continue;   // padding channels of the first layer
    const int colreal = tap * p.cin_real + ci;
#pragma unroll
    for (int a = 0; a < TM; ++a)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int co = row0 + wrow + a * 32 + 8 * (v / 4) + 4 * (lane >> 5) + (v % 4);
        if (co < p.Cout) gw[(size_t)co * (taps * p.cin_real) + colreal] = acc[a][b][v];
      }
  }
  if (want_bias && tid < BM && row0 + tid < p.Cout) p.gb[(size_t)wk * p.worker_stride + row0 + tid] = bsum;
}

// Second stage of a chunked wgrad: grid (tiles, workers, TM*TN*16 register slots).
// Each thread owns the same (output channel, reduction column) as the thread of
// the first stage that held this slot, and adds the worker's chunks in chunk
// order (fixed order: results repeat bit for bit).
template <int TM, int TN>
__global__ __launch_bounds__(kThreads) void conv_wgrad_reduce_kernel(WgradParams p, Segments seg, ChunkTable ct) {
  constexpr int BM = 64 * TM, BN = 64 * TN;
  constexpr int kTileFloats = TM * TN * 16 * kThreads;
  const int tile = blockIdx.x, wk = blockIdx.y, slot = blockIdx.z;
  const int nchunks = ct.first[wk + 1] - ct.first[wk];
  if (nchunks <= 1) return;   // written directly by the first stage
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const ConvGeom g = p.g;
  const int tiles_n = (g.K + BN - 1) / BN;
  const int tile_m = tile / tiles_n, tile_n = tile % tiles_n;
  const int row0 = tile_m * BM, col0 = tile_n * BN;
  const int wrow = (wave >> 1) * 32 * TM, wcol = (wave & 1) * 32 * TN;
  const float* all = p.partial + ((size_t)tile * ct.first[seg.K] + ct.first[wk]) * (kTileFloats + BM);
  const size_t stride = kTileFloats + BM;

  // Each wavefront adds a quarter of the chunks (16-byte loads, 8 in flight), then
  // the four quarter sums are added in wavefront order.
  __shared__ float red[4][kThreads];
  {
    const float* src = all + (size_t)slot * kThreads + lane * 4;
    const int cbeg = wave * nchunks / 4, cend = (wave + 1) * nchunks / 4;
    v4f acc4 = {0.f, 0.f, 0.f, 0.f};
    int c = cbeg;
    for (; c + 8 <= cend; c += 8) {
      v4f t[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) t[u] = *reinterpret_cast<const v4f*>(src + (size_t)(c + u) * stride);
#pragma unroll
      for (int u = 0; u < 8; ++u) acc4 += t[u];
    }
    for (; c < cend; ++c) acc4 += *reinterpret_cast<const v4f*>(src + (size_t)c * stride);
#pragma unroll
    for (int e = 0; e < 4; ++e) red[wave][lane * 4 + e] = acc4[e];
  }
  __syncthreads();
  const float s0 = (red[0][tid] + red[1][tid]) + (red[2][tid] + red[3][tid]);
  const int a = slot / (TN * 16), b = (slot / 16) % TN, v = slot % 16;
  const int kcol = col0 + wcol + b * 32 + (lane & 31);
  const int co = row0 + wrow + a * 32 + 8 * (v / 4) + 4 * (lane >> 5) + (v % 4);
  const int taps = g.ks * g.ks;
  if (kcol < g.K && co < p.Cout) {
    const int tap = kcol / g.Cs, ci = kcol - tap * g.Cs;
    if (ci < p.cin_real)
      p.gw[(size_t)wk * p.worker_stride + (size_t)co * (taps * p.cin_real) + tap * p.cin_real + ci] = s0;
  }
  if (slot == 0 && p.gb != nullptr && tile_n == 0 && tid < BM && row0 + tid < p.Cout) {
    float bs = 0.f;                      // eight loads in flight, additions in chunk order
    const float* bsrc = all + kTileFloats + tid;
    int c = 0;
    for (; c + 8 <= nchunks; c += 8) {
      float t[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) t[u] = bsrc[(size_t)(c + u) * stride];
#pragma unroll
      for (int u = 0; u < 8; ++u) bs += t[u];
    }
    for (; c < nchunks; ++c) bs += bsrc[(size_t)c * stride];
    p.gb[(size_t)wk * p.worker_stride + row0 + tid] = bs;
  }
}


// ------------------------------------------------------------------ kernel C
// Weight gradient of 3x3, stride-1, pad-1 convolutions (most of a residual net).
// Kernel B treats the nine filter taps as nine independent column blocks: the
// input is fetched and transposed nine times and dY once per column tile, and at
// 64 channels that memory traffic, not the matrix pipe, sets the pace.  Here a
// workgroup owns 64 output channels x 64 input channels x ALL nine taps and walks
// through units of 128 output positions (a strip of rows of one image, or a few
// whole small images):
//   * dY^T [64 co][128 positions] and the input patch X^T [64 ci][rows+2][W+16]
//     (with its zero halo) are transposed into LDS ONCE per unit;
//   * the B operand of tap (u, v) is the patch shifted by (u-1) rows and (v-1)
//     columns: the row shift is an address offset; the column shift of one
//     element is made in registers from the aligned 16-byte read and its two
//     neighbour words (v_alignbit), so one LDS read serves three taps;
//   * each wavefront holds 32 co x 32 ci x 9 taps = nine accumulator blocks.
// Units never straddle workers; a worker's units are cut into chunks, one
// workgroup per (tile, chunk), partial tiles are added by a second kernel in
// chunk order (bit-reproducible, no atomics).
struct Wgrad3Params {
  const bf16_t* dy;    // [rows*H*W][Cout]
  const bf16_t* src;   // [rows][H][W][Cin]
  float* gw;           // worker w: gw + w*worker_stride, [Cout][9][Cin]
  float* gb;           // may be null
  size_t worker_stride;
  int Cout, Cin, H, W;  // Cin: stored channels (a multiple of 8)
  int cin_real;        // channels of the gradient tensor (the first layer stores 3 channels padded to 8)
  int R, nimg;         // a unit is nimg images x R rows; nimg * R * W = 128
  int Wp, prows;       // patch row length W + 16 (data starts at column 8), patch rows nimg * (R + 2)
  int SX;              // bytes between channels of X^T
  int upc;             // units per chunk
  float* partial;      // [(tile * total_chunks + chunk)][144][256] (+ 64 bias sums)
  const void* zero;    // page of zeros for absent pieces
};
constexpr int kUnit = 128;
constexpr int kSA = 2 * kUnit + 16;                 // bytes between channels of dY^T
// Channel rows 8 apart are a multiple of 32 words apart: the eight channel octets that sixteen lanes
// of one transposing write cover would all land in the same banks (measured: 87 % of the LDS cycles
// of the staging writes were bank conflicts).  Every group of eight rows is therefore moved by
// another 16 bytes, which makes the writes conflict-free.  The price is on the other side: the 16
// consecutive rows that sixteen lanes of a 16-byte fragment read cover now overlap in one bank group
// (measured: fragment reads conflict-free before, 63 % conflict cycles after), still far fewer
// conflict cycles in all (5.6e7 -> 1.5e7 per launch on 64-channel 32 x 32 maps together with the
// lane swaps below).  A skew per sixteen rows leaves the reads alone but brings the write conflicts
// back (2.4e7 in all).
constexpr int kSkewPad = 128;   // room for the skew of 64 rows (7 x 16 bytes), kept a multiple of 128
__device__ inline int row_skew(int row) { return (row >> 3) * 16; }
constexpr int kTile3Floats = 9 * 16 * kThreads;    // one partial tile
constexpr int kTile3Stride = kTile3Floats + 64;

// four positions x eight channels (c[q] = the 16-byte piece of position q) -> eight
// channel rows of four positions each
// the same for a destination that is only 4-byte aligned
__device__ inline void transpose_store32(const u32x4 c[4], unsigned char* dst, int row_bytes) {
#pragma unroll
  for (int d = 0; d < 4; ++d) {
    uint32_t* lo = reinterpret_cast<uint32_t*>(dst + (2 * d) * row_bytes);
    uint32_t* hi = reinterpret_cast<uint32_t*>(dst + (2 * d + 1) * row_bytes);
    lo[0] = (c[0][d] & 0xFFFFu) | (c[1][d] << 16);
    lo[1] = (c[2][d] & 0xFFFFu) | (c[3][d] << 16);
    hi[0] = (c[0][d] >> 16) | (c[1][d] & 0xFFFF0000u);
    hi[1] = (c[2][d] >> 16) | (c[3][d] & 0xFFFF0000u);
  }
}

__device__ inline void transpose_store(const u32x4 c[4], unsigned char* dst, int row_bytes) {
#pragma unroll
  for (int d = 0; d < 4; ++d) {
    u32x2 lo, hi;
    lo[0] = (c[0][d] & 0xFFFFu) | (c[1][d] << 16);
    lo[1] = (c[2][d] & 0xFFFFu) | (c[3][d] << 16);
    hi[0] = (c[0][d] >> 16) | (c[1][d] & 0xFFFF0000u);
    hi[1] = (c[2][d] >> 16) | (c[3][d] & 0xFFFF0000u);
    *reinterpret_cast<u32x2*>(dst + (2 * d) * row_bytes) = lo;
    *reinterpret_cast<u32x2*>(dst + (2 * d + 1) * row_bytes) = hi;
  }
}

// WM = 4: maps four columns wide (a patch row is 8 elements = one 16-byte read, data in columns 2-5;
// a group of 8 reduction positions is two image rows).
// WM = 8, 16, 32: the map width is known.  The two halves of a wavefront read neighbouring windows
// of 8 columns, so the one element to the left and to the right of a window is either the zero halo
// or sits in a register of the partner lane in the other half: it comes over with a swap of the
// wavefront's halves instead of two more LDS reads per tap row (4-byte reads 16-byte-aligned rows
// apart use a quarter of the banks: measured, they were all of this kernel's read conflicts and
// more LDS time than the fragments themselves).  WM = 0: any other width, with those reads.
__device__ inline uint32_t from_partner(uint32_t send, bool upper) {
  // lanes 32-63 receive what lanes 0-31 sent, and the other way round
  const u32x2 sw = __builtin_amdgcn_permlane32_swap(send, send, false, false);
  return upper ? sw[0] : sw[1];
}

// The three taps of one filter row: q holds the window's 8 columns (two per word), pl the word
// before it (its upper half is the column to the left), pn the word after (lower half: to the right).
__device__ inline void wgrad3_taps(v16f (&acc)[9], int du, const bf16x8 fa, const u32x4 q, uint32_t pl, uint32_t pn) {
  const uint32_t m01 = __builtin_amdgcn_alignbit(q[1], q[0], 16);
  const uint32_t m12 = __builtin_amdgcn_alignbit(q[2], q[1], 16);
  const uint32_t m23 = __builtin_amdgcn_alignbit(q[3], q[2], 16);
  const u32x4 left = {__builtin_amdgcn_alignbit(q[0], pl, 16), m01, m12, m23};
  const u32x4 right = {m01, m12, m23, __builtin_amdgcn_alignbit(pn, q[3], 16)};
  acc[du * 3 + 0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa, as_bf16x8(left), acc[du * 3 + 0], 0, 0, 0);
  acc[du * 3 + 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa, as_bf16x8(q), acc[du * 3 + 1], 0, 0, 0);
  acc[du * 3 + 2] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa, as_bf16x8(right), acc[du * 3 + 2], 0, 0, 0);
}

template <int WM>
__global__ __launch_bounds__(kThreads, 2) void conv3_wgrad_kernel(Wgrad3Params p, Segments seg, ChunkTable ct) {
  constexpr bool W4 = WM == 4;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem3[];
  unsigned char* sA = smem3;                 // dY^T: 64 rows of kSA bytes
  unsigned char* sX = smem3 + 64 * kSA + kSkewPad;   // X^T: 64 rows of p.SX bytes (both arrays: + the skew)
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int j = lane & 31, h = lane >> 5;
  const int tiles_ci = (p.Cin + 63) / 64;
  const int tile = blockIdx.x;
  const int co0 = (tile / tiles_ci) * 64, ci0 = (tile % tiles_ci) * 64;
  const int wco = (wave >> 1) * 32, wci = (wave & 1) * 32;
  const int H = p.H, W = p.W, R = p.R;

  int wk = 0;
  while (wk + 1 < seg.K && (int)blockIdx.y >= ct.first[wk + 1]) ++wk;
  const int chunk_idx = blockIdx.y - ct.first[wk];
  const int nchunks = ct.first[wk + 1] - ct.first[wk];
  const int bk = seg.off[wk + 1] - seg.off[wk];
  const int upi = H / R;   // units per image when a unit is part of one image
  const int units_k = p.nimg == 1 ? bk * upi : (bk + p.nimg - 1) / p.nimg;
  const int ubeg = chunk_idx * p.upc, uend = min(units_k, ubeg + p.upc);

  // The halo columns of the patch are never written again: they stay zero.  So do the rows of
  // channels past the end of the tensor (their staging tasks are skipped altogether).
  for (int i = tid * 16; i < 64 * kSA + 64 * p.SX + 2 * kSkewPad; i += kThreads * 16)
    *reinterpret_cast<u32x4*>(smem3 + i) = u32x4{0u, 0u, 0u, 0u};

  // ---- staging tasks (the same for every unit, relative to the unit's first image and row)
  // dY: 8 channel octets x 32 groups of 4 positions
  const int a_oct = tid & 7;
  int a_rel, a_il;
  {
    const int p0 = 4 * (tid >> 3), rr = p0 / W, w = p0 - rr * W;
    a_il = rr / R;
    a_rel = (a_il * H + (rr - a_il * R)) * W + w;
  }
  const bool a_chan_ok = co0 + 8 * a_oct < p.Cout;
  unsigned char* a_dst = sA + (8 * a_oct) * kSA + row_skew(8 * a_oct) + 8 * (tid >> 3);
  // X: 8 octets x (W/4 groups of 4 columns) x patch rows, two tasks per thread
  const int wq = W >> 2;
  const int ntasks = p.prows * wq * 8;
  int x_rel[2], x_il[2], x_rr[2], x_dst[2];
  bool x_task[2];
#pragma unroll
  for (int t = 0; t < 2; ++t) {
    const int x = tid + t * kThreads;
    x_task[t] = x < ntasks;
    const int xx = x_task[t] ? x : 0;
    const int oct = xx & 7, g = xx >> 3;
    const int pr = g / wq, wg = g - pr * wq;
    x_il[t] = pr / (R + 2);
    x_rr[t] = pr - x_il[t] * (R + 2);                       // input row = first row + x_rr - 1
    x_rel[t] = ((x_il[t] * H + x_rr[t] - 1) * W + 4 * wg) * p.Cin + 8 * oct;
    x_dst[t] = (8 * oct) * p.SX + row_skew(8 * oct) + (pr * p.Wp + 4 * wg + (W4 ? 2 : 8)) * 2;
    x_task[t] = x_task[t] && ci0 + 8 * oct < p.Cin;   // false: no such piece, or a channel octet past the end
  }

  // ---- fragment addresses: k-step ks covers positions 16 ks .. 16 ks + 15, this lane the 8 at 16 ks + 8 h
  int offB[kUnit / 16];
#pragma unroll
  for (int ks = 0; ks < kUnit / 16; ++ks) {
    const int pos = (2 * ks + h) * 8, rr = pos / W, w0 = pos - rr * W;
    const int il = rr / R;
    offB[ks] = ((il * (R + 2) + (rr - il * R)) * p.Wp + (W4 ? 0 : w0 + 8)) * 2;
  }
  const unsigned char* a_frag = sA + (wco + j) * kSA + row_skew(wco + j) + h * 16;
  const unsigned char* x_frag = sX + (wci + j) * p.SX + row_skew(wci + j);
  const int row_shift = p.Wp * 2;

  v16f acc[9];
#pragma unroll
  for (int t = 0; t < 9; ++t)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[t][v] = 0.f;
  const bool want_bias = p.gb != nullptr && ci0 == 0;
  float bsum = 0.f;

  u32x4 ra[4], rx[2][4];
  const bf16_t* const zp = static_cast<const bf16_t*>(p.zero);
  auto load_unit = [&](int u) {
    int n0, r0, nvalid;
    if (p.nimg == 1) {
      const int img = u / upi;
      n0 = seg.off[wk] + img; r0 = (u - img * upi) * R; nvalid = 1;
    } else {
      n0 = seg.off[wk] + u * p.nimg; r0 = 0; nvalid = min(p.nimg, seg.off[wk + 1] - n0);
    }
    const long base_pos = ((long)n0 * H + r0) * W;
    // Loads never branch (a guarded load makes the compiler wait for each group before the
    // next): an absent piece is read from a page of zeros.
    {
      const bool in = a_chan_ok && a_il < nvalid;
      const bf16_t* src = in ? p.dy + ((base_pos + a_rel) * p.Cout + co0 + 8 * a_oct) : zp;
      const int st = in ? p.Cout : 0;
#pragma unroll
      for (int q = 0; q < 4; ++q) ra[q] = *reinterpret_cast<const u32x4*>(src + q * st);
    }
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      const int row = r0 + x_rr[t] - 1;
      const bool in = x_task[t] && x_il[t] < nvalid && row >= 0 && row < H;
      const bf16_t* src = in ? p.src + (base_pos * p.Cin + x_rel[t] + ci0) : zp;
      const int st = in ? p.Cin : 0;
#pragma unroll
      for (int q = 0; q < 4; ++q) rx[t][q] = *reinterpret_cast<const u32x4*>(src + q * st);
    }
  };
  auto store_unit = [&]() {
    if (a_chan_ok) transpose_store(ra, a_dst, kSA);
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      if (!x_task[t]) continue;   // no such patch piece, or channels that stay zero
      if (W4) transpose_store32(rx[t], sX + x_dst[t], p.SX);
      else transpose_store(rx[t], sX + x_dst[t], p.SX);
    }
  };

  load_unit(min(ubeg, max(uend - 1, 0)));
  for (int u = ubeg; u < uend; ++u) {
    __syncthreads();   // the previous unit's fragments have been read (and, first time, the zero fill is done)
    store_unit();
    __syncthreads();
    load_unit(min(u + 1, uend - 1));   // always issued: in flight during the MFMAs below
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int ks = 0; ks < kUnit / 16; ++ks) {
      const bf16x8 fa = as_bf16x8(*reinterpret_cast<const u32x4*>(a_frag + ks * 32));
      if constexpr (W4) {
        // patch rows r .. r+3 of this lane's image (16 bytes each) serve all nine taps
        u32x4 row[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) row[i] = *reinterpret_cast<const u32x4*>(x_frag + offB[ks] + i * row_shift);
        uint32_t lf[4][2], rt[4][2];   // columns 1-4 and 3-6 of every row
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const uint32_t m21 = __builtin_amdgcn_alignbit(row[i][2], row[i][1], 16);
          lf[i][0] = __builtin_amdgcn_alignbit(row[i][1], row[i][0], 16); lf[i][1] = m21;
          rt[i][0] = m21; rt[i][1] = __builtin_amdgcn_alignbit(row[i][3], row[i][2], 16);
        }
#pragma unroll
        for (int du = 0; du < 3; ++du) {
          const u32x4 left = {lf[du][0], lf[du][1], lf[du + 1][0], lf[du + 1][1]};
          const u32x4 mid = {row[du][1], row[du][2], row[du + 1][1], row[du + 1][2]};
          const u32x4 right = {rt[du][0], rt[du][1], rt[du + 1][0], rt[du + 1][1]};
          acc[du * 3 + 0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa, as_bf16x8(left), acc[du * 3 + 0], 0, 0, 0);
          acc[du * 3 + 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa, as_bf16x8(mid), acc[du * 3 + 1], 0, 0, 0);
          acc[du * 3 + 2] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa, as_bf16x8(right), acc[du * 3 + 2], 0, 0, 0);
        }
        // (keeps the next steps' patch rows from being read ahead of their turn: with them all in flight the
        // 256 registers overflowed into scratch memory)
        __builtin_amdgcn_sched_barrier(0);
      } else if constexpr (WM == 32) {
        // a map row is two reduction steps: windows A | B (this step) and C | D (the next), A and C
        // in the lower half of the wavefront, B and D in the upper
        if (ks & 1) continue;   // done together with the step before
        const bf16x8 fa2 = as_bf16x8(*reinterpret_cast<const u32x4*>(a_frag + (ks + 1) * 32));
        const bool up = h != 0;
#pragma unroll
        for (int du = 0; du < 3; ++du) {
          const u32x4 q = *reinterpret_cast<const u32x4*>(x_frag + offB[ks] + du * row_shift);
          const u32x4 q2 = *reinterpret_cast<const u32x4*>(x_frag + offB[ks + 1] + du * row_shift);
          const uint32_t r1 = from_partner(up ? q[0] : q[3], up);    // A gets B's first, B gets A's last
          const uint32_t r2 = from_partner(up ? q[3] : q2[0], up);   // C gets B's last, B gets C's first
          const uint32_t r3 = from_partner(up ? q2[0] : q2[3], up);  // C gets D's first, D gets C's last
          const uint32_t pl = up ? r1 : 0u, pn = up ? r2 : r1;
          const uint32_t pl2 = up ? r3 : r2, pn2 = up ? 0u : r3;
          wgrad3_taps(acc, du, fa, q, pl, pn);
          wgrad3_taps(acc, du, fa2, q2, pl2, pn2);
        }
      } else {
#pragma unroll
      for (int du = 0; du < 3; ++du) {
        const unsigned char* xb = x_frag + offB[ks] + du * row_shift;
        const u32x4 q = *reinterpret_cast<const u32x4*>(xb);
        uint32_t pl, pn;
        if constexpr (WM == 8) {
          pl = 0u; pn = 0u;                      // a window is a whole map row: halo on both sides
        } else if constexpr (WM == 16) {
          const bool up = h != 0;                // a map row is the two windows of this step
          const uint32_t r = from_partner(up ? q[0] : q[3], up);
          pl = up ? r : 0u; pn = up ? 0u : r;
        } else {
          pl = *reinterpret_cast<const uint32_t*>(xb - 4);
          pn = *reinterpret_cast<const uint32_t*>(xb + 16);
        }
        wgrad3_taps(acc, du, fa, q, pl, pn);
      }
      }
    }
    if (want_bias) {
      // rows of dY^T are output channels: their sums over positions are the bias gradient; every
      // wavefront adds a quarter of the unit's positions (one wavefront walking all 128 was a serial
      // chain of a thousand cycles per unit that the other three waited for at the next barrier)
      const uint32_t* rowp = reinterpret_cast<const uint32_t*>(sA + lane * kSA + row_skew(lane)) + wave * (kUnit / 8);
#pragma unroll
      for (int d = 0; d < kUnit / 8; ++d) bsum += bf16_lo(rowp[d]) + bf16_hi(rowp[d]);
    }
  }
  if (want_bias) {
    // the four quarters meet, in wavefront order
    __syncthreads();
    float* quarter = reinterpret_cast<float*>(sA);
    quarter[tid] = bsum;
    __syncthreads();
    if (tid < 64) bsum = ((quarter[tid] + quarter[64 + tid]) + quarter[128 + tid]) + quarter[192 + tid];
  }

  const int ci = ci0 + wci + j;
  if (nchunks > 1) {
    float* mine = p.partial + ((size_t)tile * ct.first[seg.K] + blockIdx.y) * kTile3Stride;
    if (ci < p.cin_real) {   // the second stage reads the same lanes only
#pragma unroll
      for (int t = 0; t < 9; ++t)
#pragma unroll
        for (int v = 0; v < 16; ++v) mine[(t * 16 + v) * kThreads + tid] = acc[t][v];
    }
    if (tid < 64) mine[kTile3Floats + tid] = bsum;
    return;
  }
  float* gw = p.gw + (size_t)wk * p.worker_stride;
  if (ci < p.cin_real) {
#pragma unroll
    for (int t = 0; t < 9; ++t)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int co = co0 + wco + 8 * (v / 4) + 4 * h + (v % 4);
        if (co < p.Cout) gw[((size_t)co * 9 + t) * p.cin_real + ci] = acc[t][v];
      }
  }
  if (want_bias && tid < 64 && co0 + tid < p.Cout) p.gb[(size_t)wk * p.worker_stride + co0 + tid] = bsum;
}

// Second stage: grid (tiles, workers, 9 taps x 4 register quarters x 4 tile quadrants).  A workgroup
// owns the (output channel, input channel) pairs one wavefront of the first stage held; each of its
// four wavefronts adds a quarter of the worker's chunks (chunk order, eight chunks in flight), the
// quarters are then added in order through LDS: a fixed summation order with four times the loads in
// flight of one wavefront walking all chunks.
__global__ __launch_bounds__(kThreads) void conv3_wgrad_reduce_kernel(Wgrad3Params p, Segments seg, ChunkTable ct) {
  __shared__ float part[4][4][64];
  const int tile = blockIdx.x, wk = blockIdx.y;
  const int quad = blockIdx.z & 3, vq = (blockIdx.z >> 2) & 3, tap = blockIdx.z >> 4;
  const int nchunks = ct.first[wk + 1] - ct.first[wk];
  if (nchunks <= 1) return;   // written directly by the first stage
  const int tid = threadIdx.x, lane = tid & 63, sub = tid >> 6;
  const int j = lane & 31, h = lane >> 5;
  const int tiles_ci = (p.Cin + 63) / 64;
  const int co0 = (tile / tiles_ci) * 64, ci0 = (tile % tiles_ci) * 64;
  const int wco = (quad >> 1) * 32, wci = (quad & 1) * 32;
  const float* all = p.partial + ((size_t)tile * ct.first[seg.K] + ct.first[wk]) * kTile3Stride;
  const float* mine = all + (size_t)(tap * 16 + vq * 4) * kThreads + quad * 64 + lane;
  const int per = (nchunks + 3) / 4;
  const int c0 = min(sub * per, nchunks), c1 = min(c0 + per, nchunks);
  float s[4] = {0.f, 0.f, 0.f, 0.f};
  const int ci = ci0 + wci + j;
  if (ci < p.cin_real) {
    int c = c0;
    for (; c + 8 <= c1; c += 8) {
      float t[8][4];
#pragma unroll
      for (int u = 0; u < 8; ++u)
#pragma unroll
        for (int e = 0; e < 4; ++e) t[u][e] = mine[(size_t)(c + u) * kTile3Stride + e * kThreads];
#pragma unroll
      for (int u = 0; u < 8; ++u)
#pragma unroll
        for (int e = 0; e < 4; ++e) s[e] += t[u][e];
    }
    for (; c < c1; ++c) {
      const float* q = mine + (size_t)c * kTile3Stride;
#pragma unroll
      for (int e = 0; e < 4; ++e) s[e] += q[e * kThreads];
    }
  }
#pragma unroll
  for (int e = 0; e < 4; ++e) part[sub][e][lane] = s[e];
  __syncthreads();
  if (sub == 0 && ci < p.cin_real) {
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const float tot = ((part[0][e][lane] + part[1][e][lane]) + part[2][e][lane]) + part[3][e][lane];
      const int v = vq * 4 + e;
      const int co = co0 + wco + 8 * (v / 4) + 4 * h + (v % 4);
      if (co < p.Cout) p.gw[(size_t)wk * p.worker_stride + ((size_t)co * 9 + tap) * p.cin_real + ci] = tot;
    }
  }
  if (blockIdx.z == 0 && p.gb != nullptr && ci0 == 0 && tid < 64 && co0 + tid < p.Cout) {
    // eight loads in flight (one dependent round trip per chunk made this the kernel's long pole);
    // the additions keep chunk order
    float bs = 0.f;
    const float* bsrc = all + kTile3Floats + tid;
    int c = 0;
    for (; c + 8 <= nchunks; c += 8) {
      float t[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) t[u] = bsrc[(size_t)(c + u) * kTile3Stride];
#pragma unroll
      for (int u = 0; u < 8; ++u) bs += t[u];
    }
    for (; c < nchunks; ++c) bs += bsrc[(size_t)c * kTile3Stride];
    p.gb[(size_t)wk * p.worker_stride + co0 + tid] = bs;
  }
}


// ---------------------------------------------------------------------------------------------
// Kernel G: weight gradient of the first layer -- 3 input channels stored as 8, 3x3 / stride 1 /
// pad 1, maps 32 wide, at most 64 output channels.
//
//   G_k[co][u][v][ci] = sum over the positions of worker k of dY[pos][co] * X[pos + (u-1, v-1)][ci]
//
// As a matrix product the output is tiny (Cout x 27) and the reduction (all positions) is
// everything, so the layer is bound by reading dY and X once: what kernel C spends on a 64 x 64
// channel tile that is 15/16 empty, and on parking and re-reading such tiles, is avoided by giving
// the product its own shape: rows = output channels (32 per block), columns = (tap, channel)
// pairs, 9 x 4 = 36 of them, column 36 = a channel of ones (its product is the bias gradient),
// reduction = positions, 16 per v_mfma_f32_32x32x16_bf16.  Both operands have the reduction as
// their SLOW index in memory ([pos][channel]); they are staged in LDS as they arrive (16-byte
// pieces) and the transposition happens in the fragment reads: eight 2-byte reads per lane and
// fragment, at immediate offsets.  A workgroup walks units of 4 image rows (128 positions) of one
// worker; its four wavefronts split the positions of a unit and keep whole accumulators, which are
// added through LDS at the end.  Chunks of one worker are added by a second small kernel in chunk
// order (fixed summation order; no atomics).
struct Wgrad1Params {
  const bf16_t* dy;     // [rows][H][32][Cout]
  const bf16_t* src;    // [rows][H][32][8]
  float* gw;            // worker k at gw + k * worker_stride, layout [Cout][3][3][cin_real]
  float* gb;            // may be null
  size_t worker_stride;
  int Cout, cin_real, H;
  int upc;              // units per chunk
  float* partial;       // [chunk][MB * 2 * 16 * 64] accumulator images
  // POOLED kernels: dy is not read; it is rebuilt from the gradient of the 2 x 2 max pooling that
  // follows the layer and the pooling's codes (one byte per pooled element: which input took it)
  const bf16_t* dpool;  // [rows][H/2][16][Cout]
  const uint8_t* code;  // [rows][H/2][16][Cout]
  int raw3;             // src is [rows][H][32][3]: a pixel is three 2-byte loads
};
constexpr int kG_W = 32, kG_R = 4, kG_Unit = kG_W * kG_R;        // 128 positions
constexpr int kG_PatchCols = kG_W + 2, kG_PatchRows = kG_R + 2;
constexpr int kG_XBytes = kG_PatchRows * kG_PatchCols * 16;

// (co, column) of accumulator register v of lane l in block (mb, nb) -> where it goes in G
__device__ inline void wgrad1_emit(const Wgrad1Params& p, float* gw, float* gb, int mb, int nb, int v, int lane,
                                   float val) {
  const int co = mb * 32 + 8 * (v / 4) + 4 * (lane >> 5) + (v % 4);
  const int col = nb * 32 + (lane & 31);
  if (co >= p.Cout) return;
  if (col < 36) {
    const int tap = col >> 2, ci = col & 3;
    if (ci < p.cin_real) gw[((size_t)co * 9 + tap) * p.cin_real + ci] = val;
  } else if (col == 36 && gb != nullptr) {
    gb[co] = val;
  }
}

// POOLED: the layer's output gradient was never written.  Every position takes the gradient of its
// pooling window where the window's code names it and zero elsewhere: 16 + 8 bytes of pooled data
// per piece (shared by the four positions of a window, so mostly cache hits) instead of 16 bytes
// of a full-resolution tensor that a pooling-backward pass would have had to write first.
template <int MB, bool POOLED>
__global__ __launch_bounds__(kThreads, 2) void conv1_wgrad_kernel(Wgrad1Params p, Segments seg, ChunkTable ct) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smemg[];
  const int SY = p.Cout * 2 + 8;                         // bytes per position of the staged dY strip
  const int stage_bytes = (kG_Unit * SY + kG_XBytes + 15) & ~15;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;

  int wk = 0;
  while (wk + 1 < seg.K && (int)blockIdx.x >= ct.first[wk + 1]) ++wk;
  const int chunk_idx = blockIdx.x - ct.first[wk];
  const int nchunks = ct.first[wk + 1] - ct.first[wk];
  const int upi = p.H / kG_R;                              // units per image
  const int units = (seg.off[wk + 1] - seg.off[wk]) * upi;
  const int ubeg = chunk_idx * p.upc, uend = min(units, ubeg + p.upc);

  // zero both stages once (halo columns of the patch are never written again)
  for (int i = tid * 16; i < 2 * stage_bytes; i += kThreads * 16) *reinterpret_cast<u32x4*>(smemg + i) = u32x4{0, 0, 0, 0};
  __syncthreads();

  // staging tasks of this thread: dY pieces (16 bytes = 8 channels of one position), one patch piece
  const int ppp = p.Cout / 8;                              // pieces per position
  const int ny = kG_Unit * ppp;                            // pieces per unit: 128 ... 1024
  constexpr int kYMax = 4;                                 // Cout <= 64
  u32x4 ry[kYMax], rx;
  u32x2 rk[kYMax];                                          // POOLED: the codes that go with ry
  // a thread's pieces are the same in every unit: where each comes from (relative to the unit) and goes
  int ysrc[kYMax], ydst[kYMax];
  uint32_t yslot[kYMax];
#pragma unroll
  for (int i = 0; i < kYMax; ++i) {
    const int q = min(tid + kThreads * i, ny - 1);         // surplus slots re-read the last piece
    const int pos = q / ppp, oct = q - pos * ppp;
    ydst[i] = pos * SY + oct * 16;                          // 8-byte aligned (SY is 8 mod 16)
    // POOLED: the unit's four rows are two pooled rows of 16; the window of position (r, c) is (r/2, c/2)
    ysrc[i] = POOLED ? (((pos >> 6) * (kG_W / 2) + ((pos & 31) >> 1)) * p.Cout + oct * 8) : q * 8;
    yslot[i] = (uint32_t)(((pos >> 5) & 1) * 2 + (pos & 1));
  }
  const bool has_x = tid < kG_PatchRows * kG_W;
  const int xr = tid / kG_W, xc = tid % kG_W;              // patch row 0..5 (image row strip*4 - 1 + xr), column
  auto fetch = [&](int u) {
    const int img = seg.off[wk] + u / upi, row0 = (u % upi) * kG_R;
    if constexpr (POOLED) {
      const size_t ubase = ((size_t)(img * (p.H >> 1) + (row0 >> 1)) * (kG_W / 2)) * p.Cout;
#pragma unroll
      for (int i = 0; i < kYMax; ++i) {
        ry[i] = *reinterpret_cast<const u32x4*>(p.dpool + ubase + ysrc[i]);
        rk[i] = *reinterpret_cast<const u32x2*>(p.code + ubase + ysrc[i]);
      }
    } else {
      const bf16_t* ybase = p.dy + ((size_t)(img * p.H + row0) * kG_W) * p.Cout;
#pragma unroll
      for (int i = 0; i < kYMax; ++i) ry[i] = *reinterpret_cast<const u32x4*>(ybase + ysrc[i]);
    }
    const int grow = row0 - 1 + xr;
    const bool in = has_x && grow >= 0 && grow < p.H;
    const bf16_t* xp = p.src + ((size_t)(img * p.H + (in ? grow : 0)) * kG_W + xc) * (p.raw3 ? 3 : 8);
    if (p.raw3) {
      const bf16_t* q = has_x ? xp : p.src;
      rx = u32x4{(uint32_t)q[0] | ((uint32_t)q[1] << 16), (uint32_t)q[2], 0u, 0u};
    } else {
      rx = *reinterpret_cast<const u32x4*>(has_x ? xp : p.src);
    }
    if (!in) rx = u32x4{0, 0, 0, 0};
    rx[2] = (rx[2] & 0xFFFF0000u) | 0x3F80u;               // channel 4 := 1.0 (the bias column reads it)
  };
  auto stash = [&](int stage) {
    unsigned char* sY = smemg + stage * stage_bytes;
    unsigned char* sX = sY + kG_Unit * SY;
#pragma unroll
    for (int i = 0; i < kYMax; ++i) {
      const int q = tid + kThreads * i;
      if (q < ny) {
        if constexpr (POOLED) {
          // keep a channel's gradient where its code names this position's place in the window
          const uint32_t slot = yslot[i];
#pragma unroll
          for (int d2 = 0; d2 < 4; ++d2) {
            const uint32_t kk = rk[i][d2 >> 1] >> (16 * (d2 & 1));
            const uint32_t lo = (kk & 0xFFu) == slot ? 0x0000FFFFu : 0u;
            const uint32_t hi = ((kk >> 8) & 0xFFu) == slot ? 0xFFFF0000u : 0u;
            ry[i][d2] &= lo | hi;
          }
        }
        unsigned char* d = sY + ydst[i];
        *reinterpret_cast<u32x2*>(d) = u32x2{ry[i][0], ry[i][1]};
        *reinterpret_cast<u32x2*>(d + 8) = u32x2{ry[i][2], ry[i][3]};
      }
    }
    if (has_x) *reinterpret_cast<u32x4*>(sX + (xr * kG_PatchCols + xc + 1) * 16) = rx;
  };

  // fragment addressing.  A: lane supplies output channel lane%32 of block mb, positions
  // 16*kb + 8*(lane/32) + i.  B: lane supplies column lane%32 of block nb.
  const int kg = lane >> 5, jl = lane & 31;
  int bbase[2];
#pragma unroll
  for (int nb = 0; nb < 2; ++nb) {
    const int col = nb * 32 + jl;
    int u = 1, v = 1, ci = 5;                              // unused columns read a zero channel
    if (col < 36) { u = (col >> 2) / 3; v = (col >> 2) % 3; ci = col & 3; }
    else if (col == 36) ci = 4;
    bbase[nb] = (u * kG_PatchCols + v + 8 * kg) * 16 + ci * 2;
  }
  const int abase = 8 * kg * SY + jl * 2;

  v16f acc[MB][2];
#pragma unroll
  for (int a = 0; a < MB; ++a)
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.f;

  if (ubeg < uend) {
    fetch(ubeg);
    stash(0);
    __syncthreads();
    int stage = 0;
    for (int u = ubeg; u < uend; ++u) {
      if (u + 1 < uend) fetch(u + 1);
      const unsigned char* sY = smemg + stage * stage_bytes;
      const unsigned char* sX = sY + kG_Unit * SY;
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        const int kb = wave + 4 * h;                        // 16 positions: image row kb/2, columns (kb%2)*16 ...
        const unsigned char* ya = sY + kb * 16 * SY + abase;
        const unsigned char* xb = sX + ((kb >> 1) * kG_PatchCols + (kb & 1) * 16) * 16;
        bf16x8 fa[MB], fb[2];
#pragma unroll
        for (int a = 0; a < MB; ++a) {
          u32x4 w;
#pragma unroll
          for (int d = 0; d < 4; ++d) {
            const uint32_t lo = *reinterpret_cast<const uint16_t*>(ya + a * 64 + (2 * d) * SY);
            const uint32_t hi = *reinterpret_cast<const uint16_t*>(ya + a * 64 + (2 * d + 1) * SY);
            w[d] = lo | (hi << 16);
          }
          fa[a] = as_bf16x8(w);
        }
#pragma unroll
        for (int b = 0; b < 2; ++b) {
          u32x4 w;
#pragma unroll
          for (int d = 0; d < 4; ++d) {
            const uint32_t lo = *reinterpret_cast<const uint16_t*>(xb + bbase[b] + (2 * d) * 16);
            const uint32_t hi = *reinterpret_cast<const uint16_t*>(xb + bbase[b] + (2 * d + 1) * 16);
            w[d] = lo | (hi << 16);
          }
          fb[b] = as_bf16x8(w);
        }
#pragma unroll
        for (int a = 0; a < MB; ++a)
#pragma unroll
          for (int b = 0; b < 2; ++b) acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[a], fb[b], acc[a][b], 0, 0, 0);
      }
      if (u + 1 < uend) stash(stage ^ 1);
      __syncthreads();
      stage ^= 1;
    }
  }

  // add the four wavefronts' accumulators (wavefront order) and write the chunk's result
  float* red = reinterpret_cast<float*>(smemg);            // [4][MB*2*16][64] floats = 32 KB at MB = 2
  constexpr int kImg = MB * 2 * 16 * 64;
#pragma unroll
  for (int a = 0; a < MB; ++a)
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int v = 0; v < 16; ++v) red[wave * kImg + ((a * 2 + b) * 16 + v) * 64 + lane] = acc[a][b][v];
  __syncthreads();
  float* gw = p.gw + (size_t)wk * p.worker_stride;
  float* gb = p.gb ? p.gb + (size_t)wk * p.worker_stride : nullptr;
  for (int e = tid; e < kImg; e += kThreads) {
    const float val = ((red[e] + red[kImg + e]) + red[2 * kImg + e]) + red[3 * kImg + e];
    if (nchunks > 1) {
      p.partial[(size_t)blockIdx.x * kImg + e] = val;
    } else {
      const int blk = e / (16 * 64), v = (e / 64) % 16, l = e % 64;
      wgrad1_emit(p, gw, gb, blk / 2, blk % 2, v, l, val);
    }
  }
}

// grid (K, MB * 32): 64 accumulator elements per workgroup; each of the four wavefronts adds a
// quarter of the worker's chunks (in chunk order, eight loads in flight), the quarters are then
// added in order through LDS: a fixed summation order with four times the loads in flight.
template <int MB>
__global__ __launch_bounds__(kThreads) void conv1_wgrad_reduce_kernel(Wgrad1Params p, Segments seg, ChunkTable ct) {
  constexpr int kImg = MB * 2 * 16 * 64;
  __shared__ float part[4][64];
  const int wk = blockIdx.x;
  const int nchunks = ct.first[wk + 1] - ct.first[wk];
  if (nchunks <= 1) return;                                 // written by the first kernel
  const int lane = threadIdx.x & 63, sub = threadIdx.x >> 6;
  const int e = blockIdx.y * 64 + lane;
  const int per = (nchunks + 3) / 4;
  const int c0 = min(sub * per, nchunks), c1 = min(c0 + per, nchunks);
  const float* src = p.partial + (size_t)ct.first[wk] * kImg + e;
  float s = 0.f;
  int c = c0;
  for (; c + 8 <= c1; c += 8) {
    float t[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) t[u] = src[(size_t)(c + u) * kImg];
#pragma unroll
    for (int u = 0; u < 8; ++u) s += t[u];
  }
  for (; c < c1; ++c) s += src[(size_t)c * kImg];
  part[sub][lane] = s;
  __syncthreads();
  if (sub != 0) return;
  s = ((part[0][lane] + part[1][lane]) + part[2][lane]) + part[3][lane];
  float* gw = p.gw + (size_t)wk * p.worker_stride;
  float* gb = p.gb ? p.gb + (size_t)wk * p.worker_stride : nullptr;
  const int blk = e / (16 * 64), v = (e / 64) % 16, l = e % 64;
  wgrad1_emit(p, gw, gb, blk / 2, blk % 2, v, l, s);
}

}  // namespace

size_t conv_wgrad_partial_floats() { return (size_t)kConvMaxPartialTiles * (2 * 2 * 16 * kThreads + 128); }

bool conv_shape_supported(const ConvGeom& g, long positions) {
  return g.Cs % 8 == 0 && g.K <= kMaxPieces * 8 && g.ks >= 1 && g.ks <= 15 && positions < (1L << 24);
}

template <int TN, int MODE>
static void launch_gemm2(hipStream_t st, const ConvParams& p, int tiles) {
  constexpr int BN = 64 * TN;
  constexpr size_t kBytes =
      (size_t)2 * (BM + BN) * (BK2 + 8) * sizeof(bf16_t) + (MODE != GEN ? 0 : kMaxPieces * sizeof(int));
  static bool configured = false;   // raising the dynamic LDS limit is a per-function, one-time host call
  if (!configured) {
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&conv_gemm2_kernel<TN, MODE>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)kBytes);
    configured = true;
  }
  hipLaunchKernelGGL((conv_gemm2_kernel<TN, MODE>), dim3(tiles), dim3(kThreads), kBytes, st, p);
}

// 3x3 / pad 1 / stride 1 (forward, or dgrad of such a layer) with channels a multiple of 32 and a
// map whose rows tile into units of 256 positions: kernel D.  Returns false if the shape does not qualify.
static bool conv3_gemm(hipStream_t st, const bf16_t* src, const bf16_t* wgt, bf16_t* out, int M, int N,
                       const ConvGeom& g, const float* bias, const bf16_t* mask, bool relu, bool accumulate,
                       bf16_t* pool, uint8_t* pool_code, bool* pooled, const bf16_t* addend) {
  const int H = g.Hs, W = g.Ws;
  if (g.raw3 || g.ks != 3 || g.stride != 1 || g.pad != 1 || g.Hp != H || g.Wp != W) return false;
  if (g.Cs % 32 != 0 || N % 8 != 0 || (long)g.rows * H * W != M) return false;
  if ((long)M * g.Cs >= (1L << 31)) return false;   // 32-bit element offsets in the kernel
  if (W < 4 || W > kUnitD || kUnitD % W != 0) return false;
  const int R = std::min(H, kUnitD / W);
  if (H % R != 0 || kUnitD % (R * W) != 0) return false;
  const int nimg = kUnitD / (R * W);
  if (nimg > 1 && R != H) return false;
  const int npatch = nimg * (R + 2) * (W + 2);
  // channels of the reduction staged at a time: 64 where the patch of a unit then fits the registers
  // that carry it to LDS (on 4 x 4 maps a unit is 16 images and their halos are most of the patch)
  const int kc = (g.Cs % 64 == 0 && npatch * 8 <= kMaxPatchPieces * kThreads) ? 64 : 32;
  const int oc = kc / 8;
  if (npatch * oc > kMaxPatchPieces * kThreads) return false;
  Conv3Params p{};
  p.src = src; p.wgt = wgt; p.out = out; p.rows = g.rows; p.H = H; p.W = W; p.Cs = g.Cs; p.N = N;
  p.R = R; p.nimg = nimg; p.flip = g.transposed ? 1 : 0; p.zero = g.zero;
  p.bias = bias; p.mask = mask; p.relu = relu ? 1 : 0; p.accumulate = accumulate ? 1 : 0;
  // the pooled copy is written from the same staged tile when a unit holds whole 2 x 2 windows
  p.pool = (pool && pool_code && !mask && !accumulate && !g.transposed && H % 2 == 0 && W % 2 == 0 && R % 2 == 0)
               ? pool : nullptr;
  p.pool_code = pool_code;
  p.addend = addend;
  *pooled = p.pool != nullptr;
  const int nb = N <= 32 ? 1 : 2;                 // a 32-channel tile for layers with at most 32 output channels
  const int tn = 32 * nb;
  const size_t stage = ((size_t)npatch + 2 * tn) * (kc + 8) * sizeof(bf16_t);
  const size_t outt = (size_t)kUnitD * (tn + 4) * sizeof(float);
  const size_t lds = std::max(stage, outt);
  if (lds > 80 * 1024) return false;
  const int big = npatch * oc > 11 * kThreads ? 1 : 0;
  const int units = nimg == 1 ? g.rows * (H / R) : (g.rows + nimg - 1) / nimg;
  const int tiles_n = (N + tn - 1) / tn;
  // several units per workgroup once there are enough workgroups to fill the chip a few times over
  int upw = 1;
  while (upw < 4 && (long)units * tiles_n / (upw * 2) >= 2048) upw *= 2;
  p.units = units; p.upw = upw;
  const dim3 grid(((units + upw - 1) / upw) * tiles_n);
  const bool w8 = W == 8 && R % 8 == 0;
  static size_t configured[2][2][2][2] = {};   // raising the dynamic LDS limit is a per-function host call
#define OMNI_CONV3(NP_, NB_, KC_, W8_)                                                                \
  {                                                                                                   \
    size_t& conf = configured[big][NB_ - 1][KC_ == 64 ? 0 : 1][W8_ ? 1 : 0];                          \
    if (lds > conf) {                                                                                 \
      (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&conv3_gemm_kernel<NP_, NB_, KC_, W8_>), \
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);                \
      conf = lds;                                                                                     \
    }                                                                                                 \
    hipLaunchKernelGGL((conv3_gemm_kernel<NP_, NB_, KC_, W8_>), grid, dim3(kThreads), lds, st, p);    \
  }
#define OMNI_CONV3_W8(NP_, NB_, KC_) { if (w8) OMNI_CONV3(NP_, NB_, KC_, true) else OMNI_CONV3(NP_, NB_, KC_, false) }
#define OMNI_CONV3_KC(NP_, NB_) { if (kc == 64) OMNI_CONV3_W8(NP_, NB_, 64) else OMNI_CONV3_W8(NP_, NB_, 32) }
  if (nb == 1) { if (big) OMNI_CONV3_KC(13, 1) else OMNI_CONV3_KC(11, 1) }
  else
  { if (big) OMNI_CONV3_KC(13, 2) else OMNI_CONV3_KC(11, 2) }
#undef OMNI_CONV3_KC
#undef OMNI_CONV3_W8
#undef OMNI_CONV3
  return true;
}

// First layer forward (8 stored channels, 3x3 / pad 1 / stride 1, at most 64 outputs): kernel F.
static bool conv1_fwd_shape(int N, const ConvGeom& g, long M) {
  const int H = g.Hs, W = g.Ws;
  if (g.transposed || g.Cs != 8 || g.ks != 3 || g.stride != 1 || g.pad != 1) return false;
  if (g.Hp != H || g.Wp != W || N % 8 != 0 || N > 64 || (long)g.rows * H * W != M) return false;
  if (W < 8 || W > kUnitD || kUnitD % W != 0) return false;
  const int R = std::min(H, kUnitD / W);
  if (H % R != 0 || kUnitD % (R * W) != 0) return false;
  const int nimg = kUnitD / (R * W);
  if (nimg > 1 && R != H) return false;
  return nimg * (R + 2) * (W + 2) <= 2 * kThreads;
}

static bool conv1_fwd(hipStream_t st, const bf16_t* src, const bf16_t* wgt, bf16_t* out, int M, int N,
                      const ConvGeom& g, const float* bias, const bf16_t* mask, bool relu, bool accumulate,
                      bf16_t* pool, uint8_t* pool_code, bool* pooled) {
  const int H = g.Hs, W = g.Ws;
  if (mask || accumulate || !conv1_fwd_shape(N, g, M)) return false;
  const int R = std::min(H, kUnitD / W);
  const int nimg = kUnitD / (R * W);
  const int npatch = nimg * (R + 2) * (W + 2);
  Conv1Params p{};
  p.raw3 = g.raw3;
  p.src = src; p.wgt = wgt; p.out = out; p.rows = g.rows; p.H = H; p.W = W; p.N = N; p.R = R; p.nimg = nimg;
  p.bias = bias; p.relu = relu ? 1 : 0; p.zero = g.zero;
  p.pool = (pool && pool_code && H % 2 == 0 && W % 2 == 0 && R % 2 == 0) ? pool : nullptr;
  p.pool_code = pool_code;
  *pooled = p.pool != nullptr;
  p.units = nimg == 1 ? g.rows * (H / R) : (g.rows + nimg - 1) / nimg;
  p.upw = 1;
  while (p.upw < 8 && p.units / (p.upw * 2) >= 1024) p.upw *= 2;
  const int nblk = N > 32 ? 2 : 1;
  const size_t lds = (size_t)((npatch + 3) & ~3) * 16 + (size_t)kUnitD * (32 * nblk + 8) * sizeof(bf16_t);
  const dim3 grid((p.units + p.upw - 1) / p.upw);
  if (nblk == 2) hipLaunchKernelGGL(conv1_fwd_kernel<2>, grid, dim3(kThreads), lds, st, p);
  else hipLaunchKernelGGL(conv1_fwd_kernel<1>, grid, dim3(kThreads), lds, st, p);
  return true;
}

bool conv_gemm_bf16(hipStream_t st, const bf16_t* src, const bf16_t* wgt, bf16_t* out, int M, int N,
                    const ConvGeom& g, const float* bias, const bf16_t* mask, bool relu, bool accumulate,
                    bf16_t* pool_out, uint8_t* pool_code, const bf16_t* addend, BnStatRequest* stats) {
  bool pooled = false;
  // 3x3 / stride 1 / pad 1: the wide-tile kernel where the shape and the amount of work allow it (it has no
  // pooling epilogue), else the 256-position one
  if (!(pool_out && pool_code) &&
      conv3_wide_bf16(st, src, wgt, out, M, N, g, bias, mask, relu, accumulate, addend, stats))
    return false;
  if (conv3_gemm(st, src, wgt, out, M, N, g, bias, mask, relu, accumulate, pool_out, pool_code, &pooled, addend))
    return pooled;
  if (!addend && conv1_fwd(st, src, wgt, out, M, N, g, bias, mask, relu, accumulate, pool_out, pool_code, &pooled))
    return pooled;
  if (g.raw3) return false;   // (callers ask conv_first_layer_raw_supported first: nothing else reads a 3-channel source)
  ConvParams p{};
  p.src = src; p.wgt = wgt; p.out = out; p.M = M; p.N = N; p.g = g;
  p.bias = bias; p.mask = mask; p.relu = relu ? 1 : 0; p.accumulate = accumulate ? 1 : 0;
  p.addend = addend;
  int tiles_m = (M + BM - 1) / BM;
  const bool chan_ok = g.Cs % BK2 == 0 && g.ks <= 3;
  const bool fast = chan_ok && (!g.transposed || g.stride == 1);
  // dgrad of a stride-2 convolution: the gathered tensor is the half-resolution output gradient
  const bool phased = chan_ok && g.transposed && g.stride == 2 && g.Hp % 2 == 0 && g.Wp % 2 == 0 &&
                      g.Hs == g.Hp / 2 && g.Ws == g.Wp / 2 && (long)g.rows * g.Hp * g.Wp == M;
  if (phased) {
    const long cls = (long)g.rows * (g.Hp / 2) * (g.Wp / 2);
    tiles_m = 4 * (int)((cls + BM - 1) / BM);   // every parity class is padded to whole tiles
  }
  const int mode = phased ? PHASED : fast ? FASTM : GEN;
  const int tiles = tiles_m * (N > 64 ? (N + 127) / 128 : (N + 63) / 64);
#define OMNI_GEMM2(TN)                                           \
  {                                                              \
    if (mode == PHASED) launch_gemm2<TN, PHASED>(st, p, tiles);  \
    else if (mode == FASTM) launch_gemm2<TN, FASTM>(st, p, tiles); \
    else launch_gemm2<TN, GEN>(st, p, tiles);                    \
  }
  if (N > 64) OMNI_GEMM2(2) else OMNI_GEMM2(1)
#undef OMNI_GEMM2
  return false;
}

// 3x3 / stride 1 / pad 1 and a map whose rows tile into units of 128 positions: kernel C.  (Also
// for a first layer with 8 stored channels on maps that are not 32 wide, which kernel G does not
// take: most of the 64-channel tile is then empty.)  Returns false if the shape does not qualify.
static bool conv3_wgrad(hipStream_t st, const bf16_t* dy, const bf16_t* src, float* gw, float* gb,
                        size_t worker_stride, int Cout, int cin_real, const ConvGeom& g, const Segments& seg,
                        float* partial) {
  const int H = g.Hs, W = g.Ws;
  if (g.ks != 3 || g.stride != 1 || g.pad != 1 || g.transposed || g.Hp != H || g.Wp != W) return false;
  if (cin_real > g.Cs || g.Cs % 8 != 0 || Cout % 8 != 0) return false;
  const bool w4 = W == 4 && H == 4;
  if (!w4 && (W % 8 != 0 || W > kUnit || kUnit % W != 0)) return false;
  const int R = std::min(H, kUnit / W);
  if (H % R != 0 || kUnit % (R * W) != 0) return false;
  const int nimg = kUnit / (R * W);
  if (nimg > 1 && R != H) return false;
  Wgrad3Params p{};
  p.dy = dy; p.src = src; p.gw = gw; p.gb = gb; p.worker_stride = worker_stride;
  p.Cout = Cout; p.Cin = g.Cs; p.cin_real = cin_real; p.H = H; p.W = W; p.R = R; p.nimg = nimg;
  p.Wp = w4 ? 8 : W + 16; p.prows = nimg * (R + 2);
  // channel stride of X^T in 4-byte words must be 4 mod 8: 16 lanes x 16 bytes then cover all 64 banks
  int words = p.prows * p.Wp / 2;
  words += (4 - words % 8 + 8) % 8;
  p.SX = words * 4;
  p.partial = partial;
  p.zero = g.zero;
  const size_t lds = (size_t)64 * kSA + (size_t)64 * p.SX + 2 * kSkewPad;   // + the row skew of both arrays
  if (lds > 80 * 1024) return false;
  const int tiles = ((Cout + 63) / 64) * ((g.Cs + 63) / 64);
  const size_t max_slots = conv_wgrad_partial_floats() / kTile3Stride;
  // units per worker, and a chunk length that gives about one workgroup per compute unit (every chunk
  // parks a partial tile of up to 148 KB that the second stage reads back: with 512 chunks that traffic
  // outweighed the extra parallelism, measured -2 % on the three-layer CNN's step with 256)
  long total_units = 0;
  int units[OMNI_MAX_WORKERS];
  for (int k = 0; k < seg.K; ++k) {
    const int bk = seg.off[k + 1] - seg.off[k];
    units[k] = nimg == 1 ? bk * (H / R) : (bk + nimg - 1) / nimg;
    total_units += units[k];
  }
  long want = std::max<long>(1, 256 / tiles);
  long upc = std::max<long>((total_units + want - 1) / want, 4);
  ChunkTable ct{};
  for (;;) {
    int acc = 0;
    for (int k = 0; k < seg.K; ++k) {
      ct.first[k] = acc;
      acc += (int)((units[k] + upc - 1) / upc);
    }
    ct.first[seg.K] = acc;
    if (acc == 0) return true;   // no rows at all
    // one chunk per worker needs no scratch (every workgroup writes its worker's gradient itself);
    // otherwise the partial tiles must fit the scratch and all workgroups should be resident at once
    // (two per compute unit): a few extra ones would run as a second round
    if (acc == seg.K) break;
    if ((size_t)tiles * acc <= max_slots && (long)tiles * acc <= std::max(256, 2 * tiles * seg.K)) break;
    upc += std::max<long>(1, upc / 16);
  }
  p.upc = (int)upc;
  // kernel variant by map width: 4, 8, 16, 32, or any other (index 4)
  const int variant = w4 ? 0 : W == 8 ? 1 : W == 16 ? 2 : W == 32 ? 3 : 4;
  using KernelFn = void (*)(Wgrad3Params, Segments, ChunkTable);
  static const KernelFn kernels[5] = {conv3_wgrad_kernel<4>, conv3_wgrad_kernel<8>, conv3_wgrad_kernel<16>,
                                      conv3_wgrad_kernel<32>, conv3_wgrad_kernel<0>};
  static size_t configured[5] = {0, 0, 0, 0, 0};   // raising the dynamic LDS limit is a per-function host call
  if (lds > configured[variant]) {
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(kernels[variant]),
                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    configured[variant] = lds;
  }
  const dim3 grid(tiles, ct.first[seg.K]);
  hipLaunchKernelGGL(kernels[variant], grid, dim3(kThreads), lds, st, p, seg, ct);
  bool chunked = false;
  for (int k = 0; k < seg.K; ++k) chunked = chunked || ct.first[k + 1] - ct.first[k] > 1;
  if (chunked)
    hipLaunchKernelGGL(conv3_wgrad_reduce_kernel, dim3(tiles, seg.K, 144), dim3(kThreads), 0, st, p, seg, ct);
  return true;
}

// The first layer (3 channels stored as 8) on 32-wide maps: kernel G.  Returns false if the shape
// does not qualify.
static bool conv1_wgrad_shape(int Cout, int cin_real, const ConvGeom& g) {
  const int H = g.Hs, W = g.Ws;
  if (g.ks != 3 || g.stride != 1 || g.pad != 1 || g.transposed || g.Hp != H || g.Wp != W) return false;
  if (g.Cs != 8 || cin_real > 4 || cin_real < 1 || W != kG_W || H % kG_R != 0) return false;
  return Cout % 8 == 0 && Cout >= 8 && Cout <= 64;
}

bool conv_wgrad_pooled_supported(int Cout, int cin_real, const ConvGeom& g) { return conv1_wgrad_shape(Cout, cin_real, g); }

bool conv_first_layer_raw_supported(int Cout, int cin_real, const ConvGeom& g, long M) {
  return cin_real == 3 && conv1_fwd_shape(Cout, g, M) && conv1_wgrad_shape(Cout, cin_real, g);
}

static bool conv1_wgrad(hipStream_t st, const bf16_t* dy, const bf16_t* src, float* gw, float* gb,
                        size_t worker_stride, int Cout, int cin_real, const ConvGeom& g, const Segments& seg,
                        float* partial, const bf16_t* dpool, const uint8_t* code) {
  const int H = g.Hs;
  if (!conv1_wgrad_shape(Cout, cin_real, g)) return false;
  const int mb = Cout > 32 ? 2 : 1;
  const size_t img_floats = (size_t)mb * 2 * 16 * 64;
  Wgrad1Params p{};
  p.dy = dy; p.src = src; p.gw = gw; p.gb = gb; p.worker_stride = worker_stride;
  p.Cout = Cout; p.cin_real = cin_real; p.H = H; p.partial = partial;
  p.dpool = dpool; p.code = code;
  p.raw3 = g.raw3;
  const bool pooled = dpool != nullptr;
  const int upi = H / kG_R;
  long total_units = 0;
  for (int k = 0; k < seg.K; ++k) total_units += (long)(seg.off[k + 1] - seg.off[k]) * upi;
  if (total_units == 0) return true;
  // about two workgroups per compute unit, at least 4 units each
  // (every worker's last chunk may be short: aim K below 512 so the total stays within it)
  const long want = std::max(64, 1024 - seg.K);
  long upc = std::max<long>((total_units + want - 1) / want, 4);
  ChunkTable ct{};
  for (;;) {
    int acc = 0;
    for (int k = 0; k < seg.K; ++k) {
      ct.first[k] = acc;
      acc += (int)(((long)(seg.off[k + 1] - seg.off[k]) * upi + upc - 1) / upc);
    }
    ct.first[seg.K] = acc;
    if (acc == seg.K || (size_t)acc * img_floats <= conv_wgrad_partial_floats()) break;
    upc += std::max<long>(1, upc / 8);
  }
  p.upc = (int)upc;
  const int SY = Cout * 2 + 8;
  const size_t stage = ((size_t)kG_Unit * SY + kG_XBytes + 15) & ~(size_t)15;
  const size_t lds = std::max(2 * stage, 4 * img_floats * sizeof(float));
  const dim3 grid(ct.first[seg.K]);
  bool chunked = false;
  for (int k = 0; k < seg.K; ++k) chunked = chunked || ct.first[k + 1] - ct.first[k] > 1;
  using KernelFn = void (*)(Wgrad1Params, Segments, ChunkTable);
  static const KernelFn kernels[2][2] = {{conv1_wgrad_kernel<1, false>, conv1_wgrad_kernel<1, true>},
                                         {conv1_wgrad_kernel<2, false>, conv1_wgrad_kernel<2, true>}};
  static size_t configured[2][2] = {};   // raising the dynamic LDS limit is a per-function host call
  const KernelFn fn = kernels[mb - 1][pooled ? 1 : 0];
  if (lds > configured[mb - 1][pooled ? 1 : 0]) {
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(fn), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    configured[mb - 1][pooled ? 1 : 0] = lds;
  }
  hipLaunchKernelGGL(fn, grid, dim3(kThreads), lds, st, p, seg, ct);
  if (chunked) {
    if (mb == 1) hipLaunchKernelGGL(conv1_wgrad_reduce_kernel<1>, dim3(seg.K, 32), dim3(kThreads), 0, st, p, seg, ct);
    else hipLaunchKernelGGL(conv1_wgrad_reduce_kernel<2>, dim3(seg.K, 64), dim3(kThreads), 0, st, p, seg, ct);
  }
  return true;
}

void conv_wgrad_bf16(hipStream_t st, const bf16_t* dy, const bf16_t* src, float* gw, float* gb,
                     size_t worker_stride, int Cout, int cin_real, const ConvGeom& g, const Segments& seg,
                     float* partial, uint32_t* counters, const bf16_t* dpool, const uint8_t* pool_code) {
  if (conv1_wgrad(st, dy, src, gw, gb, worker_stride, Cout, cin_real, g, seg, partial, dpool, pool_code)) return;
  if (dpool || g.raw3) return;   // (callers ask conv_wgrad_pooled_supported / conv_first_layer_raw_supported first)
  if (conv3_wgrad(st, dy, src, gw, gb, worker_stride, Cout, cin_real, g, seg, partial)) return;
  if (g.stride == 2 && conv3_wgrad_tr_bf16(st, dy, src, gw, gb, worker_stride, Cout, cin_real, g, seg, partial)) return;
  WgradParams p{};
  p.dy = dy; p.src = src; p.gw = gw; p.gb = gb; p.worker_stride = worker_stride;
  p.Cout = Cout; p.cin_real = cin_real; p.g = g; p.partial = partial; p.counters = counters;
  const int tm = Cout > 64 ? 2 : 1, tn = g.K > 64 ? 2 : 1;
  const int tiles = ((Cout + 64 * tm - 1) / (64 * tm)) * ((g.K + 64 * tn - 1) / (64 * tn));
  const long hw = (long)g.Hp * g.Wp;
  const long total = (long)seg.off[seg.K] * hw;
  // Chunk length: about 512 workgroups in all, two per compute unit (the reduction is where the
  // parallelism of a small filter bank lies; every extra chunk is a partial tile written and
  // read back), at least 8 slabs each, within the scratch budget.
  long want = std::max<long>(1, 512 / tiles);
  long chunk = std::max<long>((total + want - 1) / want, 8 * BK);
  chunk = (chunk + BK - 1) / BK * BK;
  ChunkTable ct{};
  for (;;) {
    int acc = 0;
    for (int k = 0; k < seg.K; ++k) {
      ct.first[k] = acc;
      acc += (int)(((long)(seg.off[k + 1] - seg.off[k]) * hw + chunk - 1) / chunk);
    }
    ct.first[seg.K] = acc;
    // one chunk per worker needs no scratch; otherwise all workgroups should be resident at once
    // (two per compute unit): a few extra ones would run as a second round
    if (acc == seg.K || ((long)tiles * acc <= kConvMaxPartialTiles && (long)tiles * acc <= std::max(512, 2 * tiles * seg.K)))
      break;
    chunk += std::max<long>(BK, chunk / 16 / BK * BK);
  }
  p.chunk = (int)chunk;
  dim3 grid(tiles, ct.first[seg.K]);
  const bool chunked = ct.first[seg.K] > seg.K;
#define OMNI_WGRAD(TM, TN)                                                                                   \
  {                                                                                                          \
    hipLaunchKernelGGL((conv_wgrad_kernel<TM, TN>), grid, dim3(kThreads), 0, st, p, seg, ct);                \
    if (chunked)                                                                                             \
      hipLaunchKernelGGL((conv_wgrad_reduce_kernel<TM, TN>), dim3(tiles, seg.K, TM * TN * 16), dim3(kThreads), \
                         0, st, p, seg, ct);                                                                 \
  }
  if (tm == 2 && tn == 2) OMNI_WGRAD(2, 2)
  else if (tm == 2) OMNI_WGRAD(2, 1)
  else if (tn == 2) OMNI_WGRAD(1, 2)
  else OMNI_WGRAD(1, 1)
#undef OMNI_WGRAD
}

}  // namespace omni
