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
// A workgroup is 4 wavefronts in a 2x2 grid over a 64x64 output tile; each
// wavefront owns one 32x32 accumulator block.  Operand slabs of BK reduction
// steps are staged through LDS with register prefetch of the next slab
// (double-buffered LDS, one barrier per slab).
//
// Filling 256 compute units when the batch is small:
//   * forward / dgrad split the reduction over gridDim.y workgroups per tile;
//     each writes its partial tile, the last one to arrive (a per-tile counter)
//     adds the partials in split order and runs the epilogue, so the sum order
//     is fixed and results repeat bit for bit;
//   * wgrad gives every workgroup one output tile position and lets it walk
//     through ALL workers' row ranges one after the other, flushing the
//     accumulator into worker k's gradient when k's rows end.  Every workgroup
//     then does the same amount of work however ragged the b_k are.  The
//     weight gradients of several layers can share one launch
//     (linear_wgrad_f32_batch): their workgroups follow each other in one grid.
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>

#include <algorithm>

#include "common.h"
#include "kernels.h"

namespace omni {

typedef float v4f __attribute__((ext_vector_type(4)));
typedef float v16f __attribute__((ext_vector_type(16)));

namespace {

constexpr int kThreads = 256;
constexpr int kTile = 64;

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

  // Loads never branch: an element outside the operand is fetched from the
  // operand's first element instead and zeroed when the slab is written to LDS
  // (`ok` carries validity bits).  Branch-free loads let the compiler keep them
  // in flight across the whole MFMA section of the current slab.
  // VEC requires the contiguous extent (kk for k-contiguous, rows for
  // row-contiguous operands) to be a multiple of 4 and 16-byte aligned rows, so a
  // 4-element piece is either wholly inside or wholly outside (one bit per piece).
  // Everything that does not change from slab to slab is worked out once per
  // thread (`Pre`): the per-slab address is one 64-bit add per piece.  The vector
  // ALU shares issue slots with the matrix pipe, so every instruction saved here
  // is matrix time gained.
  struct Pre {
    int koff[kPerThread];     // reduction offset of the piece inside a slab
    long cpart[kPerThread];   // element offset of the piece for slab start 0
    uint32_t rowok;           // bit i: the piece's rows lie inside the operand
  };
  __device__ static inline Pre prepare(int ld, int row0, int rows, int tid) {
    Pre pre;
    pre.rowok = 0;
#pragma unroll
    for (int i = 0; i < kPerThread; ++i) {
      const int c = tid + kThreads * i;
      if (!MC) {
        const int r = row0 + c / (BK / 4), kc = (c % (BK / 4)) * 4;
        pre.koff[i] = kc + 3;
        pre.cpart[i] = r < rows ? (long)r * ld + kc : (long)kc;      // absent row: row 0 stands in
        pre.rowok |= (r < rows ? 1u : 0u) << i;
      } else {
        const int kk = c / (R / 4), r = row0 + (c % (R / 4)) * 4;
        pre.koff[i] = kk;
        pre.cpart[i] = r + 3 < rows ? (long)kk * ld + r : (long)kk * ld;   // absent rows: rows 0..3 stand in
        pre.rowok |= (r + 3 < rows ? 1u : 0u) << i;
      }
    }
    return pre;
  }

  template <bool VEC>
  __device__ static inline void load(v4f (&reg)[kPerThread], uint32_t& ok, const float* __restrict__ base, int ld,
                                     int row0, int rows, int k0, int kend, int tid, const Pre& pre) {
    ok = 0;
    if (VEC) {
      const long kbase = MC ? (long)k0 * ld : (long)k0;
      const int klen = kend - k0;
#pragma unroll
      for (int i = 0; i < kPerThread; ++i) {
        const bool in = ((pre.rowok >> i) & 1u) && pre.koff[i] < klen;
        reg[i] = *reinterpret_cast<const v4f*>(base + (in ? pre.cpart[i] + kbase : 0));
        ok |= (in ? 1u : 0u) << i;
      }
      return;
    }
#pragma unroll
    for (int i = 0; i < kPerThread; ++i) {
      const int c = tid + kThreads * i;
      int gr, gk;
      if (!MC) {
        gr = row0 + c / (BK / 4);
        gk = k0 + (c % (BK / 4)) * 4;
      } else {
        gk = k0 + c / (R / 4);
        gr = row0 + (c % (R / 4)) * 4;
      }
      v4f v;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const bool in = MC ? (gk < kend && gr + e < rows) : (gr < rows && gk + e < kend);
        const size_t o = MC ? (size_t)gk * ld + gr + e : (size_t)gr * ld + gk + e;
        v[e] = base[in ? o : 0];
        ok |= (in ? 1u : 0u) << (4 * i + e);
      }
      reg[i] = v;
    }
  }

  // The mask-free form used with VEC.  A slab whose BK reduction steps all lie inside the
  // range is loaded as it is.  A slab that would run past the end of its range is moved
  // back so that it ENDS at the end of the range (start ks = max(kend - BK, 0): the caller
  // guarantees at least BK reduction steps in the operand, so this stays in bounds); the
  // steps of the slab outside [k0, kend) are zeroed in LDS afterwards (zero_outside), which
  // happens once per range.  Rows outside the operand are not zeroed at all: they only
  // feed outputs that are never stored.  The loop over full slabs then has no validity
  // bits, no selects and one address add per piece.
  __device__ static inline void load_fast(v4f (&reg)[kPerThread], const float* __restrict__ base, int ld, int ks,
                                          const Pre& pre) {
    const float* sbase = base + (MC ? (long)ks * ld : (long)ks);
#pragma unroll
    for (int i = 0; i < kPerThread; ++i) reg[i] = *reinterpret_cast<const v4f*>(sbase + pre.cpart[i]);
  }
  __device__ static inline void store_fast(const v4f (&reg)[kPerThread], float* lds, int tid, int i) {
    const int c = tid + kThreads * i;
    if (!MC) {
      const int r = c / (BK / 4), kc = (c % (BK / 4)) * 4;
      *reinterpret_cast<v4f*>(lds + r * kStride + kc) = reg[i];
    } else {
      const int kk = c / (R / 4), rc = (c % (R / 4)) * 4;
      *reinterpret_cast<v4f*>(lds + kk * kStride + rc) = reg[i];
    }
  }
  // zero the reduction steps of a staged slab outside [lo, hi)
  __device__ static inline void zero_outside(float* lds, int lo, int hi, int tid) {
    for (int idx = tid; idx < R * BK; idx += kThreads) {
      const int kk = MC ? idx / R : idx % BK;
      const int r = MC ? idx % R : idx / BK;
      if (kk < lo || kk >= hi) lds[MC ? kk * kStride + r : r * kStride + kk] = 0.f;
    }
  }

  // piece i of the thread's share of the slab
  template <bool VEC>
  __device__ static inline void store_one(const v4f (&reg)[kPerThread], uint32_t ok, float* lds, int tid, int i) {
    const int c = tid + kThreads * i;
    v4f v = reg[i];
    if (VEC) {
      const bool in = (ok >> i) & 1u;
#pragma unroll
      for (int e = 0; e < 4; ++e) v[e] = in ? v[e] : 0.f;
    } else {
#pragma unroll
      for (int e = 0; e < 4; ++e) v[e] = ((ok >> (4 * i + e)) & 1u) ? v[e] : 0.f;
    }
    if (!MC) {
      const int r = c / (BK / 4), kc = (c % (BK / 4)) * 4;
      *reinterpret_cast<v4f*>(lds + r * kStride + kc) = v;
    } else {
      const int kk = c / (R / 4), rc = (c % (R / 4)) * 4;
      *reinterpret_cast<v4f*>(lds + kk * kStride + rc) = v;
    }
  }

  template <bool VEC>
  __device__ static inline void store(const v4f (&reg)[kPerThread], uint32_t ok, float* lds, int tid) {
#pragma unroll
    for (int i = 0; i < kPerThread; ++i) store_one<VEC>(reg, ok, lds, tid, i);
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
  int xcd_remap;       // FWD / DGRAD: 1 if the workgroups are re-ordered per XCD
  int splits;          // FWD / DGRAD: reduction splits per tile
  float* partial;      // FWD / DGRAD split-K: [tiles][splits][16][256] floats
  uint32_t* counters;  // FWD / DGRAD split-K: one per tile, zero between launches
  size_t c_worker_stride;  // WGRAD: floats between consecutive workers' outputs
  float* bias_grad;        // WGRAD: per worker column sums of A (at + worker*c_worker_stride), may be null
  int c_vec;               // WGRAD: every worker's output rows are 16-byte aligned (16-byte stores allowed)
  int ngroups;             // WGRAD: consecutive workers are dealt to this many workgroups per tile (gridDim.y)
  int gfirst[9];           // WGRAD: first worker of every group; gfirst[ngroups] = K
};

// (The second launch bound caps the kernel at 256 registers: the compiler then issues the MFMAs on
// ordinary vector registers.  With accumulation registers it copied all 32 accumulator registers in
// and out around the MFMAs of every step, 64 extra vector instructions per 16 MFMAs, because the
// per-worker flush inside the loop reads and zeroes them.)
// The whole workgroup program; (bx, by) is the workgroup's place in a launch of nbx workgroups along x.
template <int BK, bool A_MC, bool B_MC, int MODE, bool VEC>
__device__ __forceinline__ void gemm_f32_body(const GemmParams& p, const Segments& seg, const int bx, const int by,
                                              const int nbx) {
  using SA = Slab<kTile, BK, A_MC>;
  using SB = Slab<kTile, BK, B_MC>;
  constexpr int kStage = SA::kFloats + SB::kFloats;
  __shared__ __attribute__((aligned(16))) float lds[2 * kStage];
  __shared__ uint32_t arrival;
  __shared__ float bred[4][kTile];                 // WGRAD: the four wavefronts' bias-gradient partial sums
  constexpr int kFlushStride = kTile + 4;          // WGRAD: row stride of the output tile staged for the flush
  static_assert(kTile * kFlushStride <= kStage, "the staged output tile must fit one LDS stage");
  auto sA = [&](int stage) { return lds + stage * kStage; };
  auto sB = [&](int stage) { return lds + stage * kStage + SA::kFloats; };

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int tiles_n = (p.N + kTile - 1) / kTile;
  const int tiles_m = (p.M + kTile - 1) / kTile;
  int tile = bx, split = 0;
  const int splits = (MODE == MODE_WGRAD) ? 1 : p.splits;
  if (MODE != MODE_WGRAD) {
    // Forward / dgrad launch tiles*splits workgroups in one dimension.  They are
    // dealt to the 8 XCDs round-robin by index; re-order them so that each XCD
    // owns a contiguous run of (split, tile) pairs, split-major: an XCD then
    // works on ONE slice of the reduction, and that slice of both operands
    // (a few MB) stays in its own L2 while all its tiles sweep over it.
    int g = bx;
    if (p.xcd_remap) {
      const int per = nbx >> 3;
      g = (bx & 7) * per + (bx >> 3);
    }
    const int tiles = tiles_m * tiles_n;
    split = g / tiles;
    tile = g - split * tiles;
  }
  // tile_n major: consecutive tiles share the same rows of B
  const int tile_n = (MODE == MODE_WGRAD) ? tile % tiles_n : tile / tiles_m;
  const int tile_m = (MODE == MODE_WGRAD) ? tile / tiles_n : tile % tiles_m;
  const int row0 = tile_m * kTile, col0 = tile_n * kTile;
  const int wrow = (wave >> 1) * 32, wcol = (wave & 1) * 32;

  // The reduction is a stream of slabs over one or more consecutive ranges
  // ("workers"); the accumulator is flushed whenever a range ends.  A slab is
  // (range index w, start k0, end of its range kend); w == nrange marks the end.
  const int nrange = (MODE == MODE_WGRAD) ? p.gfirst[by + 1] : 1;
  int w0 = 0, k00, kend0;
  if (MODE == MODE_WGRAD) {
    w0 = p.gfirst[by];
    k00 = seg.off[w0];
    kend0 = seg.off[w0 + 1];
  } else {
    const int slabs = (p.kred + BK - 1) / BK;
    const int per = (slabs + splits - 1) / splits;
    k00 = min(split * per * BK, p.kred);
    kend0 = min((split + 1) * per * BK, p.kred);
  }
#define OMNI_NEXT_SLAB(W, K0, KEND, NW, NK0, NKEND)       \
  int NW = W, NK0 = K0 + BK, NKEND = KEND;                \
  if (NK0 >= KEND) {                                      \
    NW = W + 1;                                           \
    if (MODE == MODE_WGRAD && NW < nrange) {              \
      NK0 = seg.off[NW];                                  \
      NKEND = seg.off[NW + 1];                            \
    }                                                     \
  }

  // Two accumulator chains (even / odd reduction steps) keep consecutive MFMAs independent.
  v16f acc, acc2;
#pragma unroll
  for (int v = 0; v < 16; ++v) acc[v] = acc2[v] = 0.f;
  const bool want_bias_grad = (MODE == MODE_WGRAD) && p.bias_grad != nullptr && tile_n == 0;
  float bsum = 0.f;

  // Accumulator layout of the 32x32 block: register v of lane l holds
  // row 8*(v/4) + 4*(l/32) + v%4, column l%32.
  const int j = col0 + wcol + (lane & 31);
  const int ibase = row0 + wrow + 4 * (lane >> 5);

  // Two register sets hold the slabs one and two steps ahead of the one being
  // multiplied, so every global load has two MFMA sections to arrive in.
  const typename SA::Pre preA = SA::prepare(p.lda, row0, p.M, tid);
  const typename SB::Pre preB = SB::prepare(p.ldb, col0, p.N, tid);
  v4f ra0[SA::kPerThread], rb0[SB::kPerThread], ra1[SA::kPerThread], rb1[SB::kPerThread];
  uint32_t oka0 = 0, okb0 = 0, oka1 = 0, okb1 = 0;
  OMNI_NEXT_SLAB(w0, k00, kend0, w1, k01, kend1)
  // start of the slab as it is fetched (see Slab::load_fast)
#define OMNI_KSTART(K0, KEND) ((K0) + BK <= (KEND) ? (K0) : max((KEND) - BK, 0))
  // Prefetches past the end of the stream are still issued (they re-read the
  // first slab and are discarded): a load that is issued on one path only would force
  // every later wait to assume it is not there and drain the whole queue.
  if (w1 >= nrange) { k01 = 0; kend1 = 0; }
  if (VEC) {
    SA::load_fast(ra0, p.A, p.lda, OMNI_KSTART(k00, kend0), preA);
    SB::load_fast(rb0, p.B, p.ldb, OMNI_KSTART(k00, kend0), preB);
    SA::load_fast(ra1, p.A, p.lda, OMNI_KSTART(k01, kend1), preA);
    SB::load_fast(rb1, p.B, p.ldb, OMNI_KSTART(k01, kend1), preB);
#pragma unroll
    for (int i = 0; i < SA::kPerThread; ++i) SA::store_fast(ra0, sA(0), tid, i);
#pragma unroll
    for (int i = 0; i < SB::kPerThread; ++i) SB::store_fast(rb0, sB(0), tid, i);
    if (k00 + BK > kend0) {
      const int ks = OMNI_KSTART(k00, kend0);
      __syncthreads();
      SA::zero_outside(sA(0), k00 - ks, kend0 - ks, tid);
      SB::zero_outside(sB(0), k00 - ks, kend0 - ks, tid);
    }
  } else {
    SA::template load<VEC>(ra0, oka0, p.A, p.lda, row0, p.M, k00, kend0, tid, preA);
    SB::template load<VEC>(rb0, okb0, p.B, p.ldb, col0, p.N, k00, kend0, tid, preB);
    SA::template load<VEC>(ra1, oka1, p.A, p.lda, row0, p.M, k01, kend1, tid, preA);
    SB::template load<VEC>(rb1, okb1, p.B, p.ldb, col0, p.N, k01, kend1, tid, preB);
    SA::template store<VEC>(ra0, oka0, sA(0), tid);
    SB::template store<VEC>(rb0, okb0, sB(0), tid);
  }
  __syncthreads();

  // One pipeline step: multiply slab 0 (already in LDS stage CUR, a constant of each of the two
  // copies of the step, so that every LDS address is an immediate offset), fetch the
  // slab two ahead into the free register set (LA/LB), then move the slab one
  // ahead from its register set (NA/NB) into the other LDS stage.
#define OMNI_STEP(CUR, LA, LB, LOKA, LOKB, NA, NB, NOKA, NOKB)                                               \
  {                                                                                                     \
    int w2 = nrange, k02 = 0, kend2 = 0;                                                                \
    if (w1 < nrange) {                                                                                  \
      OMNI_NEXT_SLAB(w1, k01, kend1, tw, tk0, tkend)                                                    \
      w2 = tw; k02 = tk0; kend2 = tkend;                                                                \
    }                                                                                                   \
    if (w2 >= nrange) { k02 = 0; kend2 = 0; }                                                           \
    if (VEC) {                                                                                          \
      const int ks2 = OMNI_KSTART(k02, kend2);                                                          \
      SA::load_fast(LA, p.A, p.lda, ks2, preA);                                                         \
      SB::load_fast(LB, p.B, p.ldb, ks2, preB);                                                         \
    } else {                                                                                            \
      SA::template load<VEC>(LA, LOKA, p.A, p.lda, row0, p.M, k02, kend2, tid, preA);                    \
      SB::template load<VEC>(LB, LOKB, p.B, p.ldb, col0, p.N, k02, kend2, tid, preB);                    \
    }                                                                                                   \
    __builtin_amdgcn_sched_barrier(0); /* keep the fetches ahead of the MFMA section */                 \
    /* The slab one step ahead has been in flight for a whole step: its pieces go to the other LDS */  \
    /* stage in between the MFMA groups of this slab, and the operand fragments of the next group   */  \
    /* are fetched before the current group is issued, so that the matrix pipe is not left waiting. */  \
    {                                                                                                   \
      v4f fa[2], fb[2];                                                                                 \
      fa[0] = SA::frag(sA(CUR), wrow, 0, lane);                                                         \
      fb[0] = SB::frag(sB(CUR), wcol, 0, lane);                                                         \
      _Pragma("unroll") for (int ks = 0; ks < BK / 8; ++ks) {                                           \
        if (ks + 1 < BK / 8) {                                                                          \
          fa[(ks + 1) & 1] = SA::frag(sA(CUR), wrow, ks + 1, lane);                                     \
          fb[(ks + 1) & 1] = SB::frag(sB(CUR), wcol, ks + 1, lane);                                     \
        }                                                                                               \
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[ks & 1][0], fb[ks & 1][0], acc, 0, 0, 0);         \
        acc2 = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[ks & 1][1], fb[ks & 1][1], acc2, 0, 0, 0);       \
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[ks & 1][2], fb[ks & 1][2], acc, 0, 0, 0);         \
        acc2 = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[ks & 1][3], fb[ks & 1][3], acc2, 0, 0, 0);       \
        if (VEC) {                                                                                      \
          if (ks < SA::kPerThread) SA::store_fast(NA, sA(1 - CUR), tid, ks);                            \
          else if (ks - SA::kPerThread < SB::kPerThread) SB::store_fast(NB, sB(1 - CUR), tid, ks - SA::kPerThread); \
        } else {                                                                                        \
          if (ks < SA::kPerThread) SA::template store_one<VEC>(NA, NOKA, sA(1 - CUR), tid, ks);         \
          else if (ks - SA::kPerThread < SB::kPerThread)                                                \
            SB::template store_one<VEC>(NB, NOKB, sB(1 - CUR), tid, ks - SA::kPerThread);               \
        }                                                                                               \
        __builtin_amdgcn_sched_barrier(0);                                                              \
      }                                                                                                 \
    }                                                                                                   \
    if (VEC && w1 < nrange && k01 + BK > kend1) {                                                       \
      /* the slab just staged runs past the end of its range: it was fetched moved back; clear the */  \
      /* reduction steps that are not its own (once per range; all its pieces must have landed)     */  \
      const int ks1 = OMNI_KSTART(k01, kend1);                                                          \
      __syncthreads();                                                                                  \
      SA::zero_outside(sA(1 - CUR), k01 - ks1, kend1 - ks1, tid);                                       \
      SB::zero_outside(sB(1 - CUR), k01 - ks1, kend1 - ks1, tid);                                       \
    }                                                                                                   \
    if (want_bias_grad) {                                                                               \
      /* A is the output-gradient slab [kk][row]: its column sums are the bias gradient.  Each */       \
      /* wavefront adds a quarter of the slab's reduction steps; the quarters meet at the flush. */     \
      _Pragma("unroll") for (int kk = 0; kk < BK / 4; ++kk)                                             \
        bsum += sA(CUR)[(wave * (BK / 4) + kk) * SA::kStride + lane];                                   \
    }                                                                                                   \
    if (MODE == MODE_WGRAD && w1 != w0) {                                                               \
      /* this worker's rows are done: its tile goes out (stores only; the prefetch stays in flight) */ \
      float* C = p.C + (size_t)w0 * p.c_worker_stride;                                                  \
      if (VEC && p.c_vec) {                                                                             \
        /* through the LDS stage that was just multiplied, so that every thread writes 16-byte pieces */ \
        /* of whole 256-byte rows (scattered 4-byte stores, 16 per lane, cost 3 us per launch)        */ \
        float* tile = sA(CUR);                                                                          \
        __syncthreads(); /* every wavefront is done reading this stage */                               \
        _Pragma("unroll") for (int v = 0; v < 16; ++v)                                                  \
          tile[(wrow + 4 * (lane >> 5) + 8 * (v / 4) + (v % 4)) * kFlushStride + wcol + (lane & 31)] = acc[v] + acc2[v]; \
        if (want_bias_grad) bred[wave][lane] = bsum;                                                    \
        __syncthreads();                                                                                \
        _Pragma("unroll") for (int q = 0; q < 4; ++q) {                                                 \
          const int idx = tid + kThreads * q, r = idx >> 4, c4 = (idx & 15) * 4;                         \
          if (row0 + r < p.M && col0 + c4 < p.N)                                                        \
            *reinterpret_cast<v4f*>(C + (size_t)(row0 + r) * p.ldc + col0 + c4) =                       \
                *reinterpret_cast<const v4f*>(tile + r * kFlushStride + c4);                            \
        }                                                                                               \
      } else {                                                                                          \
        if (j < p.N) {                                                                                  \
          _Pragma("unroll") for (int v = 0; v < 16; ++v) {                                              \
            const int i = ibase + 8 * (v / 4) + (v % 4);                                                \
            if (i < p.M) C[(size_t)i * p.ldc + j] = acc[v] + acc2[v];                                   \
          }                                                                                             \
        }                                                                                               \
        if (want_bias_grad) {                                                                           \
          bred[wave][lane] = bsum;                                                                      \
          __syncthreads();                                                                              \
        }                                                                                               \
      }                                                                                                 \
      if (want_bias_grad && tid < kTile && row0 + tid < p.M)                                            \
        p.bias_grad[(size_t)w0 * p.c_worker_stride + row0 + tid] =                                      \
            ((bred[0][tid] + bred[1][tid]) + bred[2][tid]) + bred[3][tid];                              \
      bsum = 0.f;                                                                                       \
      _Pragma("unroll") for (int v = 0; v < 16; ++v) acc[v] = acc2[v] = 0.f;                            \
    }                                                                                                   \
    if (w1 >= nrange) break;                                                                            \
    __syncthreads();                                                                                    \
    w0 = w1; k00 = k01; kend0 = kend1;                                                                  \
    w1 = w2; k01 = k02; kend1 = kend2;                                                                  \
  }
  for (;;) {
    OMNI_STEP(0, ra0, rb0, oka0, okb0, ra1, rb1, oka1, okb1)
    OMNI_STEP(1, ra1, rb1, oka1, okb1, ra0, rb0, oka0, okb0)
  }
#undef OMNI_STEP
#undef OMNI_NEXT_SLAB
#undef OMNI_KSTART

  if (MODE != MODE_WGRAD) {
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[v] += acc2[v];
    bool finish = true;
    if (splits > 1) {
      // Park this split's partial tile; whoever arrives last adds them up.  The
      // splits of a tile may run on different XCDs, whose L2s are not coherent
      // with each other inside a kernel.  The partial tiles therefore travel
      // through device-scope stores and loads (they bypass the XCD-private L2);
      // every thread drains its own stores, the barrier collects the workgroup,
      // and ONE wavefront then executes the device-scope release (an L2
      // write-back: done by all four wavefronts, or paired with an acquire that
      // invalidates the L2 under everybody else's feet, it cost 25 % of the
      // step) before one thread bumps the tile's arrival counter.  Without that
      // release the counter could overtake the data (seen as rare wrong tiles).
      float* mine = p.partial + ((size_t)tile * splits + split) * (16 * kThreads);
#pragma unroll
      for (int v = 0; v < 16; ++v)
        __hip_atomic_store(mine + v * kThreads + tid, acc[v], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
      __syncthreads();
      if (wave == 0) {
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
        if (tid == 0)
          arrival = __hip_atomic_fetch_add(&p.counters[tile], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
      __syncthreads();
      finish = (arrival == (uint32_t)splits - 1);
      if (finish) {
        const float* all = p.partial + (size_t)tile * splits * (16 * kThreads);
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[v] = 0.f;
        for (int s = 0; s < splits; ++s)
#pragma unroll
          for (int v = 0; v < 16; ++v)
            acc[v] += __hip_atomic_load(all + ((size_t)s * 16 + v) * kThreads + tid, __ATOMIC_RELAXED,
                                        __HIP_MEMORY_SCOPE_AGENT);
        if (tid == 0) p.counters[tile] = 0u;   // ready for the next launch
      }
    }
    if (finish && j < p.N) {
      float bj = 0.f;
      if (MODE == MODE_FWD && p.bias) bj = p.bias[j];
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int i = ibase + 8 * (v / 4) + (v % 4);
        if (i >= p.M) continue;
        float val = acc[v];
        const size_t idx = (size_t)i * p.ldc + j;
        if (MODE == MODE_FWD) {
          val += bj;
          if (p.relu) val = val > 0.f ? val : 0.f;
        } else {
          if (p.mask) val = p.mask[idx] > 0.f ? val : 0.f;
          if (p.accumulate) val += p.C[idx];
        }
        p.C[idx] = val;
      }
    }
  }
}

template <int BK, bool A_MC, bool B_MC, int MODE, bool VEC>
__global__ __launch_bounds__(kThreads, MODE == MODE_WGRAD ? 3 : 2) void gemm_f32_kernel(GemmParams p, Segments seg) {
  gemm_f32_body<BK, A_MC, B_MC, MODE, VEC>(p, seg, (int)blockIdx.x, (int)blockIdx.y, (int)gridDim.x);
}

// Weight gradients of several layers in ONE launch: the workgroups of the problems follow each other
// along x (problem i owns start[i] .. start[i+1]-1, tiles fastest, then worker groups).  A launch
// has a start-up and a drain during which the matrix pipes idle; run together, one problem's
// workgroups start while another's finish.
constexpr int kMaxBatch = 8;
struct WgradBatch {
  int n;
  int start[kMaxBatch + 1];
  GemmParams prob[kMaxBatch];
};

template <int BK, bool VEC>
__global__ __launch_bounds__(kThreads, 3) void gemm_f32_wgrad_batch_kernel(WgradBatch b, Segments seg) {
  int pi = 0;
  for (int i = 1; i < b.n; ++i)
    if ((int)blockIdx.x >= b.start[i]) pi = i;
  const GemmParams& p = b.prob[pi];
  const int local = (int)blockIdx.x - b.start[pi];
  const int tiles = ((p.M + kTile - 1) / kTile) * ((p.N + kTile - 1) / kTile);
  const int by = local / tiles;
  gemm_f32_body<BK, true, true, MODE_WGRAD, VEC>(p, seg, local - by * tiles, by, tiles);
}

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Deals the workers of a weight-gradient problem to workgroups per tile (p.gfirst, p.ngroups):
// with few tiles, groups of consecutive workers with about equal row counts (each worker stays
// whole, so nothing is summed across workgroups).  `want` is the number of workgroups to aim for.
int plan_worker_groups(GemmParams& p, const Segments& seg, int tiles, int want) {
  int G = tiles >= want ? 1 : std::min(std::min(8, seg.K), (want + tiles - 1) / tiles);
  const int B = seg.off[seg.K];
  p.gfirst[0] = 0;
  int g = 1;
  for (int w = 1; w < seg.K && g < G; ++w) {
    // start group g at the first worker whose start reaches g/G of the rows (keeping every later group non-empty)
    if ((long)seg.off[w] * G >= (long)g * B || seg.K - w <= G - g) p.gfirst[g++] = w;
  }
  G = g;
  p.gfirst[G] = seg.K;
  p.ngroups = G;
  return G;
}

template <int BK, bool A_MC, bool B_MC, int MODE>
void launch(hipStream_t st, GemmParams& p, const Segments& seg, int splits, bool vec) {
  const int tiles = ((p.M + kTile - 1) / kTile) * ((p.N + kTile - 1) / kTile);
  p.splits = splits;
  p.xcd_remap = (MODE != MODE_WGRAD && (tiles * splits) % 8 == 0) ? 1 : 0;
  dim3 grid(tiles * splits, 1, 1);
  if (MODE == MODE_WGRAD) grid = dim3(tiles, plan_worker_groups(p, seg, tiles, 512), 1);
  if (vec)
    hipLaunchKernelGGL((gemm_f32_kernel<BK, A_MC, B_MC, MODE, true>), grid, dim3(kThreads), 0, st, p, seg);
  else
    hipLaunchKernelGGL((gemm_f32_kernel<BK, A_MC, B_MC, MODE, false>), grid, dim3(kThreads), 0, st, p, seg);
}

// Number of reduction splits that brings a forward / dgrad launch to roughly two
// workgroups per compute unit, never leaving a split without at least 4 slabs.
int pick_splits(int tiles, int kred, int bk, const SplitWorkspace& sw) {
  if (!sw.partial || !sw.counters || tiles > kSplitMaxTiles) return 1;
  int s = (512 + tiles - 1) / tiles;
  const int slabs = (kred + bk - 1) / bk;
  s = std::min(s, std::max(1, slabs / 4));
  s = std::min(s, 16);
  while (s > 1 && (size_t)tiles * s * 16 * kThreads > kSplitPartialFloats) --s;
  // every split must own at least one slab
  while (s > 1 && ((slabs + s - 1) / s) * (s - 1) >= slabs) --s;
  return std::max(s, 1);
}

}  // namespace

static int gemm_tiles(int rows, int cols) { return ((rows + kTile - 1) / kTile) * ((cols + kTile - 1) / kTile); }

void linear_fwd_f32(hipStream_t st, const float* x, const float* w, const float* bias, float* y,
                    int rows, int cin, int cout, bool relu, const SplitWorkspace& sw) {
  if (linear_fwd_f32_direct(st, x, w, bias, y, rows, cin, cout, relu)) return;
  GemmParams p{};
  p.A = x; p.B = w; p.C = y; p.M = rows; p.N = cout; p.lda = cin; p.ldb = cin; p.ldc = cout;
  p.kred = cin; p.bias = bias; p.relu = relu ? 1 : 0;
  p.partial = sw.partial; p.counters = sw.counters;
  Segments seg{};
  // both operands k-contiguous; the mask-free loads need at least one whole slab of reduction steps
  const bool vec = aligned16(x) && aligned16(w) && (cin % 4 == 0) && cin >= 32;
  launch<32, false, false, MODE_FWD>(st, p, seg, pick_splits(gemm_tiles(rows, cout), cin, 32, sw), vec);
}

void linear_dgrad_f32(hipStream_t st, const float* dy, const float* w, const float* mask, float* dx,
                      int rows, int cin, int cout, bool accumulate, const SplitWorkspace& sw) {
  if (linear_dgrad_f32_direct(st, dy, w, mask, dx, rows, cin, cout, accumulate)) return;
  GemmParams p{};
  p.A = dy; p.B = w; p.C = dx; p.M = rows; p.N = cin; p.lda = cout; p.ldb = cin; p.ldc = cin;
  p.kred = cout; p.mask = mask; p.accumulate = accumulate ? 1 : 0;
  p.partial = sw.partial; p.counters = sw.counters;
  Segments seg{};
  const bool vec = aligned16(dy) && aligned16(w) && (cout % 4 == 0) && (cin % 4 == 0) && cout >= 32;
  launch<32, false, true, MODE_DGRAD>(st, p, seg, pick_splits(gemm_tiles(rows, cin), cout, 32, sw), vec);
}

static bool wgrad_params(GemmParams& p, const LinearWgradJob& j, size_t worker_stride, const Segments& seg) {
  p = GemmParams{};
  p.A = j.dy; p.B = j.x; p.C = j.gw; p.M = j.cout; p.N = j.cin; p.lda = j.cout; p.ldb = j.cin; p.ldc = j.cin;
  p.c_worker_stride = worker_stride; p.bias_grad = j.gb;
  p.c_vec = (aligned16(j.gw) && j.cin % 4 == 0 && worker_stride % 4 == 0) ? 1 : 0;
  return aligned16(j.dy) && aligned16(j.x) && (j.cout % 4 == 0) && (j.cin % 4 == 0) && seg.off[seg.K] >= 32;
}

void linear_wgrad_f32(hipStream_t st, const float* dy, const float* x, float* gw, float* gb,
                      size_t worker_stride, const Segments& seg, int cin, int cout) {
  GemmParams p;
  const LinearWgradJob job{dy, x, gw, gb, cin, cout};
  const bool vec = wgrad_params(p, job, worker_stride, seg);
  launch<32, true, true, MODE_WGRAD>(st, p, seg, 1, vec);
}

void linear_wgrad_f32_batch(hipStream_t st, const LinearWgradJob* jobs, int n, size_t worker_stride,
                            const Segments& seg, const KernelTimer* timer) {
  // problems that can take the mask-free loads share launches of up to kMaxBatch; the others go alone
  WgradBatch b{};
  // exact timing needs everything in ONE launch of the shared kernel; otherwise the events go around the launches
  bool one_launch = n >= 2 && n <= kMaxBatch;
  for (int i = 0; i < n && one_launch; ++i) {
    GemmParams p;
    one_launch = wgrad_params(p, jobs[i], worker_stride, seg);
  }
  const bool bracket = timer && !one_launch;
  if (bracket) (void)hipEventRecord(timer->start, st);
  auto flush = [&]() {
    if (b.n == 1) {
      GemmParams p = b.prob[0];
      launch<32, true, true, MODE_WGRAD>(st, p, seg, 1, true);
    } else if (b.n > 1) {
      if (timer && one_launch)
        hipExtLaunchKernelGGL((gemm_f32_wgrad_batch_kernel<32, true>), dim3(b.start[b.n]), dim3(kThreads), 0, st,
                              timer->start, timer->stop, 0, b, seg);
      else
        hipLaunchKernelGGL((gemm_f32_wgrad_batch_kernel<32, true>), dim3(b.start[b.n]), dim3(kThreads), 0, st, b, seg);
    }
    b.n = 0;
  };
  for (int i = 0; i < n; ++i) {
    GemmParams p;
    if (!wgrad_params(p, jobs[i], worker_stride, seg)) {
      launch<32, true, true, MODE_WGRAD>(st, p, seg, 1, false);
      continue;
    }
    const int tiles = gemm_tiles(p.M, p.N);
    const int G = plan_worker_groups(p, seg, tiles, 512);
    b.start[b.n + 1] = b.start[b.n] + tiles * G;
    b.prob[b.n++] = p;
    if (b.n == kMaxBatch) flush();
  }
  flush();
  if (bracket) (void)hipEventRecord(timer->stop, st);
}

}  // namespace omni
