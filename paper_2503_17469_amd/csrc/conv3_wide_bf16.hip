// Forward and stride-1 input gradient of 3x3 / pad-1 convolutions in bf16 (fp32 accumulation): the
// wide-tile variant of the patch-resident implicit GEMM (same contraction as conv_bf16.hip's kernel D:
// the inner F(.) of the gradient line of procedure Train, Algorithm 1).
//
//   out[m][co] = sum_{u,v,ci} src[n, h+u-1, w+v-1, ci] * wgt[co][u][v][ci]        (dgrad: taps mirrored)
//
// What limits the 256-position kernel is not a unit but waiting: two workgroups per compute unit leave
// 256 registers per lane, all taken by accumulators, the patch on its way to LDS and one set of
// fragments, so every group of four matrix instructions waits for its own fragment reads, and every
// filter tap for a barrier and for the weight slab that was requested one tap earlier.  Here:
//
//   * one workgroup per compute unit, one wavefront per SIMD, 512 registers per lane;
//   * a workgroup owns 512 positions x 64 output channels, a wavefront 128 x 64: 8 matrix instructions
//     per 6 fragment reads (0.75 KB of LDS per instruction instead of 1 KB) and 256 matrix cycles per
//     step of 16 reduction elements, under which the NEXT step's fragments are read (two register sets);
//   * the reduction is staged 32 channels at a time, and a slice brings its patch AND the weights of all
//     nine taps (9 x 64 x 32) into LDS together: no barrier and no wait inside a slice of 144 matrix
//     instructions per wavefront.  With one wavefront per SIMD nothing but distance hides memory
//     latency, and the memory counter retires loads in order: weight slabs requested tap by tap, in
//     between the loads of the next patch, waited for those as well (about 1 us per tap, measured).
//     All loads of the next slice are issued together when a slice begins and are first needed when it
//     ends (4608 matrix cycles later), where two barriers separate the last fragment read from the stores
//     that replace patch and weights;
//   * the product is formed TRANSPOSED (weights as the left operand): a lane then holds, for one
//     position, runs of four consecutive channels; one swap of the wavefront's halves per register pair
//     turns them into runs of eight, and the lane writes 16-byte pieces of the output row itself --
//     no staging of the output tile through LDS.
//
// Pooling in the epilogue (which needs the whole tile side by side) stays with the 256-position kernel.
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
constexpr int kTN = 64;           // output channels per workgroup
constexpr int kLdsLimit = 160 * 1024;

struct WideParams {
  const bf16_t* src;   // [rows][H][W][Cs]
  const bf16_t* wgt;   // [N][9][Cs]
  bf16_t* out;         // [rows*H*W][N]
  int rows, H, W, Cs, N;
  int R, nimg;         // a unit is nimg images x R rows; nimg * R * W = 512
  int units, upw;      // units in all, units per workgroup
  int flip;            // 1: dgrad (mirrored taps)
  const void* zero;    // zeros for absent pieces
  const float* bias;
  const bf16_t* mask;     // [rows*H*W][N] or null: the value passes where mask > 0
  const uint8_t* mask_bits;   // BITS: [rows*H*W][N/8], the mask at one bit per element (N a multiple of 64)
  const bf16_t* addend;   // [rows*H*W][N] or null: added to the product before the mask
  int relu, accumulate;
  // Workgroup g (after the XCD mapping below) takes units of ONE entry of this table: entry k owns the units
  // ufirst[k] .. ufirst[k+1]-1 and the groups gfirst[k] .. gfirst[k+1]-1 of upw units each.  One entry that
  // spans everything, or one per worker when the layer's batch-norm sums are wanted (a group's sums then
  // belong to one worker).
  int gK;
  int32_t gfirst[OMNI_MAX_WORKERS + 1], ufirst[OMNI_MAX_WORKERS + 1];
  double* stat_partial;   // STATS: [group][N][2] sums of the stored output and of its squares
};

__device__ inline bf16x8 as_bf16x8(u32x4 v) { return __builtin_bit_cast(bf16x8, v); }

// NP: 16-byte patch pieces per thread.  W8: maps 8 wide (the wavefront takes the map rows of every 64
// positions in the order 0 4 1 5 2 6 3 7: rows 4 apart are complementary in the LDS banks, neighbours are
// not).  BWD: mask / addend / accumulate in the epilogue.
constexpr int KC = 32;            // reduction channels per slice
constexpr int kRow = KC + 8;      // elements per LDS row (80 bytes): sixteen 16-byte reads of consecutive rows cover all banks
constexpr int OC = KC / 8;        // 16-byte pieces per patch position and per weight row
constexpr int KK = KC / 16;       // reduction steps per tap
static_assert(kTN * OC == kThreads, "one weight piece per thread and tap");

// One step of the statistics tree: the lane keeps half of its list (the upper half if bit DIST of its index
// is set) and adds what its partner, DIST lanes away, holds of the same half.
template <int DIST, int N, int LEN>
__device__ inline void stat_exchange(float (&sv)[LEN], int j) {
  if constexpr (LEN >= 2 * N) {
    const bool upper = (j & DIST) != 0;
#pragma unroll
    for (int i = 0; i < N; ++i) {
      const float keep = upper ? sv[N + i] : sv[i];
      const float send = upper ? sv[i] : sv[N + i];
      // ds_swizzle in bit-mask mode (groups of 32 lanes): the value comes from lane ^ DIST
      const float recv = __int_as_float(__builtin_amdgcn_ds_swizzle(__float_as_int(send), (DIST << 10) | 0x1F));
      sv[i] = keep + recv;
    }
  }
}

// MA: 32-position blocks per wavefront: 4 (a unit of 512 positions, one workgroup per compute unit) or 2 (256
// positions, two workgroups per compute unit, whose load, store and compute phases overlap each other's).
// STATS (forward, MA = 2, no bias, no ReLU): the per-channel sums of the group's stored outputs and of their
// squares go to p.stat_partial, the first pass of the batch norm that follows, without reading the tensor back.
// BITS (input gradient): the ReLU mask is read as one bit per element, 8 bytes per position and channel tile
// instead of 128.
template <int MA, int NP, bool W8, bool BWD, bool STATS = false, bool BITS = false>
__global__ __launch_bounds__(kThreads, MA == 4 ? 1 : 2) void conv3_wide_kernel(WideParams p) {
  static_assert(!STATS || (MA == 2 && !BWD), "statistics come with the forward 256-position unit only");
  static_assert(!BITS || BWD, "mask bits belong to the input gradient");
  constexpr int WPOS = 32 * MA;   // positions per wavefront
  extern __shared__ __attribute__((aligned(16))) unsigned char smemW[];
  const int W = p.W, H = p.H, R = p.R;
  const int PW = W + 2, PR = R + 2;
  const int npatch = p.nimg * PR * PW;
  bf16_t* sP = reinterpret_cast<bf16_t*>(smemW);          // [npatch][kRow]
  bf16_t* sW = sP + (size_t)npatch * kRow;                // [9][64][kRow]
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int j = lane & 31, h = lane >> 5;
  const int tiles_n = (p.N + kTN - 1) / kTN;
  // Workgroups are dealt to the 8 XCDs round-robin by index, and every XCD has an L2 of its own.  The
  // channel tiles of one group of units all read the same patches: they must run on ONE XCD, next to each
  // other in time, or every patch crosses the fabric once per channel tile (at 512 channels: eight times).
  // Workgroup b runs on XCD b % 8; there it is the (b / 8)-th: channel tile fastest, then the XCD's groups.
  const int on_xcd = blockIdx.x >> 3;
  const int tile_n = on_xcd % tiles_n;
  const int group = (on_xcd / tiles_n) * 8 + (blockIdx.x & 7);
  if (group >= p.gfirst[p.gK]) return;   // (the grid is rounded up to whole rounds of 8 groups)
  int gk = 0;
  while (gk + 1 < p.gK && group >= p.gfirst[gk + 1]) ++gk;
  const int col0 = tile_n * kTN;
  const int K = 9 * p.Cs;
  const int ubeg = p.ufirst[gk] + (group - p.gfirst[gk]) * p.upw, uend = min(p.ufirst[gk + 1], ubeg + p.upw);
  const int nslice = p.Cs / KC;

  // ---- patch staging tasks: piece x = tid + 256 t -> patch position x / OC, channel octet x % OC
  int prel[NP];
  uint32_t col_ok = 0, top = 0, bottom = 0;
  uint32_t img8[(NP + 3) / 4];
#pragma unroll
  for (int t = 0; t < (NP + 3) / 4; ++t) img8[t] = 0;
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
    img8[t / 4] |= (uint32_t)il << (8 * (t % 4));
  }
  // ---- weight staging: this thread carries row tid / OC, octet tid % OC of every tap's slab
  const int wrow = tid / OC, woct = tid % OC;
  const bool wvalid = col0 + wrow < p.N;
  const long woff = wvalid ? (long)(col0 + wrow) * K + woct * 8 : 0;
  bf16_t* const wdst = sW + wrow * kRow + woct * 8;
  // ---- fragment addresses: this wavefront's positions wave*128 + a*32 + j
  auto row_order = [](int t) { return (t >> 1) + 4 * (t & 1); };   // t: 0..7
  int pbase[MA], ipos[MA];
#pragma unroll
  for (int a = 0; a < MA; ++a) {
    int pos = wave * WPOS + a * 32 + j;
    if (W8) pos = wave * WPOS + (a >> 1) * 64 + row_order((a & 1) * 4 + (j >> 3)) * 8 + (j & 7);
    ipos[a] = pos;
    const int rr = pos / W, w = pos - rr * W;
    const int il = rr / R, r = rr - il * R;
    pbase[a] = ((il * PR + r) * PW + w) * kRow + h * 8;   // patch origin is (-1, -1): tap (u, v) adds u*PW + v
  }
  const bf16_t* const wfrag = sW + j * kRow + h * 8;

  const bf16_t* const zp = static_cast<const bf16_t*>(p.zero);
  u32x4 rp[NP], rw[9];
  auto unit_geom = [&](int unit, int& n0, int& r0, int& nvalid) {
    if (p.nimg == 1) {
      const int upi = H / R, img = unit / upi;
      n0 = img; r0 = (unit - img * upi) * R; nvalid = 1;
    } else {
      n0 = unit * p.nimg; r0 = 0; nvalid = min(p.nimg, p.rows - n0);
    }
  };
  // everything slice cs of `unit` needs, on its way to registers (all loads are unconditional)
  auto load_slice = [&](int unit, int cs) {
#pragma unroll
    for (int t = 0; t < 9; ++t)
      rw[t] = *reinterpret_cast<const u32x4*>(wvalid ? p.wgt + (woff + t * p.Cs + cs * KC) : zp);
    int n0, r0, nvalid;
    unit_geom(unit, n0, r0, nvalid);
    const int ubase = (n0 * H + r0) * W * p.Cs + cs * KC;
    const uint32_t pvalid = col_ok & ~(r0 == 0 ? top : 0u) & ~(r0 + R == H ? bottom : 0u);
#pragma unroll
    for (int t = 0; t < NP; ++t) {
      const int il = (int)(img8[t / 4] >> (8 * (t % 4))) & 255;
      const bool in = ((pvalid >> t) & 1u) && il < nvalid;
      rp[t] = *reinterpret_cast<const u32x4*>(in ? p.src + (ubase + prel[t]) : zp);
    }
  };
  auto store_slice = [&]() {
#pragma unroll
    for (int t = 0; t < 9; ++t) *reinterpret_cast<u32x4*>(wdst + t * kTN * kRow) = rw[t];
#pragma unroll
    for (int t = 0; t < NP; ++t) {
      const int x = tid + t * kThreads;
      if (x < npieces) *reinterpret_cast<u32x4*>(sP + (x / OC) * kRow + (x % OC) * 8) = rp[t];
    }
  };

  load_slice(min(ubeg, p.units - 1), 0);
  store_slice();
  __syncthreads();

  double stat_sum[2] = {0.0, 0.0};   // STATS: this lane's two (channel, moment) pairs over the group's units, see below

  for (int unit = ubeg; unit < uend; ++unit) {
    int n0, r0, nvalid;
    unit_geom(unit, n0, r0, nvalid);
    const long out_base = ((long)n0 * H + r0) * W;   // the unit's positions are contiguous rows of `out`
    const int npos = nvalid * R * W;                 // live positions of this unit

    v16f acc[MA][2];
#pragma unroll
    for (int a = 0; a < MA; ++a)
#pragma unroll
      for (int b = 0; b < 2; ++b)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.f;

    // epilogue operands of the input gradient (mask; addend or the old output), one 16-byte piece per (b, half)
    // of a block row a, in two sets.  MA = 4: the first set is fetched during the last taps, the others one
    // block row ahead.  MA = 2 (256 registers per lane): a full set that is live inside the tap loop spills, so
    // both block rows are fetched when the loop has ended and the other workgroup's matrix instructions cover the
    // wait; with the mask as bits a set is 18 registers instead of 32 and the first one does travel under the
    // last taps (except on 8-wide maps, where the seventh patch piece takes the room).
    constexpr int ESETS = 2;
    u32x4 em[ESETS][BWD && !BITS ? 4 : 1], ea[ESETS][BWD ? 4 : 1];
    u32x2 eb[ESETS];   // BITS: the mask bits of the tile's 64 channels at this lane's position (byte b*4 + q*2 + h: piece (b, q))
    auto load_epi = [&](int a, int set) {
      if (BITS) {
        const bool in = ipos[a] < npos;
        eb[set] = *reinterpret_cast<const u32x2*>(
            in ? p.mask_bits + ((size_t)(out_base + ipos[a]) * (p.N >> 3) + (col0 >> 3))
               : static_cast<const uint8_t*>(p.zero));
      }
#pragma unroll
      for (int b = 0; b < 2; ++b)
#pragma unroll
        for (int q = 0; q < 2; ++q) {
          const int c = col0 + b * 32 + q * 16 + h * 8;
          const bool in = ipos[a] < npos && c < p.N;
          const size_t idx = (size_t)(out_base + ipos[a]) * p.N + c;
          if (!BITS) em[set][b * 2 + q] = *reinterpret_cast<const u32x4*>((in && p.mask) ? p.mask + idx : zp);
          const bf16_t* other = p.addend ? p.addend : (p.accumulate ? p.out : nullptr);
          ea[set][b * 2 + q] = *reinterpret_cast<const u32x4*>((in && other) ? other + idx : zp);
        }
    };

    for (int cs = 0; cs < nslice; ++cs) {
      const bool last_slice = cs + 1 == nslice;
      // the next slice (of this unit, or the first of the next unit) sets out now: it is needed when this one ends
      load_slice(last_slice ? min(unit + 1, uend - 1) : unit, last_slice ? 0 : cs + 1);
      bf16x8 fa[2][MA], fb[2][2];   // two fragment sets: one feeds the matrix pipe while the other is read
      {
        const int toff0 = (p.flip ? 2 * PW + 2 : 0) * kRow;
#pragma unroll
        for (int b = 0; b < 2; ++b) fb[0][b] = as_bf16x8(*reinterpret_cast<const u32x4*>(wfrag + b * 32 * kRow));
#pragma unroll
        for (int a = 0; a < MA; ++a) fa[0][a] = as_bf16x8(*reinterpret_cast<const u32x4*>(sP + pbase[a] + toff0));
      }
#pragma unroll
      for (int tap = 0; tap < 9; ++tap) {
        const int u = tap / 3, v = tap - u * 3;
        const int toff = (p.flip ? (2 - u) * PW + (2 - v) : u * PW + v) * kRow;
        const int un = (tap + 1) / 3, vn = (tap + 1) - un * 3;
        const int toff_next = (p.flip ? (2 - un) * PW + (2 - vn) : un * PW + vn) * kRow;
        if (BWD && (MA == 4 || (BITS && !W8)) && tap == 6 && last_slice) load_epi(0, 0);
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) {
          const int step = tap * KK + kk;
          const int cur = step & 1, nxt = cur ^ 1;
          // (read in the order of first use: both weight fragments, then the patch fragments)
          if (kk + 1 < KK) {
#pragma unroll
            for (int b = 0; b < 2; ++b)
              fb[nxt][b] = as_bf16x8(*reinterpret_cast<const u32x4*>(wfrag + (tap * kTN + b * 32) * kRow + (kk + 1) * 16));
#pragma unroll
            for (int a = 0; a < MA; ++a)
              fa[nxt][a] = as_bf16x8(*reinterpret_cast<const u32x4*>(sP + pbase[a] + toff + (kk + 1) * 16));
          } else if (tap < 8) {
#pragma unroll
            for (int b = 0; b < 2; ++b)
              fb[nxt][b] = as_bf16x8(*reinterpret_cast<const u32x4*>(wfrag + ((tap + 1) * kTN + b * 32) * kRow));
#pragma unroll
            for (int a = 0; a < MA; ++a)
              fa[nxt][a] = as_bf16x8(*reinterpret_cast<const u32x4*>(sP + pbase[a] + toff_next));
          }
          // transposed product: rows = output channels, columns = positions
#pragma unroll
          for (int a = 0; a < MA; ++a)
#pragma unroll
            for (int b = 0; b < 2; ++b)
              acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[cur][b], fa[cur][a], acc[a][b], 0, 0, 0);
          // issue order of this step: a fragment read of the next step behind each of the first matrix
          // instructions (left to itself the scheduler reads every fragment right before its use and waits)
          if (step + 1 < 9 * KK) {
#pragma unroll
            for (int i = 0; i < MA + 2; ++i) {
              __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);   // one matrix instruction
              __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);   // one LDS read
            }
            if (MA > 2) __builtin_amdgcn_sched_group_barrier(0x008, MA - 2, 0);
          }
          __builtin_amdgcn_sched_barrier(0);
        }
      }
      // the slice is done: the next one replaces patch and weights once every wavefront has read its last fragment
      __syncthreads();
      store_slice();
      __syncthreads();
    }

    // ---- epilogue, straight from registers.  Register v of block (a, b) in lane (j, h) is channel
    // b*32 + 8 (v/4) + 4 h + v%4 of position ipos[a].  Swapping registers v and v + 4 between the
    // wavefront's halves leaves lane (j, 0) with channels 0-7 (and 16-23), lane (j, 1) with 8-15 (24-31).
    constexpr bool AFFINE = !BWD && !STATS;   // bias and ReLU exist in the plain forward only
    float bias8[AFFINE ? 4 : 1][8];
    if (AFFINE && p.bias) {
#pragma unroll
      for (int bq = 0; bq < 4; ++bq) {
        const int c = min(col0 + (bq >> 1) * 32 + (bq & 1) * 16 + h * 8, p.N - 8);
        const v4f b0 = *reinterpret_cast<const v4f*>(p.bias + c), b1 = *reinterpret_cast<const v4f*>(p.bias + c + 4);
#pragma unroll
        for (int e = 0; e < 4; ++e) { bias8[bq][e] = b0[e]; bias8[bq][4 + e] = b1[e]; }
      }
    }
    if (BWD && MA == 2 && !(BITS && !W8)) load_epi(0, 0);
    if (BWD && MA == 2) load_epi(1, 1);
    // STATS: sv[which*32 + (b*2+q)*8 + e]: sums over this lane's positions of the stored values (which = 0) and
    // of their squares (1)
    float sv[STATS ? 64 : 1];
    if (STATS) {
#pragma unroll
      for (int i = 0; i < 64; ++i) sv[STATS ? i : 0] = 0.f;
    }
#pragma unroll
    for (int a = 0; a < MA; ++a) {
      const bool row_in = ipos[a] < npos;
      const size_t row = (size_t)(out_base + ipos[a]) * p.N;
      if (BWD && MA == 4 && a + 1 < MA) load_epi(a + 1, (a + 1) & 1);
      if (BWD && ESETS == 1 && a > 0) load_epi(a, 0);
#pragma unroll
      for (int b = 0; b < 2; ++b)
#pragma unroll
        for (int q = 0; q < 2; ++q) {
          float val[8];
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const u32x2 sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(acc[a][b][8 * q + e]),
                                                              __float_as_uint(acc[a][b][8 * q + 4 + e]), false, false);
            val[e] = __uint_as_float(sw[0]);
            val[4 + e] = __uint_as_float(sw[1]);
          }
          const int c = col0 + b * 32 + q * 16 + h * 8;
          if (!row_in || c >= p.N) continue;   // N is a multiple of 8: a piece is wholly inside or outside
          if (AFFINE && p.bias) {
#pragma unroll
            for (int e = 0; e < 8; ++e) val[e] += bias8[AFFINE ? b * 2 + q : 0][e];
          }
          if (AFFINE && p.relu) {
#pragma unroll
            for (int e = 0; e < 8; ++e) val[e] = val[e] > 0.f ? val[e] : 0.f;
          }
          if (BWD) {
            const u32x4 mk = em[a & (ESETS - 1)][BITS ? 0 : b * 2 + q], ad = ea[a & (ESETS - 1)][b * 2 + q];
            if (p.addend) {
#pragma unroll
              for (int d = 0; d < 4; ++d) { val[2 * d] += bf16_lo(ad[d]); val[2 * d + 1] += bf16_hi(ad[d]); }
            }
            if (BITS) {
              const uint32_t byte = eb[a & (ESETS - 1)][b] >> (8 * (2 * q + h));
#pragma unroll
              for (int e = 0; e < 8; ++e) val[e] = ((byte >> e) & 1u) ? val[e] : 0.f;
            } else if (p.mask) {
#pragma unroll
              for (int d = 0; d < 4; ++d) {
                val[2 * d] = bf16_lo(mk[d]) > 0.f ? val[2 * d] : 0.f;
                val[2 * d + 1] = bf16_hi(mk[d]) > 0.f ? val[2 * d + 1] : 0.f;
              }
            }
            if (p.accumulate) {
#pragma unroll
              for (int d = 0; d < 4; ++d) { val[2 * d] += bf16_lo(ad[d]); val[2 * d + 1] += bf16_hi(ad[d]); }
            }
          }
          if (!STATS) {
            Piece<bf16_t>::store(p.out + row + c, val);
          } else {
            u32x4 t;
#pragma unroll
            for (int d = 0; d < 4; ++d) t[d] = pack_bf16(val[2 * d], val[2 * d + 1]);
            *reinterpret_cast<u32x4*>(p.out + row + c) = t;
#pragma unroll
            for (int d = 0; d < 4; ++d) {
              const float lo = bf16_lo(t[d]), hi = bf16_hi(t[d]);   // the values as stored
              const int i = (b * 2 + q) * 8 + 2 * d;
              sv[STATS ? i : 0] += lo;
              sv[STATS ? i + 1 : 0] += hi;
              sv[STATS ? 32 + i : 0] = fmaf(lo, lo, sv[STATS ? 32 + i : 0]);
              sv[STATS ? 32 + i + 1 : 0] = fmaf(hi, hi, sv[STATS ? 32 + i + 1 : 0]);
            }
          }
        }
    }
    if (STATS) {
      // The 32 lanes of a half hold 64 sums each over different positions.  Five exchange steps (lane distance
      // 16, 8, 4, 2, 1): a lane keeps one half of its list and adds the partner's copy of that half, so the list
      // halves while the positions covered double: a fixed tree, 62 additions instead of 320 for 64 separate
      // reductions.  Lane j ends with entries 2 j' and 2 j' + 1, j' = its bits in the order they were used:
      // which = bit 4 of j, b = bit 3, q = bit 2, e = 4 * bit 1 + 2 * bit 0 (+ 1 for the second entry).
      stat_exchange<16, 32>(sv, j);
      stat_exchange<8, 16>(sv, j);
      stat_exchange<4, 8>(sv, j);
      stat_exchange<2, 4>(sv, j);
      stat_exchange<1, 2>(sv, j);
      stat_sum[0] += (double)sv[0];
      stat_sum[1] += (double)sv[STATS ? 1 : 0];
    }
  }
  if (STATS) {
    // the four wavefronts' sums meet in LDS (nobody reads patch or weights any more), added in wavefront order
    double* red = reinterpret_cast<double*>(smemW);   // [4][2][64]
    const int which = (j >> 4) & 1;
    const int ch = ((j >> 3) & 1) * 32 + ((j >> 2) & 1) * 16 + h * 8 + ((j >> 1) & 1) * 4 + (j & 1) * 2;
    red[(wave * 2 + which) * 64 + ch] = stat_sum[0];
    red[(wave * 2 + which) * 64 + ch + 1] = stat_sum[1];
    __syncthreads();
    if (tid < 128) {
      const int c = tid & 63, w = tid >> 6;
      const double tot = ((red[(0 * 2 + w) * 64 + c] + red[(1 * 2 + w) * 64 + c]) + red[(2 * 2 + w) * 64 + c]) +
                         red[(3 * 2 + w) * 64 + c];
      if (col0 + c < p.N) p.stat_partial[((size_t)group * p.N + col0 + c) * 2 + w] = tot;
    }
  }
}

template <int MA, int NP, bool W8, bool BWD, bool STATS, bool BITS>
void launch_variant(hipStream_t st, const WideParams& p, dim3 grid, size_t lds) {
  static size_t configured = 0;   // raising the dynamic LDS limit is a per-function host call
  const void* fn = reinterpret_cast<const void*>(&conv3_wide_kernel<MA, NP, W8, BWD, STATS, BITS>);
  if (lds > configured) {
    (void)hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    configured = lds;
  }
  hipLaunchKernelGGL((conv3_wide_kernel<MA, NP, W8, BWD, STATS, BITS>), grid, dim3(kThreads), lds, st, p);
}

template <int MA, int NP, bool W8>
void launch_wide(hipStream_t st, const WideParams& p, dim3 grid, size_t lds, bool bwd, bool stats) {
  if (bwd) {
    if (p.mask_bits) return launch_variant<MA, NP, W8, true, false, true>(st, p, grid, lds);
    return launch_variant<MA, NP, W8, true, false, false>(st, p, grid, lds);
  }
  if constexpr (MA == 2 && !W8) {
    if (stats) return launch_variant<MA, NP, W8, false, true, false>(st, p, grid, lds);
  }
  launch_variant<MA, NP, W8, false, false, false>(st, p, grid, lds);
}

}  // namespace

namespace {
// Unit geometry for units of `unit` positions: R rows of nimg images; false if the map does not tile that way.
bool unit_shape(int H, int W, int unit, int& R, int& nimg) {
  if (W < 4 || W > unit || unit % W != 0) return false;
  R = std::min(H, unit / W);
  if (H % R != 0 || unit % (R * W) != 0) return false;
  nimg = unit / (R * W);
  return (nimg == 1 || R == H) && nimg <= 255;
}
}  // namespace

bool conv3_wide_bf16(hipStream_t st, const bf16_t* src, const bf16_t* wgt, bf16_t* out, int M, int N,
                     const ConvGeom& g, const float* bias, const bf16_t* mask, bool relu, bool accumulate,
                     const bf16_t* addend, BnStatRequest* stats) {
  const int H = g.Hs, W = g.Ws;
  if (g.raw3 || g.ks != 3 || g.stride != 1 || g.pad != 1 || g.Hp != H || g.Wp != W) return false;
  if (g.Cs % 32 != 0 || N % 8 != 0 || N <= 32 || (long)g.rows * H * W != M) return false;
  if ((long)M * std::max(g.Cs, N) >= (1L << 31)) return false;   // 32-bit element offsets in the kernel
  const int tiles_n = (N + kTN - 1) / kTN;
  // Units of 256 positions with two workgroups per compute unit where both fit LDS (one workgroup's loads,
  // stores and epilogue then run under the other's matrix instructions); units of 512 with one otherwise.
  // Two 256-register kernels also share a SIMD with the weight-gradient kernels of the side streams; a
  // 512-register wavefront has its SIMD to itself, and the two chains then merely take turns.
  const bool bwd = mask || addend || accumulate;
  if (bwd && (bias || relu)) return false;   // the input-gradient epilogue carries neither (32 registers it needs elsewhere)
  int ma = 0, R = 0, nimg = 0, npatch = 0;
  size_t lds = 0;
  for (int cand : {2, 4}) {
    int r, n;
    if (!unit_shape(H, W, 128 * cand, r, n)) continue;
    const int np_ = n * (r + 2) * (W + 2);
    const size_t l = ((size_t)np_ + 9 * kTN) * kRow * sizeof(bf16_t);   // patch + the nine taps' weights of a slice
    if (l > (size_t)kLdsLimit / (cand == 2 ? 2 : 1)) continue;
    ma = cand; R = r; nimg = n; npatch = np_; lds = l;
    break;
  }
  if (!ma) return false;
  const int units = nimg == 1 ? g.rows * (H / R) : (g.rows + nimg - 1) / nimg;
  if ((long)units * tiles_n < 32) return false;   // too little work to fill the chip this way: the generic kernels spread it better
  const bool w8 = W == 8 && R % 8 == 0;
  const int need = (npatch * OC + kThreads - 1) / kThreads;   // patch pieces per thread
  WideParams p{};
  p.src = src; p.wgt = wgt; p.out = out; p.rows = g.rows; p.H = H; p.W = W; p.Cs = g.Cs; p.N = N;
  p.R = R; p.nimg = nimg; p.flip = g.transposed ? 1 : 0; p.zero = g.zero;
  p.bias = bias; p.mask = mask; p.addend = addend; p.relu = relu ? 1 : 0; p.accumulate = accumulate ? 1 : 0;
  p.mask_bits = (bwd && mask && N % kTN == 0) ? g.mask_bits : nullptr;
  // several units per workgroup (the next unit's patch and weights travel under the current one's taps) while
  // the grid still covers the chip a few times over
  int upw = 1;
  while (upw < 8 && (long)units * tiles_n / (upw * 2) >= (ma == 2 ? 2048 : 1024)) upw *= 2;
  // Batch-norm sums on the way out: units of one image (so a unit has one owner), no bias, no ReLU, and groups
  // that do not cross from one worker to the next, few enough for the statistics scratch.
  bool with_stats = false;
  p.gK = 1;
  p.ufirst[0] = 0; p.ufirst[1] = units;
  if (stats && stats->partial && stats->seg && ma == 2 && nimg == 1 && !w8 && !bwd && !bias && !relu && N % kTN == 0 &&
      stats->seg->off[stats->seg->K] == g.rows) {
    const Segments& seg = *stats->seg;
    const int upi = H / R;
    int u = upw;
    auto groups_at = [&](int per) {
      long n = 0;
      for (int k = 0; k < seg.K; ++k) n += ((long)(seg.off[k + 1] - seg.off[k]) * upi + per - 1) / per;
      return n;
    };
    while (groups_at(u) > (long)seg.K * kBnMaxSplits && u < 64) u *= 2;
    if (groups_at(u) <= (long)seg.K * kBnMaxSplits) {
      with_stats = true;
      upw = u;
      p.gK = seg.K;
      for (int k = 0; k <= seg.K; ++k) p.ufirst[k] = seg.off[k] * upi;
      p.stat_partial = stats->partial;
    }
  }
  p.units = units; p.upw = upw;
  p.gfirst[0] = 0;
  for (int k = 0; k < p.gK; ++k) p.gfirst[k + 1] = p.gfirst[k] + (p.ufirst[k + 1] - p.ufirst[k] + upw - 1) / upw;
  const int groups = p.gfirst[p.gK];
  const dim3 grid(((groups + 7) / 8) * 8 * tiles_n);   // whole rounds of 8 groups: see the kernel's index mapping
  if (ma == 2) {
    if (w8 && need <= 7) launch_wide<2, 7, true>(st, p, grid, lds, bwd, with_stats);
    else if (!w8 && need <= 6) launch_wide<2, 6, false>(st, p, grid, lds, bwd, with_stats);
    else return false;
  } else {
    if (w8 && need <= 13) launch_wide<4, 13, true>(st, p, grid, lds, bwd, false);
    else if (!w8 && need <= 11) launch_wide<4, 11, false>(st, p, grid, lds, bwd, false);
    else if (!w8 && need <= 18) launch_wide<4, 18, false>(st, p, grid, lds, bwd, false);
    else return false;
  }
  if (with_stats) {
    for (int k = 0; k <= p.gK; ++k) stats->table.first[k] = p.gfirst[k];
    stats->done = true;
  }
  return true;
}

}  // namespace omni
