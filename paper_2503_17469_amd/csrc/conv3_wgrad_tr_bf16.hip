// Weight gradient of 3x3 / pad-1 convolutions of stride 2 in bf16 with fp32 accumulation, per worker
// (the gradient line of procedure Train, Algorithm 1, for one layer's filter bank):
//
//   G_k[co][u][v][ci] = sum over the output positions (n, h, w) of worker k of
//                       dY[n, h, w, co] * X[n, S h + u - 1, S w + v - 1, ci]
//
// As a matrix product the reduction runs over positions, which is the SLOW index of both operands in memory
// ([position][channel]).  The generic weight-gradient kernel gathers and transposes the input once per filter
// tap and channel tile (nine LDS tiles per tap-less patch, operands fetched up to 12 times on the 512-channel
// layers); the stride-1 kernel stores both operands transposed, which ties it to unit stride (a tap is a shift
// by one element inside a row of X^T).  Here both operands stay as they arrive:
//
//   * LDS holds the dY rows of a unit of 64 output positions ([position][128 output channels]) and the unit's
//     input patch, halo included, once ([patch position][32 input channels]); 16-byte pieces, no shuffling;
//   * the matrix operands are formed by the transposing LDS read of gfx950 (ds_read_b64_tr_b16): sixteen lanes
//     hand in four positions x sixteen channels (8 bytes each) and receive, per lane, one channel at those four
//     positions -- the reduction index moves into the lane's registers on the way out of LDS.  A tap is just
//     another address, so the stride costs nothing;
//   * a workgroup owns 128 output channels x 32 input channels x 9 taps (one 32 x 32 block per tap and
//     wavefront: 144 accumulator registers), walks the units of one chunk of ONE worker's positions, and writes
//     the worker's gradient itself or, if the worker has several chunks, a partial tile that a second kernel adds
//     in chunk order (no atomics: bit-reproducible).
//
// Layers with a bias are left to the generic kernel (the convolutions this is for are followed by a batch norm).
#include <hip/hip_runtime.h>

#include <algorithm>

#include "bf16.h"
#include "common.h"
#include "kernels.h"

namespace omni {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef short v4s __attribute__((ext_vector_type(4)));

namespace {

constexpr int kThreads = 256;
constexpr int kUnit = 64;          // output positions per unit
constexpr int kCo = 128;           // output channels per workgroup (32 per wavefront)
constexpr int kCi = 32;            // input channels per workgroup
constexpr int kSA = (kCo + 16) * 2;   // bytes per dY row in LDS: 72 banks, so four rows 8 banks apart start in different bank octets
constexpr int kNA = kUnit * (kCo / 8) / kThreads;   // dY pieces per thread (4)
constexpr int kNX = 6;             // patch pieces per thread (up to 384 patch positions x 4 pieces)
constexpr int kTileFloats = 9 * 16 * kThreads;

struct TrParams {
  const bf16_t* dy;    // [rows*Ho*Wo][Cout]
  const bf16_t* src;   // [rows][H][W][Cin]
  float* gw;           // worker w: gw + w*worker_stride, [Cout][9][cin_real]
  size_t worker_stride;
  int Cout, Cin, cin_real;
  int Ho, Wo, H, W;
  int R, nimg;         // a unit is nimg images x R output rows; nimg * R * Wo = 64
  int PR, PW;          // patch rows and columns per image: S (R - 1) + 3, S (Wo - 1) + 3
  int upc;             // units per chunk
  float* partial;      // [(tile * total_chunks + chunk)][144][256]
  const void* zero;    // zeros for absent pieces
};
struct TrChunks { int32_t first[OMNI_MAX_WORKERS + 1]; };   // first chunk of every worker; first[K] = total

__device__ inline bf16x8 tr_pair(const unsigned char* lds_a, const unsigned char* lds_b) {
  typedef __attribute__((address_space(3))) v4s lds_v4s;
  const v4s lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4s*)lds_a);
  const v4s hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4s*)lds_b);
  typedef short v8s __attribute__((ext_vector_type(8)));
  const v8s both = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
  return __builtin_bit_cast(bf16x8, both);
}

// S: stride of the forward convolution.  Bytes per patch position in LDS: 64 of data + padding such that the
// four positions one transposing read covers (S patch positions apart) start 8 banks apart.
template <int S>
__global__ __launch_bounds__(kThreads, 2) void conv3_wgrad_tr_kernel(TrParams p, Segments seg, TrChunks ct) {
  constexpr int SX = S == 2 ? 80 : 96;
  extern __shared__ __attribute__((aligned(16))) unsigned char smemT[];
  unsigned char* sA = smemT;                       // [64][kSA]
  unsigned char* sX = smemT + kUnit * kSA;         // [npatch][SX]
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int tiles_ci = (p.Cin + kCi - 1) / kCi;
  const int tile = blockIdx.x;
  const int co0 = (tile / tiles_ci) * kCo, ci0 = (tile % tiles_ci) * kCi;
  const int Ho = p.Ho, Wo = p.Wo, H = p.H, W = p.W, R = p.R, PR = p.PR, PW = p.PW;

  int wk = 0;
  while (wk + 1 < seg.K && (int)blockIdx.y >= ct.first[wk + 1]) ++wk;
  const int chunk_idx = blockIdx.y - ct.first[wk];
  const int nchunks = ct.first[wk + 1] - ct.first[wk];
  const int bk = seg.off[wk + 1] - seg.off[wk];
  const int upi = Ho / R;   // units per image when a unit is part of one image
  const int units_k = p.nimg == 1 ? bk * upi : (bk + p.nimg - 1) / p.nimg;
  const int ubeg = chunk_idx * p.upc, uend = min(units_k, ubeg + p.upc);

  // ---- staging tasks, relative to the unit's first image and output row
  // dY: piece x = tid + 256 t -> position x / 16, channel octet x % 16 (a unit's positions are contiguous rows of dY)
  const int a_oct = tid & 15;
  const bool a_chan_ok = co0 + 8 * a_oct < p.Cout;
  // X: piece x = tid + 256 t -> patch position x / 4, channel octet x % 4
  const int x_oct = tid & 3;
  const bool x_chan_ok = ci0 + 8 * x_oct < p.Cin;
  const int npatch = p.nimg * PR * PW;
  int x_rel[kNX];        // element offset from the unit's first input pixel (row S r0 - 1, column -1)
  uint32_t x_ok = 0, x_top = 0, x_bottom = 0, x_img = 0;   // x_img: 4 bits per piece
#pragma unroll
  for (int t = 0; t < kNX; ++t) {
    const int pp = min((tid + t * kThreads) >> 2, npatch - 1);
    const int il = pp / (PR * PW), rem = pp - il * (PR * PW);
    const int pr = rem / PW, pc = rem - pr * PW;
    x_rel[t] = ((il * H + pr) * W + pc) * p.Cin + 8 * x_oct;
    const bool col_in = pc >= 1 && pc <= W;   // input column pc - 1
    x_ok |= (((tid + t * kThreads) >> 2) < npatch && col_in && x_chan_ok ? 1u : 0u) << t;
    x_top |= (pr == 0 ? 1u : 0u) << t;
    x_bottom |= (pr == PR - 1 ? 1u : 0u) << t;
    x_img |= (uint32_t)il << (4 * t);
  }

  // ---- fragment addresses.  Sixteen lanes (group g = lane / 16, s = lane % 16) hand in, for read q of
  // reduction step ks, position 16 ks + 8 (g / 2) + 4 q + s / 4 and channels 16 (g % 2) + 4 (s % 4) .. + 3;
  // lane 16 g + i then holds channel 16 (g % 2) + i at the four positions 16 ks + 8 (g / 2) + 4 q + 0..3:
  // with both reads, the eight reduction elements 8 (lane / 32) .. + 7 of row / column lane % 32 that the
  // 32 x 32 x 16 matrix instruction expects.
  const int g = lane >> 4, s = lane & 15;
  const int chan = 16 * (g & 1) + 4 * (s & 3);
  const unsigned char* a_base = sA + (8 * (g >> 1) + (s >> 2)) * kSA + (wave * 32 + chan) * 2;
  // patch byte offset of a position of the unit (tap (0, 0))
  auto patch_off = [&](int pos) {
    const int il = pos / (R * Wo), rem = pos - il * (R * Wo);
    const int r = rem / Wo, w = rem - r * Wo;
    return ((il * PR + S * r) * PW + S * w) * SX;
  };
  // The sixteen positions of a reduction step start at a multiple of 16, which is the start of a map row or
  // (maps 32 or more wide) the middle of one, and never reach into the next image: the offset of position
  // 16 ks + i is that of 16 ks (the same for every lane: scalar arithmetic) plus that of i.
  int xb[2];       // this lane's part, for read q
#pragma unroll
  for (int q = 0; q < 2; ++q) xb[q] = patch_off(8 * (g >> 1) + 4 * q + (s >> 2)) + chan * 2;

  v16f acc[9];
#pragma unroll
  for (int t = 0; t < 9; ++t)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[t][v] = 0.f;

  u32x4 ra[kNA], rx[kNX];
  const bf16_t* const zp = static_cast<const bf16_t*>(p.zero);
  auto load_unit = [&](int u) {
    int n0, r0, nvalid;
    if (p.nimg == 1) {
      const int img = u / upi;
      n0 = seg.off[wk] + img; r0 = (u - img * upi) * R; nvalid = 1;
    } else {
      n0 = seg.off[wk] + u * p.nimg; r0 = 0; nvalid = min(p.nimg, seg.off[wk + 1] - n0);
    }
    // loads never branch: an absent piece is read from a page of zeros
    const long base_pos = ((long)n0 * Ho + r0) * Wo;
    const int live = nvalid * R * Wo;   // positions of images that exist
#pragma unroll
    for (int t = 0; t < kNA; ++t) {
      const int pos = (tid + t * kThreads) >> 4;
      const bool in = a_chan_ok && pos < live;
      ra[t] = *reinterpret_cast<const u32x4*>(in ? p.dy + ((base_pos + pos) * p.Cout + co0 + 8 * a_oct) : zp);
    }
    const long base_in = (((long)n0 * H + (S * r0 - 1)) * W - 1) * p.Cin + ci0;
    const uint32_t ok = x_ok & ~(r0 == 0 ? x_top : 0u) & ~(S * (r0 + R - 1) + 1 >= H ? x_bottom : 0u);
#pragma unroll
    for (int t = 0; t < kNX; ++t) {
      const int il = (int)(x_img >> (4 * t)) & 15;
      const bool in = ((ok >> t) & 1u) && il < nvalid;
      rx[t] = *reinterpret_cast<const u32x4*>(in ? p.src + (base_in + x_rel[t]) : zp);
    }
  };
  auto store_unit = [&]() {
#pragma unroll
    for (int t = 0; t < kNA; ++t) {
      const int x = tid + t * kThreads;
      *reinterpret_cast<u32x4*>(sA + (x >> 4) * kSA + (x & 15) * 16) = ra[t];
    }
#pragma unroll
    for (int t = 0; t < kNX; ++t) {
      const int x = tid + t * kThreads;
      if ((x >> 2) < npatch) *reinterpret_cast<u32x4*>(sX + (x >> 2) * SX + (x & 3) * 16) = rx[t];
    }
  };

  if (ubeg < uend) load_unit(ubeg);
  for (int u = ubeg; u < uend; ++u) {
    __syncthreads();   // the previous unit's fragments have been read
    store_unit();
    __syncthreads();
    load_unit(min(u + 1, uend - 1));   // always issued: in flight during the matrix instructions below
#pragma unroll
    for (int ks = 0; ks < kUnit / 16; ++ks) {
      const bf16x8 fa = tr_pair(a_base + (16 * ks) * kSA, a_base + (16 * ks + 4) * kSA);
      const int kofs = patch_off(16 * ks);
      const unsigned char* x0 = sX + xb[0] + kofs;
      const unsigned char* x1 = sX + xb[1] + kofs;
#pragma unroll
      for (int tap = 0; tap < 9; ++tap) {
        const int toff = ((tap / 3) * PW + (tap % 3)) * SX;
        const bf16x8 fb = tr_pair(x0 + toff, x1 + toff);
        acc[tap] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa, fb, acc[tap], 0, 0, 0);
      }
    }
  }

  // register v of lane (j = lane % 32, h = lane / 32) is output channel wave*32 + 8 (v/4) + 4 h + v%4, input channel j
  const int j = lane & 31, h = lane >> 5;
  const int ci = ci0 + j;
  if (nchunks > 1) {
    float* mine = p.partial + ((size_t)tile * ct.first[seg.K] + blockIdx.y) * kTileFloats;
#pragma unroll
    for (int t = 0; t < 9; ++t)
#pragma unroll
      for (int v = 0; v < 16; ++v) mine[(t * 16 + v) * kThreads + tid] = acc[t][v];
    return;
  }
  if (ci < p.cin_real) {
    float* gw = p.gw + (size_t)wk * p.worker_stride;
#pragma unroll
    for (int t = 0; t < 9; ++t)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int co = co0 + wave * 32 + 8 * (v / 4) + 4 * h + (v % 4);
        if (co < p.Cout) gw[((size_t)co * 9 + t) * p.cin_real + ci] = acc[t][v];
      }
  }
}

// Second stage: grid (tiles, workers, 36); a thread adds one (tap, four registers, lane) entry of every chunk of
// the worker in chunk order.
__global__ __launch_bounds__(kThreads) void conv3_wgrad_tr_reduce_kernel(TrParams p, Segments seg, TrChunks ct) {
  const int tile = blockIdx.x, wk = blockIdx.y;
  const int nchunks = ct.first[wk + 1] - ct.first[wk];
  if (nchunks <= 1) return;   // written directly by the first stage
  const int tap = blockIdx.z >> 2, vq = blockIdx.z & 3;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int j = lane & 31, h = lane >> 5;
  const int tiles_ci = (p.Cin + kCi - 1) / kCi;
  const int co0 = (tile / tiles_ci) * kCo, ci0 = (tile % tiles_ci) * kCi;
  const int ci = ci0 + j;
  if (ci >= p.cin_real) return;
  const float* mine = p.partial + ((size_t)tile * ct.first[seg.K] + ct.first[wk]) * kTileFloats +
                      (size_t)(tap * 16 + vq * 4) * kThreads + tid;
  float sum[4] = {0.f, 0.f, 0.f, 0.f};
  int c = 0;
  for (; c + 4 <= nchunks; c += 4) {   // sixteen loads in flight; the additions keep chunk order
    float t[4][4];
#pragma unroll
    for (int u = 0; u < 4; ++u)
#pragma unroll
      for (int e = 0; e < 4; ++e) t[u][e] = mine[(size_t)(c + u) * kTileFloats + e * kThreads];
#pragma unroll
    for (int u = 0; u < 4; ++u)
#pragma unroll
      for (int e = 0; e < 4; ++e) sum[e] += t[u][e];
  }
  for (; c < nchunks; ++c)
#pragma unroll
    for (int e = 0; e < 4; ++e) sum[e] += mine[(size_t)c * kTileFloats + e * kThreads];
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const int v = vq * 4 + e;
    const int co = co0 + wave * 32 + 8 * (v / 4) + 4 * h + (v % 4);
    if (co < p.Cout) p.gw[(size_t)wk * p.worker_stride + ((size_t)co * 9 + tap) * p.cin_real + ci] = sum[e];
  }
}

}  // namespace

bool conv3_wgrad_tr_bf16(hipStream_t st, const bf16_t* dy, const bf16_t* src, float* gw, float* gb,
                         size_t worker_stride, int Cout, int cin_real, const ConvGeom& g, const Segments& seg,
                         float* partial) {
  const int S = g.stride, Ho = g.Hp, Wo = g.Wp, H = g.Hs, W = g.Ws;
  // (the kernel is written for any stride; stride-1 layers are not sent here: the transposed-patch kernel of
  // conv_bf16.hip measured faster on every map width, by 0.07 to 0.64 ms per ResNet-18 step)
  if (gb || g.ks != 3 || g.pad != 1 || g.transposed || g.raw3 || S != 2) return false;
  if (H != S * Ho || W != S * Wo || g.Cs % 8 != 0 || Cout % 8 != 0 || cin_real > g.Cs) return false;
  // (a reduction step of sixteen positions must lie inside one map row or be made of whole rows of one image)
  if (Wo < 4 || Wo > kUnit || (Wo % 16 != 0 && 16 % Wo != 0)) return false;
  const int R = std::min(Ho, kUnit / Wo);
  if (Ho % R != 0 || kUnit % (R * Wo) != 0 || (R * Wo) % 16 != 0) return false;
  const int nimg = kUnit / (R * Wo);
  if ((nimg > 1 && R != Ho) || nimg > 15) return false;
  const int PR = S * (R - 1) + 3, PW = S * (Wo - 1) + 3;
  const int npatch = nimg * PR * PW;
  if (npatch * 4 > kNX * kThreads) return false;
  if ((long)g.rows * H * W * g.Cs >= (1L << 31) || (long)g.rows * Ho * Wo * Cout >= (1L << 31)) return false;
  TrParams p{};
  p.dy = dy; p.src = src; p.gw = gw; p.worker_stride = worker_stride;
  p.Cout = Cout; p.Cin = g.Cs; p.cin_real = cin_real; p.Ho = Ho; p.Wo = Wo; p.H = H; p.W = W;
  p.R = R; p.nimg = nimg; p.PR = PR; p.PW = PW; p.partial = partial; p.zero = g.zero;
  const int tiles = ((Cout + kCo - 1) / kCo) * ((g.Cs + kCi - 1) / kCi);
  const size_t max_slots = conv_wgrad_partial_floats() / kTileFloats;
  long units[OMNI_MAX_WORKERS], total_units = 0;
  for (int k = 0; k < seg.K; ++k) {
    const long bk = seg.off[k + 1] - seg.off[k];
    units[k] = nimg == 1 ? bk * (Ho / R) : (bk + nimg - 1) / nimg;
    total_units += units[k];
  }
  // about 512 workgroups in all (two per compute unit), at least 8 units each
  long want = std::max<long>(1, 512 / tiles);
  long upc = std::max<long>((total_units + want - 1) / want, 8);
  TrChunks ct{};
  for (;;) {
    int acc = 0;
    for (int k = 0; k < seg.K; ++k) {
      ct.first[k] = acc;
      acc += (int)((units[k] + upc - 1) / upc);
    }
    ct.first[seg.K] = acc;
    if (acc == 0) return true;   // no rows at all
    // one chunk per worker needs no scratch; otherwise the partial tiles must fit it
    if (acc == seg.K) break;
    if ((size_t)tiles * acc <= max_slots && (long)tiles * acc <= std::max(512, 2 * tiles * seg.K)) break;
    upc += std::max<long>(1, upc / 16);
  }
  p.upc = (int)upc;
  const size_t lds = (size_t)kUnit * kSA + (size_t)npatch * 80;   // (80 bytes per patch position at stride 2: see the kernel)
  const dim3 grid(tiles, ct.first[seg.K]);
  hipLaunchKernelGGL(conv3_wgrad_tr_kernel<2>, grid, dim3(kThreads), lds, st, p, seg, ct);
  bool chunked = false;
  for (int k = 0; k < seg.K; ++k) chunked = chunked || ct.first[k + 1] - ct.first[k] > 1;
  if (chunked)
    hipLaunchKernelGGL(conv3_wgrad_tr_reduce_kernel, dim3(tiles, seg.K, 36), dim3(kThreads), 0, st, p, seg, ct);
  return true;
}

}  // namespace omni
