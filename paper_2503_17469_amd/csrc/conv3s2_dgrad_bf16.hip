// Input gradient of a residual block's ENTRY in bf16 (fp32 accumulation): the block input x feeds a
// 3x3 / stride-2 / pad-1 convolution and, beside it, the 1x1 / stride-2 projection of the shortcut; both
// send gradients back to x (the inner F(.) of the gradient line of procedure Train, Algorithm 1):
//
//   dx[n, h, w, ci] = mask * ( sum_{u,v,co} dy[n, (h+1-u)/2, (w+1-v)/2, co] * wt[ci][u][v][co]      (both quotients whole)
//                            + [h, w even] sum_co dys[n, h/2, w/2, co] * wts[ci][co] )
//
// Launched separately through the generic kernel these were its slowest calls (two passes over the
// full-resolution dx, each re-reading the mask; 128-row tiles with two to eight reduction slabs each).
// Here ONE pass writes dx:
//   * a workgroup owns 512 positions of dx (whole rows of whole images) x 64 channels; the positions
//     split into the four parity classes (h mod 2, w mod 2) of 128 each, and a wavefront takes 32 of
//     every class: a class meets only the filter taps of matching parity (1, 2, 2 or 4 of the 9), so
//     no dead tap is ever multiplied, and the classes' different tap counts balance inside every wavefront;
//   * the half-resolution patch of dy (one extra row and column: odd positions reach one further) and the
//     weights of all nine taps are staged per slice of 32 reduction channels, as in conv3_wide_bf16.hip;
//     the shortcut's slices follow with a patch of dys and one weight slab, feeding class (0, 0) only;
//   * the product is formed transposed and written straight from registers in 16-byte pieces, with the
//     ReLU mask of x (and an addend or the old dx, if another consumer of x wrote first) fetched per piece.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <type_traits>

#include "bf16.h"
#include "common.h"
#include "kernels.h"

namespace omni {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float v16f __attribute__((ext_vector_type(16)));

namespace {

constexpr int kThreads = 256;
constexpr int kUnit = 512;        // positions of dx per unit
constexpr int kTN = 64;           // channels of dx per workgroup
constexpr int KC = 32;            // reduction channels per slice
constexpr int kRow = KC + 8;      // elements per LDS row
constexpr int OC = KC / 8;
constexpr int KK = KC / 16;
constexpr int NPP = 4;            // patch pieces per thread (up to 256 patch positions)

struct S2Params {
  const bf16_t* dy;    // [rows][H/2][W/2][Cs]
  const bf16_t* wt;    // [N][9][Cs]
  const bf16_t* dys;   // [rows][H/2][W/2][Cs2] or null
  const bf16_t* wts;   // [N][Cs2]
  bf16_t* dx;          // [rows*H*W][N]
  int rows, H, W, Cs, Cs2, N;
  int R, nimg;         // a unit is nimg images x R rows of dx; nimg * R * W = 512
  int units, upw;
  const void* zero;
  const bf16_t* mask;
  const uint8_t* mask_bits;   // may be null: the mask at one bit per element, [rows*H*W][N/8] (N a multiple of 64)
  const bf16_t* addend;
  int accumulate;
};

__device__ inline bf16x8 as_bf16x8(u32x4 v) { return __builtin_bit_cast(bf16x8, v); }

__global__ __launch_bounds__(kThreads, 1) void conv3s2_dgrad_kernel(S2Params p) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smemS[];
  const int W = p.W, H = p.H, R = p.R;
  const int H2 = H >> 1, W2 = W >> 1, R2 = R >> 1;
  const int PW2 = W2 + 1, PR2 = R2 + 1;
  const int npatch = p.nimg * PR2 * PW2;
  bf16_t* sP = reinterpret_cast<bf16_t*>(smemS);          // [npatch][kRow]
  bf16_t* sW = sP + (size_t)npatch * kRow;                // [9][64][kRow]
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int j = lane & 31, h = lane >> 5;
  const int tiles_n = (p.N + kTN - 1) / kTN;
  // (workgroup b runs on XCD b % 8: the channel tiles of a group of units, which read the same patches, share one)
  const int on_xcd = blockIdx.x >> 3;
  const int tile_n = on_xcd % tiles_n;
  const int group = (on_xcd / tiles_n) * 8 + (blockIdx.x & 7);
  if (group * p.upw >= p.units) return;
  const int col0 = tile_n * kTN;
  const int ubeg = group * p.upw, uend = min(p.units, ubeg + p.upw);
  const int nslice = p.Cs / KC, nslice2 = p.dys ? p.Cs2 / KC : 0;
  const int nall = nslice + nslice2;

  // ---- patch staging tasks: piece x = tid + 256 t -> patch position x / OC, channel octet x % OC
  int prel[NPP];
  uint32_t img8 = 0, prow8 = 0, pcol_ok = 0;
  const int npieces = npatch * OC;
#pragma unroll
  for (int t = 0; t < NPP; ++t) {
    const int x = tid + t * kThreads;
    const int pp = min(x, npieces - 1) / OC;
    const int il = pp / (PR2 * PW2), rem = pp - il * (PR2 * PW2);
    const int pr = rem / PW2, pc = rem - pr * PW2;
    prel[t] = (il * H2 + pr) * W2 + pc;   // source position relative to the unit's first (channels: see load_slice)
    img8 |= (uint32_t)il << (8 * t);
    prow8 |= (uint32_t)pr << (8 * t);
    pcol_ok |= (x < npieces && pc < W2 ? 1u : 0u) << t;   // (the extra column lies outside the image)
  }
  const int poct = tid % OC;   // (256 is a multiple of OC: a thread's pieces all carry the same octet)
  // ---- weight staging: this thread carries row tid / OC, octet tid % OC of every tap's slab
  const int wrow = tid / OC;
  const bool wvalid = col0 + wrow < p.N;
  bf16_t* const wdst = sW + wrow * kRow + poct * 8;
  // ---- this wavefront's positions: the 32 class positions wave*32 + j of every parity class
  const int per_img = R2 * W2;
  const int q = wave * 32 + j;
  const int qil = q / per_img, qrem = q - qil * per_img;
  const int qi = qrem / W2, qj = qrem - qi * W2;
  const int pbase = ((qil * PR2 + qi) * PW2 + qj) * kRow + h * 8;
  int ipos[4];   // position within the unit of class (ph, pw) = (a >> 1, a & 1)
#pragma unroll
  for (int a = 0; a < 4; ++a) ipos[a] = (qil * R + 2 * qi + (a >> 1)) * W + 2 * qj + (a & 1);
  const bf16_t* const wfrag = sW + j * kRow + h * 8;

  const bf16_t* const zp = static_cast<const bf16_t*>(p.zero);
  // Two staging sets: a slice is requested TWO slices before it is needed (a slice is at most 36 matrix instructions
  // per wavefront, about half a microsecond: one slice of distance left every slice waiting for memory).
  u32x4 rp[2][NPP], rw[2][9];
  auto unit_geom = [&](int unit, int& n0, int& r0, int& nvalid) {
    if (p.nimg == 1) {
      const int upi = H / R, img = unit / upi;
      n0 = img; r0 = (unit - img * upi) * R; nvalid = 1;
    } else {
      n0 = unit * p.nimg; r0 = 0; nvalid = min(p.nimg, p.rows - n0);
    }
  };
  // slice s of `unit`: s < nslice: 32 channels of dy with all nine taps' weights; else of dys with its one slab
  auto load_slice = [&](int set, int unit, int s) {
    const bool main = s < nslice;
    const bf16_t* src = main ? p.dy : p.dys;
    const int cs_total = main ? p.Cs : p.Cs2;
    const int c0 = (main ? s : s - nslice) * KC;
    const bf16_t* wsrc = main ? p.wt + ((long)(col0 + wrow) * 9 * p.Cs + c0 + poct * 8)
                              : p.wts + ((long)(col0 + wrow) * p.Cs2 + c0 + poct * 8);
#pragma unroll
    for (int t = 0; t < 9; ++t)
      rw[set][t] = *reinterpret_cast<const u32x4*>((wvalid && (main || t == 0)) ? wsrc + (main ? t * p.Cs : 0) : zp);
    int n0, r0, nvalid;
    unit_geom(unit, n0, r0, nvalid);
    const long ubase = ((long)n0 * H2 + (r0 >> 1)) * W2;
#pragma unroll
    for (int t = 0; t < NPP; ++t) {
      const int il = (int)(img8 >> (8 * t)) & 255, pr = (int)(prow8 >> (8 * t)) & 255;
      const bool in = ((pcol_ok >> t) & 1u) && il < nvalid && (r0 >> 1) + pr < H2;
      rp[set][t] = *reinterpret_cast<const u32x4*>(in ? src + ((ubase + prel[t]) * cs_total + c0 + poct * 8) : zp);
    }
  };
  auto store_slice = [&](int set) {
#pragma unroll
    for (int t = 0; t < 9; ++t) *reinterpret_cast<u32x4*>(wdst + t * kTN * kRow) = rw[set][t];
#pragma unroll
    for (int t = 0; t < NPP; ++t) {
      const int x = tid + t * kThreads;
      if (x < npieces) *reinterpret_cast<u32x4*>(sP + (x / OC) * kRow + (x % OC) * 8) = rp[set][t];
    }
  };
  // the slice `ahead` slices after (unit, s), running on into the next unit of this workgroup
  auto load_ahead = [&](int set, int unit, int s, int ahead) {
    int u = unit, t = s + ahead;
    if (t >= nall) { t -= nall; u = min(unit + 1, uend - 1); }
    load_slice(set, u, t);
  };

  // (nall is even -- the launcher sees to it -- so slice s of every unit lives in set s & 1)
  load_slice(0, min(ubeg, p.units - 1), 0);
  store_slice(0);
  load_ahead(1, min(ubeg, p.units - 1), 0, 1);
  __syncthreads();

  for (int unit = ubeg; unit < uend; ++unit) {
    int n0, r0, nvalid;
    unit_geom(unit, n0, r0, nvalid);
    const long out_base = ((long)n0 * H + r0) * W;
    const int npos = nvalid * R * W;

    v16f acc[4][2];
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
      for (int b = 0; b < 2; ++b)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.f;

    auto slice = [&](int s, auto set_tag) {
      constexpr int SET = decltype(set_tag)::value;
      load_ahead(SET, unit, s, 2);   // (set SET held this slice until the end of the slice before: free now)
      if (s < nslice) {
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) {
          // class (ph, pw) meets tap (u, v) when ph + 1 - u and pw + 1 - v are even; its source lies (du, dv) =
          // ((ph + 1 - u) / 2, (pw + 1 - v) / 2) from the class position's own half-resolution coordinates
#pragma unroll
          for (int u = 0; u < 3; ++u)
#pragma unroll
            for (int v = 0; v < 3; ++v) {
              const int ph = (u + 1) & 1, pw = (v + 1) & 1;
              const int du = (ph + 1 - u) >> 1, dv = (pw + 1 - v) >> 1;
              const int a = ph * 2 + pw;
              const bf16x8 fa = as_bf16x8(*reinterpret_cast<const u32x4*>(sP + pbase + (du * PW2 + dv) * kRow + kk * 16));
#pragma unroll
              for (int b = 0; b < 2; ++b) {
                const bf16x8 fb = as_bf16x8(*reinterpret_cast<const u32x4*>(wfrag + ((u * 3 + v) * kTN + b * 32) * kRow + kk * 16));
                acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb, fa, acc[a][b], 0, 0, 0);
              }
            }
        }
      } else {
        // the shortcut's 1x1 / stride-2 projection reaches the even-even positions only
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) {
          const bf16x8 fa = as_bf16x8(*reinterpret_cast<const u32x4*>(sP + pbase + kk * 16));
#pragma unroll
          for (int b = 0; b < 2; ++b) {
            const bf16x8 fb = as_bf16x8(*reinterpret_cast<const u32x4*>(wfrag + (b * 32) * kRow + kk * 16));
            acc[0][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb, fa, acc[0][b], 0, 0, 0);
          }
        }
      }
      __syncthreads();
      store_slice(SET ^ 1);   // the next slice, requested a slice ago
      __syncthreads();
    };
    for (int s = 0; s < nall; s += 2) {
      slice(s, std::integral_constant<int, 0>{});
      slice(s + 1, std::integral_constant<int, 1>{});
    }

    // ---- epilogue, straight from registers (see conv3_wide_bf16.hip): after the swap of the wavefront's halves
    // lane (j, h) holds channels b*32 + q*16 + 8h .. +7 of its position of class a
    u32x4 em[2][4], ea[2][4];   // mask and addend / old dx of class a: fetched one class ahead
    u32x2 eb[2];                // the mask as bits: the 8 bytes of the tile's 64 channels at this lane's position
    auto load_epi = [&](int a, int set) {
      const size_t row = (size_t)(out_base + ipos[a]) * p.N;
      const bf16_t* other = p.addend ? p.addend : (p.accumulate ? p.dx : nullptr);
      const bf16_t* mask = p.mask_bits ? nullptr : p.mask;
      eb[set] = *reinterpret_cast<const u32x2*>((ipos[a] < npos && p.mask_bits)
                                                    ? p.mask_bits + ((size_t)(out_base + ipos[a]) * (p.N >> 3) + (col0 >> 3))
                                                    : static_cast<const uint8_t*>(p.zero));
#pragma unroll
      for (int bq = 0; bq < 4; ++bq) {
        const int c = col0 + (bq >> 1) * 32 + (bq & 1) * 16 + h * 8;
        const bool in = ipos[a] < npos && c < p.N;
        em[set][bq] = *reinterpret_cast<const u32x4*>((in && mask) ? mask + row + c : zp);
        ea[set][bq] = *reinterpret_cast<const u32x4*>((in && other) ? other + row + c : zp);
      }
    };
    load_epi(0, 0);
#pragma unroll
    for (int a = 0; a < 4; ++a) {
      const bool row_in = ipos[a] < npos;
      const size_t row = (size_t)(out_base + ipos[a]) * p.N;
      if (a + 1 < 4) load_epi(a + 1, (a + 1) & 1);
#pragma unroll
      for (int b = 0; b < 2; ++b)
#pragma unroll
        for (int qq = 0; qq < 2; ++qq) {
          float val[8];
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const u32x2 sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(acc[a][b][8 * qq + e]),
                                                              __float_as_uint(acc[a][b][8 * qq + 4 + e]), false, false);
            val[e] = __uint_as_float(sw[0]);
            val[4 + e] = __uint_as_float(sw[1]);
          }
          const int c = col0 + b * 32 + qq * 16 + h * 8;
          if (!row_in || c >= p.N) continue;
          const u32x4 mk = em[a & 1][b * 2 + qq], ad = ea[a & 1][b * 2 + qq];
          if (p.addend) {
#pragma unroll
            for (int d = 0; d < 4; ++d) { val[2 * d] += bf16_lo(ad[d]); val[2 * d + 1] += bf16_hi(ad[d]); }
          }
          if (p.mask_bits) {
            const uint32_t byte = eb[a & 1][b] >> (8 * (2 * qq + h));
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
          Piece<bf16_t>::store(p.dx + row + c, val);
        }
    }
  }
}

}  // namespace

bool conv3s2_dgrad_supported(int rows, int H, int W, int Cin, int Cout, int Cout_sc) {
  if (H % 2 || W % 2 || Cin % 8 != 0 || Cin <= 32 || Cout % KC != 0 || Cout_sc % KC != 0) return false;
  if ((Cout / KC + Cout_sc / KC) % 2 != 0) return false;   // (slices alternate between two staging sets)
  if ((long)rows * H * W * std::max(Cin, std::max(Cout, Cout_sc)) >= (1L << 31)) return false;   // 32-bit element offsets
  if (W < 4 || W > kUnit || kUnit % W != 0) return false;
  const int R = std::min(H, kUnit / W);
  if (R % 2 || H % R != 0 || kUnit % (R * W) != 0) return false;
  const int nimg = kUnit / (R * W);
  if ((nimg > 1 && R != H) || nimg > 255) return false;
  const int npatch = nimg * (R / 2 + 1) * (W / 2 + 1);
  if (npatch * OC > NPP * kThreads || R / 2 + 1 > 255) return false;
  const int tiles_n = (Cin + kTN - 1) / kTN;
  const int units = nimg == 1 ? rows * (H / R) : (rows + nimg - 1) / nimg;
  return (long)units * tiles_n >= 32;   // (less work than that: the generic kernel spreads it better)
}

bool conv3s2_dgrad_bf16(hipStream_t st, const bf16_t* dy, const bf16_t* wt, int Cout, const bf16_t* dy_sc,
                        const bf16_t* wt_sc, int Cout_sc, bf16_t* dx, int rows, int H, int W, int Cin,
                        const bf16_t* mask, bool accumulate, const bf16_t* addend, const void* zero,
                        const uint8_t* mask_bits) {
  if (!conv3s2_dgrad_supported(rows, H, W, Cin, Cout, dy_sc ? Cout_sc : 0)) return false;
  if (dy_sc && !wt_sc) return false;
  const int R = std::min(H, kUnit / W);
  const int nimg = kUnit / (R * W);
  const int npatch = nimg * (R / 2 + 1) * (W / 2 + 1);
  const int tiles_n = (Cin + kTN - 1) / kTN;
  const int units = nimg == 1 ? rows * (H / R) : (rows + nimg - 1) / nimg;
  S2Params p{};
  p.dy = dy; p.wt = wt; p.dys = dy_sc; p.wts = wt_sc; p.dx = dx;
  p.rows = rows; p.H = H; p.W = W; p.Cs = Cout; p.Cs2 = dy_sc ? Cout_sc : 0; p.N = Cin;
  p.R = R; p.nimg = nimg; p.zero = zero; p.mask = mask; p.addend = addend; p.accumulate = accumulate ? 1 : 0;
  p.mask_bits = (mask && Cin % kTN == 0) ? mask_bits : nullptr;
  int upw = 1;
  while (upw < 8 && (long)units * tiles_n / (upw * 2) >= 1024) upw *= 2;
  p.units = units; p.upw = upw;
  const int groups = (units + upw - 1) / upw;
  const dim3 grid(((groups + 7) / 8) * 8 * tiles_n);
  const size_t lds = ((size_t)npatch + 9 * kTN) * kRow * sizeof(bf16_t);
  static size_t configured = 0;
  if (lds > configured) {
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&conv3s2_dgrad_kernel),
                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    configured = lds;
  }
  hipLaunchKernelGGL(conv3s2_dgrad_kernel, grid, dim3(kThreads), lds, st, p);
  return true;
}

}  // namespace omni
