// bfloat16 storage helpers for device code: values travel as raw 16-bit words.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

namespace omni {

typedef uint16_t bf16_t;   // raw bits of a bfloat16
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef float v4f __attribute__((ext_vector_type(4)));

__device__ inline float bf16_to_f32(bf16_t h) { return __uint_as_float((uint32_t)h << 16); }
__device__ inline float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ inline float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xFFFF0000u); }

// Round to nearest, ties to even, two values per instruction: gfx950 converts in hardware
// (v_cvt_pk_bf16_f32; the same rounding in integer arithmetic cost about five instructions per value,
// which showed in every epilogue that stores bf16).
__device__ inline uint32_t pack_bf16(float lo, float hi) {
  typedef float f32x2 __attribute__((ext_vector_type(2)));
  typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2{lo, hi}, bf16x2));
}
__device__ inline bf16_t f32_to_bf16(float f) { return (bf16_t)(pack_bf16(f, 0.f) & 0xFFFFu); }

// One 16-byte piece of a row as floats: 4 fp32 or 8 bf16.
template <typename T> struct Piece;
template <> struct Piece<float> {
  static constexpr int EL = 4;
  __device__ static inline void load(const float* p, float (&v)[4]) {
    const v4f t = *reinterpret_cast<const v4f*>(p);
    v[0] = t[0]; v[1] = t[1]; v[2] = t[2]; v[3] = t[3];
  }
  __device__ static inline void store(float* p, const float (&v)[4]) {
    *reinterpret_cast<v4f*>(p) = v4f{v[0], v[1], v[2], v[3]};
  }
  __device__ static inline float get(const float* p) { return *p; }
};
template <> struct Piece<bf16_t> {
  static constexpr int EL = 8;
  __device__ static inline void load(const bf16_t* p, float (&v)[8]) {
    const u32x4 t = *reinterpret_cast<const u32x4*>(p);
#pragma unroll
    for (int d = 0; d < 4; ++d) {
      v[2 * d] = bf16_lo(t[d]);
      v[2 * d + 1] = bf16_hi(t[d]);
    }
  }
  __device__ static inline void store(bf16_t* p, const float (&v)[8]) {
    u32x4 t;
#pragma unroll
    for (int d = 0; d < 4; ++d) t[d] = pack_bf16(v[2 * d], v[2 * d + 1]);
    *reinterpret_cast<u32x4*>(p) = t;
  }
  __device__ static inline float get(const bf16_t* p) { return bf16_to_f32(*p); }
};

}  // namespace omni
