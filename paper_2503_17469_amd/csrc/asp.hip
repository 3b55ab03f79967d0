// Asynchronous training, Algorithm 2: the update a worker's push leaves on the
// parameter-server model, dst = base - eta_k * g_k with eta_k = eta * b_k / B
// (equation aspvariableSGD).  Bandwidth-bound: one read of the model, one of
// the gradient, one write.
#include <hip/hip_runtime.h>

#include <cmath>

#include "common.h"

namespace omni {

typedef float v4f __attribute__((ext_vector_type(4)));

namespace {

// dst and base may be the same buffer (each element is read before it is written by the
// same thread), so neither is marked restrict.
__global__ __launch_bounds__(256) void asp_update_kernel(float* dst, const float* base,
                                                         const float* __restrict__ grad, size_t P, float eta) {
  const size_t n4 = P / 4;
  const size_t nthreads = (size_t)gridDim.x * blockDim.x;
  const size_t t = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  for (size_t i0 = t; i0 < n4; i0 += 2 * nthreads) {
    const size_t i1 = i0 + nthreads;
    const bool has1 = i1 < n4;
    const size_t j1 = has1 ? i1 : i0;
    const v4f th0 = *reinterpret_cast<const v4f*>(base + 4 * i0);
    const v4f th1 = *reinterpret_cast<const v4f*>(base + 4 * j1);
    const v4f g0 = __builtin_nontemporal_load(reinterpret_cast<const v4f*>(grad + 4 * i0));
    const v4f g1 = __builtin_nontemporal_load(reinterpret_cast<const v4f*>(grad + 4 * j1));
    *reinterpret_cast<v4f*>(dst + 4 * i0) = th0 - eta * g0;
    if (has1) *reinterpret_cast<v4f*>(dst + 4 * i1) = th1 - eta * g1;
  }
  if (t < P - 4 * n4) {
    const size_t i = 4 * n4 + t;
    dst[i] = base[i] - eta * grad[i];
  }
}

}  // namespace
}  // namespace omni

extern "C" int omni_asp_update(void* stream, float* dst, const float* base, const float* grad, size_t P, float lr,
                               int32_t b_k, int32_t B, int32_t lr_scaling) {
  using omni::fail;
  if (!dst || !base || !grad) return fail(OMNI_EINVAL, "omni_asp_update: NULL argument");
  if (P < 1) return fail(OMNI_EINVAL, "omni_asp_update: P must be at least 1");
  if ((reinterpret_cast<uintptr_t>(dst) & 15u) || (reinterpret_cast<uintptr_t>(base) & 15u) ||
      (reinterpret_cast<uintptr_t>(grad) & 15u))
    return fail(OMNI_EINVAL, "omni_asp_update: dst/base/grad must be 16-byte aligned");
  if (!std::isfinite(lr)) return fail(OMNI_EINVAL, "omni_asp_update: lr is not finite");
  if (b_k < 1 || B < b_k) return fail(OMNI_EINVAL, "omni_asp_update: need 1 <= b_k <= B (b_k=%d B=%d)", b_k, B);
  if (dst != base) {
    // partial overlap would let one thread overwrite what another still has to read
    const uintptr_t d = reinterpret_cast<uintptr_t>(dst), s = reinterpret_cast<uintptr_t>(base);
    const uintptr_t bytes = (uintptr_t)P * 4u;
    if (d < s + bytes && s < d + bytes) return fail(OMNI_EINVAL, "omni_asp_update: dst and base overlap partially");
  }
  const float eta = lr_scaling ? (float)((double)lr * ((double)b_k / (double)B)) : lr;
  const size_t n4 = P / 4;
  size_t blocks = (n4 + 511) / 512;
  if (blocks > 2048) blocks = 2048;
  if (blocks < 1) blocks = 1;
  hipLaunchKernelGGL(omni::asp_update_kernel, dim3((unsigned)blocks), dim3(256), 0, static_cast<hipStream_t>(stream),
                     dst, base, grad, P, eta);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(OMNI_EHIP, "omni_asp_update: launch failed: %s", hipGetErrorString(e));
  return OMNI_OK;
}
