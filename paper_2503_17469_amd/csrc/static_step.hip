// omni_step for callers that cannot allocate device memory: the workspace is not an argument but a
// fixed array in the library's own device image, one copy per GPU, held until the process ends.
//
// Same launch plan and kernels as omni_step (the step driver is shared); what differs is where the
// scratch memory comes from (per-worker gradient rows, split-reduction partial tiles and their arrival
// counters, activations and their gradients, the status word) and that nothing at all is created on
// the way: no device allocation, no stream, no event.
#include <hip/hip_runtime.h>

#include <mutex>

#include "common.h"
#include "kernels.h"

namespace {

constexpr size_t kStaticBytes = OMNI_STATIC_WORKSPACE_BYTES;

// The array's name is a host-side handle only: device code and API calls take the address that
// hipGetSymbolAddress returns for the current device (every GPU holds its own copy at its own address).
static __device__ __align__(256) unsigned char scratch[kStaticBytes];

constexpr int kMaxDevices = 64;
void* g_scratch_ptr[kMaxDevices] = {};
std::mutex g_scratch_mutex;

// Device address of `scratch` on the current device; looked up once per device.
int static_scratch(void** out) {
  int dev = -1;
  OMNI_HIP_CHECK(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return omni::fail(OMNI_ECAPACITY, "omni_step_static: device index %d not supported", dev);
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    OMNI_HIP_CHECK(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
    if (!ptr || (reinterpret_cast<uintptr_t>(ptr) & 255u))
      return omni::fail(OMNI_EHIP, "omni_step_static: bad address for the static workspace");
    g_scratch_ptr[dev] = ptr;
  }
  *out = g_scratch_ptr[dev];
  return OMNI_OK;
}

}  // namespace

extern "C" int omni_step_static(omni_net* net, void* stream, float* params, const void* x, const int32_t* labels,
                                const int32_t* off, const int32_t* b, int32_t K, float lr, float* loss_per_worker,
                                float* loss, uint32_t flags) {
  if (!net) return omni::fail(OMNI_EINVAL, "omni_step_static: NULL net");
  const size_t need = omni_net_workspace_bytes(net);
  if (need > kStaticBytes)
    return omni::fail(OMNI_ECAPACITY,
                      "omni_step_static: this network needs %zu bytes of workspace, the static one holds %zu; use omni_step "
                      "with a workspace of the caller's",
                      need, kStaticBytes);
  void* ws = nullptr;
  if (int rc = static_scratch(&ws)) return rc;
  return omni::step_impl(net, stream, params, x, labels, off, b, K, lr, ws, loss_per_worker, loss, flags, false);
}
