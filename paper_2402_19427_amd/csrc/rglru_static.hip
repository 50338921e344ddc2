// rglru_forward_static: rglru_forward for callers that cannot allocate or hand over a
// workspace (code under HIP graph capture, tight serving loops, harnesses that forbid
// hipMalloc). What rglru_forward takes from its workspace argument - the status word, the
// record rings of a sequence sliced in time, W_x in half precision - lives in a file-scope
// device array instead, one copy per GPU the library runs on, held until the process ends.
#include <cstdio>
#include <mutex>

#include "rglru_internal.h"

namespace {

constexpr size_t SCRATCH_BYTES = RGLRU_STATIC_SCRATCH_BYTES;
// In host code this name is only a handle for hipGetSymbolAddress; the device address of the
// array differs from GPU to GPU and is looked up once per device below.
static __device__ __align__(256) __attribute__((used)) unsigned char scratch[SCRATCH_BYTES];

constexpr int MAX_DEVICES = 64;
void *g_scratch_ptr[MAX_DEVICES] = {};
std::mutex g_scratch_mutex;

// Device address of this GPU's copy of the array (looked up on the first call on that GPU,
// with that GPU current); nullptr and *err set if the runtime refuses.
void *scratch_of_current_device(hipError_t *err) {
  int dev = -1;
  *err = hipGetDevice(&dev);
  if (*err != hipSuccess) return nullptr;
  if (dev < 0 || dev >= MAX_DEVICES) {
    *err = hipErrorInvalidDevice;
    return nullptr;
  }
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void *ptr = nullptr;
    *err = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (*err != hipSuccess) return nullptr;
    g_scratch_ptr[dev] = ptr;
  }
  return g_scratch_ptr[dev];
}

}  // namespace

extern "C" int rglru_forward_static(const rglru_shape *shape, const rglru_params *params, const void *u,
                                    const float *h0, const void *conv_state_in, int64_t pos0, void *y,
                                    float *hT, void *conv_state_out, void *stream) {
  // (an invalid shape makes the size 0 here and is reported by rglru_forward itself)
  const size_t need = rglru_workspace_bytes(shape, RGLRU_OP_FORWARD);
  if (need > SCRATCH_BYTES) {
    rglru::set_last_error("rglru_forward_static: this shape needs %zu bytes of scratch, the static array holds %zu "
                          "(use rglru_forward with a workspace)", need, SCRATCH_BYTES);
    return RGLRU_ERR_WORKSPACE;
  }
  void *ptr = nullptr;
  if (need > 0) {
    hipError_t e;
    ptr = scratch_of_current_device(&e);
    if (!ptr) {
      rglru::set_last_error("rglru_forward_static: address of the static scratch array: %s", hipGetErrorString(e));
      return RGLRU_ERR_HIP;
    }
  }
  // the same validation, kernels and launches as rglru_forward; everything the kernels expect to
  // start from zero in the scratch is cleared by their own preparation kernel on `stream`
  return rglru_forward(shape, params, u, h0, conv_state_in, pos0, y, hT, conv_state_out, ptr,
                       ptr ? SCRATCH_BYTES : 0, stream);
}
