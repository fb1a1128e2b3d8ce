// Weight gradient for callers that cannot allocate device memory (code under stream capture, serving loops,
// harnesses that forbid hipMalloc): the split partial sums that lms_conv_wgrad keeps in a caller workspace live
// in a fixed array of this code object instead.
#include <hip/hip_runtime.h>

#include <mutex>

#include "graph.hpp"
#include "kernels.hpp"

namespace lms {
lms_status desc_to_geom(const lms_conv_desc* d, ConvGeom& g);
}

namespace {

constexpr uint64_t SCRATCH_BYTES = 64ull << 20;
// One copy per device the code object is loaded on, held until the process ends.  In host code this name is only a
// handle for hipGetSymbolAddress; kernels get the address that call returns.
static __device__ __align__(256) unsigned char scratch[SCRATCH_BYTES];

constexpr int MAX_DEVICES = 64;
std::mutex g_lock;
void* g_ptr[MAX_DEVICES] = {};

// Device address of `scratch` on the current device, looked up once per device.
hipError_t scratch_ptr(void** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= MAX_DEVICES) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> hold(g_lock);
  if (!g_ptr[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!p) return hipErrorInvalidSymbol;
    g_ptr[dev] = p;
  }
  *out = g_ptr[dev];
  return hipSuccess;
}

}  // namespace

extern "C" {

uint64_t lms_static_scratch_bytes(void) { return SCRATCH_BYTES; }

lms_status lms_conv_wgrad_static(const lms_conv_desc* d, const void* x, const void* dy, float* dw, void* stream) {
  if (!d || !x || !dy || !dw) { lms::set_error("lms_conv_wgrad_static: null argument"); return LMS_EINVAL; }
  lms::ConvGeom g;
  if (lms::desc_to_geom(d, g) != LMS_OK) { lms::set_error("lms_conv_wgrad_static: bad descriptor"); return LMS_EINVAL; }
  const uint64_t need = lms::conv_wgrad_ws(g);
  if (need > SCRATCH_BYTES) {
    lms::set_error("lms_conv_wgrad_static: this geometry needs %llu bytes of partial sums, the fixed scratch holds %llu; "
                   "use lms_conv_wgrad with a workspace", (unsigned long long)need, (unsigned long long)SCRATCH_BYTES);
    return LMS_EINVAL;
  }
  void* ws = nullptr;
  hipError_t e = scratch_ptr(&ws);
  if (e == hipSuccess) e = lms::conv_wgrad(g, x, dy, dw, ws, (hipStream_t)stream);
  if (e != hipSuccess) { lms::set_error("lms_conv_wgrad_static: %s", hipGetErrorString(e)); return LMS_EHIP; }
  return LMS_OK;
}

}  // extern "C"
