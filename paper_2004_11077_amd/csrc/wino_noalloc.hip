// wino_conv2d_noalloc: the whole-layer call for callers that cannot allocate or pass device
// scratch memory.  The workspace wino_conv2d takes from its caller (V unless pretransformed,
// U, M) lives here in a file-scope device array of WINO_NOALLOC_MAX_BYTES; each GPU the
// library runs on holds its own copy of that array from the moment the library's device code
// is loaded on it until the process ends.
//
// In host code the array's name is only a handle: its device address is looked up once per
// device with hipGetSymbolAddress (with that device current) and kept; every use below goes
// through that address.  Nothing in the workspace has to start at zero: every byte a kernel of
// the layer reads was written by an earlier kernel of the same call (the zero padding of a
// fragment-order V is written by a fill kernel inside the call).  All calls on one GPU share
// the one array, so two calls that overlap in time on the same GPU (different streams or
// threads) race; calls on one stream are ordered and safe.
#include <hip/hip_runtime.h>

#include <mutex>

#include "../../include/wino.h"
#include "wino_kernels.hpp"

namespace {

static __device__ __align__(256) unsigned char scratch[WINO_NOALLOC_MAX_BYTES];

constexpr int kMaxDevices = 64;
void* g_scratch_ptr[kMaxDevices];   // device address of `scratch` per device, null until looked up
std::mutex g_scratch_mu;

}  // namespace

extern "C" int wino_conv2d_noalloc(const wino_conv_desc_t* d, const void* x, const void* w_or_V,
                                   void* y, const wino_scales_t* s, void* hip_stream) {
  size_t want = 0;
  if (int rc = wino_workspace_bytes(d, &want)) return rc;
  if (want > (size_t)WINO_NOALLOC_MAX_BYTES)
    return wino::report_error(WINO_EWORKSPACE,
                              "this layer needs %zu bytes of workspace, the built-in scratch of "
                              "wino_conv2d_noalloc holds %zu", want, (size_t)WINO_NOALLOC_MAX_BYTES);
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess)
    return wino::report_error(WINO_EHIP, "hipGetDevice: %s", hipGetErrorString(e));
  if (dev < 0 || dev >= kMaxDevices)
    return wino::report_error(WINO_EUNSUPPORTED, "device ordinal %d beyond %d", dev, kMaxDevices - 1);
  void* ptr = nullptr;
  {
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    ptr = g_scratch_ptr[dev];
    if (!ptr) {
      e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
      if (e != hipSuccess || !ptr)
        return wino::report_error(WINO_EHIP, "hipGetSymbolAddress(scratch): %s", hipGetErrorString(e));
      g_scratch_ptr[dev] = ptr;
    }
  }
  return wino_conv2d(d, x, w_or_V, y, s, ptr, (size_t)WINO_NOALLOC_MAX_BYTES, hip_stream);
}
