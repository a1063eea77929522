// abl_backward_noalloc: the layer backward for callers that cannot allocate.  Its workspace is a
// fixed array in device memory that belongs to the library; the kernels are those of abl_backward
// and receive the array's device address as their workspace argument.

#include <mutex>

#include "abl_internal.h"

namespace {

constexpr size_t kStaticScratchBytes = (size_t)ABL_NOALLOC_SCRATCH_BYTES;
constexpr int kMaxDevices = 64;

// One copy per GPU that loads the library, at an address of that GPU's own.  In host code the
// name is only a handle for hipGetSymbolAddress - never a device address.
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

std::mutex g_lock;
void* g_scratch_ptr[kMaxDevices];  // device address of `scratch` per device, filled on first use

// Device address of this device's copy of `scratch` (nullptr on failure).
void* static_scratch() {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
  std::lock_guard<std::mutex> hold(g_lock);
  if (g_scratch_ptr[dev] == nullptr) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess) {
      (void)hipGetLastError();
      return nullptr;
    }
    g_scratch_ptr[dev] = p;
  }
  return g_scratch_ptr[dev];
}

}  // namespace

extern "C" {

size_t abl_noalloc_scratch_limit(void) { return kStaticScratchBytes; }

int abl_backward_noalloc(void* stream, const abl_shape* shape, int K, uint32_t flags, const void* packed,
                         const void* stats, const float* dy, const float* W, float* dx, float* dW, float* dgamma,
                         float* dbeta) {
  const size_t need = abl_scratch_bytes(shape, K);
  if (need == 0) {
    // invalid shape or K: let the checked path name the error (it enqueues nothing); any non-null
    // aligned value serves as the workspace argument of a call that fails before using it
    return abl_backward(stream, shape, K, flags, packed, stats, dy, W, reinterpret_cast<void*>(256), 0, dx, dW,
                        dgamma, dbeta);
  }
  if (need > kStaticScratchBytes) return ABL_ERR_SCRATCH;
  void* ws = static_scratch();
  if (ws == nullptr) return ABL_ERR_HIP;
  // Nothing in the workspace has to start at zero: every partial row and partial copy that a
  // kernel of the backward reads has been written by an earlier kernel of the same call.
  return abl_backward(stream, shape, K, flags, packed, stats, dy, W, ws, kStaticScratchBytes, dx, dW, dgamma,
                      dbeta);
}

}  // extern "C"
