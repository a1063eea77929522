// Memory-bandwidth probes: what a plain read-only, write-only and copy kernel reach on this
// device.  They measure the ceiling that the element-wise passes of the method (Eq. 1-3, 8-10)
// are compared with; they compute nothing of the method.

#include "abl_internal.h"

namespace abl {
namespace {

typedef float vec4f __attribute__((ext_vector_type(4)));
constexpr int kProbeThreads = 256;

// One 16-byte access per thread, consecutive lanes on consecutive addresses: the plainest
// possible stream (measured best here among 1-16 accesses per thread and persistent grids).
__global__ __launch_bounds__(kProbeThreads) void probe_read_kernel(const vec4f* __restrict__ src, int64_t n4,
                                                                   float* __restrict__ sink) {
  const int64_t i = (int64_t)blockIdx.x * kProbeThreads + threadIdx.x;
  if (i >= n4) return;
  const vec4f v = src[i];
  // never true for the finite test pattern; keeps the load alive without a store
  if (v.x + v.y + v.z + v.w == 1.2345e38f) sink[0] = v.x;
}

__global__ __launch_bounds__(kProbeThreads) void probe_write_kernel(vec4f* __restrict__ dst, int64_t n4, float val) {
  const int64_t i = (int64_t)blockIdx.x * kProbeThreads + threadIdx.x;
  if (i >= n4) return;
  dst[i] = vec4f{val, val, val, val};
}

__global__ __launch_bounds__(kProbeThreads) void probe_copy_kernel(const vec4f* __restrict__ src,
                                                                   vec4f* __restrict__ dst, int64_t n4) {
  const int64_t i = (int64_t)blockIdx.x * kProbeThreads + threadIdx.x;
  if (i >= n4) return;
  dst[i] = src[i];
}

}  // namespace
}  // namespace abl

extern "C" int abl_hbm_probe(void* stream, int mode, const void* src, void* dst, size_t bytes) {
  using namespace abl;
  if (mode < 0 || mode > 2) return ABL_ERR_ARG;
  if (bytes == 0 || bytes % 16 != 0 || bytes > ((size_t)1 << 40)) return ABL_ERR_SHAPE;
  const bool need_src = mode != 1, need_dst = true;  // mode 0 uses dst as its 16-byte sink
  if ((need_src && (src == nullptr || (reinterpret_cast<uintptr_t>(src) & 15u))) ||
      (need_dst && (dst == nullptr || (reinterpret_cast<uintptr_t>(dst) & 15u))))
    return ABL_ERR_ARG;
  const int64_t n4 = (int64_t)(bytes / 16);
  const unsigned blocks = (unsigned)((n4 + kProbeThreads - 1) / kProbeThreads);
  hipStream_t st = (hipStream_t)stream;
  if (mode == 0)
    probe_read_kernel<<<blocks, kProbeThreads, 0, st>>>(static_cast<const vec4f*>(src), n4, static_cast<float*>(dst));
  else if (mode == 1)
    probe_write_kernel<<<blocks, kProbeThreads, 0, st>>>(static_cast<vec4f*>(dst), n4, 1.0f);
  else
    probe_copy_kernel<<<blocks, kProbeThreads, 0, st>>>(static_cast<const vec4f*>(src), static_cast<vec4f*>(dst), n4);
  return hip_status();
}
