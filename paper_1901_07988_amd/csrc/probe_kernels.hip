// Probes of the device's ceilings: what a plain read-only, write-only and copy kernel reach of
// the memory system, and what a loop of independent matrix-core instructions reaches of the
// matrix cores.  They measure what the element-wise passes (Eq. 1-3, 8-10) and the contractions
// (Eq. 4-5) of the method are compared with; they compute nothing of the method.

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

// Matrix-core probe: every wave issues `iters` rounds of eight independent MFMAs (eight
// accumulator tiles, so no instruction waits for the previous one's result); operands stay in
// registers.  MODE 0: v_mfma_f32_16x16x4_f32 (2048 flops each), MODE 1: v_mfma_f32_16x16x32_bf16
// (16384 flops each).
constexpr int kMfmaProbeBlocks = 2048, kMfmaProbeAcc = 8;
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

template <int MODE>
__global__ __launch_bounds__(kProbeThreads) void probe_mfma_kernel(float* __restrict__ out, int iters, float seed) {
  floatx4 acc[kMfmaProbeAcc];
#pragma unroll
  for (int i = 0; i < kMfmaProbeAcc; ++i) acc[i] = floatx4{0.f, 0.f, 0.f, 0.f};
  const float av = seed + (float)threadIdx.x * 1e-6f, bv = seed;
  bf16x8 a8, b8;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    a8[i] = (__bf16)(av + (float)i);
    b8[i] = (__bf16)bv;
  }
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < kMfmaProbeAcc; ++i) {
      if constexpr (MODE == 0) acc[i] = __builtin_amdgcn_mfma_f32_16x16x4f32(av, bv, acc[i], 0, 0, 0);
      else acc[i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a8, b8, acc[i], 0, 0, 0);
    }
  }
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < kMfmaProbeAcc; ++i) s += acc[i][0] + acc[i][1] + acc[i][2] + acc[i][3];
  out[(size_t)blockIdx.x * kProbeThreads + threadIdx.x] = s;
}

}  // namespace
}  // namespace abl

extern "C" size_t abl_mfma_probe_out_bytes(void) {
  return (size_t)abl::kMfmaProbeBlocks * abl::kProbeThreads * sizeof(float);
}

extern "C" double abl_mfma_probe_flops(int mode, int iters) {
  if (mode < 0 || mode > 1 || iters < 1) return 0.0;
  const double per = mode == 0 ? 2.0 * 16 * 16 * 4 : 2.0 * 16 * 16 * 32;
  return (double)abl::kMfmaProbeBlocks * (abl::kProbeThreads / 64) * (double)iters * abl::kMfmaProbeAcc * per;
}

extern "C" int abl_mfma_probe(void* stream, int mode, int iters, void* out, size_t out_bytes) {
  using namespace abl;
  if (mode < 0 || mode > 1 || iters < 1 || iters > (1 << 24)) return ABL_ERR_ARG;
  if (out == nullptr || (reinterpret_cast<uintptr_t>(out) & 15u)) return ABL_ERR_ARG;
  if (out_bytes < abl_mfma_probe_out_bytes()) return ABL_ERR_SCRATCH;
  hipStream_t st = (hipStream_t)stream;
  if (mode == 0) probe_mfma_kernel<0><<<kMfmaProbeBlocks, kProbeThreads, 0, st>>>(static_cast<float*>(out), iters, 1.0f);
  else probe_mfma_kernel<1><<<kMfmaProbeBlocks, kProbeThreads, 0, st>>>(static_cast<float*>(out), iters, 1.0f);
  return hip_status();
}

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
