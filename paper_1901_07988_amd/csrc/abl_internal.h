// Internal declarations shared by the HIP translation units of libabl (not part of the ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "abl.h"

namespace abl {

// Planes of the per-channel `stats` block, each C 4-byte values.
enum StatPlane { P_MEAN = 0, P_VAR, P_RSTD, P_GAMMA, P_BETA, P_CQ, P_STEP, P_FB };

constexpr int kMaxPartialBlocks = 512;   // upper bound on per-block reduction partials

// Bytes of partial-sum workspace for the per-channel reductions over [M,C].
size_t bn_partial_bytes(int64_t M, int C);

// ---- batch-norm / quantizer kernels (bn_kernels.hip) ----
int launch_bn_stats(hipStream_t st, const float* x, int64_t M, int C, const float* gamma,
                    const float* beta, int K, void* scratch, void* stats);
int launch_bn_relu_pack(hipStream_t st, const float* x, int64_t M, int C, int K, const void* stats,
                        float* a3, void* packed);
int launch_pack(hipStream_t st, const float* a2, int64_t M, int C, int K, const void* stats,
                void* packed);
int launch_unpack(hipStream_t st, const void* packed, int64_t M, int C, int K, const void* stats,
                  float* a2t);
int launch_bn_bwd(hipStream_t st, const void* packed, const void* stats, const float* da3, int64_t M,
                  int C, int K, bool accum, void* scratch, float* dx, float* dgamma, float* dbeta);

// Convolution geometry passed to the kernels by value.
struct ConvGeom {
  int N, H, W, Cin, Cout, R, S, stride, pad, Ho, Wo;
};

inline int out_dim(int in, int pad, int f, int stride) { return (in + 2 * pad - f) / stride + 1; }

inline ConvGeom geom_of(const abl_shape& s) {
  ConvGeom g;
  g.N = s.N; g.H = s.H; g.W = s.W; g.Cin = s.Cin; g.Cout = s.Cout;
  g.R = s.R; g.S = s.S; g.stride = s.stride; g.pad = s.pad;
  g.Ho = out_dim(s.H, s.pad, s.R, s.stride);
  g.Wo = out_dim(s.W, s.pad, s.S, s.stride);
  return g;
}

// ---- stride-1 convolutions with the input tile staged once in LDS (conv_halo.hip) ----
// mode 0: forward, mode 1: gradient to the input.
bool halo_conv_supported(const ConvGeom& g);
int launch_halo_conv(hipStream_t st, const ConvGeom& g, int mode, const float* in, const float* w,
                     const float* skip, float* out);

// Weight gradient of stride-1 3x3 convolutions from the packed activation, all taps per pass.
// halo_wgrad_partial_bytes returns 0 when the shape is not supported.
size_t halo_wgrad_partial_bytes(const ConvGeom& g);
int launch_halo_wgrad(hipStream_t st, const ConvGeom& g, int K, const void* packed, const float* stats,
                      const float* dy, void* scratch, float* dw);

// ---- convolution kernels (conv_kernels.hip) ----
size_t wgrad_partial_bytes(const abl_shape& s);
int launch_conv_fwd(hipStream_t st, const abl_shape& s, const float* a3, const float* w,
                    const float* skip, float* y);
int launch_conv_dgrad(hipStream_t st, const abl_shape& s, const float* dy, const float* w,
                      float* da3);
int launch_conv_wgrad_packed(hipStream_t st, const abl_shape& s, int K, const void* packed,
                             const void* stats, const float* dy, void* scratch, float* dw);

// v where ok, zeros elsewhere - written per component so that it stays in registers
__device__ inline float4 keep_if(bool ok, const float4& v) {
  return make_float4(ok ? v.x : 0.f, ok ? v.y : 0.f, ok ? v.z : 0.f, ok ? v.w : 0.f);
}

inline int hip_status() { return hipGetLastError() == hipSuccess ? ABL_OK : ABL_ERR_HIP; }

}  // namespace abl
