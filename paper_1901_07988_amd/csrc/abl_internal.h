// Internal declarations shared by the HIP translation units of libabl (not part of the ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "abl.h"

namespace abl {

// Planes of the per-channel `stats` block, each C 4-byte values.
enum StatPlane { P_MEAN = 0, P_VAR, P_RSTD, P_GAMMA, P_BETA, P_CQ, P_STEP, P_FB };

constexpr int kMaxPartialBlocks = 1024;  // upper bound on per-block reduction partials

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

// ---- convolution kernels (conv_kernels.hip) ----
size_t wgrad_partial_bytes(const abl_shape& s);
int launch_conv_fwd(hipStream_t st, const abl_shape& s, const float* a3, const float* w,
                    const float* skip, float* y);
int launch_conv_dgrad(hipStream_t st, const abl_shape& s, const float* dy, const float* w,
                      float* da3);
int launch_conv_wgrad_packed(hipStream_t st, const abl_shape& s, int K, const void* packed,
                             const void* stats, const float* dy, void* scratch, float* dw);

inline int out_dim(int in, int pad, int f, int stride) { return (in + 2 * pad - f) / stride + 1; }

inline int hip_status() { return hipGetLastError() == hipSuccess ? ABL_OK : ABL_ERR_HIP; }

}  // namespace abl
