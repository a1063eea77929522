// Internal declarations shared by the HIP translation units of libabl (not part of the ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "abl.h"

namespace abl {

// Planes of the per-channel `stats` block, each C 4-byte values.
enum StatPlane { P_MEAN = 0, P_VAR, P_RSTD, P_GAMMA, P_BETA, P_CQ, P_STEP, P_FB };

constexpr int kMaxPartialBlocks = 512;  // upper bound on per-block reduction partials

// Bytes of partial-sum workspace for the per-channel reductions over [M,C].
size_t bn_partial_bytes(int64_t M, int C);

// ---- batch-norm / quantizer kernels (bn_kernels.hip) ----
int launch_bn_stats(hipStream_t st, const float* x, int64_t M, int C, const float* gamma,
                    const float* beta, int K, void* scratch, void* stats);
// naive: a3 = ReLU of the dequantized code instead of the exact A3 (the baseline of Sec. 4).
// slope: 0 = ReLU (Eq. 3); > 0 = leaky ReLU (Sec. 3.4), in every launcher below that takes one.
int launch_bn_relu_pack(hipStream_t st, const float* x, int64_t M, int C, int K, const void* stats,
                        float* a3, void* packed, bool naive = false, float slope = 0.0f);
int launch_pack(hipStream_t st, const float* a2, int64_t M, int C, int K, const void* stats,
                void* packed);
// act: apply the non-linearity to the dequantized values (the A3~ the weight gradient contracts).
int launch_unpack(hipStream_t st, const void* packed, int64_t M, int C, int K, const void* stats,
                  float* a2t, bool act = false, float slope = 0.0f);
// The second halves of the two reductions, for partial sums produced elsewhere (conv epilogues).
size_t bn_means_offset(int C);
int launch_bn_stats_finalize(hipStream_t st, const double* partial, int nb, const float* shift_row, int64_t M,
                             int C, const float* gamma, const float* beta, int K, void* stats);
// dwsum (nullable): a weight gradient left as `copies` partial copies of n floats by the conv
// backward kernel; the finalize launch also sums them into dw (fixed order).
struct DwSum {
  const float* partial;
  int copies;
  int64_t n;
  float* dw;
};
int launch_sgd_momentum(hipStream_t st, int64_t n, float lr, float mu, float wd, float* w, const float* grad,
                        float* v);
// Backward of BN + ReLU from dA3 and the codes (Eq. 6-8): both passes.
int launch_bn_bwd(hipStream_t st, const void* packed, const void* stats, const float* da3, int64_t M,
                  int C, int K, bool accum, void* scratch, float* dx, float* dgamma, float* dbeta,
                  const DwSum* dwsum = nullptr, float slope = 0.0f);
int launch_bn_bwd_finish(hipStream_t st, const void* packed, const void* stats, const float* da3, int64_t M,
                         int C, int K, bool accum, void* scratch, int nb, float* dx, float* dgamma,
                         float* dbeta, const DwSum* dwsum = nullptr, float slope = 0.0f);

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
int launch_halo_conv(hipStream_t st, const ConvGeom& g, int mode, bool bf16, const float* in, const float* w,
                     const float* skip, float* out, double* out_partial = nullptr);
// Forward with Eq. 1-3 and Eq. 9 applied while the input patch is staged: reads x, writes y and
// the packed codes; A3 never reaches memory.  Supported for 'same' stride-1 convolutions.
bool halo_fused_supported(const ConvGeom& g);
// out_partial (nullable): [tiles][2][Cout] doubles = per-tile sum(y), sum(y^2) of the output,
// the first pass of the next layer's statistics.  halo_tile_count gives `tiles` (0: unsupported).
int halo_tile_count(const ConvGeom& g, int mode);
int launch_halo_fwd_fused(hipStream_t st, const ConvGeom& g, int K, bool bf16, const float* x,
                          const void* stats, const float* w, const float* skip, float* y, void* packed,
                          double* out_partial);
// Gradient to the conv input with the first pass of the BN backward (Eq. 6-7 sums from the
// layer's packed codes) in the epilogue: partial = [tiles][2][Cin] doubles.
int launch_halo_dgrad_reduce(hipStream_t st, const ConvGeom& g, int K, bool bf16, const float* dy,
                             const float* w, const void* packed, const void* stats, float* da3,
                             double* partial);

// Weight gradient of stride-1 3x3 convolutions from the packed activation, all taps per pass.
// halo_wgrad_partial_bytes returns 0 when the shape is not supported.
size_t halo_wgrad_partial_bytes(const ConvGeom& g);
int launch_halo_wgrad(hipStream_t st, const ConvGeom& g, int K, bool bf16, const void* packed, const float* stats,
                      const float* dy, void* scratch, float* dw);

// Whole conv backward of a 3x3 'same' stride-1 layer with 16 input and 16 output channels:
// dA3, the Eq. 6-7 partial sums ([tiles][2][16] doubles) and dW in one pass over dy and the codes.
// halo_bwd16_tiles returns 0 when the shape is not supported.  wscratch: as for launch_halo_wgrad.
int halo_bwd16_tiles(const ConvGeom& g);
// dw == nullptr: the per-tile copies of dW ([tiles][3][3][16][16]) are left in wscratch unsummed.
int launch_halo_bwd16(hipStream_t st, const ConvGeom& g, int K, bool bf16, const float* dy, const float* w,
                      const void* packed, const void* stats, float* da3, double* partial, void* wscratch,
                      float* dw);

// ---- convolution kernels (conv_kernels.hip) ----
size_t wgrad_partial_bytes(const abl_shape& s);
// sums / rows (nullable): where the kernel can, it leaves per-block fp64 sums of y and y^2
// ([rows][2][Cout], *rows <= kMaxPartialBlocks) for the next layer's statistics; *rows = 0 if not.
int launch_conv_fwd(hipStream_t st, const abl_shape& s, bool bf16, const float* a3, const float* w,
                    const float* skip, float* y, double* sums = nullptr, int* rows = nullptr);
int launch_conv_dgrad(hipStream_t st, const abl_shape& s, bool bf16, const float* dy, const float* w,
                      float* da3);
// Forward of a 1x1 stride-1 convolution without padding with Eq. 1-3 and Eq. 9 applied while the
// A tile is staged: reads x, writes y and the packed codes; A3 never reaches memory.  y must not
// alias x.
// 1x1 stride-1 convolutions without padding whose channel counts allow it (contraction a
// multiple of 64, outputs a multiple of 16) run as plain GEMMs with the activation operand
// loaded straight into MFMA layout.  mode 0 forward (skip nullable), 1 dgrad.
bool pointwise_supported(const ConvGeom& g, int mode);
int launch_pointwise_conv(hipStream_t st, const ConvGeom& g, int mode, bool bf16, const float* in, const float* w,
                          const float* skip, float* out, double* sums = nullptr, int* rows = nullptr);
int launch_pointwise_fwd_fused(hipStream_t st, const ConvGeom& g, int K, bool bf16, const float* x, const float* stats,
                               const float* w, const float* skip, float* y, void* packed, double* sums = nullptr,
                               int* rows = nullptr);
// dgrad (Eq. 5) with the Eq. 6-7 sums taken in its epilogue from the layer's codes: one row of
// [2][Cin] doubles per block, *rows of them (<= kMaxPartialBlocks), for launch_bn_bwd_finish.
int launch_pointwise_dgrad_reduce(hipStream_t st, const ConvGeom& g, int K, bool bf16, const float* dy, const float* w,
                                  const void* packed, const void* stats, float* da3, double* sums, int* rows);
bool igemm_fused_supported(const abl_shape& s);
int launch_conv_fwd_fused(hipStream_t st, const abl_shape& s, int K, bool bf16, const float* x, const void* stats,
                          const float* w, const float* skip, float* y, void* packed, double* sums = nullptr,
                          int* rows = nullptr);
// K = 32: `packed` is an fp32 tensor, used as it is or (relu32) as the pre-ReLU activation A2.
// defer (nullable): where the kernel leaves split partial copies, describe them there instead of
// summing them (copies = 0 when dw is already complete) - for launch_bn_bwd_finish.
int launch_conv_wgrad_packed(hipStream_t st, const abl_shape& s, int K, bool bf16, const void* packed,
                             const void* stats, const float* dy, void* scratch, float* dw, bool relu32 = false,
                             DwSum* defer = nullptr);

// ---- ABL_MATH_BF16 contractions on the 32-deep bf16 matrix instruction (conv_bf16.hip) ----
// Forward (mode 0) / gradient to the input (mode 1) of any stride, filter and padding whose
// contraction channels are a multiple of 32 and output channels a multiple of 64.
bool bf16_gemm_supported(const ConvGeom& g, int mode);
// sums / rows (nullable, mode 0): [*rows][2][Cout] doubles = per-block sum(y), sum(y^2) of the output;
// *rows = 0 when the kernel leaves none (more blocks than kMaxPartialBlocks).
int launch_bf16_gemm(hipStream_t st, const ConvGeom& g, int mode, const float* in, const float* w, const float* skip,
                     float* out, double* sums = nullptr, int* rows = nullptr);
// Gradient to the conv input with the Eq. 6-7 sums from the layer's codes (K = 4 / 8) in the epilogue of
// whichever bf16 kernel takes the shape: partial = [rows][2][Cin] doubles; bf16_dgrad_reduce_rows = 0 if none does.
int bf16_dgrad_reduce_rows(const ConvGeom& g);
int launch_bf16_dgrad_reduce(hipStream_t st, const ConvGeom& g, int K, const float* dy, const float* w,
                             const void* packed, const void* stats, float* da3, double* partial);
// 3x3 'same' stride-1 convolutions whose whole image fits in LDS as bf16 (up to 208 pixels, e.g.
// 14x14 with 256 channels): one block per image and 64 output channels.
// sums (nullable, mode 0): [N][2][Cout] doubles = per-image sum(y), sum(y^2) of the output.
bool image_bf16_supported(const ConvGeom& g, int mode);
int launch_image_bf16(hipStream_t st, const ConvGeom& g, int mode, const float* in, const float* w,
                      const float* skip, float* out, double* sums);

// ---- fp32 3x3 'same' stride-1 convolutions with the whole image resident in LDS (conv_image.hip) ----
// Images of up to 208 pixels (14x14, 7x7 ...), 16, 32 or a multiple of 64 contraction channels,
// output channels a multiple of 64, at most kMaxPartialBlocks images and at least 224 blocks: one
// block per image and 64 output channels.
// sums (nullable, mode 0): [N][2][Cout] doubles = per-image sum(y), sum(y^2) of the output.
bool image_f32_supported(const ConvGeom& g, int mode);
int launch_image_f32(hipStream_t st, const ConvGeom& g, int mode, const float* in, const float* w,
                     const float* skip, float* out, double* sums);
// Gradient to the conv input with the Eq. 6-7 sums from the layer's packed codes (K = 4 / 8) in the
// epilogue: partial = [N][2][Cin] doubles, one row per image.
int launch_image_dgrad_reduce(hipStream_t st, const ConvGeom& g, int K, const float* dy, const float* w,
                              const void* packed, const void* stats, float* da3, double* partial);

// Weight gradient of the same layers (14-pixel-wide images) from the K-bit codes (K = 4 / 8): one
// block per 32 x 64 tile of (input, output) channels and share of the images, each share leaving
// its own copy of dW in `copies` ([image_wgrad_copies][R][S][Cin][Cout] floats) for the caller to
// sum.  image_wgrad_copies returns 0 when the shape is not supported.  bf16: operands rounded to bf16,
// 16 pixels per MFMA.
int image_wgrad_copies(const ConvGeom& g, int K);
int launch_image_wgrad(hipStream_t st, const ConvGeom& g, int K, bool bf16, const void* packed, const float* stats,
                       const float* dy, float* copies);

// Weight gradient of a 1x1 stride-1 layer from its K-bit codes with the block's 64 x 256 tile of dW in
// registers (fp32; Cin a multiple of 64, Cout of 256, N H W of 16).  Each share of the pixels
// writes its own copy of dW in `copies` ([rows_wgrad_copies][Cin][Cout] floats) for the caller to sum.
// rows_wgrad_copies returns 0 when the shape is not supported.
// bf16: operands rounded to bf16 and contracted 32 pixels per MFMA (N H W a multiple of 32).
int rows_wgrad_copies(const ConvGeom& g, int K, bool bf16);
int launch_rows_wgrad(hipStream_t st, const ConvGeom& g, int K, bool bf16, const void* packed, const float* stats,
                      const float* dy, float* copies);

// 1x1 stride-1 convolutions (channel counts in multiples of 64) with the block's whole output tile in
// accumulator registers and the operands loaded straight from global memory, for shapes that give
// about one block per compute unit.  rows_f32_blocks: number of row blocks = rows of the sums
// ([blocks][2][C] doubles: of y in mode 0, Eq. 6-7 in launch_rows_dgrad_reduce), 0 = not supported.
int rows_f32_blocks(const ConvGeom& g, int mode);
int launch_rows_f32(hipStream_t st, const ConvGeom& g, int mode, const float* in, const float* w, const float* skip,
                    float* out, double* sums);
int launch_rows_dgrad_reduce(hipStream_t st, const ConvGeom& g, int K, const float* dy, const float* w,
                             const void* packed, const void* stats, float* da3, double* partial);

// ---- Eq. 9 / Eq. 10 for one value.  Callers must be compiled with floating-point contraction
// off: the codes are compared bit for bit with an IEEE fp32 evaluation.
// floor() limited to +-2^24 so that the integer conversion is defined for any input.
__device__ inline float limit_floor(float u) {
  const float lim = 16777216.0f;
  // one instruction: the median of (u, -lim, lim); a NaN input gives the smallest of the other
  // two, -lim, as the comparison form (u >= -lim ? u : -lim) does
  return __builtin_amdgcn_fmed3f(floorf(u), -lim, lim);
}

// Eq. 9 for one value (cq = 2^K/(6 gamma), fb = floor(beta*cq)).  K = 32 is exact storage: the
// "code" is the value's bit pattern.
template <int K>
__device__ inline uint32_t quant_code(float a2, float cq, int32_t fb) {
  if constexpr (K == 32) {
    return __float_as_uint(a2);
  } else {
    const float u = limit_floor(a2 * cq);
    int32_t v = (int32_t)u + (1 << (K - 1)) - fb;
    v = v < 0 ? 0 : v;
    v = v > (1 << K) - 1 ? (1 << K) - 1 : v;
    return (uint32_t)v;
  }
}

// Eq. 10 for one code.
template <int K>
__device__ inline float dequant(uint32_t q, float step, int32_t fb) {
  if constexpr (K == 32) {
    return __uint_as_float(q);
  } else {
    const int32_t j = (int32_t)q - (1 << (K - 1)) + fb;
    const float t = (float)j + 0.5f;
    return step * t;
  }
}

// Sum over the 16 lanes of a row (lanes that differ in bits 0-3); every lane gets the total.
// (Data-parallel-primitive moves within the row: swap neighbours, swap pairs, mirror each half,
// mirror the row.)
template <int CTRL>
__device__ inline double dpp_move(double v) {
  const unsigned long long u = __double_as_longlong(v);
  const int lo = __builtin_amdgcn_update_dpp(0, (int)(unsigned)u, CTRL, 0xf, 0xf, false);
  const int hi = __builtin_amdgcn_update_dpp(0, (int)(unsigned)(u >> 32), CTRL, 0xf, 0xf, false);
  return __longlong_as_double(((unsigned long long)(unsigned)hi << 32) | (unsigned)lo);
}
__device__ inline double row16_sum(double v) {
  v += dpp_move<0xB1>(v);   // quad_perm [1,0,3,2]
  v += dpp_move<0x4E>(v);   // quad_perm [2,3,0,1]
  v += dpp_move<0x141>(v);  // row_half_mirror
  v += dpp_move<0x140>(v);  // row_mirror
  return v;
}

typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef short shortx4 __attribute__((ext_vector_type(4)));

// D = A(16x4) * B(4x16) + C on the fp32 matrix cores; lane l supplies A[l%16][l/16] and
// B[l/16][l%16] and holds D[4*(l/16) + r][l%16], r = 0..3.
__device__ inline floatx4 mfma16(float a, float b, floatx4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0);
}

// fp32 -> bf16, round to nearest even, by the hardware's packed convert (v_cvt_pk_bf16_f32).
typedef __bf16 bf16x4_t __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
// eight floats -> the 8-deep bf16 operand of one lane of v_mfma_f32_16x16x32_bf16
__device__ inline bf16x8_t to_bf16x8(const float (&v)[8]) {
  return bf16x8_t{(__bf16)v[0], (__bf16)v[1], (__bf16)v[2], (__bf16)v[3],
                  (__bf16)v[4], (__bf16)v[5], (__bf16)v[6], (__bf16)v[7]};
}
__device__ inline shortx4 to_bf16x4(const float4& v) {
  const bf16x4_t b = {(__bf16)v.x, (__bf16)v.y, (__bf16)v.z, (__bf16)v.w};
  return __builtin_bit_cast(shortx4, b);
}

// Contract four consecutive k (one float4 per lane and operand row) into every accumulator
// tile.  fp32: four 16x16x4 MFMAs per tile, component e of the float4 = k-step e, the lane
// group l/16 = k within the step.  bf16: operands rounded to bf16, ONE 16x16x16 MFMA per
// tile, lane group l/16 supplies k = 4*(l/16) + e; accumulation stays fp32.
template <bool BF16, int MT, int NT>
__device__ inline void mma_k4(const float4 (&af)[MT], const float4 (&bf)[NT], floatx4 (&acc)[MT][NT]) {
  if constexpr (BF16) {
    shortx4 a[MT], b[NT];
#pragma unroll
    for (int i = 0; i < MT; ++i) a[i] = to_bf16x4(af[i]);
#pragma unroll
    for (int j = 0; j < NT; ++j) b[j] = to_bf16x4(bf[j]);
#pragma unroll
    for (int i = 0; i < MT; ++i)
#pragma unroll
      for (int j = 0; j < NT; ++j)
        acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(a[i], b[j], acc[i][j], 0, 0, 0);
  } else {
    // k-step outermost: consecutive MFMAs write different accumulators
#pragma unroll
    for (int i = 0; i < MT; ++i)
#pragma unroll
      for (int j = 0; j < NT; ++j) acc[i][j] = mfma16(af[i].x, bf[j].x, acc[i][j]);
#pragma unroll
    for (int i = 0; i < MT; ++i)
#pragma unroll
      for (int j = 0; j < NT; ++j) acc[i][j] = mfma16(af[i].y, bf[j].y, acc[i][j]);
#pragma unroll
    for (int i = 0; i < MT; ++i)
#pragma unroll
      for (int j = 0; j < NT; ++j) acc[i][j] = mfma16(af[i].z, bf[j].z, acc[i][j]);
#pragma unroll
    for (int i = 0; i < MT; ++i)
#pragma unroll
      for (int j = 0; j < NT; ++j) acc[i][j] = mfma16(af[i].w, bf[j].w, acc[i][j]);
  }
}

// The same contraction for the first NB (compile-time, <= NT) tiles of the second operand only;
// the others are left untouched and cost no matrix-core time.
template <bool BF16, int MT, int NT, int NB>
__device__ inline void mma_k4_first(const float4 (&af)[MT], const float4 (&bf)[NT], floatx4 (&acc)[MT][NT]) {
  static_assert(NB <= NT, "at most all tiles");
  if constexpr (BF16) {
    shortx4 a[MT], b[NB > 0 ? NB : 1];
#pragma unroll
    for (int i = 0; i < MT; ++i) a[i] = to_bf16x4(af[i]);
#pragma unroll
    for (int j = 0; j < NB; ++j) b[j] = to_bf16x4(bf[j]);
#pragma unroll
    for (int i = 0; i < MT; ++i)
#pragma unroll
      for (int j = 0; j < NB; ++j)
        acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(a[i], b[j], acc[i][j], 0, 0, 0);
  } else {
#pragma unroll
    for (int i = 0; i < MT; ++i)
#pragma unroll
      for (int j = 0; j < NB; ++j) acc[i][j] = mfma16(af[i].x, bf[j].x, acc[i][j]);
#pragma unroll
    for (int i = 0; i < MT; ++i)
#pragma unroll
      for (int j = 0; j < NB; ++j) acc[i][j] = mfma16(af[i].y, bf[j].y, acc[i][j]);
#pragma unroll
    for (int i = 0; i < MT; ++i)
#pragma unroll
      for (int j = 0; j < NB; ++j) acc[i][j] = mfma16(af[i].z, bf[j].z, acc[i][j]);
#pragma unroll
    for (int i = 0; i < MT; ++i)
#pragma unroll
      for (int j = 0; j < NB; ++j) acc[i][j] = mfma16(af[i].w, bf[j].w, acc[i][j]);
  }
}

// v where ok, zeros elsewhere - written per component so that it stays in registers
__device__ inline float4 keep_if(bool ok, const float4& v) {
  return make_float4(ok ? v.x : 0.f, ok ? v.y : 0.f, ok ? v.z : 0.f, ok ? v.w : 0.f);
}

inline int hip_status() { return hipGetLastError() == hipSuccess ? ABL_OK : ABL_ERR_HIP; }

}  // namespace abl
