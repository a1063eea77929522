// C ABI of libabl: argument validation, workspace carving and the order in which the
// kernels of one layer step (and of a residual stack) are enqueued.  No device code here.

#include "abl_internal.h"

using namespace abl;

namespace {

inline size_t up256(size_t v) { return (v + 255) / 256 * 256; }

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

inline bool bad_ptr(const void* p) { return p == nullptr || !aligned16(p); }

// K = 32 is exact storage (the fp32 A2 itself is kept, Sec. 3.2's alpha = 1); the fused kernels
// and the conv -> BN -> ReLU grouping take the two quantized widths only.
int check_k(int K) { return (K == 4 || K == 8 || K == 32) ? ABL_OK : ABL_ERR_ARG; }
int check_k48(int K) { return (K == 4 || K == 8) ? ABL_OK : ABL_ERR_ARG; }

int check_shape(const abl_shape* s) {
  if (s == nullptr) return ABL_ERR_ARG;
  if (s->N < 1 || s->H < 1 || s->W < 1 || s->Cin < 1 || s->Cout < 1 || s->R < 1 || s->S < 1 ||
      s->stride < 1 || s->pad < 0)
    return ABL_ERR_SHAPE;
  if (s->H + 2 * s->pad < s->R || s->W + 2 * s->pad < s->S) return ABL_ERR_SHAPE;
  const int64_t lim = 2147483647LL;
  const int64_t e_in = (int64_t)s->N * s->H * s->W * s->Cin;
  const int64_t e_out = (int64_t)s->N * out_dim(s->H, s->pad, s->R, s->stride) *
                        out_dim(s->W, s->pad, s->S, s->stride) * s->Cout;
  const int64_t e_w = (int64_t)s->R * s->S * s->Cin * s->Cout;
  if (e_in > lim || e_out > lim || e_w > lim) return ABL_ERR_SHAPE;
  return ABL_OK;
}

int check_mc(int64_t M, int32_t C) {
  if (M < 1 || C < 1) return ABL_ERR_SHAPE;
  if (M * C > 2147483647LL) return ABL_ERR_SHAPE;
  return ABL_OK;
}

inline int64_t rows_of(const abl_shape& s) { return (int64_t)s.N * s.H * s.W; }

size_t packed_bytes_of(int64_t E, int K) { return (size_t)(((E * K + 7) / 8 + 127) / 128 * 128); }

}  // namespace

extern "C" {

const char* abl_error_string(int code) {
  switch (code) {
    case ABL_OK: return "ok";
    case ABL_ERR_ARG: return "invalid argument (null or misaligned pointer, unsupported K or flag)";
    case ABL_ERR_SHAPE: return "invalid shape";
    case ABL_ERR_SCRATCH: return "scratch buffer too small";
    case ABL_ERR_HIP: return "HIP launch failure";
    default: return "unknown error";
  }
}

size_t abl_packed_bytes(const abl_shape* s, int K) {
  if (check_shape(s) != ABL_OK || check_k(K) != ABL_OK) return 0;
  return packed_bytes_of(rows_of(*s) * s->Cin, K);
}

size_t abl_stats_bytes(const abl_shape* s) {
  if (check_shape(s) != ABL_OK) return 0;
  return (size_t)ABL_STATS_PLANES * 4 * (size_t)s->Cin;
}

size_t abl_bn_scratch_bytes(int64_t M, int32_t C) {
  if (check_mc(M, C) != ABL_OK) return 0;
  return bn_partial_bytes(M, C);
}

size_t abl_wgrad_scratch_bytes(const abl_shape* s) {
  if (check_shape(s) != ABL_OK) return 0;
  return wgrad_partial_bytes(*s);
}

size_t abl_scratch_bytes(const abl_shape* s, int K) {
  if (check_shape(s) != ABL_OK || check_k(K) != ABL_OK) return 0;
  const size_t act = up256((size_t)rows_of(*s) * s->Cin * sizeof(float));
  return act + up256(bn_partial_bytes(rows_of(*s), s->Cin)) + wgrad_partial_bytes(*s);
}

int abl_bn_stats(void* stream, const float* x, int64_t M, int32_t C, const float* gamma,
                 const float* beta, int K, void* scratch, size_t scratch_bytes, void* stats) {
  if (int e = check_k(K)) return e;
  if (int e = check_mc(M, C)) return e;
  if (bad_ptr(x) || bad_ptr(gamma) || bad_ptr(beta) || bad_ptr(scratch) || bad_ptr(stats)) return ABL_ERR_ARG;
  if (scratch_bytes < bn_partial_bytes(M, C)) return ABL_ERR_SCRATCH;
  return launch_bn_stats((hipStream_t)stream, x, M, C, gamma, beta, K, scratch, stats);
}

int abl_bn_relu_pack(void* stream, const float* x, int64_t M, int32_t C, int K, const void* stats,
                     float* a3, void* packed) {
  if (int e = check_k(K)) return e;
  if (int e = check_mc(M, C)) return e;
  if (bad_ptr(x) || bad_ptr(stats) || bad_ptr(a3) || bad_ptr(packed)) return ABL_ERR_ARG;
  return launch_bn_relu_pack((hipStream_t)stream, x, M, C, K, stats, a3, packed);
}

int abl_pack(void* stream, const float* a2, int64_t M, int32_t C, int K, const void* stats,
             void* packed) {
  if (int e = check_k(K)) return e;
  if (int e = check_mc(M, C)) return e;
  if (bad_ptr(a2) || bad_ptr(stats) || bad_ptr(packed)) return ABL_ERR_ARG;
  return launch_pack((hipStream_t)stream, a2, M, C, K, stats, packed);
}

int abl_unpack(void* stream, const void* packed, int64_t M, int32_t C, int K, const void* stats,
               float* a2t) {
  if (int e = check_k(K)) return e;
  if (int e = check_mc(M, C)) return e;
  if (bad_ptr(packed) || bad_ptr(stats) || bad_ptr(a2t)) return ABL_ERR_ARG;
  return launch_unpack((hipStream_t)stream, packed, M, C, K, stats, a2t);
}

int abl_bn_bwd(void* stream, const void* packed, const void* stats, const float* da3, int64_t M,
               int32_t C, int K, uint32_t flags, void* scratch, size_t scratch_bytes, float* dx,
               float* dgamma, float* dbeta) {
  if (int e = check_k(K)) return e;
  if (int e = check_mc(M, C)) return e;
  if (flags & ~(uint32_t)ABL_ACCUM_DX) return ABL_ERR_ARG;
  if (bad_ptr(packed) || bad_ptr(stats) || bad_ptr(da3) || bad_ptr(scratch) || bad_ptr(dx) ||
      bad_ptr(dgamma) || bad_ptr(dbeta))
    return ABL_ERR_ARG;
  if (scratch_bytes < bn_partial_bytes(M, C)) return ABL_ERR_SCRATCH;
  return launch_bn_bwd((hipStream_t)stream, packed, stats, da3, M, C, K, (flags & ABL_ACCUM_DX) != 0,
                       scratch, dx, dgamma, dbeta);
}

int abl_conv_fwd(void* stream, const abl_shape* s, uint32_t flags, const float* a3, const float* W,
                 const float* skip, float* y) {
  if (int e = check_shape(s)) return e;
  if (flags & ~(uint32_t)ABL_MATH_BF16) return ABL_ERR_ARG;
  if (bad_ptr(a3) || bad_ptr(W) || bad_ptr(y) || (skip != nullptr && !aligned16(skip))) return ABL_ERR_ARG;
  return launch_conv_fwd((hipStream_t)stream, *s, (flags & ABL_MATH_BF16) != 0, a3, W, skip, y);
}

int abl_conv_dgrad(void* stream, const abl_shape* s, uint32_t flags, const float* dy, const float* W,
                   float* da3) {
  if (int e = check_shape(s)) return e;
  if (flags & ~(uint32_t)ABL_MATH_BF16) return ABL_ERR_ARG;
  if (bad_ptr(dy) || bad_ptr(W) || bad_ptr(da3)) return ABL_ERR_ARG;
  return launch_conv_dgrad((hipStream_t)stream, *s, (flags & ABL_MATH_BF16) != 0, dy, W, da3);
}

int abl_conv_wgrad_packed(void* stream, const abl_shape* s, int K, uint32_t flags, const void* packed,
                          const void* stats, const float* dy, void* scratch, size_t scratch_bytes,
                          float* dW) {
  if (int e = check_shape(s)) return e;
  if (flags & ~(uint32_t)ABL_MATH_BF16) return ABL_ERR_ARG;
  if (int e = check_k(K)) return e;
  if (bad_ptr(packed) || bad_ptr(stats) || bad_ptr(dy) || bad_ptr(scratch) || bad_ptr(dW)) return ABL_ERR_ARG;
  if (scratch_bytes < wgrad_partial_bytes(*s)) return ABL_ERR_SCRATCH;
  return launch_conv_wgrad_packed((hipStream_t)stream, *s, K, (flags & ABL_MATH_BF16) != 0, packed, stats, dy,
                                  scratch, dW, K == 32);
}

}  // extern "C"

namespace {

// Which forward kernel a layer with separate input and output takes: 1 = the 'same' stride-1 kernel
// with the Eq. 1-3 / Eq. 9 prologue, 2 = the 1x1 kernel with it, 0 = pack pass + plain contraction.
inline bool aliased(const void* a, const void* b) { return a == b; }
int forward_fused_path(const abl_shape& s, const ConvGeom& g, int K, bool bf16, bool naive) {
  // bf16 operands: the contraction runs on the 32-deep bf16 matrix instruction with bf16 tiles in
  // LDS (its kernel has no BN prologue), so the layer takes the separate stages
  // - where the contraction is heavy enough to pay for the separate normalise-ReLU-pack pass
  // (measured: from 512 flops per input element on; below, e.g. 1x1 256->64 at 56x56, reading x
  // once in the fused kernel wins)
  const bool bf16_gemm = bf16 && bf16_gemm_supported(g, 0) && 2 * g.Cout * g.R * g.S >= 512;
  if (K == 32 || naive || bf16_gemm) return 0;
  // (Not for the small images of the image-resident kernel: the pack pass plus that kernel is
  // faster than the fused one - 14x14 256->256: 7 + 120 us against 146.)
  if (halo_fused_supported(g) && !(!bf16 && image_f32_supported(g, 0))) return 1;
  // With the prologue every block along the output channels repeats the normalization of its
  // input rows; measured against the separate pack kernel this pays up to 256 output channels.
  // (Not for the long contractions that the register-resident 1x1 kernel takes: the pack pass plus
  // that kernel is faster - 1024 -> 256 at 14x14: 17.6 + 55 us against 81.)
  if (igemm_fused_supported(s) && s.Cout <= 256 && !(!bf16 && rows_f32_blocks(g, 0) > 0)) return 2;
  return 0;
}

// Forward: statistics -> (normalise, ReLU, quantize, pack) -> convolution.  A3 lives in the
// workspace only until the convolution has read it (Sec. 3.2: full-precision intermediates
// are overwritten as soon as they have been used); 'same' stride-1 convolutions do not even
// write it.
//   in_partial / in_nb : first-pass sums of x's statistics left by the producer of x (nullable)
//   out_partial        : where to leave the first-pass sums of y's statistics (nullable);
//                        *out_nb = number of partial rows written, 0 if this layer could not
int forward_impl(hipStream_t st, const abl_shape* s, int K, uint32_t flags, const float* x, const float* W,
                 const float* gamma, const float* beta, const float* skip, void* scratch, float* y,
                 void* packed, void* stats, const double* in_partial, int in_nb, double* out_partial,
                 int* out_nb) {
  const int64_t M = rows_of(*s);
  const size_t act = up256((size_t)M * s->Cin * sizeof(float));
  float* a3 = static_cast<float*>(scratch);
  void* red = static_cast<char*>(scratch) + act;
  const bool bf16 = (flags & ABL_MATH_BF16) != 0;
  const bool naive = (flags & ABL_NAIVE_FWD) != 0 && K != 32;
  if (out_nb != nullptr) *out_nb = 0;
  if (in_partial != nullptr && in_nb > 0) {
    if (int e = launch_bn_stats_finalize(st, in_partial, in_nb, nullptr, M, s->Cin, gamma, beta, K, stats)) return e;
  } else {
    if (int e = launch_bn_stats(st, x, M, s->Cin, gamma, beta, K, red, stats)) return e;
  }
  const ConvGeom g = geom_of(*s);
  const int path = aliased(x, y) ? 0 : forward_fused_path(*s, g, K, bf16, naive);
  // 'same' stride-1 convolutions normalise, quantize and pack while they stage their input
  // patch: x is read once and A3 never reaches memory.  (Not when y aliases x: a block would
  // overwrite input pixels that a neighbouring block has not staged yet.)
  if (path == 1) {
    const int tiles = halo_tile_count(g, 0);
    const bool want = out_partial != nullptr && tiles > 0 && tiles <= kMaxPartialBlocks;
    if (int e = launch_halo_fwd_fused(st, g, K, bf16, x, stats, W, skip, y, packed, want ? out_partial : nullptr))
      return e;
    if (want && out_nb != nullptr) *out_nb = tiles;
    return ABL_OK;
  }
  // 1x1 convolutions do the same while they stage their A tile
  if (path == 2) return launch_conv_fwd_fused(st, *s, K, bf16, x, stats, W, skip, y, packed, out_partial, out_nb);
  if (int e = launch_bn_relu_pack(st, x, M, s->Cin, K, stats, a3, packed, naive)) return e;
  return launch_conv_fwd(st, *s, bf16, a3, W, skip, y, out_partial, out_nb);
}

}  // namespace

extern "C" {

int abl_forward_is_fused(const abl_shape* s, int K, uint32_t flags) {
  if (int e = check_shape(s)) return -e;
  if (int e = check_k(K)) return -e;
  if (flags & ~(uint32_t)(ABL_MATH_BF16 | ABL_NAIVE_FWD)) return -ABL_ERR_ARG;
  return forward_fused_path(*s, geom_of(*s), K, (flags & ABL_MATH_BF16) != 0, (flags & ABL_NAIVE_FWD) != 0 && K != 32) != 0
             ? 1
             : 0;
}

int abl_forward(void* stream, const abl_shape* s, int K, uint32_t flags, const float* x, const float* W,
                const float* gamma, const float* beta, const float* skip, void* scratch,
                size_t scratch_bytes, float* y, void* packed, void* stats) {
  if (int e = check_shape(s)) return e;
  if (int e = check_k(K)) return e;
  if (flags & ~(uint32_t)(ABL_MATH_BF16 | ABL_NAIVE_FWD)) return ABL_ERR_ARG;
  if (bad_ptr(x) || bad_ptr(W) || bad_ptr(gamma) || bad_ptr(beta) || bad_ptr(scratch) || bad_ptr(y) ||
      bad_ptr(packed) || bad_ptr(stats) || (skip != nullptr && !aligned16(skip)))
    return ABL_ERR_ARG;
  if (scratch_bytes < abl_scratch_bytes(s, K)) return ABL_ERR_SCRATCH;
  return forward_impl((hipStream_t)stream, s, K, flags, x, W, gamma, beta, skip, scratch, y, packed, stats,
                      nullptr, 0, nullptr, nullptr);
}

// Backward: dgrad (exact) and wgrad (from the packed copy) consume dy; then the BN/ReLU
// backward turns dA3 into dx.  dx may alias dy because dy is dead once both contractions
// have been enqueued ahead of the kernel that writes dx.
int abl_backward(void* stream, const abl_shape* s, int K, uint32_t flags, const void* packed,
                 const void* stats, const float* dy, const float* W, void* scratch, size_t scratch_bytes,
                 float* dx, float* dW, float* dgamma, float* dbeta) {
  if (int e = check_shape(s)) return e;
  if (int e = check_k(K)) return e;
  if (flags & ~(uint32_t)(ABL_ACCUM_DX | ABL_MATH_BF16)) return ABL_ERR_ARG;
  if (bad_ptr(packed) || bad_ptr(stats) || bad_ptr(dy) || bad_ptr(W) || bad_ptr(scratch) || bad_ptr(dx) ||
      bad_ptr(dW) || bad_ptr(dgamma) || bad_ptr(dbeta))
    return ABL_ERR_ARG;
  if (scratch_bytes < abl_scratch_bytes(s, K)) return ABL_ERR_SCRATCH;
  hipStream_t st = (hipStream_t)stream;
  const int64_t M = rows_of(*s);
  const size_t act = up256((size_t)M * s->Cin * sizeof(float));
  const size_t redb = up256(bn_partial_bytes(M, s->Cin));
  float* da3 = static_cast<float*>(scratch);
  void* red = static_cast<char*>(scratch) + act;
  void* wpart = static_cast<char*>(scratch) + act + redb;
  const bool bf16 = (flags & ABL_MATH_BF16) != 0;
  const bool accum = (flags & ABL_ACCUM_DX) != 0;
  const ConvGeom g = geom_of(*s);
  // Stride-1 convolutions with a filter larger than 1x1 take the Eq. 6-7 sums in the epilogue of
  // the dgrad kernel (dA3 is still in registers there), which saves the reduce pass over dA3.
  // bf16 operands with a dgrad on the 32-deep bf16 matrix instruction: the separate stages
  const bool bf16_gemm = bf16 && bf16_gemm_supported(g, 1);
  // 16-channel 3x3 layers: both contractions and the Eq. 6-7 sums in one kernel
  if (const int t16 = K != 32 ? halo_bwd16_tiles(g) : 0) {
    if (int e = launch_halo_bwd16(st, g, K, bf16, dy, W, packed, stats, da3, static_cast<double*>(red), wpart,
                                  nullptr))
      return e;
    // the second pass of the Eq. 7 sums and the sum of the per-tile copies of dW share a launch
    const DwSum dwsum{static_cast<const float*>(wpart), t16, (int64_t)9 * 16 * 16, dW};
    return launch_bn_bwd_finish(st, packed, stats, da3, M, s->Cin, K, accum, red, t16, dx, dgamma, dbeta, &dwsum);
  }
  // small images (3x3 'same' stride 1): the image-resident kernel, one row of sums per image
  if (K != 32 && !bf16 && image_f32_supported(g, 1)) {
    if (int e = launch_image_dgrad_reduce(st, g, K, dy, W, packed, stats, da3, static_cast<double*>(red))) return e;
    DwSum dwsum;
    if (int e = launch_conv_wgrad_packed(st, *s, K, bf16, packed, stats, dy, wpart, dW, false, &dwsum)) return e;
    return launch_bn_bwd_finish(st, packed, stats, da3, M, s->Cin, K, accum, red, g.N, dx, dgamma, dbeta,
                                dwsum.copies > 0 ? &dwsum : nullptr);
  }
  // bf16 operands on the 32-deep matrix instruction: the same sums in the epilogue of its kernels
  if (const int nr = (K != 32 && bf16_gemm) ? bf16_dgrad_reduce_rows(g) : 0) {
    if (int e = launch_bf16_dgrad_reduce(st, g, K, dy, W, packed, stats, da3, static_cast<double*>(red))) return e;
    DwSum dwsum;
    if (int e = launch_conv_wgrad_packed(st, *s, K, bf16, packed, stats, dy, wpart, dW, false, &dwsum)) return e;
    return launch_bn_bwd_finish(st, packed, stats, da3, M, s->Cin, K, accum, red, nr, dx, dgamma, dbeta,
                                dwsum.copies > 0 ? &dwsum : nullptr);
  }
  const int tiles = K != 32 && !bf16_gemm && halo_conv_supported(g) ? halo_tile_count(g, 1) : 0;
  if (tiles > 0 && tiles <= kMaxPartialBlocks) {
    if (int e = launch_halo_dgrad_reduce(st, g, K, bf16, dy, W, packed, stats, da3, static_cast<double*>(red)))
      return e;
    // split partial copies of dW are summed by the launch that finishes the Eq. 7 sums
    DwSum dwsum;
    if (int e = launch_conv_wgrad_packed(st, *s, K, bf16, packed, stats, dy, wpart, dW, false, &dwsum)) return e;
    return launch_bn_bwd_finish(st, packed, stats, da3, M, s->Cin, K, accum, red, tiles, dx, dgamma, dbeta,
                                dwsum.copies > 0 ? &dwsum : nullptr);
  }
  // 1x1 layers with a long contraction: the register-resident kernel, one row of sums per row block
  if (const int nrb = (K != 32 && !bf16) ? rows_f32_blocks(g, 1) : 0) {
    if (int e = launch_rows_dgrad_reduce(st, g, K, dy, W, packed, stats, da3, static_cast<double*>(red))) return e;
    DwSum dwsum;
    if (int e = launch_conv_wgrad_packed(st, *s, K, bf16, packed, stats, dy, wpart, dW, false, &dwsum)) return e;
    return launch_bn_bwd_finish(st, packed, stats, da3, M, s->Cin, K, accum, red, nrb, dx, dgamma, dbeta,
                                dwsum.copies > 0 ? &dwsum : nullptr);
  }
  // 1x1 stride-1 layers: the same sums in the epilogue of the pointwise dgrad kernel
  if (K != 32 && !bf16_gemm && pointwise_supported(g, 1)) {
    int rows = 0;
    if (int e = launch_pointwise_dgrad_reduce(st, g, K, bf16, dy, W, packed, stats, da3, static_cast<double*>(red),
                                              &rows))
      return e;
    if (rows > 0) {
      DwSum dwsum;
      if (int e = launch_conv_wgrad_packed(st, *s, K, bf16, packed, stats, dy, wpart, dW, false, &dwsum)) return e;
      return launch_bn_bwd_finish(st, packed, stats, da3, M, s->Cin, K, accum, red, rows, dx, dgamma, dbeta,
                                  dwsum.copies > 0 ? &dwsum : nullptr);
    }
    // (long contractions: the kernel computed dA3 only)
    DwSum dwsum;
    if (int e = launch_conv_wgrad_packed(st, *s, K, bf16, packed, stats, dy, wpart, dW, false, &dwsum)) return e;
    return launch_bn_bwd(st, packed, stats, da3, M, s->Cin, K, accum, red, dx, dgamma, dbeta,
                         dwsum.copies > 0 ? &dwsum : nullptr);
  }
  if (int e = launch_conv_dgrad(st, *s, bf16, dy, W, da3)) return e;
  // exact storage keeps the pre-ReLU A2: the weight gradient applies Eq. 3 on the way in
  DwSum dwsum;
  if (int e = launch_conv_wgrad_packed(st, *s, K, bf16, packed, stats, dy, wpart, dW, K == 32, &dwsum)) return e;
  return launch_bn_bwd(st, packed, stats, da3, M, s->Cin, K, accum, red, dx, dgamma, dbeta,
                       dwsum.copies > 0 ? &dwsum : nullptr);
}

// ---- the layer with a leaky ReLU (Sec. 3.4) ---------------------------------------------------
// Same stages as above with the slope passed to the element-wise kernels.  The contraction
// kernels know the plain ReLU only, so the backward first rebuilds A3~ = leaky(Eq. 10) in the
// workspace and hands it to the weight gradient as a full-precision operand; dA3 then takes
// its place.

static int check_slope(float slope) { return (slope >= 0.0f && slope <= 1.0f) ? ABL_OK : ABL_ERR_ARG; }

int abl_leaky_forward(void* stream, const abl_shape* s, int K, uint32_t flags, float slope, const float* x,
                      const float* W, const float* gamma, const float* beta, const float* skip, void* scratch,
                      size_t scratch_bytes, float* y, void* packed, void* stats) {
  if (int e = check_shape(s)) return e;
  if (int e = check_k(K)) return e;
  if (int e = check_slope(slope)) return e;
  if (flags & ~(uint32_t)ABL_MATH_BF16) return ABL_ERR_ARG;
  if (bad_ptr(x) || bad_ptr(W) || bad_ptr(gamma) || bad_ptr(beta) || bad_ptr(scratch) || bad_ptr(y) ||
      bad_ptr(packed) || bad_ptr(stats) || (skip != nullptr && !aligned16(skip)))
    return ABL_ERR_ARG;
  if (scratch_bytes < abl_scratch_bytes(s, K)) return ABL_ERR_SCRATCH;
  hipStream_t st = (hipStream_t)stream;
  const int64_t M = rows_of(*s);
  float* a3 = static_cast<float*>(scratch);
  void* red = static_cast<char*>(scratch) + up256((size_t)M * s->Cin * sizeof(float));
  if (int e = launch_bn_stats(st, x, M, s->Cin, gamma, beta, K, red, stats)) return e;
  if (int e = launch_bn_relu_pack(st, x, M, s->Cin, K, stats, a3, packed, false, slope)) return e;
  return launch_conv_fwd(st, *s, (flags & ABL_MATH_BF16) != 0, a3, W, skip, y);
}

int abl_leaky_backward(void* stream, const abl_shape* s, int K, uint32_t flags, float slope, const void* packed,
                       const void* stats, const float* dy, const float* W, void* scratch, size_t scratch_bytes,
                       float* dx, float* dW, float* dgamma, float* dbeta) {
  if (int e = check_shape(s)) return e;
  if (int e = check_k(K)) return e;
  if (int e = check_slope(slope)) return e;
  if (flags & ~(uint32_t)(ABL_ACCUM_DX | ABL_MATH_BF16)) return ABL_ERR_ARG;
  if (bad_ptr(packed) || bad_ptr(stats) || bad_ptr(dy) || bad_ptr(W) || bad_ptr(scratch) || bad_ptr(dx) ||
      bad_ptr(dW) || bad_ptr(dgamma) || bad_ptr(dbeta))
    return ABL_ERR_ARG;
  if (scratch_bytes < abl_scratch_bytes(s, K)) return ABL_ERR_SCRATCH;
  hipStream_t st = (hipStream_t)stream;
  const int64_t M = rows_of(*s);
  const size_t act = up256((size_t)M * s->Cin * sizeof(float));
  float* buf = static_cast<float*>(scratch);  // A3~, then dA3
  void* red = static_cast<char*>(scratch) + act;
  void* wpart = static_cast<char*>(scratch) + act + up256(bn_partial_bytes(M, s->Cin));
  const bool bf16 = (flags & ABL_MATH_BF16) != 0;
  if (int e = launch_unpack(st, packed, M, s->Cin, K, stats, buf, true, slope)) return e;
  DwSum dwsum;
  if (int e = launch_conv_wgrad_packed(st, *s, 32, bf16, buf, stats, dy, wpart, dW, false, &dwsum)) return e;
  if (int e = launch_conv_dgrad(st, *s, bf16, dy, W, buf)) return e;
  return launch_bn_bwd(st, packed, stats, buf, M, s->Cin, K, (flags & ABL_ACCUM_DX) != 0, red, dx, dgamma, dbeta,
                       dwsum.copies > 0 ? &dwsum : nullptr, slope);
}

// ---- the two fused kernels of the layer step, callable on their own --------------------------

int abl_bn_conv_fwd(void* stream, const abl_shape* s, int K, uint32_t flags, const float* x, const void* stats,
                    const float* W, const float* skip, float* y, void* packed) {
  if (int e = check_shape(s)) return e;
  if (int e = check_k48(K)) return e;
  if (flags & ~(uint32_t)ABL_MATH_BF16) return ABL_ERR_ARG;
  if (bad_ptr(x) || bad_ptr(stats) || bad_ptr(W) || bad_ptr(y) || bad_ptr(packed) ||
      (skip != nullptr && !aligned16(skip)) || static_cast<const void*>(x) == static_cast<const void*>(y))
    return ABL_ERR_ARG;
  const ConvGeom g = geom_of(*s);
  if (igemm_fused_supported(*s))
    return launch_conv_fwd_fused((hipStream_t)stream, *s, K, (flags & ABL_MATH_BF16) != 0, x, stats, W, skip, y,
                                 packed);
  if (!halo_fused_supported(g)) return ABL_ERR_SHAPE;
  return launch_halo_fwd_fused((hipStream_t)stream, g, K, (flags & ABL_MATH_BF16) != 0, x, stats, W, skip, y,
                               packed, nullptr);
}

int abl_conv_dgrad_bn_reduce(void* stream, const abl_shape* s, int K, uint32_t flags, const float* dy,
                             const float* W, const void* packed, const void* stats, void* scratch,
                             size_t scratch_bytes, float* da3, int32_t* rows) {
  if (int e = check_shape(s)) return e;
  if (int e = check_k48(K)) return e;
  if (flags & ~(uint32_t)ABL_MATH_BF16) return ABL_ERR_ARG;
  if (bad_ptr(dy) || bad_ptr(W) || bad_ptr(packed) || bad_ptr(stats) || bad_ptr(scratch) || bad_ptr(da3) ||
      rows == nullptr)
    return ABL_ERR_ARG;
  const ConvGeom g = geom_of(*s);
  if (scratch_bytes < bn_partial_bytes(rows_of(*s), s->Cin)) return ABL_ERR_SCRATCH;
  if (const int nrb = !(flags & ABL_MATH_BF16) ? rows_f32_blocks(g, 1) : 0) {   // 1x1, long contraction
    *rows = nrb;
    return launch_rows_dgrad_reduce((hipStream_t)stream, g, K, dy, W, packed, stats, da3,
                                    static_cast<double*>(scratch));
  }
  if (!halo_conv_supported(g) && pointwise_supported(g, 1)) {  // 1x1 stride 1: the pointwise kernel's epilogue
    int r = 0;
    if (int e = launch_pointwise_dgrad_reduce((hipStream_t)stream, g, K, (flags & ABL_MATH_BF16) != 0, dy, W, packed,
                                              stats, da3, static_cast<double*>(scratch), &r))
      return e;
    *rows = r;
    // contractions of more than 256 channels run without the sums: dA3 is written, no rows
    return r > 0 ? ABL_OK : ABL_ERR_SHAPE;
  }
  if (!(flags & ABL_MATH_BF16) && image_f32_supported(g, 1)) {  // small images: one row of sums per image
    *rows = g.N;
    return launch_image_dgrad_reduce((hipStream_t)stream, g, K, dy, W, packed, stats, da3,
                                     static_cast<double*>(scratch));
  }
  const int tiles = halo_conv_supported(g) ? halo_tile_count(g, 1) : 0;
  if (tiles <= 0 || tiles > kMaxPartialBlocks) return ABL_ERR_SHAPE;
  *rows = tiles;
  return launch_halo_dgrad_reduce((hipStream_t)stream, g, K, (flags & ABL_MATH_BF16) != 0, dy, W, packed, stats,
                                  da3, static_cast<double*>(scratch));
}

int abl_conv_bwd_bn_reduce(void* stream, const abl_shape* s, int K, uint32_t flags, const float* dy, const float* W,
                           const void* packed, const void* stats, void* scratch, size_t scratch_bytes, float* da3,
                           float* dW, int32_t* rows) {
  if (int e = check_shape(s)) return e;
  if (int e = check_k48(K)) return e;
  if (flags & ~(uint32_t)ABL_MATH_BF16) return ABL_ERR_ARG;
  if (bad_ptr(dy) || bad_ptr(W) || bad_ptr(packed) || bad_ptr(stats) || bad_ptr(scratch) || bad_ptr(da3) ||
      (dW != nullptr && !aligned16(dW)) || rows == nullptr)
    return ABL_ERR_ARG;
  const ConvGeom g = geom_of(*s);
  const int tiles = halo_bwd16_tiles(g);
  if (tiles <= 0) return ABL_ERR_SHAPE;
  const size_t redb = up256(bn_partial_bytes(rows_of(*s), s->Cin));
  if (scratch_bytes < redb + wgrad_partial_bytes(*s)) return ABL_ERR_SCRATCH;
  *rows = tiles;
  return launch_halo_bwd16((hipStream_t)stream, g, K, (flags & ABL_MATH_BF16) != 0, dy, W, packed, stats, da3,
                           static_cast<double*>(scratch), static_cast<char*>(scratch) + redb, dW);
}

// ---- the same layer grouped as conv -> BN -> ReLU ------------------------------------------
// Same kernels in another order: F3 -> F1 -> F2 | B3 -> B4 -> B1, B2.  What is packed is still
// the pre-ReLU BN output A2, now with Cout channels at the output resolution.

static inline int64_t out_rows(const abl_shape& s) {
  return (int64_t)s.N * out_dim(s.H, s.pad, s.R, s.stride) * out_dim(s.W, s.pad, s.S, s.stride);
}

size_t abl_postact_packed_bytes(const abl_shape* s, int K) {
  if (check_shape(s) != ABL_OK || check_k48(K) != ABL_OK) return 0;
  return packed_bytes_of(out_rows(*s) * s->Cout, K);
}

size_t abl_postact_stats_bytes(const abl_shape* s) {
  if (check_shape(s) != ABL_OK) return 0;
  return (size_t)ABL_STATS_PLANES * 4 * (size_t)s->Cout;
}

size_t abl_postact_scratch_bytes(const abl_shape* s, int K) {
  if (check_shape(s) != ABL_OK || check_k48(K) != ABL_OK) return 0;
  const size_t act = up256((size_t)out_rows(*s) * s->Cout * sizeof(float));
  return act + up256(bn_partial_bytes(out_rows(*s), s->Cout)) + wgrad_partial_bytes(*s);
}

int abl_postact_forward(void* stream, const abl_shape* s, int K, uint32_t flags, const float* x,
                        const float* W, const float* gamma, const float* beta, void* scratch,
                        size_t scratch_bytes, float* y, void* packed, void* stats) {
  if (int e = check_shape(s)) return e;
  if (int e = check_k48(K)) return e;
  if (flags & ~(uint32_t)ABL_MATH_BF16) return ABL_ERR_ARG;
  if (bad_ptr(x) || bad_ptr(W) || bad_ptr(gamma) || bad_ptr(beta) || bad_ptr(scratch) || bad_ptr(y) ||
      bad_ptr(packed) || bad_ptr(stats))
    return ABL_ERR_ARG;
  if (scratch_bytes < abl_postact_scratch_bytes(s, K)) return ABL_ERR_SCRATCH;
  hipStream_t st = (hipStream_t)stream;
  const int64_t Mo = out_rows(*s);
  float* t = static_cast<float*>(scratch);  // conv output, consumed by the BN kernels
  void* red = static_cast<char*>(scratch) + up256((size_t)Mo * s->Cout * sizeof(float));
  if (int e = launch_conv_fwd(st, *s, (flags & ABL_MATH_BF16) != 0, x, W, nullptr, t)) return e;
  if (int e = launch_bn_stats(st, t, Mo, s->Cout, gamma, beta, K, red, stats)) return e;
  return launch_bn_relu_pack(st, t, Mo, s->Cout, K, stats, y, packed);
}

int abl_postact_backward(void* stream, const abl_shape* s, int K, uint32_t flags, const void* packed,
                         const void* stats, const float* dy, const float* W, const void* xin,
                         const void* xin_stats, void* scratch, size_t scratch_bytes, float* dx, float* dW,
                         float* dgamma, float* dbeta) {
  if (int e = check_shape(s)) return e;
  if (int e = check_k48(K)) return e;
  if (flags & ~(uint32_t)(ABL_MATH_BF16 | ABL_XIN_F32 | ABL_XIN_PACKED)) return ABL_ERR_ARG;
  const bool xin_f32 = (flags & ABL_XIN_F32) != 0, xin_packed = (flags & ABL_XIN_PACKED) != 0;
  if (xin_f32 == xin_packed) return ABL_ERR_ARG;  // exactly one of the two
  if (bad_ptr(packed) || bad_ptr(stats) || bad_ptr(dy) || bad_ptr(W) || bad_ptr(xin) || bad_ptr(scratch) ||
      bad_ptr(dW) || bad_ptr(dgamma) || bad_ptr(dbeta) || (dx != nullptr && !aligned16(dx)) ||
      (xin_packed && bad_ptr(xin_stats)))
    return ABL_ERR_ARG;
  if (scratch_bytes < abl_postact_scratch_bytes(s, K)) return ABL_ERR_SCRATCH;
  hipStream_t st = (hipStream_t)stream;
  const bool bf16 = (flags & ABL_MATH_BF16) != 0;
  const int64_t Mo = out_rows(*s);
  const size_t act = up256((size_t)Mo * s->Cout * sizeof(float));
  const size_t redb = up256(bn_partial_bytes(Mo, s->Cout));
  float* dt = static_cast<float*>(scratch);  // gradient w.r.t. the conv output
  void* red = static_cast<char*>(scratch) + act;
  void* wpart = static_cast<char*>(scratch) + act + redb;
  // Eq. 6-8 first: they turn dy into the gradient of the conv output
  if (int e = launch_bn_bwd(st, packed, stats, dy, Mo, s->Cout, K, false, red, dt, dgamma, dbeta)) return e;
  // Eq. 5: the weight gradient needs the conv input - the exact tensor at the bottom of a
  // network, otherwise the previous layer's packed copy (its A3 is rebuilt on the fly)
  if (int e = launch_conv_wgrad_packed(st, *s, xin_f32 ? 32 : K, bf16, xin, xin_stats, dt, wpart, dW)) return e;
  if (dx != nullptr) return launch_conv_dgrad(st, *s, bf16, dt, W, dx);
  return ABL_OK;
}

// ---- residual stack ---------------------------------------------------------------------

// Workspace of a stack: [cross-layer statistics partials | the largest per-layer workspace].
static size_t stack_xpart_bytes(const abl_layer* layers, int32_t L) {
  int cmax = 1;
  for (int i = 0; i < L; ++i) {
    if (layers[i].shape.Cin > cmax) cmax = layers[i].shape.Cin;
    if (layers[i].shape.Cout > cmax) cmax = layers[i].shape.Cout;
  }
  return up256((size_t)kMaxPartialBlocks * 2 * (size_t)cmax * sizeof(double));
}

size_t abl_stack_scratch_bytes(const abl_layer* layers, int32_t L, int K) {
  if (layers == nullptr || L < 1) return 0;
  size_t m = 0;
  for (int i = 0; i < L; ++i) {
    const size_t b = abl_scratch_bytes(&layers[i].shape, K);
    if (b == 0) return 0;
    if (b > m) m = b;
  }
  return stack_xpart_bytes(layers, L) + m;
}

size_t abl_stack_buffer_bytes(const abl_layer* layers, int32_t L) {
  if (layers == nullptr || L < 1) return 0;
  size_t m = 0;
  for (int i = 0; i < L; ++i) {
    const abl_shape& s = layers[i].shape;
    if (check_shape(&s) != ABL_OK) return 0;
    const size_t in = (size_t)rows_of(s) * s.Cin * sizeof(float);
    const size_t out = (size_t)s.N * out_dim(s.H, s.pad, s.R, s.stride) * out_dim(s.W, s.pad, s.S, s.stride) *
                       s.Cout * sizeof(float);
    if (in > m) m = in;
    if (out > m) m = out;
  }
  return up256(m);
}

}  // extern "C"

namespace {

// A group is `skip_every` consecutive layers; the shortcut is taken when the group's output
// shape equals its input shape.  Layers after the last complete group form a plain chain.
struct GroupInfo {
  bool in_group;  // layer belongs to a complete group
  bool first, last;
  bool shortcut;  // group has an identity shortcut
};

GroupInfo group_info(const abl_layer* layers, int L, int skip_every, int i) {
  GroupInfo gi{false, false, false, false};
  if (skip_every <= 0) return gi;
  const int g0 = (i / skip_every) * skip_every;
  if (g0 + skip_every > L) return gi;
  gi.in_group = true;
  gi.first = i == g0;
  gi.last = i == g0 + skip_every - 1;
  const abl_shape& a = layers[g0].shape;
  const abl_shape& b = layers[g0 + skip_every - 1].shape;
  gi.shortcut = a.N == b.N && a.H == out_dim(b.H, b.pad, b.R, b.stride) &&
                a.W == out_dim(b.W, b.pad, b.S, b.stride) && a.Cin == b.Cout;
  return gi;
}

// Which of the two buffers a layer reads (x / dx) and writes (y / dy): true = S.
//  * In a group the first layer reads S and writes T, middle layers run in place on T, the last
//    layer writes S (+ the shortcut).
//  * Layers outside the groups (a plain chain, or what is left after the last complete group)
//    alternate S -> T -> S ... so that input and output are different buffers and the fused
//    forward kernels apply; when their number is odd the first of them runs in place on S, so
//    that the chain ends in S.
void layer_buffers(const abl_layer* layers, int L, int skip_every, int i, bool* x_is_s, bool* y_is_s) {
  const GroupInfo gi = group_info(layers, L, skip_every, i);
  if (gi.in_group) {
    *x_is_s = gi.first;
    *y_is_s = gi.last;
    return;
  }
  const int a = skip_every > 0 ? (L / skip_every) * skip_every : 0;  // first layer outside the groups
  const int len = L - a;
  int pos = i - a;
  if (len % 2 == 1) {
    if (pos == 0) {
      *x_is_s = *y_is_s = true;
      return;
    }
    --pos;
  }
  *x_is_s = pos % 2 == 0;
  *y_is_s = !*x_is_s;
}

// backward: which per-layer pointers the direction needs (parameters, store and statistics always;
// the gradient outputs in the backward pass).  Everything is validated before the first launch.
int check_stack(const abl_layer* layers, int L, int K, int skip_every, const float* s, const float* t,
                void* scratch, size_t scratch_bytes, bool backward) {
  if (layers == nullptr || L < 1 || skip_every < 0) return ABL_ERR_ARG;
  if (int e = check_k(K)) return e;
  if (bad_ptr(s) || bad_ptr(t) || bad_ptr(scratch)) return ABL_ERR_ARG;
  for (int i = 0; i < L; ++i) {
    if (int e = check_shape(&layers[i].shape)) return e;
    if (i > 0) {  // layer i consumes layer i-1's output
      const abl_shape& p = layers[i - 1].shape;
      const abl_shape& c = layers[i].shape;
      if (c.N != p.N || c.H != out_dim(p.H, p.pad, p.R, p.stride) ||
          c.W != out_dim(p.W, p.pad, p.S, p.stride) || c.Cin != p.Cout)
        return ABL_ERR_SHAPE;
    }
  }
  for (int i = 0; i < L; ++i) {
    const abl_layer& l = layers[i];
    if (bad_ptr(l.W) || bad_ptr(l.packed) || bad_ptr(l.stats)) return ABL_ERR_ARG;
    if (!backward && (bad_ptr(l.gamma) || bad_ptr(l.beta))) return ABL_ERR_ARG;
    if (backward && (bad_ptr(l.dW) || bad_ptr(l.dgamma) || bad_ptr(l.dbeta))) return ABL_ERR_ARG;
  }
  if (scratch_bytes < abl_stack_scratch_bytes(layers, L, K)) return ABL_ERR_SCRATCH;
  return ABL_OK;
}

// Inspection copy of a layer's input (or incoming gradient) before the layer runs.
int trace_copy(hipStream_t st, float* const* trace, int i, const float* src, size_t floats) {
  if (trace == nullptr || trace[i] == nullptr) return ABL_OK;
  return hipMemcpyAsync(trace[i], src, floats * sizeof(float), hipMemcpyDeviceToDevice, st) == hipSuccess
             ? ABL_OK
             : ABL_ERR_HIP;
}

}  // namespace

extern "C" {

// Buffer plan (Fig. 2): S holds the residual stream, T the straight path.  The first layer
// of a group reads S and writes T, middle layers run in place on T (a layer's input is dead
// once A3 is in the workspace), the last layer writes S = conv + S; layers outside the groups
// alternate between the two buffers (layer_buffers).
int abl_stack_forward_traced(void* stream, const abl_layer* layers, int32_t L, int K, uint32_t flags,
                             int32_t skip_every, float* buf_s, float* buf_t, void* scratch,
                             size_t scratch_bytes, float* const* trace) {
  if (flags & ~(uint32_t)(ABL_MATH_BF16 | ABL_NAIVE_FWD)) return ABL_ERR_ARG;
  if (int e = check_stack(layers, L, K, skip_every, buf_s, buf_t, scratch, scratch_bytes, false)) return e;
  if (trace != nullptr)
    for (int i = 0; i < L; ++i)
      if (trace[i] != nullptr && !aligned16(trace[i])) return ABL_ERR_ARG;
  const size_t xbytes = stack_xpart_bytes(layers, L);
  double* xpart = static_cast<double*>(scratch);
  void* lscratch = static_cast<char*>(scratch) + xbytes;
  int in_nb = 0;
  for (int i = 0; i < L; ++i) {
    const abl_layer& l = layers[i];
    const GroupInfo gi = group_info(layers, L, skip_every, i);
    bool x_is_s, y_is_s;
    layer_buffers(layers, L, skip_every, i, &x_is_s, &y_is_s);
    const float* x = x_is_s ? buf_s : buf_t;
    float* y = y_is_s ? buf_s : buf_t;
    const float* skip = gi.in_group && gi.last && gi.shortcut ? buf_s : nullptr;
    if (int e = trace_copy((hipStream_t)stream, trace, i, x, (size_t)rows_of(l.shape) * l.shape.Cin)) return e;
    // layer i's convolution leaves the first-pass statistics of its output (= layer i+1's input)
    // in `xpart` when it can; layer i+1 then only runs the finalize kernel
    int out_nb = 0;
    if (int e = forward_impl((hipStream_t)stream, &l.shape, K, flags, x, l.W, l.gamma, l.beta, skip, lscratch, y,
                             l.packed, l.stats, in_nb > 0 ? xpart : nullptr, in_nb,
                             i + 1 < L ? xpart : nullptr, &out_nb))
      return e;
    in_nb = out_nb;
  }
  return ABL_OK;
}

int abl_stack_forward(void* stream, const abl_layer* layers, int32_t L, int K, uint32_t flags,
                      int32_t skip_every, float* buf_s, float* buf_t, void* scratch,
                      size_t scratch_bytes) {
  return abl_stack_forward_traced(stream, layers, L, K, flags, skip_every, buf_s, buf_t, scratch, scratch_bytes,
                                  nullptr);
}

// Mirror image: S holds the gradient of the residual stream.  The last layer of a group reads
// S and writes T, middle layers run in place on T, the first layer adds its dx into S
// (gradients through a shortcut are copied and added, Sec. 3.4).  Without a shortcut the
// first layer overwrites S.
int abl_stack_backward_traced(void* stream, const abl_layer* layers, int32_t L, int K, uint32_t flags,
                              int32_t skip_every, float* buf_s, float* buf_t, void* scratch,
                              size_t scratch_bytes, float* const* trace) {
  if (flags & ~(uint32_t)ABL_MATH_BF16) return ABL_ERR_ARG;
  if (int e = check_stack(layers, L, K, skip_every, buf_s, buf_t, scratch, scratch_bytes, true)) return e;
  if (trace != nullptr)
    for (int i = 0; i < L; ++i)
      if (trace[i] != nullptr && !aligned16(trace[i])) return ABL_ERR_ARG;
  const size_t xbytes = stack_xpart_bytes(layers, L);
  for (int i = L - 1; i >= 0; --i) {
    const abl_layer& l = layers[i];
    const GroupInfo gi = group_info(layers, L, skip_every, i);
    bool x_is_s, y_is_s;
    layer_buffers(layers, L, skip_every, i, &x_is_s, &y_is_s);
    const float* dy = y_is_s ? buf_s : buf_t;
    float* dx = x_is_s ? buf_s : buf_t;
    uint32_t f = flags;
    if (gi.in_group && gi.first && gi.shortcut) f |= ABL_ACCUM_DX;
    const abl_shape& sh = l.shape;
    const size_t out_floats = (size_t)sh.N * out_dim(sh.H, sh.pad, sh.R, sh.stride) *
                              out_dim(sh.W, sh.pad, sh.S, sh.stride) * sh.Cout;
    if (int e = trace_copy((hipStream_t)stream, trace, i, dy, out_floats)) return e;
    if (int e = abl_backward(stream, &l.shape, K, f, l.packed, l.stats, dy, l.W,
                             static_cast<char*>(scratch) + xbytes, scratch_bytes - xbytes, dx, l.dW, l.dgamma,
                             l.dbeta))
      return e;
  }
  return ABL_OK;
}

int abl_stack_backward(void* stream, const abl_layer* layers, int32_t L, int K, uint32_t flags,
                       int32_t skip_every, float* buf_s, float* buf_t, void* scratch,
                       size_t scratch_bytes) {
  return abl_stack_backward_traced(stream, layers, L, K, flags, skip_every, buf_s, buf_t, scratch, scratch_bytes,
                                   nullptr);
}

int abl_sgd_momentum(void* stream, int64_t n, float lr, float momentum, float weight_decay, float* w,
                     const float* grad, float* v) {
  if (n < 0) return ABL_ERR_ARG;
  if (n == 0) return ABL_OK;
  if (bad_ptr(w) || bad_ptr(grad) || bad_ptr(v)) return ABL_ERR_ARG;
  if (n >= (int64_t)1 << 40) return ABL_ERR_SHAPE;
  return launch_sgd_momentum((hipStream_t)stream, n, lr, momentum, weight_decay, w, grad, v);
}

}  // extern "C"
