// Oracle for approximate-activation backprop (Chakrabarti & Moseley, arXiv 1901.07988).
//
// TEST INFRASTRUCTURE ONLY.  A plain, slow, CPU implementation of what one
// pre-activation layer (BatchNorm -> scale & bias -> ReLU -> convolution) computes
// in the forward pass (Sec. 3.1, Eq. 1-4), of the K-bit quantizer / dequantizer
// (Sec. 3.2, Eq. 9-10) and of the backward pass (Sec. 3.1, Eq. 5-8).  It shares
// no code with the GPU library; only tests, the smoke check and the benchmark's
// CPU-baseline leg may load it.
//
// Conventions (the paper fixes the tensor roles, Sec. 3.1: first dim = sample,
// last dim = channel; everything else is this file's reading, listed in the
// design notes):
//   * activations are NHWC, row-major, M = N*H*W rows of C channels;
//   * weights are [R][S][Cin][Cout]; the "linear transform" is a
//     cross-correlation with zero padding, no bias, no dilation;
//   * Mean/Var/Sum run over every dim except the channel; Var is the biased one
//     (divide by M) - Eq. 8 is the derivative of exactly that estimator;
//   * every elementwise operation is done in the storage type T (float or double)
//     as its own rounded IEEE operation (build with -ffp-contract=off); every sum
//     is accumulated in double.
//
// All functions are instantiated for T = float ("_f32": the arithmetic the GPU
// path decides codes in) and T = double ("_f64": finite-difference checks).
// The OpenMP pragmas only parallelise independent outputs; no sum is reordered.

#include <cmath>
#include <cstddef>
#include <cstdint>

namespace {

// ---- Eq. 1 (statistics): per-channel mean and biased variance -------------------
template <typename T>
void bn_stats(const T* x, int64_t M, int C, T* mean, T* var) {
#pragma omp parallel for schedule(static)
  for (int c = 0; c < C; ++c) {
    double s = 0.0;
    for (int64_t m = 0; m < M; ++m) s += (double)x[m * C + c];
    const double mu = s / (double)M;
    double ss = 0.0;
    for (int64_t m = 0; m < M; ++m) {
      const double d = (double)x[m * C + c] - mu;
      ss += d * d;
    }
    mean[c] = (T)mu;
    var[c] = (T)(ss / (double)M);
  }
}

// ---- Eq. 1 (scale): (sigma^2 + eps)^(-1/2), evaluated in double, stored in T ----
template <typename T>
void bn_rstd(const T* var, int C, T eps, T* rstd) {
  for (int c = 0; c < C; ++c) rstd[c] = (T)(1.0 / std::sqrt((double)var[c] + (double)eps));
}

// ---- Eq. 1-3: normalise, scale & bias, ReLU ---------------------------------------
// slope: 0 for the ReLU of Eq. 3; in (0, 1] the "leaky" ReLU that Sec. 3.4 admits (negative
// inputs are scaled by `slope` instead of being zeroed; the gradient still depends on the sign only).
template <typename T>
void bn_relu(const T* x, int64_t M, int C, const T* mean, const T* rstd, const T* gamma,
             const T* beta, T slope, T* a2, T* a3) {
#pragma omp parallel for schedule(static)
  for (int64_t m = 0; m < M; ++m)
    for (int c = 0; c < C; ++c) {
      const T d = x[m * C + c] - mean[c];
      const T a1 = d * rstd[c];          // Eq. 1
      const T g = gamma[c] * a1;
      const T v = g + beta[c];           // Eq. 2
      a2[m * C + c] = v;
      a3[m * C + c] = v > (T)0 ? v : (slope != (T)0 ? slope * v : (T)0);  // Eq. 3
    }
}

// ---- Eq. 9/10 per-channel constants ----------------------------------------------
// cq = 2^K (6 gamma)^-1 ; step = 2^-K (6 gamma) ; fb = floor(beta * cq).
// Floors are limited to +-2^24 before the integer conversion so that the
// conversion is defined for any finite input.
template <typename T>
T limit_floor(T u) {
  const T lim = (T)16777216.0;
  u = std::floor(u);
  if (!(u >= -lim)) u = -lim;  // also catches NaN
  if (u > lim) u = lim;
  return u;
}

template <typename T>
void quant_consts(const T* gamma, const T* beta, int C, int K, T* cq, T* step, int32_t* fb) {
  const T two_k = (T)std::ldexp(1.0, K);
  for (int c = 0; c < C; ++c) {
    const T six_g = (T)6 * gamma[c];
    cq[c] = two_k / six_g;
    step[c] = six_g / two_k;
    fb[c] = (int32_t)limit_floor<T>(beta[c] * cq[c]);
  }
}

// ---- Eq. 9: integer codes in [0, 2^K - 1] ------------------------------------------
template <typename T>
void quantize(const T* a2, int64_t M, int C, const T* cq, const int32_t* fb, int K, int32_t* q) {
  const int64_t half = (int64_t)1 << (K - 1);
  const int64_t top = ((int64_t)1 << K) - 1;
#pragma omp parallel for schedule(static)
  for (int64_t m = 0; m < M; ++m)
    for (int c = 0; c < C; ++c) {
      const T u = limit_floor<T>(a2[m * C + c] * cq[c]);
      int64_t v = (int64_t)u + half - (int64_t)fb[c];
      if (v < 0) v = 0;
      if (v > top) v = top;
      q[m * C + c] = (int32_t)v;
    }
}

// ---- Eq. 10: bin-midpoint reconstruction -------------------------------------------
template <typename T>
void dequantize(const int32_t* q, int64_t M, int C, const T* step, const int32_t* fb, int K,
                T* a2t) {
  const int64_t half = (int64_t)1 << (K - 1);
#pragma omp parallel for schedule(static)
  for (int64_t m = 0; m < M; ++m)
    for (int c = 0; c < C; ++c) {
      const int64_t j = (int64_t)q[m * C + c] - half + (int64_t)fb[c];
      const T t = (T)j + (T)0.5;
      a2t[m * C + c] = step[c] * t;
    }
}

// ---- Eq. 4: y[n,ho,wo,co] = sum_{r,s,ci} a3[n, ho*st+r-pad, wo*st+s-pad, ci] W[r,s,ci,co]
template <typename T>
void conv_fwd(const T* a3, const T* w, int N, int H, int W, int Cin, int Cout, int R, int S,
              int st, int pad, T* y) {
  const int Ho = (H + 2 * pad - R) / st + 1, Wo = (W + 2 * pad - S) / st + 1;
#pragma omp parallel for collapse(2) schedule(static)
  for (int n = 0; n < N; ++n)
    for (int ho = 0; ho < Ho; ++ho)
      for (int wo = 0; wo < Wo; ++wo)
        for (int co = 0; co < Cout; ++co) {
          double acc = 0.0;
          for (int r = 0; r < R; ++r) {
            const int h = ho * st + r - pad;
            if (h < 0 || h >= H) continue;
            for (int s = 0; s < S; ++s) {
              const int x = wo * st + s - pad;
              if (x < 0 || x >= W) continue;
              const T* ap = a3 + (((int64_t)n * H + h) * W + x) * Cin;
              const T* wp = w + ((int64_t)(r * S + s) * Cin) * Cout + co;
              for (int ci = 0; ci < Cin; ++ci) acc += (double)ap[ci] * (double)wp[(int64_t)ci * Cout];
            }
          }
          y[(((int64_t)n * Ho + ho) * Wo + wo) * Cout + co] = (T)acc;
        }
}

// ---- Eq. 5, second half: gradient to the conv input --------------------------------
// da3[n,h,w,ci] = sum over every (ho,wo,r,s,co) whose window touches (h,w).
template <typename T>
void conv_dgrad(const T* dy, const T* w, int N, int H, int W, int Cin, int Cout, int R, int S,
                int st, int pad, T* da3) {
  const int Ho = (H + 2 * pad - R) / st + 1, Wo = (W + 2 * pad - S) / st + 1;
#pragma omp parallel for collapse(2) schedule(static)
  for (int n = 0; n < N; ++n)
    for (int h = 0; h < H; ++h)
      for (int x = 0; x < W; ++x)
        for (int ci = 0; ci < Cin; ++ci) {
          double acc = 0.0;
          for (int ho = 0; ho < Ho; ++ho) {
            const int r = h + pad - ho * st;
            if (r < 0 || r >= R) continue;
            for (int wo = 0; wo < Wo; ++wo) {
              const int s = x + pad - wo * st;
              if (s < 0 || s >= S) continue;
              const T* gp = dy + (((int64_t)n * Ho + ho) * Wo + wo) * Cout;
              const T* wp = w + ((int64_t)(r * S + s) * Cin + ci) * Cout;
              for (int co = 0; co < Cout; ++co) acc += (double)gp[co] * (double)wp[co];
            }
          }
          da3[(((int64_t)n * H + h) * W + x) * Cin + ci] = (T)acc;
        }
}

// ---- Eq. 5, first half: gradient to the weights -------------------------------------
template <typename T>
void conv_wgrad(const T* a3, const T* dy, int N, int H, int W, int Cin, int Cout, int R, int S,
                int st, int pad, T* dw) {
  const int Ho = (H + 2 * pad - R) / st + 1, Wo = (W + 2 * pad - S) / st + 1;
#pragma omp parallel for collapse(3) schedule(static)
  for (int r = 0; r < R; ++r)
    for (int s = 0; s < S; ++s)
      for (int ci = 0; ci < Cin; ++ci)
        for (int co = 0; co < Cout; ++co) {
          double acc = 0.0;
          for (int n = 0; n < N; ++n)
            for (int ho = 0; ho < Ho; ++ho) {
              const int h = ho * st + r - pad;
              if (h < 0 || h >= H) continue;
              for (int wo = 0; wo < Wo; ++wo) {
                const int x = wo * st + s - pad;
                if (x < 0 || x >= W) continue;
                acc += (double)a3[(((int64_t)n * H + h) * W + x) * Cin + ci] *
                       (double)dy[(((int64_t)n * Ho + ho) * Wo + wo) * Cout + co];
              }
            }
          dw[((int64_t)(r * S + s) * Cin + ci) * Cout + co] = (T)acc;
        }
}

// ---- Eq. 6-8: ReLU, scale & bias and BatchNorm backward from a (possibly approximate)
// copy a2t of the pre-ReLU activation.  A1 is rebuilt by inverting Eq. 2.
template <typename T>
void bn_relu_bwd(const T* a2t, const T* da3, int64_t M, int C, const T* rstd, const T* gamma,
                 const T* beta, T slope, T* dx, T* dgamma, T* dbeta) {
#pragma omp parallel for schedule(static)
  for (int c = 0; c < C; ++c) {
    double sum_da2 = 0.0, sum_a1_da2 = 0.0, sum_da1 = 0.0, sum_a1_da1 = 0.0;
    for (int64_t m = 0; m < M; ++m) {
      const T v = a2t[m * C + c];
      const T da2 = v > (T)0 ? da3[m * C + c] : (slope != (T)0 ? slope * da3[m * C + c] : (T)0);  // Eq. 6
      const T a1 = (v - beta[c]) / gamma[c];          // inverse of Eq. 2
      const T da1 = gamma[c] * da2;                   // Eq. 7
      sum_da2 += (double)da2;
      sum_a1_da2 += (double)a1 * (double)da2;
      sum_da1 += (double)da1;
      sum_a1_da1 += (double)a1 * (double)da1;
    }
    dbeta[c] = (T)sum_da2;      // Eq. 7
    dgamma[c] = (T)sum_a1_da2;  // Eq. 7
    const T mean_da1 = (T)(sum_da1 / (double)M);
    const T mean_a1_da1 = (T)(sum_a1_da1 / (double)M);
    for (int64_t m = 0; m < M; ++m) {
      const T v = a2t[m * C + c];
      const T da2 = v > (T)0 ? da3[m * C + c] : (slope != (T)0 ? slope * da3[m * C + c] : (T)0);
      const T a1 = (v - beta[c]) / gamma[c];
      const T da1 = gamma[c] * da2;
      const T t1 = da1 - mean_da1;
      const T t2 = a1 * mean_a1_da1;
      const T t3 = t1 - t2;
      dx[m * C + c] = rstd[c] * t3;  // Eq. 8
    }
  }
}

// ---- storage of the K-bit codes: flat NHWC element order, little-endian in the byte ---
// K=8: byte e holds code e.  K=4: byte e/2 holds code 2j in bits 0-3 and code
// 2j+1 in bits 4-7.  Other K (1,2,16): codes are laid out LSB-first the same way.
void pack_codes(const int32_t* q, int64_t E, int K, uint8_t* out, int64_t out_bytes) {
  for (int64_t i = 0; i < out_bytes; ++i) out[i] = 0;
  for (int64_t e = 0; e < E; ++e) {
    const uint64_t bit = (uint64_t)e * (uint64_t)K;
    uint32_t v = (uint32_t)q[e];
    for (int b = 0; b < K; ++b)
      if ((v >> b) & 1u) out[(bit + b) >> 3] |= (uint8_t)(1u << ((bit + b) & 7));
  }
}

void unpack_codes(const uint8_t* in, int64_t E, int K, int32_t* q) {
  for (int64_t e = 0; e < E; ++e) {
    const uint64_t bit = (uint64_t)e * (uint64_t)K;
    uint32_t v = 0;
    for (int b = 0; b < K; ++b)
      if ((in[(bit + b) >> 3] >> ((bit + b) & 7)) & 1u) v |= 1u << b;
    q[e] = (int32_t)v;
  }
}

}  // namespace

#define ORC_INSTANTIATE(T, SUF)                                                                    \
  extern "C" void orc_bn_stats_##SUF(const T* x, int64_t M, int C, T* mean, T* var) {              \
    bn_stats<T>(x, M, C, mean, var);                                                               \
  }                                                                                                \
  extern "C" void orc_bn_rstd_##SUF(const T* var, int C, T eps, T* rstd) {                         \
    bn_rstd<T>(var, C, eps, rstd);                                                                 \
  }                                                                                                \
  extern "C" void orc_bn_relu_##SUF(const T* x, int64_t M, int C, const T* mean, const T* rstd,    \
                                    const T* gamma, const T* beta, T slope, T* a2, T* a3) {        \
    bn_relu<T>(x, M, C, mean, rstd, gamma, beta, slope, a2, a3);                                   \
  }                                                                                                \
  extern "C" void orc_quant_consts_##SUF(const T* gamma, const T* beta, int C, int K, T* cq,       \
                                         T* step, int32_t* fb) {                                   \
    quant_consts<T>(gamma, beta, C, K, cq, step, fb);                                              \
  }                                                                                                \
  extern "C" void orc_quantize_##SUF(const T* a2, int64_t M, int C, const T* cq,                   \
                                     const int32_t* fb, int K, int32_t* q) {                       \
    quantize<T>(a2, M, C, cq, fb, K, q);                                                           \
  }                                                                                                \
  extern "C" void orc_dequantize_##SUF(const int32_t* q, int64_t M, int C, const T* step,          \
                                       const int32_t* fb, int K, T* a2t) {                         \
    dequantize<T>(q, M, C, step, fb, K, a2t);                                                      \
  }                                                                                                \
  extern "C" void orc_conv_fwd_##SUF(const T* a3, const T* w, int N, int H, int W, int Cin,        \
                                     int Cout, int R, int S, int st, int pad, T* y) {              \
    conv_fwd<T>(a3, w, N, H, W, Cin, Cout, R, S, st, pad, y);                                      \
  }                                                                                                \
  extern "C" void orc_conv_dgrad_##SUF(const T* dy, const T* w, int N, int H, int W, int Cin,      \
                                       int Cout, int R, int S, int st, int pad, T* da3) {          \
    conv_dgrad<T>(dy, w, N, H, W, Cin, Cout, R, S, st, pad, da3);                                  \
  }                                                                                                \
  extern "C" void orc_conv_wgrad_##SUF(const T* a3, const T* dy, int N, int H, int W, int Cin,     \
                                       int Cout, int R, int S, int st, int pad, T* dw) {           \
    conv_wgrad<T>(a3, dy, N, H, W, Cin, Cout, R, S, st, pad, dw);                                  \
  }                                                                                                \
  extern "C" void orc_bn_relu_bwd_##SUF(const T* a2t, const T* da3, int64_t M, int C,              \
                                        const T* rstd, const T* gamma, const T* beta, T slope,     \
                                        T* dx, T* dgamma, T* dbeta) {                              \
    bn_relu_bwd<T>(a2t, da3, M, C, rstd, gamma, beta, slope, dx, dgamma, dbeta);                   \
  }

ORC_INSTANTIATE(float, f32)
ORC_INSTANTIATE(double, f64)

extern "C" void orc_pack_codes(const int32_t* q, int64_t E, int K, uint8_t* out, int64_t out_bytes) {
  pack_codes(q, E, K, out, out_bytes);
}
extern "C" void orc_unpack_codes(const uint8_t* in, int64_t E, int K, int32_t* q) {
  unpack_codes(in, E, K, q);
}
