// Batch-norm / quantizer kernels of the approximate-activation layer for gfx950.
//
//   bn_stats      Eq. 1 statistics (Sec. 3.1) + per-channel constants of Eq. 9/10 (Sec. 3.2)
//   bn_relu_pack  Eq. 1-3 and Eq. 9 fused: one read of x, writes A3 (fp32) and the K-bit codes
//   pack/unpack   Eq. 9 / Eq. 10 alone
//   bn_bwd        Eq. 6-8 from the K-bit codes: reduce pass, then apply pass
//
// All of them stream [M,C] row-major tensors once and are HBM-bound.  A block is a
// TX x TY arrangement of 256 threads: a thread owns VEC consecutive channels (so its
// per-channel constants live in registers) and walks rows ty, ty+TY, ...; a wave
// therefore touches whole contiguous rows.  Reductions are two-pass with a fixed order
// (no atomics), so every result is reproducible bit for bit.
//
// The codes must equal those of a CPU evaluation of Eq. 9 in IEEE fp32, so the
// quantizer arithmetic is written one rounded operation at a time and this file is
// compiled with floating-point contraction off.

#include "abl_internal.h"

#pragma clang fp contract(off)

namespace abl {
namespace {

constexpr int kThreads = 256;
constexpr int kUnroll = 4;
// fp32 tensors at least this large are written with streaming (non-temporal) stores
constexpr int64_t kStreamBytes = 64ll << 20;

struct RowGeom {
  int CV;     // channel groups per row (C / VEC)
  int TX;     // channel groups per block
  int TY;     // rows per block pass
  int gridX;  // blocks across channel groups
  int gridY;  // blocks across rows
  int rpt;    // rows per thread
};

// reduce == true bounds gridY (partials) and keeps >= 64 rows per block so that the
// partial sums stay below 1/16 of the tensor's bytes.  rows: rows in flight per thread of the
// element-wise kernel this geometry is for (its ROWS template parameter).
RowGeom make_geom(int64_t M, int C, int VEC, bool reduce, int rows = kUnroll) {
  RowGeom g;
  g.CV = C / VEC;
  g.TX = g.CV < 64 ? g.CV : 64;
  g.TY = kThreads / g.TX;
  g.gridX = (g.CV + g.TX - 1) / g.TX;
  const int64_t passes = (M + g.TY - 1) / g.TY;  // rows / TY
  // blocks across rows we would like: two per compute unit for the element-wise passes (measured
  // on the 16-channel layer's Eq. 8 pass: 6.7 -> 5.9 us against four, 8.3 -> 6.6 us with
  // accumulation), up to the partial-row limit for reductions
  int64_t want = (reduce ? 2048 : 512) / g.gridX;
  if (want < 1) want = 1;
  int64_t rpt = (passes + want - 1) / want;
  if (reduce) {
    const int64_t min_rpt = (64 + g.TY - 1) / g.TY;
    if (rpt < min_rpt) rpt = min_rpt;
    const int64_t cap = (passes + kMaxPartialBlocks - 1) / kMaxPartialBlocks;
    if (rpt < cap) rpt = cap;
  } else {
    // one batch of rows per thread and no loop: measured best from 50 MB tensors up
    // (pack on 205 MB: 4.5 -> 5.3 TB/s against 16 rows per thread)
    if (rpt > rows) rpt = rows;
  }
  if (rpt < 1) rpt = 1;
  g.rpt = (int)rpt;
  g.gridY = (int)((passes + rpt - 1) / rpt);
  if (g.gridY < 1) g.gridY = 1;
  return g;
}

template <int VEC>
__device__ inline void load_vec(const float* __restrict__ p, float (&v)[VEC]) {
  if constexpr (VEC % 4 == 0) {
#pragma unroll
    for (int i = 0; i < VEC / 4; ++i) {
      const float4 t = reinterpret_cast<const float4*>(p)[i];
      v[4 * i + 0] = t.x; v[4 * i + 1] = t.y; v[4 * i + 2] = t.z; v[4 * i + 3] = t.w;
    }
  } else {
#pragma unroll
    for (int i = 0; i < VEC; ++i) v[i] = p[i];
  }
}

template <int VEC>
__device__ inline void load_vec_i(const int32_t* __restrict__ p, int32_t (&v)[VEC]) {
  if constexpr (VEC % 4 == 0) {
#pragma unroll
    for (int i = 0; i < VEC / 4; ++i) {
      const int4 t = reinterpret_cast<const int4*>(p)[i];
      v[4 * i + 0] = t.x; v[4 * i + 1] = t.y; v[4 * i + 2] = t.z; v[4 * i + 3] = t.w;
    }
  } else {
#pragma unroll
    for (int i = 0; i < VEC; ++i) v[i] = p[i];
  }
}

// STREAM: the stores carry the non-temporal hint (large tensors that will not be re-read from
// cache before they are evicted anyway).
template <int VEC, bool STREAM = false>
__device__ inline void store_vec(float* __restrict__ p, const float (&v)[VEC]) {
  if constexpr (VEC % 4 == 0) {
    typedef float vec4f __attribute__((ext_vector_type(4)));
#pragma unroll
    for (int i = 0; i < VEC / 4; ++i) {
      const vec4f t = {v[4 * i], v[4 * i + 1], v[4 * i + 2], v[4 * i + 3]};
      if constexpr (STREAM) __builtin_nontemporal_store(t, reinterpret_cast<vec4f*>(p) + i);
      else reinterpret_cast<vec4f*>(p)[i] = t;
    }
  } else {
#pragma unroll
    for (int i = 0; i < VEC; ++i) p[i] = v[i];
  }
}

// Packed word of VEC codes: K*VEC bits (32 or 16).
template <int K, int VEC>
struct PackedWord {
  static_assert(K * VEC == 32 || K * VEC == 16, "unsupported packing");
  using type = typename std::conditional<K * VEC == 32, uint32_t, uint16_t>::type;
};

// What a thread holds of one row's stored activation: VEC K-bit codes in one word, or (K = 32,
// exact storage) the VEC fp32 values themselves.
template <int K, int VEC>
struct Stored {
  using raw_t = uint32_t;
  static __device__ inline raw_t load(const void* __restrict__ packed, int64_t e) {
    return reinterpret_cast<const typename PackedWord<K, VEC>::type*>(packed)[e / VEC];
  }
  static __device__ inline float value(const raw_t& w, int v, float step, int32_t fb) {
    return dequant<K>((w >> (K * v)) & ((1u << K) - 1), step, fb);  // Eq. 10
  }
};
template <int VEC>
struct Stored<32, VEC> {
  struct raw_t {
    float f[VEC];
  };
  static __device__ inline raw_t load(const void* __restrict__ packed, int64_t e) {
    raw_t r;
    load_vec<VEC>(reinterpret_cast<const float*>(packed) + e, r.f);
    return r;
  }
  static __device__ inline float value(const raw_t& w, int v, float, int32_t) { return w.f[v]; }
};

struct ThreadPos {
  int tx, ty;
  int c0;       // first channel of this thread
  bool active;
};

template <int VEC>
__device__ inline ThreadPos thread_pos(const RowGeom& g) {
  ThreadPos p;
  p.tx = threadIdx.x % g.TX;
  p.ty = threadIdx.x / g.TX;
  const int cg = blockIdx.x * g.TX + p.tx;
  p.active = p.ty < g.TY && cg < g.CV;
  p.c0 = p.active ? cg * VEC : 0;
  return p;
}

// ------------------------------------------------------------------------------------------
// Eq. 1 statistics, pass 1: per-block sums of (x - k) and (x - k)^2 in fp64, k = first row
// (a per-channel shift that keeps E[x^2] - E[x]^2 well conditioned when |mean| >> sigma).
// partial layout: [gridY][2][C] doubles.
template <int VEC>
__global__ __launch_bounds__(kThreads) void stats_partial_kernel(const float* __restrict__ x, int64_t M,
                                                                 int C, RowGeom g,
                                                                 double* __restrict__ partial) {
  __shared__ double red[2 * VEC][kThreads];  // [value][thread]: conflict-free
  const ThreadPos p = thread_pos<VEC>(g);
  double s[VEC], ss[VEC];
  float k[VEC];
#pragma unroll
  for (int v = 0; v < VEC; ++v) s[v] = ss[v] = 0.0;
  load_vec<VEC>(x + p.c0, k);
  const int64_t row0 = (int64_t)blockIdx.y * g.TY * g.rpt + p.ty;
  for (int i = 0; i < g.rpt; i += kUnroll) {
    float xv[kUnroll][VEC];
    bool ok[kUnroll];
#pragma unroll
    for (int j = 0; j < kUnroll; ++j) {
      const int64_t r = row0 + (int64_t)(i + j) * g.TY;
      ok[j] = p.active && (i + j) < g.rpt && r < M;
      load_vec<VEC>(x + (ok[j] ? r : 0) * C + p.c0, xv[j]);
    }
#pragma unroll
    for (int j = 0; j < kUnroll; ++j)
      if (ok[j]) {
#pragma unroll
        for (int v = 0; v < VEC; ++v) {
          const double d = (double)xv[j][v] - (double)k[v];
          s[v] += d;
          ss[v] += d * d;
        }
      }
  }
#pragma unroll
  for (int v = 0; v < VEC; ++v) {
    red[v][threadIdx.x] = s[v];
    red[VEC + v][threadIdx.x] = ss[v];
  }
  __syncthreads();
  // tree over ty (threads tx + TX*ty), fixed order
  int span = 1;
  while (span < g.TY) span <<= 1;
  for (int h = span >> 1; h >= 1; h >>= 1) {
    if (p.ty < h && p.ty + h < g.TY) {
#pragma unroll
      for (int v = 0; v < 2 * VEC; ++v) red[v][threadIdx.x] += red[v][threadIdx.x + h * g.TX];
    }
    __syncthreads();
  }
  if (p.active && p.ty == 0) {
    double* out = partial + (int64_t)blockIdx.y * 2 * C + p.c0;
#pragma unroll
    for (int v = 0; v < VEC; ++v) {
      out[v] = red[v][threadIdx.x];
      out[C + v] = red[VEC + v][threadIdx.x];
    }
  }
}

// Sums `nb` partial rows of two per-channel quantities in a fixed order.  A block of 1024
// threads covers 16 channels: thread = (part 0..31, quantity 0..1, channel 0..15); every thread
// adds up its interleaved share of the rows, then the 32 parts are combined by a tree in LDS.
// Returns the two totals of channel blockIdx.x*16 + (threadIdx.x & 15) to threads < 16.
constexpr int kFinThreads = 1024;
// One part's share of the rows (part, part + 32, ...; at most ROWS of them): every row is
// requested before the first is added - one memory round trip - and the adds keep their order.
template <int ROWS>
__device__ inline double sum_part_rows(const double* __restrict__ src, int part, int nb, int C) {
  double r[ROWS];
#pragma unroll
  for (int k = 0; k < ROWS; ++k) {
    const int i = part + 32 * k;
    r[k] = src[(int64_t)(i < nb ? i : 0) * 2 * C];
  }
  double a = 0.0;
#pragma unroll
  for (int k = 0; k < ROWS; ++k) a += (part + 32 * k < nb) ? r[k] : 0.0;
  return a;
}

__device__ inline void reduce_partials(const double* __restrict__ partial, int nb, int C,
                                       double (&out)[2], double (*sm)[32]) {
  const int v = threadIdx.x & 31, part = threadIdx.x >> 5;
  const int c = blockIdx.x * 16 + (v & 15), q = v >> 4;
  double a = 0.0;
  if (c < C) {
    static_assert(kMaxPartialBlocks == 512, "at most 16 rows per part");
    const double* src = partial + (int64_t)q * C + c;
    if (nb <= 64) a = sum_part_rows<2>(src, part, nb, C);
    else if (nb <= 128) a = sum_part_rows<4>(src, part, nb, C);
    else if (nb <= 256) a = sum_part_rows<8>(src, part, nb, C);
    else if (nb <= 512) a = sum_part_rows<16>(src, part, nb, C);
    else
      for (int i = part; i < nb; i += 32) a += src[(int64_t)i * 2 * C];
  }
  sm[part][v] = a;
  __syncthreads();
  for (int h = 16; h >= 1; h >>= 1) {
    if (part < h) sm[part][v] += sm[part + h][v];
    __syncthreads();
  }
  out[0] = sm[0][threadIdx.x & 15];
  out[1] = sm[0][16 + (threadIdx.x & 15)];
}

// Eq. 1 statistics, pass 2, and the per-channel constants of Eq. 9/10.
__global__ __launch_bounds__(kFinThreads) void stats_finalize_kernel(const double* __restrict__ partial, int nb,
                                                                  const float* __restrict__ x, int64_t M,
                                                                  int C, const float* __restrict__ gamma,
                                                                  const float* __restrict__ beta, int K,
                                                                  float* __restrict__ stats) {
  __shared__ double sm[32][32];
  const int c = blockIdx.x * 16 + (threadIdx.x & 15);
  double t[2];
  reduce_partials(partial, nb, C, t, sm);
  if (c >= C || threadIdx.x >= 16) return;
  const double k = x != nullptr ? (double)x[c] : 0.0;  // the shift the partial sums were taken with
  const double mk = t[0] / (double)M;
  double var = t[1] / (double)M - mk * mk;
  var = var > 0.0 ? var : 0.0;
  const float mean_f = (float)(k + mk);
  const float var_f = (float)var;
  const float rstd = (float)(1.0 / sqrt((double)var_f + (double)ABL_BN_EPS));
  const float gm = gamma[c], bt = beta[c];
  // K = 32 (exact storage) has no quantizer: the constants are written as zeros
  const float two_k = K < 32 ? (float)(1 << K) : 0.0f;
  const float six_g = 6.0f * gm;
  // double division then one rounding == correctly rounded fp32 division
  const float cq = K < 32 ? (float)((double)two_k / (double)six_g) : 0.0f;
  const float step = K < 32 ? (float)((double)six_g / (double)two_k) : 0.0f;
  const int32_t fb = K < 32 ? (int32_t)limit_floor(bt * cq) : 0;
  stats[P_MEAN * C + c] = mean_f;
  stats[P_VAR * C + c] = var_f;
  stats[P_RSTD * C + c] = rstd;
  stats[P_GAMMA * C + c] = gm;
  stats[P_BETA * C + c] = bt;
  stats[P_CQ * C + c] = cq;
  stats[P_STEP * C + c] = step;
  reinterpret_cast<int32_t*>(stats)[P_FB * C + c] = fb;
}

// ------------------------------------------------------------------------------------------
// Forward elementwise pass.  MODE 0: x -> A3 and codes (Eq. 1-3, 9).  MODE 1: a2 -> codes (Eq. 9).
// ROWS: rows in flight per thread.
template <int K, int VEC, int MODE, bool STREAM, int ROWS>
__global__ __launch_bounds__(kThreads) void quant_pack_kernel(const float* __restrict__ in, int64_t M, int C,
                                                              RowGeom g, const float* __restrict__ stats,
                                                              float* __restrict__ a3,
                                                              void* __restrict__ packed, int pad_bytes,
                                                              float slope) {
  const ThreadPos p = thread_pos<VEC>(g);
  const bool leaky = slope != 0.0f;
  if (blockIdx.x == 0 && blockIdx.y == 0 && (int)threadIdx.x < pad_bytes)  // zero the 128-byte row tail
    reinterpret_cast<uint8_t*>(packed)[(M * C * K) / 8 + threadIdx.x] = 0;
  if (!p.active) return;
  float mean[VEC], rstd[VEC], gm[VEC], bt[VEC], cq[VEC];
  int32_t fb[VEC];
  if constexpr (MODE == 0) {
    load_vec<VEC>(stats + P_MEAN * C + p.c0, mean);
    load_vec<VEC>(stats + P_RSTD * C + p.c0, rstd);
    load_vec<VEC>(stats + P_GAMMA * C + p.c0, gm);
    load_vec<VEC>(stats + P_BETA * C + p.c0, bt);
  }
  load_vec<VEC>(stats + P_CQ * C + p.c0, cq);
  load_vec_i<VEC>(reinterpret_cast<const int32_t*>(stats) + P_FB * C + p.c0, fb);
  const int64_t row0 = (int64_t)blockIdx.y * g.TY * g.rpt + p.ty;
  for (int i = 0; i < g.rpt; i += ROWS) {
    float xv[ROWS][VEC];
    bool ok[ROWS];
#pragma unroll
    for (int j = 0; j < ROWS; ++j) {
      const int64_t r = row0 + (int64_t)(i + j) * g.TY;
      ok[j] = (i + j) < g.rpt && r < M;
      load_vec<VEC>(in + (ok[j] ? r : 0) * C + p.c0, xv[j]);
    }
#pragma unroll
    for (int j = 0; j < ROWS; ++j)
      if (ok[j]) {
        const int64_t r = row0 + (int64_t)(i + j) * g.TY;
        uint32_t word = 0;
        float out[VEC], kept[VEC];
#pragma unroll
        for (int v = 0; v < VEC; ++v) {
          float a2;
          if constexpr (MODE == 0) {
            const float d = xv[j][v] - mean[v];
            const float a1 = d * rstd[v];   // Eq. 1
            const float t = gm[v] * a1;
            a2 = t + bt[v];                 // Eq. 2
            out[v] = a2 > 0.0f ? a2 : (leaky ? slope * a2 : 0.0f);  // Eq. 3 (leaky: Sec. 3.4)
          } else {
            a2 = xv[j][v];
          }
          if constexpr (K == 32) kept[v] = a2;  // exact storage keeps the value itself
          else word |= quant_code<K>(a2, cq[v], fb[v]) << (K * v);
        }
        const int64_t e = r * C + p.c0;
        if constexpr (MODE == 0) store_vec<VEC, STREAM>(a3 + e, out);
        if constexpr (K == 32) {
          store_vec<VEC, false>(reinterpret_cast<float*>(packed) + e, kept);
        } else {
          using word_t = typename PackedWord<K, VEC>::type;
          reinterpret_cast<word_t*>(packed)[e / VEC] = (word_t)word;
        }
      }
  }
}

// Eq. 10: codes -> fp32; with `act` the non-linearity on top (negative values times `slope`).
template <int K, int VEC, bool STREAM>
__global__ __launch_bounds__(kThreads) void unpack_kernel(const void* __restrict__ packed, int64_t M, int C,
                                                          RowGeom g, const float* __restrict__ stats,
                                                          float* __restrict__ a2t, int act, float slope) {
  using S = Stored<K, VEC>;
  const ThreadPos p = thread_pos<VEC>(g);
  if (!p.active) return;
  float step[VEC];
  int32_t fb[VEC];
  load_vec<VEC>(stats + P_STEP * C + p.c0, step);
  load_vec_i<VEC>(reinterpret_cast<const int32_t*>(stats) + P_FB * C + p.c0, fb);
  const int64_t row0 = (int64_t)blockIdx.y * g.TY * g.rpt + p.ty;
  for (int i = 0; i < g.rpt; i += kUnroll) {
    typename S::raw_t w[kUnroll];
    bool ok[kUnroll];
#pragma unroll
    for (int j = 0; j < kUnroll; ++j) {
      const int64_t r = row0 + (int64_t)(i + j) * g.TY;
      ok[j] = (i + j) < g.rpt && r < M;
      w[j] = S::load(packed, (ok[j] ? r : 0) * C + p.c0);
    }
#pragma unroll
    for (int j = 0; j < kUnroll; ++j)
      if (ok[j]) {
        const int64_t r = row0 + (int64_t)(i + j) * g.TY;
        float out[VEC];
#pragma unroll
        for (int v = 0; v < VEC; ++v) {
          const float a = S::value(w[j], v, step[v], fb[v]);
          out[v] = (act == 0 || a > 0.0f) ? a : slope * a;  // act: Eq. 3 (slope 0) or its leaky version
        }
        store_vec<VEC, STREAM>(a2t + r * C + p.c0, out);
      }
  }
}

// ------------------------------------------------------------------------------------------
// Backward, pass 1 (Eq. 6-7): per-block sums of dA2 and A1~ * dA2, fp64, [gridY][2][C].
template <int K, int VEC>
__global__ __launch_bounds__(kThreads) void bwd_reduce_kernel(const void* __restrict__ packed,
                                                              const float* __restrict__ da3, int64_t M, int C,
                                                              RowGeom g, const float* __restrict__ stats,
                                                              double* __restrict__ partial, float slope) {
  using S = Stored<K, VEC>;
  __shared__ double red[2 * VEC][kThreads];  // [value][thread]: conflict-free
  const ThreadPos p = thread_pos<VEC>(g);
  const bool leaky = slope != 0.0f;
  float step[VEC], bt[VEC], ig[VEC];
  int32_t fb[VEC];
  load_vec<VEC>(stats + P_STEP * C + p.c0, step);
  load_vec<VEC>(stats + P_BETA * C + p.c0, bt);
  load_vec<VEC>(stats + P_GAMMA * C + p.c0, ig);
  load_vec_i<VEC>(reinterpret_cast<const int32_t*>(stats) + P_FB * C + p.c0, fb);
  double s1[VEC], s2[VEC];
#pragma unroll
  for (int v = 0; v < VEC; ++v) {
    ig[v] = 1.0f / ig[v];
    s1[v] = s2[v] = 0.0;
  }
  const int64_t row0 = (int64_t)blockIdx.y * g.TY * g.rpt + p.ty;
  for (int i = 0; i < g.rpt; i += kUnroll) {
    float gv[kUnroll][VEC];
    typename S::raw_t w[kUnroll];
    bool ok[kUnroll];
#pragma unroll
    for (int j = 0; j < kUnroll; ++j) {
      const int64_t r = row0 + (int64_t)(i + j) * g.TY;
      ok[j] = p.active && (i + j) < g.rpt && r < M;
      const int64_t e = (ok[j] ? r : 0) * C + p.c0;
      load_vec<VEC>(da3 + e, gv[j]);
      w[j] = S::load(packed, e);
    }
#pragma unroll
    for (int j = 0; j < kUnroll; ++j)
      if (ok[j]) {
#pragma unroll
        for (int v = 0; v < VEC; ++v) {
          const float a2t = S::value(w[j], v, step[v], fb[v]);
          const float da2 = a2t > 0.0f ? gv[j][v] : (leaky ? slope * gv[j][v] : 0.0f);  // Eq. 6
          const float a1t = (a2t - bt[v]) * ig[v];          // inverse of Eq. 2
          s1[v] += (double)da2;
          s2[v] += (double)a1t * (double)da2;
        }
      }
  }
#pragma unroll
  for (int v = 0; v < VEC; ++v) {
    red[v][threadIdx.x] = s1[v];
    red[VEC + v][threadIdx.x] = s2[v];
  }
  __syncthreads();
  int span = 1;
  while (span < g.TY) span <<= 1;
  for (int h = span >> 1; h >= 1; h >>= 1) {
    if (p.ty < h && p.ty + h < g.TY) {
#pragma unroll
      for (int v = 0; v < 2 * VEC; ++v) red[v][threadIdx.x] += red[v][threadIdx.x + h * g.TX];
    }
    __syncthreads();
  }
  if (p.active && p.ty == 0) {
    double* out = partial + (int64_t)blockIdx.y * 2 * C + p.c0;
#pragma unroll
    for (int v = 0; v < VEC; ++v) {
      out[v] = red[v][threadIdx.x];
      out[C + v] = red[VEC + v][threadIdx.x];
    }
  }
}

// Backward, pass 1b: dbeta, dgamma (Eq. 7) and the two per-channel means of Eq. 8.
// means layout: [2][C] floats = Mean(dA1), Mean(A1~ * dA1) with dA1 = gamma * dA2.
__global__ __launch_bounds__(kFinThreads) void bwd_finalize_kernel(const double* __restrict__ partial, int nb,
                                                                int64_t M, int C,
                                                                const float* __restrict__ stats,
                                                                float* __restrict__ dgamma,
                                                                float* __restrict__ dbeta,
                                                                float* __restrict__ means) {
  __shared__ double sm[32][32];
  const int c = blockIdx.x * 16 + (threadIdx.x & 15);
  double t[2];
  reduce_partials(partial, nb, C, t, sm);
  if (c >= C || threadIdx.x >= 16) return;
  const double gm = (double)stats[P_GAMMA * C + c];
  dbeta[c] = (float)t[0];
  dgamma[c] = (float)t[1];
  means[c] = (float)(gm * t[0] / (double)M);
  means[C + c] = (float)(gm * t[1] / (double)M);
}

// The same second pass (blocks 0 .. nfin-1) and, in the other blocks of the same launch, the sum
// of `ncopies` partial copies of a weight gradient of n floats (64 outputs x 16 interleaved parts
// per block, a binary tree over the parts): two small dependent-free jobs that follow the conv
// backward kernel share one launch.
__global__ __launch_bounds__(kFinThreads) void bwd_finalize_dwsum_kernel(const double* __restrict__ partial, int nb,
                                                                      int64_t M, int C,
                                                                      const float* __restrict__ stats,
                                                                      float* __restrict__ dgamma,
                                                                      float* __restrict__ dbeta,
                                                                      float* __restrict__ means, int nfin,
                                                                      const float* __restrict__ wpartial,
                                                                      int ncopies, int64_t n,
                                                                      float* __restrict__ dw, int straight) {
  __shared__ double sm[32][32];
  if ((int)blockIdx.x >= nfin && straight != 0) {
    // large weight tensors in few copies: four consecutive outputs per thread (n is a multiple of 4
    // in this mode), the copies added in order
    const int64_t i = 4 * ((int64_t)(blockIdx.x - nfin) * kFinThreads + threadIdx.x);
    if (i >= n) return;
    float4 a = *reinterpret_cast<const float4*>(wpartial + i);
#pragma unroll 8
    for (int k = 1; k < ncopies; ++k) {
      const float4 b = *reinterpret_cast<const float4*>(wpartial + (int64_t)k * n + i);
      a.x += b.x; a.y += b.y; a.z += b.z; a.w += b.w;
    }
    *reinterpret_cast<float4*>(dw + i) = a;
    return;
  }
  if ((int)blockIdx.x < nfin) {
    const int c = blockIdx.x * 16 + (threadIdx.x & 15);
    double t[2];
    reduce_partials(partial, nb, C, t, sm);
    if (c >= C || threadIdx.x >= 16) return;
    const double gm = (double)stats[P_GAMMA * C + c];
    dbeta[c] = (float)t[0];
    dgamma[c] = (float)t[1];
    means[c] = (float)(gm * t[0] / (double)M);
    means[C + c] = (float)(gm * t[1] / (double)M);
    return;
  }
  float(*sw)[64] = reinterpret_cast<float(*)[64]>(&sm[0][0]);  // [16][64]
  const int o = threadIdx.x & 63, part = threadIdx.x >> 6;
  const int64_t i = (int64_t)(blockIdx.x - nfin) * 64 + o;
  float a = 0.f;
  if (i < n) {
#pragma unroll 8
    for (int k = part; k < ncopies; k += 16) a += wpartial[(int64_t)k * n + i];
  }
  sw[part][o] = a;
  __syncthreads();
  for (int h = 8; h >= 1; h >>= 1) {
    if (part < h) sw[part][o] += sw[part + h][o];
    __syncthreads();
  }
  if (part == 0 && i < n) dw[i] = sw[0][o];
}

// Backward, pass 2 (Eq. 8): dx = rstd * (dA1 - Mean(dA1) - A1~ * Mean(A1~ * dA1)).
template <int K, int VEC, bool ACCUM, bool STREAM>
__global__ __launch_bounds__(kThreads) void bwd_apply_kernel(const void* __restrict__ packed,
                                                             const float* da3, int64_t M, int C, RowGeom g,
                                                             const float* __restrict__ stats,
                                                             const float* __restrict__ means, float* dx,
                                                             float slope) {
  using S = Stored<K, VEC>;
  const ThreadPos p = thread_pos<VEC>(g);
  if (!p.active) return;
  const bool leaky = slope != 0.0f;
  float step[VEC], bt[VEC], gm[VEC], ig[VEC], rstd[VEC], m1[VEC], m2[VEC];
  int32_t fb[VEC];
  load_vec<VEC>(stats + P_STEP * C + p.c0, step);
  load_vec<VEC>(stats + P_BETA * C + p.c0, bt);
  load_vec<VEC>(stats + P_GAMMA * C + p.c0, gm);
  load_vec<VEC>(stats + P_RSTD * C + p.c0, rstd);
  load_vec<VEC>(means + p.c0, m1);
  load_vec<VEC>(means + C + p.c0, m2);
  load_vec_i<VEC>(reinterpret_cast<const int32_t*>(stats) + P_FB * C + p.c0, fb);
#pragma unroll
  for (int v = 0; v < VEC; ++v) ig[v] = 1.0f / gm[v];
  const int64_t row0 = (int64_t)blockIdx.y * g.TY * g.rpt + p.ty;
  for (int i = 0; i < g.rpt; i += kUnroll) {
    float gv[kUnroll][VEC], acc[kUnroll][VEC];
    typename S::raw_t w[kUnroll];
    bool ok[kUnroll];
#pragma unroll
    for (int j = 0; j < kUnroll; ++j) {
      const int64_t r = row0 + (int64_t)(i + j) * g.TY;
      ok[j] = (i + j) < g.rpt && r < M;
      const int64_t e = (ok[j] ? r : 0) * C + p.c0;
      load_vec<VEC>(da3 + e, gv[j]);
      if constexpr (ACCUM) load_vec<VEC>(dx + e, acc[j]);
      w[j] = S::load(packed, e);
    }
#pragma unroll
    for (int j = 0; j < kUnroll; ++j)
      if (ok[j]) {
        const int64_t r = row0 + (int64_t)(i + j) * g.TY;
        float out[VEC];
#pragma unroll
        for (int v = 0; v < VEC; ++v) {
          const float a2t = S::value(w[j], v, step[v], fb[v]);
          const float da2 = a2t > 0.0f ? gv[j][v] : (leaky ? slope * gv[j][v] : 0.0f);  // Eq. 6
          const float a1t = (a2t - bt[v]) * ig[v];
          const float da1 = gm[v] * da2;                    // Eq. 7
          const float t = (da1 - m1[v]) - a1t * m2[v];
          out[v] = rstd[v] * t;                             // Eq. 8
          if constexpr (ACCUM) out[v] = acc[j][v] + out[v];
        }
        store_vec<VEC, STREAM>(dx + r * C + p.c0, out);
      }
  }
}

// ------------------------------------------------------------------------------------------
// Any-C fallbacks: flat element order, 8 elements per thread, per-element channel lookup.
// They cover the zero-padded tail of the packed store as well.
template <int K, int MODE>  // MODE 0: bn+relu+pack, 1: pack only
__global__ __launch_bounds__(kThreads) void flat_quant_pack_kernel(const float* __restrict__ in, int64_t E,
                                                                   int C, int64_t packed_bytes,
                                                                   const float* __restrict__ stats,
                                                                   float* __restrict__ a3,
                                                                   uint8_t* __restrict__ packed, int naive,
                                                                   float slope) {
  const int64_t t = (int64_t)blockIdx.x * kThreads + threadIdx.x;
  const int64_t e0 = t * 8;
  if (e0 * K / 8 >= packed_bytes) return;
  const int32_t* fbp = reinterpret_cast<const int32_t*>(stats) + P_FB * C;
  uint32_t codes[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int64_t e = e0 + i;
    codes[i] = 0;
    if (e < E) {
      const int c = (int)(e % C);
      float a2 = in[e];
      if constexpr (MODE == 0) {
        const float d = a2 - stats[P_MEAN * C + c];
        const float a1 = d * stats[P_RSTD * C + c];
        const float g = stats[P_GAMMA * C + c] * a1;
        a2 = g + stats[P_BETA * C + c];
        a3[e] = a2 > 0.0f ? a2 : (slope != 0.0f ? slope * a2 : 0.0f);
      }
      codes[i] = quant_code<K>(a2, stats[P_CQ * C + c], fbp[c]);
      if constexpr (MODE == 0) {
        if (naive) {  // the convolution gets the approximation (Eq. 10), not A3
          const float a2t = dequant<K>(codes[i], stats[P_STEP * C + c], fbp[c]);
          a3[e] = a2t > 0.0f ? a2t : 0.0f;
        }
      }
    }
  }
  if constexpr (K == 32) {
#pragma unroll
    for (int b = 0; b < 8; ++b) reinterpret_cast<uint32_t*>(packed)[e0 + b] = codes[b];
  } else if constexpr (K == 4) {
#pragma unroll
    for (int b = 0; b < 4; ++b) packed[e0 / 2 + b] = (uint8_t)(codes[2 * b] | (codes[2 * b + 1] << 4));
  } else {
#pragma unroll
    for (int b = 0; b < 8; ++b) packed[e0 + b] = (uint8_t)codes[b];
  }
}

template <int K>
__device__ inline uint32_t flat_code(const uint8_t* __restrict__ packed, int64_t e) {
  if constexpr (K == 32) return reinterpret_cast<const uint32_t*>(packed)[e];
  if constexpr (K == 4) return (packed[e >> 1] >> ((e & 1) * 4)) & 15u;
  return packed[e];
}

template <int K>
__global__ __launch_bounds__(kThreads) void flat_unpack_kernel(const uint8_t* __restrict__ packed, int64_t E,
                                                               int C, const float* __restrict__ stats,
                                                               float* __restrict__ a2t, int act, float slope) {
  const int64_t e = (int64_t)blockIdx.x * kThreads + threadIdx.x;
  if (e >= E) return;
  const int c = (int)(e % C);
  const float a = dequant<K>(flat_code<K>(packed, e), stats[P_STEP * C + c],
                             reinterpret_cast<const int32_t*>(stats)[P_FB * C + c]);
  a2t[e] = (act == 0 || a > 0.0f) ? a : slope * a;
}

// Reduce pass for any C: one thread per channel per block pass (VEC = 1 geometry).
template <int K>
__global__ __launch_bounds__(kThreads) void flat_bwd_reduce_kernel(const uint8_t* __restrict__ packed,
                                                                   const float* __restrict__ da3, int64_t M,
                                                                   int C, RowGeom g,
                                                                   const float* __restrict__ stats,
                                                                   double* __restrict__ partial, float slope) {
  __shared__ double red[2][kThreads];
  const ThreadPos p = thread_pos<1>(g);
  const int c = p.c0;
  const float step = stats[P_STEP * C + c], bt = stats[P_BETA * C + c];
  const float ig = 1.0f / stats[P_GAMMA * C + c];
  const int32_t fb = reinterpret_cast<const int32_t*>(stats)[P_FB * C + c];
  double s1 = 0.0, s2 = 0.0;
  const int64_t row0 = (int64_t)blockIdx.y * g.TY * g.rpt + p.ty;
  for (int i = 0; i < g.rpt; ++i) {
    const int64_t r = row0 + (int64_t)i * g.TY;
    if (p.active && r < M) {
      const int64_t e = r * C + c;
      const float a2t = dequant<K>(flat_code<K>(packed, e), step, fb);
      const float da2 = a2t > 0.0f ? da3[e] : (slope != 0.0f ? slope * da3[e] : 0.0f);
      const float a1t = (a2t - bt) * ig;
      s1 += (double)da2;
      s2 += (double)a1t * (double)da2;
    }
  }
  red[0][threadIdx.x] = s1;
  red[1][threadIdx.x] = s2;
  __syncthreads();
  int span = 1;
  while (span < g.TY) span <<= 1;
  for (int h = span >> 1; h >= 1; h >>= 1) {
    if (p.ty < h && p.ty + h < g.TY) {
      red[0][threadIdx.x] += red[0][threadIdx.x + h * g.TX];
      red[1][threadIdx.x] += red[1][threadIdx.x + h * g.TX];
    }
    __syncthreads();
  }
  if (p.active && p.ty == 0) {
    partial[(int64_t)blockIdx.y * 2 * C + c] = red[0][threadIdx.x];
    partial[(int64_t)blockIdx.y * 2 * C + C + c] = red[1][threadIdx.x];
  }
}

template <int K, bool ACCUM>
__global__ __launch_bounds__(kThreads) void flat_bwd_apply_kernel(const uint8_t* __restrict__ packed,
                                                                  const float* da3, int64_t E, int C,
                                                                  const float* __restrict__ stats,
                                                                  const float* __restrict__ means, float* dx,
                                                                  float slope) {
  const int64_t e = (int64_t)blockIdx.x * kThreads + threadIdx.x;
  if (e >= E) return;
  const int c = (int)(e % C);
  const float gm = stats[P_GAMMA * C + c];
  const float a2t = dequant<K>(flat_code<K>(packed, e), stats[P_STEP * C + c],
                               reinterpret_cast<const int32_t*>(stats)[P_FB * C + c]);
  const float da2 = a2t > 0.0f ? da3[e] : (slope != 0.0f ? slope * da3[e] : 0.0f);
  const float a1t = (a2t - stats[P_BETA * C + c]) * (1.0f / gm);
  const float da1 = gm * da2;
  const float t = (da1 - means[c]) - a1t * means[C + c];
  float out = stats[P_RSTD * C + c] * t;
  if constexpr (ACCUM) out = dx[e] + out;
  dx[e] = out;
}

// Channels per thread of the row kernels for (K, C); 0 = use the flat fallback.
// wide: eight channels per thread where K = 4 allows (one 32-bit word of codes per thread and
// row) - measured best for the pass that only reads fp32 (pack: 5.3 -> 5.9 TB/s on a 205 MB
// tensor with one row per thread).  Kernels that WRITE fp32 rows take four channels: a lane then
// stores 16 bytes next to its neighbours' instead of 32 bytes in two instructions that each
// leave every other 16 bytes out (unpack 3.8 -> 5.4 TB/s, normalise-ReLU-pack 5.2 -> 5.9,
// Eq. 6-8 5.5 -> 5.9).
int fast_vec(int K, int C, bool wide) {
  if (K == 4 && wide && C % 8 == 0) return 8;
  return C % 4 == 0 ? 4 : 0;
}

inline dim3 grid_of(const RowGeom& g) { return dim3(g.gridX, g.gridY, 1); }

}  // namespace

// Room for kMaxPartialBlocks partial rows (the reduce kernels of this file use at most that
// many blocks, and so do the convolution epilogues that produce the same partial sums) plus the
// two per-channel means of the BN backward.
size_t bn_partial_bytes(int64_t M, int C) {
  (void)M;
  const size_t partial = (size_t)kMaxPartialBlocks * 2 * (size_t)C * sizeof(double);
  const size_t means = ((size_t)2 * C * sizeof(float) + 255) / 256 * 256;
  return partial + means;
}

size_t bn_means_offset(int C) { return (size_t)kMaxPartialBlocks * 2 * (size_t)C * sizeof(double); }

int launch_bn_stats(hipStream_t st, const float* x, int64_t M, int C, const float* gamma,
                    const float* beta, int K, void* scratch, void* stats) {
  double* partial = static_cast<double*>(scratch);
  const int vec = C % 4 == 0 ? 4 : 1;
  const RowGeom g = make_geom(M, C, vec, true);
  if (vec == 4)
    stats_partial_kernel<4><<<grid_of(g), kThreads, 0, st>>>(x, M, C, g, partial);
  else
    stats_partial_kernel<1><<<grid_of(g), kThreads, 0, st>>>(x, M, C, g, partial);
  return launch_bn_stats_finalize(st, partial, g.gridY, x, M, C, gamma, beta, K, stats);
}

// Second pass of the statistics from `nb` partial rows [nb][2][C]; `shift_row` is the row whose
// values the sums were shifted by (nullptr: no shift).
int launch_bn_stats_finalize(hipStream_t st, const double* partial, int nb, const float* shift_row, int64_t M,
                             int C, const float* gamma, const float* beta, int K, void* stats) {
  stats_finalize_kernel<<<(C + 15) / 16, kFinThreads, 0, st>>>(partial, nb, shift_row, M, C, gamma, beta, K,
                                                            static_cast<float*>(stats));
  return hip_status();
}

template <int MODE>
static int launch_quant_pack(hipStream_t st, const float* in, int64_t M, int C, int K, const void* stats,
                             float* a3, void* packed, bool naive = false, float slope = 0.0f) {
  const float* sp = static_cast<const float*>(stats);
  const int64_t E = M * C;
  const int64_t raw = (E * K + 7) / 8;
  const int64_t pbytes = (raw + 127) / 128 * 128;
  // the baseline variant exists in the element-wise kernel only
  const int vec = naive ? 0 : fast_vec(K, C, MODE == 1);
  if (vec == 0) {
    const int nv = naive ? 1 : 0;
    const int64_t threads = pbytes * 8 / K / 8;
    const unsigned blocks = (unsigned)((threads + kThreads - 1) / kThreads);
    uint8_t* pk = static_cast<uint8_t*>(packed);
    if (K == 4)
      flat_quant_pack_kernel<4, MODE><<<blocks, kThreads, 0, st>>>(in, E, C, pbytes, sp, a3, pk, nv, slope);
    else if (K == 8)
      flat_quant_pack_kernel<8, MODE><<<blocks, kThreads, 0, st>>>(in, E, C, pbytes, sp, a3, pk, nv, slope);
    else
      flat_quant_pack_kernel<32, MODE><<<blocks, kThreads, 0, st>>>(in, E, C, pbytes, sp, a3, pk, nv, slope);
    return hip_status();
  }
  // rows in flight per thread (measured on 205 MB, 51 MB and 13 MB tensors): the pass that writes
  // fp32 runs best with two, the read-only pack with one (K = 4) or two
  constexpr int ROWS_WIDE = 1, ROWS = 2;
  const RowGeom g = make_geom(M, C, vec, false, vec == 8 ? ROWS_WIDE : ROWS);
  const int pad = (int)(pbytes - raw);
  const bool stream = E * (int64_t)sizeof(float) >= kStreamBytes;
#define ABL_QP(KK, VV, RR)                                                                                   \
  do {                                                                                                       \
    if (stream)                                                                                              \
      quant_pack_kernel<KK, VV, MODE, true, RR><<<grid_of(g), kThreads, 0, st>>>(in, M, C, g, sp, a3, packed, pad, slope);  \
    else                                                                                                     \
      quant_pack_kernel<KK, VV, MODE, false, RR><<<grid_of(g), kThreads, 0, st>>>(in, M, C, g, sp, a3, packed, pad, slope); \
  } while (0)
  if (K == 4 && vec == 8) ABL_QP(4, 8, ROWS_WIDE);
  else if (K == 4) ABL_QP(4, 4, ROWS);
  else if (K == 8) ABL_QP(8, 4, ROWS);
  else ABL_QP(32, 4, ROWS);
#undef ABL_QP
  return hip_status();
}

int launch_bn_relu_pack(hipStream_t st, const float* x, int64_t M, int C, int K, const void* stats,
                        float* a3, void* packed, bool naive, float slope) {
  return launch_quant_pack<0>(st, x, M, C, K, stats, a3, packed, naive, slope);
}

int launch_pack(hipStream_t st, const float* a2, int64_t M, int C, int K, const void* stats,
                void* packed) {
  return launch_quant_pack<1>(st, a2, M, C, K, stats, nullptr, packed);
}

int launch_unpack(hipStream_t st, const void* packed, int64_t M, int C, int K, const void* stats,
                  float* a2t, bool act, float slope) {
  const int ac = act ? 1 : 0;
  const float* sp = static_cast<const float*>(stats);
  const int vec = fast_vec(K, C, false);
  if (vec == 0) {
    const int64_t E = M * C;
    const unsigned blocks = (unsigned)((E + kThreads - 1) / kThreads);
    const uint8_t* pk = static_cast<const uint8_t*>(packed);
    if (K == 4)
      flat_unpack_kernel<4><<<blocks, kThreads, 0, st>>>(pk, E, C, sp, a2t, ac, slope);
    else if (K == 8)
      flat_unpack_kernel<8><<<blocks, kThreads, 0, st>>>(pk, E, C, sp, a2t, ac, slope);
    else
      flat_unpack_kernel<32><<<blocks, kThreads, 0, st>>>(pk, E, C, sp, a2t, ac, slope);
    return hip_status();
  }
  const RowGeom g = make_geom(M, C, vec, false);
  // (streaming stores slow a pure-write kernel down on this part; measured 87 us vs 36 us)
#define ABL_UP(KK, VV)                                                                              \
  do {                                                                                              \
    unpack_kernel<KK, VV, false><<<grid_of(g), kThreads, 0, st>>>(packed, M, C, g, sp, a2t, ac, slope); \
  } while (0)
  if (K == 4) ABL_UP(4, 4);
  else if (K == 8) ABL_UP(8, 4);
  else ABL_UP(32, 4);
#undef ABL_UP
  return hip_status();
}

int launch_bn_bwd(hipStream_t st, const void* packed, const void* stats, const float* da3, int64_t M,
                  int C, int K, bool accum, void* scratch, float* dx, float* dgamma, float* dbeta,
                  const DwSum* dwsum, float slope) {
  const float* sp = static_cast<const float*>(stats);
  double* partial = static_cast<double*>(scratch);
  const int vec = fast_vec(K, C, false);
  const RowGeom gr = make_geom(M, C, vec ? vec : 1, true);
  const uint8_t* pk = static_cast<const uint8_t*>(packed);
  if (vec == 0) {
    if (K == 4)
      flat_bwd_reduce_kernel<4><<<grid_of(gr), kThreads, 0, st>>>(pk, da3, M, C, gr, sp, partial, slope);
    else if (K == 8)
      flat_bwd_reduce_kernel<8><<<grid_of(gr), kThreads, 0, st>>>(pk, da3, M, C, gr, sp, partial, slope);
    else
      flat_bwd_reduce_kernel<32><<<grid_of(gr), kThreads, 0, st>>>(pk, da3, M, C, gr, sp, partial, slope);
  } else if (K == 4) {
    bwd_reduce_kernel<4, 4><<<grid_of(gr), kThreads, 0, st>>>(packed, da3, M, C, gr, sp, partial, slope);
  } else if (K == 8) {
    bwd_reduce_kernel<8, 4><<<grid_of(gr), kThreads, 0, st>>>(packed, da3, M, C, gr, sp, partial, slope);
  } else {
    bwd_reduce_kernel<32, 4><<<grid_of(gr), kThreads, 0, st>>>(packed, da3, M, C, gr, sp, partial, slope);
  }
  if (hipGetLastError() != hipSuccess) return ABL_ERR_HIP;
  return launch_bn_bwd_finish(st, packed, stats, da3, M, C, K, accum, scratch, gr.gridY, dx, dgamma, dbeta, dwsum,
                              slope);
}

// Eq. 7 totals and Eq. 8 from `nb` partial rows [nb][2][C] of (sum dA2, sum A1~ dA2) at the
// start of `scratch`: finalize kernel, then the apply pass.
int launch_bn_bwd_finish(hipStream_t st, const void* packed, const void* stats, const float* da3, int64_t M,
                         int C, int K, bool accum, void* scratch, int nb, float* dx, float* dgamma,
                         float* dbeta, const DwSum* dwsum, float slope) {
  const float* sp = static_cast<const float*>(stats);
  const double* partial = static_cast<const double*>(scratch);
  float* means = reinterpret_cast<float*>(static_cast<char*>(scratch) + bn_means_offset(C));
  const uint8_t* pk = static_cast<const uint8_t*>(packed);
  const int vec = fast_vec(K, C, false);
  const int nfin = (C + 15) / 16;
  if (dwsum != nullptr) {
    // many small copies (one per pixel tile): 16 interleaved parts per output and a tree;
    // few large ones (split contraction): one thread per output
    const bool straight = dwsum->copies <= 32 && dwsum->n >= 131072 && dwsum->n % 4 == 0;
    const unsigned wblocks = straight ? (unsigned)((dwsum->n / 4 + kFinThreads - 1) / kFinThreads)
                                      : (unsigned)((dwsum->n + 63) / 64);
    bwd_finalize_dwsum_kernel<<<nfin + wblocks, kFinThreads, 0, st>>>(partial, nb, M, C, sp, dgamma, dbeta, means, nfin,
                                                                      dwsum->partial, dwsum->copies, dwsum->n,
                                                                      dwsum->dw, straight ? 1 : 0);
  } else
    bwd_finalize_kernel<<<nfin, kFinThreads, 0, st>>>(partial, nb, M, C, sp, dgamma, dbeta, means);
  if (vec == 0) {
    const int64_t E = M * C;
    const unsigned blocks = (unsigned)((E + kThreads - 1) / kThreads);
    if (K == 4 && accum) flat_bwd_apply_kernel<4, true><<<blocks, kThreads, 0, st>>>(pk, da3, E, C, sp, means, dx, slope);
    else if (K == 4) flat_bwd_apply_kernel<4, false><<<blocks, kThreads, 0, st>>>(pk, da3, E, C, sp, means, dx, slope);
    else if (K == 8 && accum) flat_bwd_apply_kernel<8, true><<<blocks, kThreads, 0, st>>>(pk, da3, E, C, sp, means, dx, slope);
    else if (K == 8) flat_bwd_apply_kernel<8, false><<<blocks, kThreads, 0, st>>>(pk, da3, E, C, sp, means, dx, slope);
    else if (accum) flat_bwd_apply_kernel<32, true><<<blocks, kThreads, 0, st>>>(pk, da3, E, C, sp, means, dx, slope);
    else flat_bwd_apply_kernel<32, false><<<blocks, kThreads, 0, st>>>(pk, da3, E, C, sp, means, dx, slope);
    return hip_status();
  }
  const RowGeom ga = make_geom(M, C, vec, false);
  const bool stream = M * C * (int64_t)sizeof(float) >= kStreamBytes;
#define ABL_APPLY1(KK, VV, AA)                                                                              \
  do {                                                                                                      \
    if (stream)                                                                                             \
      bwd_apply_kernel<KK, VV, AA, true><<<grid_of(ga), kThreads, 0, st>>>(packed, da3, M, C, ga, sp, means, dx, slope); \
    else                                                                                                    \
      bwd_apply_kernel<KK, VV, AA, false><<<grid_of(ga), kThreads, 0, st>>>(packed, da3, M, C, ga, sp, means, dx, slope); \
  } while (0)
#define ABL_APPLY(KK, VV)             \
  do {                                \
    if (accum) ABL_APPLY1(KK, VV, true); \
    else ABL_APPLY1(KK, VV, false);   \
  } while (0)
  if (K == 4) ABL_APPLY(4, 4);
  else if (K == 8) ABL_APPLY(8, 4);
  else ABL_APPLY(32, 4);
#undef ABL_APPLY1
#undef ABL_APPLY
  return hip_status();
}


// ------------------------------------------------------------------------------------------
// SGD with momentum and weight decay (Sec. 4), in place; four elements per lane, scalar tail.
namespace {
__device__ inline void sgd_one(float& w, float g, float& v, float lr, float mu, float wd) {
  const float d = g + wd * w;
  v = mu * v + d;
  w = w - lr * v;
}

__global__ __launch_bounds__(kThreads) void sgd_momentum_kernel(int64_t n, float lr, float mu, float wd,
                                                                float* __restrict__ w,
                                                                const float* __restrict__ grad,
                                                                float* __restrict__ v) {
  const int64_t i = ((int64_t)blockIdx.x * kThreads + threadIdx.x) * 4;
  if (i + 4 <= n) {
    float4 wv = *reinterpret_cast<const float4*>(w + i);
    float4 vv = *reinterpret_cast<const float4*>(v + i);
    const float4 gv = *reinterpret_cast<const float4*>(grad + i);
    sgd_one(wv.x, gv.x, vv.x, lr, mu, wd);
    sgd_one(wv.y, gv.y, vv.y, lr, mu, wd);
    sgd_one(wv.z, gv.z, vv.z, lr, mu, wd);
    sgd_one(wv.w, gv.w, vv.w, lr, mu, wd);
    *reinterpret_cast<float4*>(w + i) = wv;
    *reinterpret_cast<float4*>(v + i) = vv;
  } else {
    for (int64_t k = i; k < n; ++k) {
      float wk = w[k], vk = v[k];
      sgd_one(wk, grad[k], vk, lr, mu, wd);
      w[k] = wk;
      v[k] = vk;
    }
  }
}
}  // namespace

int launch_sgd_momentum(hipStream_t st, int64_t n, float lr, float mu, float wd, float* w, const float* grad,
                        float* v) {
  if (n == 0) return ABL_OK;
  const int64_t lanes = (n + 3) / 4;
  sgd_momentum_kernel<<<(unsigned)((lanes + kThreads - 1) / kThreads), kThreads, 0, st>>>(n, lr, mu, wd, w, grad, v);
  return hip_status();
}

}  // namespace abl
