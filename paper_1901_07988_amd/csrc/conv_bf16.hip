// ABL_MATH_BF16 contractions for gfx950 (CDNA4): Eq. 4 (forward) and the second half of Eq. 5
// (gradient to the conv input) as implicit GEMMs on v_mfma_f32_16x16x32_bf16.
//
//   Out[p][n] = sum_{tap, c} A[p][(tap, c)] * B[(tap, c)][n]        (fp32 accumulation)
//   MODE 0 forward: p = (n, ho, wo), A = a3[n, ho*st + r - pad, wo*st + s - pad, c], c < Cin,
//                   B = W[r][s][c][n], n < Cout
//   MODE 1 dgrad  : p = (n, h, w),   A = dy[n, (h + pad - r)/st, (w + pad - s)/st, c], c < Cout
//                   (where the division is exact and lands inside dy), B = W[r][s][n][c], n < Cin
//
// Operands are rounded to bf16 ONCE, by the hardware's packed convert, on their way from global
// memory into LDS, and stay bf16 there: a tile row holds the 32 contraction channels of one chunk
// contiguously (80-byte pitch: conflict-free 16-byte fragment reads), so one ds_read_b128 is a
// lane's whole operand of one MFMA (8 consecutive k).  Block tile 128 pixels x BN channels, four
// waves as 2 x 2, LDS tiles double buffered with the next chunk's global loads in flight during
// the MFMAs.  The forward's weights arrive with the output channel contiguous and are transposed
// on the way: a lane packs rows k, k+1 of four channels into 32-bit words and the lane order is
// chosen so that those writes hit 64 different banks.
// The MFMA computes the transposed tile (first operand = weights), so a lane ends up with four
// consecutive channels of one pixel: 16-byte stores and shortcut loads.

#include <mutex>
#include <set>
#include <utility>

#include "abl_internal.h"

namespace abl {
namespace {

constexpr int kThreads = 256;
constexpr int BM = 128;   // pixels per block
constexpr int BK = 32;    // contraction channels per chunk = k of one MFMA
constexpr int LDK = 40;   // bf16 per LDS tile row (32 + 8 pad): 80 bytes, 16-byte aligned

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

// two floats -> one 32-bit word of two bf16 (round to nearest even), lo in bits 0-15
__device__ inline uint32_t pack_bf16(float lo, float hi) {
  const bf16x2 v = {(__bf16)lo, (__bf16)hi};
  return __builtin_bit_cast(uint32_t, v);
}

// EPI: 0 = none; 1 (forward) = per-block sums of y and y^2 per channel, the first pass of the next
// layer's Eq. 1; 4 / 8 (gradient) = the Eq. 6-7 sums from the layer's K-bit codes, the first pass of
// the BN backward.  Row m0 / BM of sums = [blocks][2][Ng] doubles.
template <int MODE, int BN, int EPI>
__global__ __launch_bounds__(kThreads) void gemm_bf16_kernel(const float* __restrict__ in,
                                                             const float* __restrict__ wgt, const float* skip,
                                                             float* out, ConvGeom g, double* __restrict__ sums,
                                                             const uint8_t* __restrict__ codes,
                                                             const float* __restrict__ stats) {
  constexpr int WM = BM / 2, WN = BN / 2;     // wave tile
  constexpr int MT = WM / 16, NT = WN / 16;
  constexpr int A_PASSES = BM * (BK / 4) / kThreads;   // float4 of the A tile per thread: 4
  constexpr int B_F4 = BN * (BK / 4) / kThreads;       // float4 of the B tile per thread: 2 or 4
  constexpr int B_PAIRS = B_F4 / 2;                    // forward: items of two float4 (rows k, k + 1)
  static_assert(BM * (BK / 4) % kThreads == 0 && BN * (BK / 4) % kThreads == 0, "whole items per thread");

  __shared__ __attribute__((aligned(16))) unsigned short lds[2 * (BM + BN) * LDK];
  unsigned short* const As0 = lds;                  // [2][BM][LDK]
  unsigned short* const Bs0 = lds + 2 * BM * LDK;   // [2][BN][LDK]

  const int Hi = MODE == 0 ? g.H : g.Ho, Wi = MODE == 0 ? g.W : g.Wo;
  const int Hq = MODE == 0 ? g.Ho : g.H, Wq = MODE == 0 ? g.Wo : g.W;
  const int Cg = MODE == 0 ? g.Cin : g.Cout;   // contraction channels (multiple of 32)
  const int Ng = MODE == 0 ? g.Cout : g.Cin;   // output channels (multiple of BN)
  const int64_t Mg = (int64_t)g.N * Hq * Wq;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int li = lane & 15, lk = lane >> 4;
  const int wm0 = (wave >> 1) * WM, wn0 = (wave & 1) * WN;
  // ids 8 apart share an XCD (and its L2): the blocks that read the same pixel rows for
  // different output-channel blocks run there back to back
  const int nblk_n = Ng / BN;
  const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
  const int64_t m0 = ((int64_t)(slot / nblk_n) * 8 + xcd) * BM;
  const int n0 = (slot % nblk_n) * BN;
  if (m0 >= Mg) return;

  // A tile: thread = (row a_row + 32 i, channels 4 a_kq .. +3 of the chunk)
  const int a_kq = tid & 7, a_row = tid >> 3;
  int a_n[A_PASSES], a_h[A_PASSES], a_w[A_PASSES];
  bool a_ok[A_PASSES];
#pragma unroll
  for (int i = 0; i < A_PASSES; ++i) {
    const int64_t p = m0 + a_row + 32 * i;
    a_ok[i] = p < Mg;
    const int pp = a_ok[i] ? (int)p : 0;
    const int wq = pp % Wq;
    const int t = pp / Wq;
    const int hq = t % Hq;
    a_n[i] = t / Hq;
    a_h[i] = MODE == 0 ? hq * g.stride - g.pad : hq + g.pad;
    a_w[i] = MODE == 0 ? wq * g.stride - g.pad : wq + g.pad;
  }
  int a_off[A_PASSES];  // element offset of channel 0 of the thread's pixel for the current tap, -1 = zero
  auto set_tap = [&](int tap) __attribute__((always_inline)) {
    const int r = tap / g.S, s = tap - r * g.S;
#pragma unroll
    for (int i = 0; i < A_PASSES; ++i) {
      int hi, wi;
      bool ok = a_ok[i];
      if (MODE == 0) {
        hi = a_h[i] + r;
        wi = a_w[i] + s;
      } else {
        const int hh = a_h[i] - r, ww = a_w[i] - s;
        hi = hh / g.stride;
        wi = ww / g.stride;
        ok = ok && hh >= 0 && ww >= 0 && hi * g.stride == hh && wi * g.stride == ww;
      }
      ok = ok && hi >= 0 && hi < Hi && wi >= 0 && wi < Wi;
      a_off[i] = ok ? ((a_n[i] * Hi + hi) * Wi + wi) * Cg : -1;
    }
  };
  // B tile.  dgrad: W[tap][n][k] has k contiguous - thread = (row n, channels 4 q .. +3), as the A
  // tile.  Forward: W[tap][k][n] has n contiguous - thread = (k pair kp = lane % 16, four
  // channels 4 gq .. +3 with gq = lane / 16 + 4 (wave + 4 j)): it reads rows 2 kp and 2 kp + 1 and
  // writes four words [n][2 kp, 2 kp + 1]; per write instruction the 64 lanes cover 16 kp x 4 gq,
  // whose word addresses n * 20 + kp fall into 64 different banks.
  const int b_kp = lane & 15, b_g = lane >> 4;
  const int taps = g.R * g.S;
  const int cchunks = Cg / BK;
  const int iters = taps * cchunks;

  floatx4 ra[A_PASSES];
  floatx4 rb[B_F4];
  uint32_t a_live = 0;
  int f_tap = 0, f_c0 = 0;
  set_tap(0);
  auto fetch = [&]() __attribute__((always_inline)) {
    // every load is unconditional (a lane outside the image reads element 0 and is zeroed when the
    // tile is staged): no branch separates the loads, so all of them are in flight together
#pragma unroll
    for (int i = 0; i < A_PASSES; ++i) {
      const bool ok = a_off[i] >= 0;
      ra[i] = *reinterpret_cast<const floatx4*>(in + (ok ? a_off[i] + f_c0 + 4 * a_kq : 0));
      a_live = ok ? (a_live | (1u << i)) : (a_live & ~(1u << i));
    }
    if (MODE == 0) {
      const float* wb = wgt + ((int64_t)f_tap * g.Cin + f_c0) * g.Cout + n0;
#pragma unroll
      for (int j = 0; j < B_PAIRS; ++j) {
        const int gq = b_g + 4 * (wave + 4 * j);
        const float* src = wb + (int64_t)(2 * b_kp) * g.Cout + 4 * gq;
        rb[2 * j] = *reinterpret_cast<const floatx4*>(src);
        rb[2 * j + 1] = *reinterpret_cast<const floatx4*>(src + g.Cout);
      }
    } else {
      const float* wb = wgt + (int64_t)f_tap * g.Cin * g.Cout + f_c0;
#pragma unroll
      for (int j = 0; j < B_F4; ++j) {
        const int idx = tid + kThreads * j;
        rb[j] = *reinterpret_cast<const floatx4*>(wb + (int64_t)(n0 + (idx >> 3)) * g.Cout + 4 * (idx & 7));
      }
    }
    f_c0 += BK;
    if (f_c0 >= Cg) {
      f_c0 = 0;
      ++f_tap;
      if (f_tap < taps) set_tap(f_tap);
    }
  };
  auto stage = [&](int buf) __attribute__((always_inline)) {
    unsigned short* As = As0 + buf * BM * LDK;
    unsigned short* Bs = Bs0 + buf * BN * LDK;
#pragma unroll
    for (int i = 0; i < A_PASSES; ++i) {
      const bool ok = (a_live >> i) & 1u;
      uint2 v;
      v.x = ok ? pack_bf16(ra[i][0], ra[i][1]) : 0u;
      v.y = ok ? pack_bf16(ra[i][2], ra[i][3]) : 0u;
      *reinterpret_cast<uint2*>(&As[(a_row + 32 * i) * LDK + 4 * a_kq]) = v;
    }
    if (MODE == 0) {
#pragma unroll
      for (int j = 0; j < B_PAIRS; ++j) {
        const int gq = b_g + 4 * (wave + 4 * j);
#pragma unroll
        for (int e = 0; e < 4; ++e)
          *reinterpret_cast<uint32_t*>(&Bs[(4 * gq + e) * LDK + 2 * b_kp]) = pack_bf16(rb[2 * j][e], rb[2 * j + 1][e]);
      }
    } else {
#pragma unroll
      for (int j = 0; j < B_F4; ++j) {
        const int idx = tid + kThreads * j;
        uint2 v;
        v.x = pack_bf16(rb[j][0], rb[j][1]);
        v.y = pack_bf16(rb[j][2], rb[j][3]);
        *reinterpret_cast<uint2*>(&Bs[(idx >> 3) * LDK + 4 * (idx & 7)]) = v;
      }
    }
  };

  floatx4 acc[NT][MT];  // acc[j][i][r]: pixel wm0 + 16 i + li, channel wn0 + 16 j + 4 lk + r
#pragma unroll
  for (int j = 0; j < NT; ++j)
#pragma unroll
    for (int i = 0; i < MT; ++i) acc[j][i] = floatx4{0.f, 0.f, 0.f, 0.f};

  fetch();
  stage(0);
  __syncthreads();
  for (int it = 0; it < iters; ++it) {
    const int cur = it & 1;
    if (it + 1 < iters) fetch();
    const unsigned short* As = As0 + cur * BM * LDK;
    const unsigned short* Bs = Bs0 + cur * BN * LDK;
    bf16x8 af[MT], bf[NT];
#pragma unroll
    for (int i = 0; i < MT; ++i) af[i] = *reinterpret_cast<const bf16x8*>(&As[(wm0 + 16 * i + li) * LDK + 8 * lk]);
#pragma unroll
    for (int j = 0; j < NT; ++j) bf[j] = *reinterpret_cast<const bf16x8*>(&Bs[(wn0 + 16 * j + li) * LDK + 8 * lk]);
#pragma unroll
    for (int j = 0; j < NT; ++j)
#pragma unroll
      for (int i = 0; i < MT; ++i) acc[j][i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(bf[j], af[i], acc[j][i], 0, 0, 0);
    if (it + 1 < iters) stage(cur ^ 1);
    __syncthreads();
  }

  // epilogue: the lane holds channels n0 + wn0 + 16 j + 4 lk .. +3 of pixel m0 + wm0 + 16 i + li.
  // One 16-channel tile after the other, so that the sums of one tile only are live (all of them
  // at once cost the kernel a resident block per SIMD).
  if constexpr (EPI == 0) {
    // no sums: one pixel after the other, so that a wave's stores to a pixel's channels follow each other
#pragma unroll
    for (int i = 0; i < MT; ++i) {
      const int64_t p = m0 + wm0 + 16 * i + li;
      if (p >= Mg) continue;
#pragma unroll
      for (int j = 0; j < NT; ++j) {
        const int64_t o = p * Ng + n0 + wn0 + 16 * j + 4 * lk;
        float4 v = make_float4(acc[j][i][0], acc[j][i][1], acc[j][i][2], acc[j][i][3]);
        if (skip != nullptr) {
          const float4 sv = *reinterpret_cast<const float4*>(skip + o);
          v.x += sv.x; v.y += sv.y; v.z += sv.z; v.w += sv.w;
        }
        *reinterpret_cast<float4*>(out + o) = v;
      }
    }
    return;
  }
  double* red = reinterpret_cast<double*>(lds);   // [2][2][BN], free since the barrier that ended the main loop
#pragma unroll
  for (int j = 0; j < NT; ++j) {
    const int c = n0 + wn0 + 16 * j + 4 * lk;
    double s1[4] = {0.0, 0.0, 0.0, 0.0}, s2[4] = {0.0, 0.0, 0.0, 0.0};
    floatx4 e_st, e_bt, e_ig;
    int4 e_fb;
    if constexpr (EPI > 1) {
      e_st = *reinterpret_cast<const floatx4*>(stats + P_STEP * Ng + c);
      e_bt = *reinterpret_cast<const floatx4*>(stats + P_BETA * Ng + c);
      const floatx4 gm = *reinterpret_cast<const floatx4*>(stats + P_GAMMA * Ng + c);
      e_ig = floatx4{1.0f / gm[0], 1.0f / gm[1], 1.0f / gm[2], 1.0f / gm[3]};
      e_fb = *reinterpret_cast<const int4*>(stats + P_FB * Ng + c);
    }
#pragma unroll
    for (int i = 0; i < MT; ++i) {
      const int64_t p = m0 + wm0 + 16 * i + li;
      if (p >= Mg) continue;
      const int64_t o = p * Ng + c;
      float4 v = make_float4(acc[j][i][0], acc[j][i][1], acc[j][i][2], acc[j][i][3]);
      if (skip != nullptr) {
        const float4 sv = *reinterpret_cast<const float4*>(skip + o);
        v.x += sv.x; v.y += sv.y; v.z += sv.z; v.w += sv.w;
      }
      *reinterpret_cast<float4*>(out + o) = v;
      if constexpr (EPI == 1) {
        const float vv[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          s1[r] += (double)vv[r];
          s2[r] += (double)vv[r] * (double)vv[r];
        }
      } else if constexpr (EPI > 1) {
        const uint32_t cw = EPI == 4 ? (uint32_t) * reinterpret_cast<const uint16_t*>(codes + (o >> 1))
                                     : *reinterpret_cast<const uint32_t*>(codes + o);
        const float vv[4] = {v.x, v.y, v.z, v.w};
        const int32_t fbv[4] = {e_fb.x, e_fb.y, e_fb.z, e_fb.w};
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const uint32_t code = (cw >> (EPI * r)) & ((1u << EPI) - 1u);
          const int32_t q = (int32_t)code - (1 << (EPI - 1)) + fbv[r];
          const float a2t = e_st[r] * ((float)q + 0.5f);            // Eq. 10
          const float da2 = a2t > 0.0f ? vv[r] : 0.0f;              // Eq. 6
          const float a1t = (a2t - e_bt[r]) * e_ig[r];              // inverse of Eq. 2
          s1[r] += (double)da2;
          s2[r] += (double)a1t * (double)da2;
        }
      }
    }
    if constexpr (EPI != 0) {
      // fixed order: the 16 pixel lanes by a butterfly, then (below) the two waves that share the channels
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        double t1 = s1[r], t2 = s2[r];
#pragma unroll
        for (int d = 1; d < 16; d <<= 1) {
          t1 += __shfl_xor(t1, d, 64);
          t2 += __shfl_xor(t2, d, 64);
        }
        if (li == 0) {
          red[(0 * 2 + (wave >> 1)) * BN + wn0 + 16 * j + 4 * lk + r] = t1;
          red[(1 * 2 + (wave >> 1)) * BN + wn0 + 16 * j + 4 * lk + r] = t2;
        }
      }
    }
  }
  if constexpr (EPI != 0) {
    __syncthreads();
    for (int c = tid; c < 2 * BN; c += kThreads) {
      const int qv = c / BN, ch = c % BN;
      sums[((m0 / BM) * 2 + qv) * Ng + n0 + ch] = red[(qv * 2 + 0) * BN + ch] + red[(qv * 2 + 1) * BN + ch];
    }
  }
}

// ---- 3x3 'same' stride-1 convolutions on small images: the whole image stays in LDS -------------
// One block = one image x 64 output channels.  The image, rounded to bf16 once, sits in LDS with
// its zero border for the whole contraction ((H+2)(W+2) positions of Cg channels, 135 KB for
// 14x14x256: what the 160 KB of LDS per compute unit are for), so every input element is fetched
// and converted once per block instead of once per filter tap.  The four waves split the
// CONTRACTION (tap, 32-channel chunk) between them and each keeps the block's whole output tile
// (up to 13 x 4 MFMA tiles) in registers: an activation fragment is then read from LDS once per
// block and k-step, the waves share no weights (each streams its own k-steps' fragments straight
// from the L2 into registers, converted on arrival) and the main loop has no barrier.  The four
// partial tiles are added through LDS at the end in a fixed wave order; the wave that owns an
// output-channel tile adds the shortcut, stores, and takes the per-channel sums of the output for
// the next layer's Eq. 1 statistics.
constexpr int IMG_NB = 64;       // output channels per block

template <int MODE, int MT, int EPI>
__global__ __launch_bounds__(kThreads, 1) void image_bf16_kernel(const float* __restrict__ in,
                                                                 const float* __restrict__ wgt,
                                                                 const float* skip, float* out,
                                                                 double* __restrict__ sums, ConvGeom g,
                                                                 const uint8_t* __restrict__ codes,
                                                                 const float* __restrict__ stats) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const int H = g.H, W = g.W, HW = H * W, PW = W + 2;
  const int Cg = MODE == 0 ? g.Cin : g.Cout;   // contraction channels: a power of two, 32 .. 1024
  const int Ng = MODE == 0 ? g.Cout : g.Cin;   // output channels: a multiple of 64
  const int pitch = 2 * Cg + 16;               // bytes per patch position: 16-byte fragments of 16
                                               // consecutive positions fall into different banks
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int li = lane & 15, lk = lane >> 4;
  // ids 8 apart share an XCD and its L2: the blocks of one image (same input) run there
  const int nblk = Ng / IMG_NB;
  const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
  const int img = (slot / nblk) * 8 + xcd;
  const int n0 = (slot % nblk) * IMG_NB;
  if (img >= g.N) return;

  // ---- the image -> LDS (bf16), border positions zeroed
  {
    const int c4sh = __builtin_ctz((unsigned)Cg) - 2;   // log2 of float4 per pixel
    const int total = HW << c4sh;
    const uint32_t wmagic = 65536u / (unsigned)W + 1u;  // pix / W for pix * W < 65536
    const floatx4* src = reinterpret_cast<const floatx4*>(in + (size_t)img * HW * Cg);
    // No branch anywhere below (a guarded load or store makes the compiler wait for everything in
    // flight): a lane past the end repeats the last item, which rewrites the same value.
    constexpr int U = 13;   // loads in flight per lane: four round trips for 14x14x256
    for (int f0 = 0; f0 < total; f0 += kThreads * U) {
      floatx4 v[U];
      int fi[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int f = f0 + tid + kThreads * u;
        fi[u] = f < total ? f : total - 1;
        v[u] = src[fi[u]];
      }
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int pix = fi[u] >> c4sh, c4 = fi[u] - (pix << c4sh);
        const int h = (int)(((unsigned)pix * wmagic) >> 16), w = pix - h * W;
        uint2 o;
        o.x = pack_bf16(v[u][0], v[u][1]);
        o.y = pack_bf16(v[u][2], v[u][3]);
        *reinterpret_cast<uint2*>(smem + ((h + 1) * PW + w + 1) * pitch + c4 * 8) = o;
      }
    }
    const int per = pitch >> 4;                         // 16-byte pieces per position
    const int border = 2 * PW + 2 * H;
    const int nz = border * per;
    for (int i0 = 0; i0 < nz; i0 += kThreads) {
      const int it = i0 + tid < nz ? i0 + tid : nz - 1;
      const int bp = it / per, piece = it - bp * per;
      int pos;
      if (bp < PW) pos = bp;
      else if (bp < 2 * PW) pos = (H + 1) * PW + (bp - PW);
      else pos = (((bp - 2 * PW) >> 1) + 1) * PW + (((bp - 2 * PW) & 1) ? PW - 1 : 0);
      *reinterpret_cast<uint4*>(smem + pos * pitch + piece * 16) = make_uint4(0u, 0u, 0u, 0u);
    }
  }

  // ---- fragment addresses.  acc[jj] is the output-channel tile (wave + jj) % 4, so that a wave's
  // own tile (the one it finishes) is acc[0] whatever the wave.
  int a_base[MT];
#pragma unroll
  for (int i = 0; i < MT; ++i) {
    int m = 16 * i + li;
    m = m < HW ? m : HW - 1;   // rows past the image: any valid address, never stored
    const int h = m / W, w = m - h * W;
    a_base[i] = (h * PW + w) * pitch + lk * 16;
    asm volatile("" : "+v"(a_base[i]));   // kept in its register, not recomputed in the loop
  }
  const int cch_sh = __builtin_ctz((unsigned)Cg) - 5;   // log2 of 32-channel chunks
  const int T = 9 << cch_sh;
  const int ks_begin = wave * T / 4, ks_end = (wave + 1) * T / 4;

  // raw weights of one k-step: the lane's 8 contraction channels of its column in 4 tiles.
  // Uniform part of the address in scalar registers, the lane's part a 32-bit offset.
  floatx4 raw[4][2];
  uint32_t w_lane[8];   // forward: byte offsets of the 8 rows; gradient: [0] only
#pragma unroll
  for (int e = 0; e < 8; ++e)
    w_lane[e] = 4u * (MODE == 0 ? (uint32_t)((8 * lk + e) * g.Cout + li) : (uint32_t)(li * g.Cout + 8 * lk));
  auto load_w_tile = [&](int ks, int jj) __attribute__((always_inline)) {
    const int tap = ks >> cch_sh, c0 = (ks - (tap << cch_sh)) * BK;
    const int nt = n0 + 16 * ((wave + jj) & 3);
    if (MODE == 0) {
      // W[tap][c][n]: rows c0 + 8 lk + e of column n
      const char* wb = reinterpret_cast<const char*>(wgt + ((size_t)(tap * g.Cin + c0) * g.Cout + nt));
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        // (opaque to the optimizer: the 32-bit offset stays a 32-bit register operand of the load
        // beside the scalar base instead of being widened to a 64-bit address outside the loop)
        asm volatile("" : "+v"(w_lane[e]));
        raw[jj][e >> 2][e & 3] = *reinterpret_cast<const float*>(wb + w_lane[e]);
      }
    } else {
      // gradient to the input: tap (r', s') of the patch pairs with W[2 - r'][2 - s'][n][c]
      const char* wb = reinterpret_cast<const char*>(wgt + ((size_t)((8 - tap) * g.Cin + nt) * g.Cout + c0));
      asm volatile("" : "+v"(w_lane[0]));
      raw[jj][0] = *reinterpret_cast<const floatx4*>(wb + w_lane[0]);
      raw[jj][1] = *reinterpret_cast<const floatx4*>(wb + w_lane[0] + 16);
    }
  };
  auto a_offset = [&](int ks) __attribute__((always_inline)) {
    const int tap = ks >> cch_sh, cc = ks - (tap << cch_sh);
    const int r = tap / 3, s = tap - 3 * r;
    return (r * PW + s) * pitch + cc * (BK * 2);
  };

  floatx4 acc[4][MT];
#pragma unroll
  for (int jj = 0; jj < 4; ++jj)
#pragma unroll
    for (int i = 0; i < MT; ++i) acc[jj][i] = floatx4{0.f, 0.f, 0.f, 0.f};

  // Per k-step: convert the weights that arrived during the previous one and issue the 4 x MT
  // MFMAs, with the requests for the next k-step's weights behind the first four tiles.
  if (ks_begin < ks_end) {
#pragma unroll
    for (int jj = 0; jj < 4; ++jj) load_w_tile(ks_begin, jj);
  }
  __syncthreads();
  // One set of activation fragments, refreshed in place: a tile's fragment of the next k-step is
  // requested as soon as its four MFMAs of this k-step have been issued, a whole k-step ahead.
  bf16x8 a[MT];
  if (ks_begin < ks_end) {
    const int off = a_offset(ks_begin);
#pragma unroll
    for (int i = 0; i < MT; ++i) a[i] = *reinterpret_cast<const bf16x8*>(smem + a_base[i] + off);
  }
  for (int ks = ks_begin; ks < ks_end; ++ks) {
    bf16x8 wf[4];
#pragma unroll
    for (int jj = 0; jj < 4; ++jj) {
      const uint4 q = make_uint4(pack_bf16(raw[jj][0][0], raw[jj][0][1]), pack_bf16(raw[jj][0][2], raw[jj][0][3]),
                                 pack_bf16(raw[jj][1][0], raw[jj][1][1]), pack_bf16(raw[jj][1][2], raw[jj][1][3]));
      wf[jj] = __builtin_bit_cast(bf16x8, q);
    }
    const int kn = ks + 1 < ks_end ? ks + 1 : ks;   // the last k-step asks for its own operands again: no branch
    const int offn = a_offset(kn);
    __builtin_amdgcn_sched_barrier(0);
    // the order below is the schedule
#pragma unroll
    for (int i = 0; i < MT; ++i) {
#pragma unroll
      for (int jj = 0; jj < 4; ++jj)
        // written out so that the accumulator stays in one place (result register = addend
        // register): left to the register allocator, some tiles get a result register of their
        // own and are copied back every k-step.  The matrix core's results are not read before
        // the wait states after the loop.
        asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(acc[jj][i]) : "v"(wf[jj]), "v"(a[i]));
      a[i] = *reinterpret_cast<const bf16x8*>(smem + a_base[i] + offn);
      constexpr int WT = MT < 4 ? MT : 4;   // the next k-step's weights behind the first four tiles
      if (i < WT) load_w_tile(kn, i);
      __builtin_amdgcn_sched_barrier(0);
    }
  }

  // the last MFMAs' results are read below by instructions the compiler does not know to depend
  // on a matrix-core result: more wait states than the longest such hazard (18)
  asm volatile("s_nop 15\n\ts_nop 15");
  // ---- the four partial tiles -> one: wave w sends acc[jj], jj = 1..3, to the owner (w + jj) % 4,
  // which adds what it receives in the order jj = 1, 2, 3 of the senders
  __syncthreads();   // every wave has finished reading the image
#pragma unroll
  for (int jj = 1; jj < 4; ++jj) {
    const int owner = (wave + jj) & 3;
    unsigned char* dst = smem + (size_t)((owner * 3 + (jj - 1)) * MT) * 1024 + lane * 16;
#pragma unroll
    for (int i = 0; i < MT; ++i) *reinterpret_cast<floatx4*>(dst + i * 1024) = acc[jj][i];
  }
  __syncthreads();
  const int nch = n0 + 16 * wave + 4 * lk;
  floatx4 v[MT];
  size_t o[MT];   // element offset of the lane's four channels; rows past the image: the last pixel's
#pragma unroll
  for (int i = 0; i < MT; ++i) {
    v[i] = acc[0][i];
#pragma unroll
    for (int q = 0; q < 3; ++q) {
      const floatx4 t = *reinterpret_cast<const floatx4*>(smem + (size_t)((wave * 3 + q) * MT + i) * 1024 + lane * 16);
      v[i][0] += t[0]; v[i][1] += t[1]; v[i][2] += t[2]; v[i][3] += t[3];
    }
    const int m = 16 * i + li;
    o[i] = ((size_t)img * HW + (m < HW ? m : HW - 1)) * Ng + nch;
  }
  if (MODE == 0 && skip != nullptr) {
    // all the shortcut loads together, none of them guarded
    floatx4 sv[MT];
#pragma unroll
    for (int i = 0; i < MT; ++i) sv[i] = *reinterpret_cast<const floatx4*>(skip + o[i]);
#pragma unroll
    for (int i = 0; i < MT; ++i) {
      v[i][0] += sv[i][0]; v[i][1] += sv[i][1]; v[i][2] += sv[i][2]; v[i][3] += sv[i][3];
    }
  }
  double s1[4] = {0.0, 0.0, 0.0, 0.0}, s2[4] = {0.0, 0.0, 0.0, 0.0};
  if constexpr (MODE == 1 && EPI != 0) {
    // Eq. 6-7 from the layer's K-bit codes: the codes of the lane's four channels per pixel
    uint32_t cw[MT];
#pragma unroll
    for (int i = 0; i < MT; ++i)
      cw[i] = EPI == 4 ? (uint32_t) * reinterpret_cast<const uint16_t*>(codes + (o[i] >> 1))
                       : *reinterpret_cast<const uint32_t*>(codes + o[i]);
    const floatx4 st4 = *reinterpret_cast<const floatx4*>(stats + P_STEP * Ng + nch);
    const floatx4 bt4 = *reinterpret_cast<const floatx4*>(stats + P_BETA * Ng + nch);
    const floatx4 gm4 = *reinterpret_cast<const floatx4*>(stats + P_GAMMA * Ng + nch);
    const int4 fb4 = *reinterpret_cast<const int4*>(stats + P_FB * Ng + nch);
    const int32_t fbv[4] = {fb4.x, fb4.y, fb4.z, fb4.w};
    float ig[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) ig[r] = 1.0f / gm4[r];
#pragma unroll
    for (int i = 0; i < MT; ++i) {
      if (16 * i + li < HW) {
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const uint32_t code = (cw[i] >> (EPI * r)) & ((1u << EPI) - 1u);
          const int32_t q = (int32_t)code - (1 << (EPI - 1)) + fbv[r];
          const float a2t = st4[r] * ((float)q + 0.5f);        // Eq. 10
          const float da2 = a2t > 0.0f ? v[i][r] : 0.0f;       // Eq. 6
          const float a1t = (a2t - bt4[r]) * ig[r];            // inverse of Eq. 2
          s1[r] += (double)da2;
          s2[r] += (double)a1t * (double)da2;
        }
      }
    }
  }
#pragma unroll
  for (int i = 0; i < MT; ++i) {
    if (16 * i + li < HW) {
      *reinterpret_cast<floatx4*>(out + o[i]) = v[i];
      if (MODE == 0 && sums != nullptr) {
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          s1[r] += (double)v[i][r];
          s2[r] += (double)v[i][r] * (double)v[i][r];
        }
      }
    }
  }
  if (sums != nullptr && (MODE == 0 || EPI != 0)) {
    // row `img` of [N][2][Ng]: the two sums over the image, added over the 16 pixel lanes
#pragma unroll
    for (int r = 0; r < 4; ++r) {
#pragma unroll
      for (int d = 1; d < 16; d <<= 1) {
        s1[r] += __shfl_xor(s1[r], d, 64);
        s2[r] += __shfl_xor(s2[r], d, 64);
      }
    }
    if (li == 0) {
      double* row = sums + (size_t)img * 2 * Ng;
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        row[nch + r] = s1[r];
        row[Ng + nch + r] = s2[r];
      }
    }
  }
}

}  // namespace

bool bf16_gemm_supported(const ConvGeom& g, int mode) {
  const int Cg = mode == 0 ? g.Cin : g.Cout, Ng = mode == 0 ? g.Cout : g.Cin;
  if (Cg % BK != 0 || Ng % 64 != 0) return false;
  // 32-bit element offsets in the kernel
  const int64_t e_in = (int64_t)g.N * g.H * g.W * g.Cin, e_out = (int64_t)g.N * g.Ho * g.Wo * g.Cout;
  return e_in < ((int64_t)1 << 31) && e_out < ((int64_t)1 << 31);
}

int launch_image_bf16_epi(hipStream_t st, const ConvGeom& g, int K, const float* dy, const float* w, float* da3,
                          double* partial, const uint8_t* codes, const float* stats);

namespace {
// rows of sums the kernel leaves (one per block of 128 pixels), 0 if more than the partial buffers hold
int gemm_sum_rows(const ConvGeom& g, int mode) {
  const int64_t Mg = mode == 0 ? (int64_t)g.N * g.Ho * g.Wo : (int64_t)g.N * g.H * g.W;
  const int64_t nb = (Mg + BM - 1) / BM;
  return nb <= kMaxPartialBlocks ? (int)nb : 0;
}

template <int MODE, int EPI>
int launch_gemm(hipStream_t st, const ConvGeom& g, const float* in, const float* w, const float* skip, float* out,
                double* sums, const uint8_t* codes, const float* stats) {
  const int Ng = MODE == 0 ? g.Cout : g.Cin;
  const int64_t Mg = MODE == 0 ? (int64_t)g.N * g.Ho * g.Wo : (int64_t)g.N * g.H * g.W;
  const int64_t mblk = ((Mg + BM - 1) / BM + 7) / 8 * 8;  // whole XCD rounds; blocks past the end return
  // 128 output channels per block when that still leaves two blocks per compute unit
  // (not with the Eq. 6-7 epilogue: its registers would cost the wide tile a resident block per SIMD)
  const bool wide = EPI <= 1 && Ng % 128 == 0 && mblk * (Ng / 128) >= 512;
  const unsigned grid = (unsigned)(mblk * (Ng / (wide ? 128 : 64)));
  if (wide) gemm_bf16_kernel<MODE, 128, EPI><<<grid, kThreads, 0, st>>>(in, w, skip, out, g, sums, codes, stats);
  else gemm_bf16_kernel<MODE, 64, EPI><<<grid, kThreads, 0, st>>>(in, w, skip, out, g, sums, codes, stats);
  return hip_status();
}
}  // namespace

int launch_bf16_gemm(hipStream_t st, const ConvGeom& g, int mode, const float* in, const float* w, const float* skip,
                     float* out, double* sums, int* rows) {
  if (!bf16_gemm_supported(g, mode)) return ABL_ERR_SHAPE;
  if (rows != nullptr) *rows = 0;
  if (mode == 0) {
    const int nr = sums != nullptr && rows != nullptr ? gemm_sum_rows(g, 0) : 0;
    if (nr > 0) {
      *rows = nr;
      return launch_gemm<0, 1>(st, g, in, w, skip, out, sums, nullptr, nullptr);
    }
    return launch_gemm<0, 0>(st, g, in, w, skip, out, nullptr, nullptr, nullptr);
  }
  return launch_gemm<1, 0>(st, g, in, w, nullptr, out, nullptr, nullptr, nullptr);
}

int bf16_dgrad_reduce_rows(const ConvGeom& g) {
  if (image_bf16_supported(g, 1)) return g.N <= kMaxPartialBlocks ? g.N : 0;
  return bf16_gemm_supported(g, 1) ? gemm_sum_rows(g, 1) : 0;
}

int launch_bf16_dgrad_reduce(hipStream_t st, const ConvGeom& g, int K, const float* dy, const float* w,
                             const void* packed, const void* stats, float* da3, double* partial) {
  if ((K != 4 && K != 8) || bf16_dgrad_reduce_rows(g) == 0) return ABL_ERR_SHAPE;
  const uint8_t* codes = static_cast<const uint8_t*>(packed);
  const float* sp = static_cast<const float*>(stats);
  if (image_bf16_supported(g, 1)) return launch_image_bf16_epi(st, g, K, dy, w, da3, partial, codes, sp);
  if (K == 4) return launch_gemm<1, 4>(st, g, dy, w, nullptr, da3, partial, codes, sp);
  return launch_gemm<1, 8>(st, g, dy, w, nullptr, da3, partial, codes, sp);
}

namespace {
int image_mt(const ConvGeom& g) {
  const int tiles = (g.H * g.W + 15) / 16;
  return tiles <= 4 ? 4 : tiles <= 8 ? 8 : tiles <= 13 ? 13 : 0;
}
size_t image_lds_bytes(const ConvGeom& g, int mode) {
  const int Cg = mode == 0 ? g.Cin : g.Cout;
  const size_t patch = (size_t)(g.H + 2) * (g.W + 2) * (2 * Cg + 16);
  const size_t red = (size_t)12 * image_mt(g) * 1024;
  return patch > red ? patch : red;
}
}  // namespace

bool image_bf16_supported(const ConvGeom& g, int mode) {
  const int Cg = mode == 0 ? g.Cin : g.Cout, Ng = mode == 0 ? g.Cout : g.Cin;
  if (g.R != 3 || g.S != 3 || g.stride != 1 || g.pad != 1) return false;
  if (Cg < 32 || Cg > 1024 || (Cg & (Cg - 1)) != 0 || Ng % IMG_NB != 0) return false;
  if (image_mt(g) == 0 || g.H * g.W * g.W >= 65536) return false;
  if (image_lds_bytes(g, mode) > (size_t)160 * 1024) return false;
  const int64_t e_in = (int64_t)g.N * g.H * g.W * g.Cin, e_out = (int64_t)g.N * g.Ho * g.Wo * g.Cout;
  return e_in < ((int64_t)1 << 31) && e_out < ((int64_t)1 << 31);
}

namespace {
// more than the default 64 KB of LDS per block has to be asked for, once per kernel and device
// (the full 160 KB, so that the answer does not depend on the first shape seen)
int allow_full_lds_bf16(const void* kern) {
  static std::mutex mu;
  static std::set<std::pair<int, const void*>> done;
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) {
    (void)hipGetLastError();
    return ABL_ERR_HIP;
  }
  const std::pair<int, const void*> key(dev, kern);
  std::lock_guard<std::mutex> lock(mu);
  if (done.find(key) == done.end()) {
    if (hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024) != hipSuccess) {
      (void)hipGetLastError();
      return ABL_ERR_HIP;
    }
    done.insert(key);
  }
  return ABL_OK;
}

template <int MODE, int EPI>
int launch_image(hipStream_t st, const ConvGeom& g, const float* in, const float* w, const float* skip, float* out,
                 double* sums, const uint8_t* codes, const float* stats) {
  const int Ng = MODE == 0 ? g.Cout : g.Cin;
  const int mt = image_mt(g);
  const size_t lds = image_lds_bytes(g, MODE);
  const unsigned grid = (unsigned)((g.N + 7) / 8 * 8 * (Ng / IMG_NB));
  auto kern = mt == 4 ? image_bf16_kernel<MODE, 4, EPI> : mt == 8 ? image_bf16_kernel<MODE, 8, EPI>
                                                                   : image_bf16_kernel<MODE, 13, EPI>;
  if (int e = allow_full_lds_bf16(reinterpret_cast<const void*>(kern))) return e;
  kern<<<grid, kThreads, lds, st>>>(in, w, skip, out, sums, g, codes, stats);
  return hip_status();
}
}  // namespace

int launch_image_bf16(hipStream_t st, const ConvGeom& g, int mode, const float* in, const float* w,
                      const float* skip, float* out, double* sums) {
  if (!image_bf16_supported(g, mode)) return ABL_ERR_SHAPE;
  if (mode == 0) return launch_image<0, 0>(st, g, in, w, skip, out, sums, nullptr, nullptr);
  return launch_image<1, 0>(st, g, in, w, nullptr, out, nullptr, nullptr, nullptr);
}

int launch_image_bf16_epi(hipStream_t st, const ConvGeom& g, int K, const float* dy, const float* w, float* da3,
                          double* partial, const uint8_t* codes, const float* stats) {
  if (!image_bf16_supported(g, 1)) return ABL_ERR_SHAPE;
  if (K == 4) return launch_image<1, 4>(st, g, dy, w, nullptr, da3, partial, codes, stats);
  return launch_image<1, 8>(st, g, dy, w, nullptr, da3, partial, codes, stats);
}

}  // namespace abl
