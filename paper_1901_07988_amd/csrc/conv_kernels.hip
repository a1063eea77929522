// Convolution contractions of the approximate-activation layer for gfx950 (CDNA4):
//   conv_fwd     Eq. 4            y   = A3 (*) W            (+ identity shortcut, Sec. 3.4)
//   conv_dgrad   Eq. 5, 2nd half  dA3 = dy (*)^T W          (exact: does not touch activations)
//   conv_wgrad   Eq. 5, 1st half  dW  = A3~^T (*) dy        with A3~ = max(0, dequant(codes))
//                                 rebuilt in registers on the way to LDS (Eq. 10, Eq. 3)
//
// All three are implicit GEMMs on the fp32 matrix cores (v_mfma_f32_16x16x4_f32,
// 64-lane wavefronts): operand tiles are staged in LDS with the contraction index
// contiguous, so a lane fetches four consecutive k of its row with one ds_read_b128 and
// feeds four MFMAs from it.  NHWC activations, [R][S][Cin][Cout] weights.

#include "abl_internal.h"

// the fused forward evaluates Eq. 1-3 and Eq. 9 here: one rounded fp32 operation at a time
#pragma clang fp contract(off)

namespace abl {
namespace {


constexpr int kThreads = 256;


// ------------------------------------------------------------------------------------------
// Implicit GEMM  Out[p][n] = sum_{tap,c} A[p][(tap,c)] * B[(tap,c)][n]
//   MODE 0 (forward): p = (n,ho,wo), A = a3[n, ho*st+r-pad, wo*st+s-pad, c], c < Cin,
//                     B = W[r][s][c][n], n < Cout
//   MODE 1 (dgrad):   p = (n,h,w),   A = dy[n, (h+pad-r)/st, (w+pad-s)/st, c], c < Cout,
//                     (only where the division is exact and lands inside dy)
//                     B = W[r][s][n][c], n < Cin
// Block tile BM x BN, K chunk 16 channels of one filter tap, 4 waves of WM x WN.  The LDS
// tiles are double buffered: the global loads of chunk i+1 are in flight while chunk i is
// contracted, and one barrier per chunk separates "everyone has read buffer b" from
// "buffer b is overwritten".
// FUSE = K (4 or 8; forward of 1x1 stride-1 convolutions without padding only): `in` is the layer
// input x; BatchNorm, scale & bias and ReLU (Eq. 1-3) are applied to the A tile on its way into
// LDS and the blocks of the first output-channel block also write the K-bit codes (Eq. 9), so A3
// never reaches memory.  pack_pad: zero bytes after the last code.
// CLS (dgrad of a strided convolution): an input pixel (h, w) receives the taps with
// (h + pad - r) and (w + pad - s) divisible by the stride only - with stride 2, one, two, two or
// four of nine, and for a 1x1 filter three pixels in four receive nothing.  The pixels are
// therefore enumerated class by class ((h mod stride, w mod stride), each class's tiles after the
// previous one's), so that a block's pixels share their taps and the block contracts just those
// (all taps for every pixel, with the misses zeroed, is four times the matrix work).
template <int BM, int BN, int WM, int WN, int BK, int MODE, bool BF16, int FUSE, bool CLS = false>
__global__ __launch_bounds__(kThreads) void igemm_kernel(const float* __restrict__ in,
                                                         const float* __restrict__ wgt,
                                                         const float* skip, float* out, ConvGeom g,
                                                         const float* __restrict__ stats,
                                                         void* __restrict__ packed, int pack_pad) {
  constexpr int LDK = BK + 4;
  constexpr int KQ = BK / 4;                               // float4 per tile row
  constexpr int WAVES_N = BN / WN, WAVES_M = BM / WM;
  static_assert(WAVES_M * WAVES_N == 4, "four waves per block");
  constexpr int MT = WM / 16, NT = WN / 16;
  constexpr int ROWS = kThreads / KQ;                      // A rows staged per pass
  static_assert(BM % ROWS == 0, "A tile rows are staged ROWS at a time");
  constexpr int A_PASSES = BM / ROWS;
  constexpr int B_F4 = BK * BN / 4;                        // float4 per B chunk
  constexpr int B_PASSES = (B_F4 + kThreads - 1) / kThreads;

  extern __shared__ __attribute__((aligned(16))) float lds[];
  float* As0 = lds;                      // [2][BM * LDK]
  float* Bs0 = lds + 2 * BM * LDK;       // [2][BN * LDK]

  // A-operand tensor dims, output pixel grid, GEMM extents
  const int Hi = MODE == 0 ? g.H : g.Ho, Wi = MODE == 0 ? g.W : g.Wo;
  const int Hq = MODE == 0 ? g.Ho : g.H, Wq = MODE == 0 ? g.Wo : g.W;
  const int Cg = MODE == 0 ? g.Cin : g.Cout;
  const int Ng = MODE == 0 ? g.Cout : g.Cin;
  const int64_t Mg = (int64_t)g.N * Hq * Wq;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm0 = (wave / WAVES_N) * WM, wn0 = (wave % WAVES_N) * WN;
  // Workgroups go round-robin to the 8 XCDs, each with its own L2.  The blocks that share an
  // A tile (same pixel rows, different output channels) are therefore given ids 8 apart, so
  // they run on one XCD back to back and the tile comes from HBM once.
  const int nblk_n = (Ng + BN - 1) / BN;
  const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
  int64_t m0 = ((int64_t)(slot / nblk_n) * 8 + xcd) * BM;
  const int n0 = (slot % nblk_n) * BN;
  if (FUSE != 0 && blockIdx.x == 0 && (int)threadIdx.x < pack_pad)  // tail of the last 128-byte row
    static_cast<uint8_t*>(packed)[((int64_t)g.N * g.H * g.W * g.Cin * FUSE) / 8 + threadIdx.x] = 0;
  // CLS: the block's class (ph, pw), its grid Hc x Wc of pixels (ph + stride h', pw + stride w'),
  // their number Mc; m0 becomes the first of the block's pixels in the class's own numbering
  int ph = 0, pw = 0, Hc = 0, Wc = 0;
  int64_t Mc = 0;
  if constexpr (CLS) {
    const int st = g.stride;
    int64_t mt = m0 / BM;
    bool found = false;
    for (int c = 0; c < st * st && !found; ++c) {
      ph = c / st;
      pw = c - ph * st;
      Hc = g.H > ph ? (g.H - ph + st - 1) / st : 0;
      Wc = g.W > pw ? (g.W - pw + st - 1) / st : 0;
      Mc = (int64_t)g.N * Hc * Wc;
      const int64_t tiles = (Mc + BM - 1) / BM;
      if (mt < tiles) found = true;
      else mt -= tiles;
    }
    if (!found) return;
    m0 = mt * BM;
  } else {
    if (m0 >= Mg) return;
  }
  // pixel row `q` of the block's numbering -> (image, h, w) of the output pixel
  auto pixel_of = [&](int64_t q, int& n, int& hq, int& wq) __attribute__((always_inline)) {
    const int pp = (int)q;
    if constexpr (CLS) {
      const int wc = pp % Wc, t = pp / Wc;
      wq = wc * g.stride + pw;
      hq = (t % Hc) * g.stride + ph;
      n = t / Hc;
    } else {
      wq = pp % Wq;
      const int t = pp / Wq;
      hq = t % Hq;
      n = t / Hq;
    }
  };
  const int64_t Mrows = CLS ? Mc : Mg;

  // rows of the A tile this thread fetches (one float4 = 4 channels per row and pass)
  const int a_kq = tid % KQ, a_row = tid / KQ;
  int a_n[A_PASSES], a_h[A_PASSES], a_w[A_PASSES];
  bool a_ok[A_PASSES];
#pragma unroll
  for (int i = 0; i < A_PASSES; ++i) {
    const int64_t p = m0 + a_row + ROWS * i;
    a_ok[i] = p < Mrows;
    int hq, wq;
    pixel_of(a_ok[i] ? p : 0, a_n[i], hq, wq);
    if (MODE == 0) {
      a_h[i] = hq * g.stride - g.pad;
      a_w[i] = wq * g.stride - g.pad;
    } else {
      a_h[i] = hq + g.pad;
      a_w[i] = wq + g.pad;
    }
  }

  // The MFMA computes the transposed tile (first operand = weights): a lane ends up with four
  // consecutive output channels of one pixel, stored and read (shortcut) 16 bytes at a time.
  floatx4 acc[NT][MT];  // acc[j][i][r]: pixel wm0 + 16i + li, channel wn0 + 16j + 4lk + r
#pragma unroll
  for (int j = 0; j < NT; ++j)
#pragma unroll
    for (int i = 0; i < MT; ++i) acc[j][i] = floatx4{0.f, 0.f, 0.f, 0.f};

  const int cchunks = (Cg + BK - 1) / BK;
  const int taps = g.R * g.S;
  // CLS: the taps that reach this class (bit t of the mask), walked in ascending order
  uint64_t tap_mask = ~0ull;
  int ntaps = taps;
  if constexpr (CLS) {
    tap_mask = 0;
    ntaps = 0;
    for (int t = 0; t < taps; ++t) {
      const int r = t / g.S, sx = t - r * g.S;
      if ((ph + g.pad - r) % g.stride == 0 && (pw + g.pad - sx) % g.stride == 0) {
        tap_mask |= 1ull << t;
        ++ntaps;
      }
    }
  }
  auto next_tap = [&](int t) __attribute__((always_inline)) {  // first tap of the block at or after t
    if constexpr (CLS) {
      while (t < taps && !((tap_mask >> t) & 1ull)) ++t;
    }
    return t;
  };
  const int iters = ntaps * cchunks;
  float4 ra[A_PASSES], rb[B_PASSES];

  // Fetch state.  Chunks are fetched in order, so everything that depends on the filter tap
  // (bounds, the division for strided dgrad, the pixel offset) is recomputed only when the tap
  // changes; within a tap a chunk is `offset + channel`.
  int a_off[A_PASSES];  // element offset of channel 0 of this thread's pixel for the tap, -1 = zero
  int f_tap = next_tap(0), f_c0 = 0;
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
  // per-thread part of the weight address
  int b_thr[B_PASSES];
  bool b_ok[B_PASSES];
#pragma unroll
  for (int j = 0; j < B_PASSES; ++j) {
    const int idx = tid + kThreads * j;
    if (MODE == 0) {  // column n of four consecutive k rows
      const int n = n0 + idx % BN;
      b_ok[j] = idx < B_F4 && n < Ng;
      b_thr[j] = 4 * (idx / BN) * g.Cout + n;
    } else {          // row n, float4 along k
      const int nn = n0 + idx / KQ;
      b_ok[j] = idx < B_F4 && nn < Ng;
      b_thr[j] = nn * g.Cout + 4 * (idx % KQ);
    }
  }
  if (f_tap < taps) set_tap(f_tap);

  // per-channel constants of the 4 channels this thread stages (fused forward)
  float4 k_mean, k_rstd, k_gamma, k_beta, k_cq;
  int4 k_fb;
  int k_c = 0, k_chunk = 0;
  // bit i / j: pass i of the A tile / pass j of the B tile holds real data.  The zeroing of the
  // rest happens when the tile is staged, so that nothing waits for the loads before the MFMAs
  // of the current chunk.
  uint32_t a_live = 0, b_live = 0;
  auto fetch = [&]() __attribute__((always_inline)) {
    // every load is issued unconditionally (out-of-range lanes read element 0 and are zeroed
    // afterwards): no branches between the loads, so they are all in flight together
    const int c = f_c0 + 4 * a_kq;
#pragma unroll
    for (int i = 0; i < A_PASSES; ++i) {
      const bool ok = a_off[i] >= 0 && c < Cg;
      ra[i] = *reinterpret_cast<const float4*>(in + (ok ? a_off[i] + c : 0));
      a_live = ok ? (a_live | (1u << i)) : (a_live & ~(1u << i));
    }
    if (FUSE != 0) {
      k_mean = *reinterpret_cast<const float4*>(stats + P_MEAN * g.Cin + c);
      k_rstd = *reinterpret_cast<const float4*>(stats + P_RSTD * g.Cin + c);
      k_gamma = *reinterpret_cast<const float4*>(stats + P_GAMMA * g.Cin + c);
      k_beta = *reinterpret_cast<const float4*>(stats + P_BETA * g.Cin + c);
      k_cq = *reinterpret_cast<const float4*>(stats + P_CQ * g.Cin + c);
      k_fb = *reinterpret_cast<const int4*>(reinterpret_cast<const int32_t*>(stats) + P_FB * g.Cin + c);
      k_c = c;
      k_chunk = f_c0 / BK;
    }
    const float* wb = MODE == 0 ? wgt + ((int64_t)f_tap * g.Cin + f_c0) * g.Cout
                                : wgt + (int64_t)f_tap * g.Cin * g.Cout + f_c0;
#pragma unroll
    for (int j = 0; j < B_PASSES; ++j) {
      const int idx = tid + kThreads * j;
      if (MODE == 0) {
        const bool ok = b_ok[j] && f_c0 + 4 * (idx / BN) < Cg;
        const float* src = ok ? wb + b_thr[j] : wgt;
        const int64_t ld = ok ? g.Cout : 0;
        rb[j] = make_float4(src[0], src[ld], src[2 * ld], src[3 * ld]);
        b_live = ok ? (b_live | (1u << j)) : (b_live & ~(1u << j));
      } else {
        const bool ok = b_ok[j] && f_c0 + 4 * (idx % KQ) < Cg;
        rb[j] = *reinterpret_cast<const float4*>(ok ? wb + b_thr[j] : wgt);
        b_live = ok ? (b_live | (1u << j)) : (b_live & ~(1u << j));
      }
    }
    f_c0 += BK;
    if (f_c0 >= Cg) {
      f_c0 = 0;
      f_tap = next_tap(f_tap + 1);
      if (f_tap < taps) set_tap(f_tap);
    }
  };

  auto stage = [&](int buf) __attribute__((always_inline)) {
    float* As = As0 + buf * BM * LDK;
    float* Bs = Bs0 + buf * BN * LDK;
#pragma unroll
    for (int i = 0; i < A_PASSES; ++i) {
      float4 v = FUSE != 0 ? ra[i] : keep_if((a_live >> i) & 1u, ra[i]);
      if (FUSE != 0) {
        // a 1x1 convolution has one tap, so a_off[] still belongs to the chunk in ra[]
        const bool ok = a_off[i] >= 0;
        const float xs[4] = {v.x, v.y, v.z, v.w};
        const float mean[4] = {k_mean.x, k_mean.y, k_mean.z, k_mean.w};
        const float rstd[4] = {k_rstd.x, k_rstd.y, k_rstd.z, k_rstd.w};
        const float gm[4] = {k_gamma.x, k_gamma.y, k_gamma.z, k_gamma.w};
        const float bt[4] = {k_beta.x, k_beta.y, k_beta.z, k_beta.w};
        const float cq[4] = {k_cq.x, k_cq.y, k_cq.z, k_cq.w};
        const int32_t fb[4] = {k_fb.x, k_fb.y, k_fb.z, k_fb.w};
        float a2[4], a3[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const float d = xs[e] - mean[e];
          const float a1 = d * rstd[e];  // Eq. 1
          const float t = gm[e] * a1;
          a2[e] = t + bt[e];             // Eq. 2
          a3[e] = (ok && a2[e] > 0.0f) ? a2[e] : 0.0f;  // Eq. 3
        }
        v = make_float4(a3[0], a3[1], a3[2], a3[3]);
        // block-uniform: the output-channel blocks of a pixel tile take turns over the chunks in
        // quantizing, so that each has the same amount of vector work
        if (k_chunk % nblk_n == n0 / BN) {
          uint32_t word = 0;
#pragma unroll
          for (int e = 0; e < 4; ++e)
            word |= quant_code<(FUSE != 0 ? FUSE : 4)>(a2[e], cq[e], fb[e]) << ((FUSE != 0 ? FUSE : 4) * e);  // Eq. 9
          if (ok) {
            const int64_t e0 = (int64_t)a_off[i] + k_c;  // flat element index of the first of 4 codes
            if (FUSE == 4) reinterpret_cast<uint16_t*>(packed)[e0 >> 2] = (uint16_t)word;
            else reinterpret_cast<uint32_t*>(packed)[e0 >> 2] = word;
          }
        }
      }
      *reinterpret_cast<float4*>(&As[(a_row + ROWS * i) * LDK + 4 * a_kq]) = v;
    }
#pragma unroll
    for (int j = 0; j < B_PASSES; ++j) {
      const int idx = tid + kThreads * j;
      if (B_F4 % kThreads == 0 || idx < B_F4) {
        const float4 v = keep_if((b_live >> j) & 1u, rb[j]);
        if (MODE == 0) {
          *reinterpret_cast<float4*>(&Bs[(idx % BN) * LDK + 4 * (idx / BN)]) = v;
        } else {
          *reinterpret_cast<float4*>(&Bs[(idx / KQ) * LDK + 4 * (idx % KQ)]) = v;
        }
      }
    }
  };

  const int li = lane & 15, lk = lane >> 4;
  auto compute = [&](int cur) __attribute__((always_inline)) {
    const float* As = As0 + cur * BM * LDK;
    const float* Bs = Bs0 + cur * BN * LDK;
#pragma unroll
    for (int kg = 0; kg < BK / 16; ++kg) {
      float4 af[MT], bf[NT];
#pragma unroll
      for (int i = 0; i < MT; ++i)
        af[i] = *reinterpret_cast<const float4*>(&As[(wm0 + 16 * i + li) * LDK + 16 * kg + 4 * lk]);
#pragma unroll
      for (int j = 0; j < NT; ++j)
        bf[j] = *reinterpret_cast<const float4*>(&Bs[(wn0 + 16 * j + li) * LDK + 16 * kg + 4 * lk]);
      mma_k4<BF16, NT, MT>(bf, af, acc);
    }
  };
  // The loads of chunk i+1 are issued before chunk i is contracted and written to the other
  // LDS buffer afterwards; one barrier per chunk.
  if (iters > 0) {  // (a class that no tap reaches: its pixels are zeros)
    fetch();
    stage(0);
  }
  __syncthreads();
  for (int it = 0; it < iters; ++it) {
    const int cur = it & 1;
    if (it + 1 < iters) fetch();
    compute(cur);
    if (it + 1 < iters) stage(cur ^ 1);
    __syncthreads();
  }

  // epilogue: the lane holds channels n0 + wn0 + 16j + 4lk .. +3 of pixel m0 + wm0 + 16i + li.
  // Channel counts that are not a multiple of 4 take the element-wise path.
  const bool full = !CLS && m0 + BM <= Mg && n0 + BN <= Ng;
  const bool vec4 = (Ng & 3) == 0;
#pragma unroll
  for (int i = 0; i < MT; ++i) {
    int64_t p = m0 + wm0 + 16 * i + li;
    const bool p_ok = full || p < Mrows;
    if constexpr (CLS) {  // the class's numbering -> the pixel's row in the tensor
      int n, hq, wq;
      pixel_of(p_ok ? p : 0, n, hq, wq);
      p = ((int64_t)n * g.H + hq) * g.W + wq;
    }
    if (vec4) {
      bool ok[NT];
#pragma unroll
      for (int j = 0; j < NT; ++j) ok[j] = p_ok && (full || n0 + wn0 + 16 * j + 4 * lk < Ng);
      if (skip != nullptr) {
        float4 sv[NT];
#pragma unroll
        for (int j = 0; j < NT; ++j)
          sv[j] = *reinterpret_cast<const float4*>(skip + (ok[j] ? p * Ng + n0 + wn0 + 16 * j + 4 * lk : 0));
#pragma unroll
        for (int j = 0; j < NT; ++j) {
          acc[j][i][0] += sv[j].x; acc[j][i][1] += sv[j].y; acc[j][i][2] += sv[j].z; acc[j][i][3] += sv[j].w;
        }
      }
#pragma unroll
      for (int j = 0; j < NT; ++j)
        if (ok[j])
          *reinterpret_cast<float4*>(out + p * Ng + n0 + wn0 + 16 * j + 4 * lk) =
              make_float4(acc[j][i][0], acc[j][i][1], acc[j][i][2], acc[j][i][3]);
    } else {
#pragma unroll
      for (int j = 0; j < NT; ++j)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const int n = n0 + wn0 + 16 * j + 4 * lk + r;
          if (p_ok && n < Ng) {
            float v = acc[j][i][r];
            if (skip != nullptr) v += skip[p * Ng + n];
            out[p * Ng + n] = v;
          }
        }
    }
  }
}

// ------------------------------------------------------------------------------------------
// Weight gradient from the packed activation.  One block = one filter tap x TM input
// channels x TN output channels x one slice of the output pixels; a chunk of 64 pixels is
// staged in LDS (activations dequantized + ReLU'd to fp32 on the way in; K == 32: `packed` is
// an fp32 tensor: the conv input itself, or with relu32 the pre-ReLU activation A2 of exact
// storage).  Small tiles: each wave contracts 16 of the pixels into its own accumulators and
// the four waves are summed in a fixed order at the end.  QUAD (64-channel-wide tiles): each
// wave owns a quadrant of the tile and contracts all 64 pixels, so nothing is summed and the
// accumulators are a quarter of the size.  The summation order over pixels is fixed either
// way.  partial layout: [split][R][S][Cin][Cout].
template <int TM, int TN, int K, bool BF16, bool QUAD = false>
__global__ __launch_bounds__(kThreads, 3) void wgrad_kernel(const uint32_t* __restrict__ packed,
                                                         const float* __restrict__ stats,
                                                         const float* __restrict__ dy,
                                                         float* __restrict__ partial, ConvGeom g,
                                                         int chunks, int nsplit, int relu32) {
  constexpr int CH = 64;                                  // pixels per chunk
  constexpr int LDA = (TM % 32 == 0) ? TM + (TN == 128 ? 8 : 16) : TM;
  constexpr int LDB = (TN % 32 == 0) ? TN + (TN == 128 ? 8 : 16) : TN;
  constexpr int CPW = 32 / K;                             // codes per 32-bit word
  constexpr int GA = TM / CPW;                            // words per pixel of the A tile
  constexpr int A_PASSES = (CH * GA + kThreads - 1) / kThreads;
  constexpr int GB = TN / 4;                              // float4 per pixel of the B tile
  constexpr int B_PASSES = (CH * GB + kThreads - 1) / kThreads;
  // QUAD: the four waves own the quadrants of the tile and each contracts all 64 pixels;
  // otherwise every wave owns the whole tile and a quarter of the pixels.
  static_assert(!QUAD || (TM % 32 == 0 && TN % 32 == 0), "quadrants are whole 16x16 tiles");
  constexpr int MT = (QUAD ? TM / 2 : TM) / 16, NT = (QUAD ? TN / 2 : TN) / 16;
  constexpr int SM_AB = CH * (LDA + LDB), SM_RED = QUAD ? 0 : TM * TN;
  __shared__ __attribute__((aligned(16))) float sm[SM_AB > SM_RED ? SM_AB : SM_RED];
  float* As = sm;
  float* Bs = sm + CH * LDA;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int tiles_m = (g.Cin + TM - 1) / TM, tiles_n = (g.Cout + TN - 1) / TN;
  // ids 8 apart share an XCD (and its L2): each XCD takes an equal, contiguous run of the
  // (pixel slice, tile) pairs, so the tiles of one slice run there back to back
  const int ntiles = g.R * g.S * tiles_m * tiles_n;
  const int per_xcd = (nsplit * ntiles + 7) >> 3;
  const int item = (int)(blockIdx.x & 7) * per_xcd + (int)(blockIdx.x >> 3);
  if ((int)(blockIdx.x >> 3) >= per_xcd || item >= nsplit * ntiles) return;
  const int split_idx = item / ntiles;
  int t = item - split_idx * ntiles;
  const int tn = t % tiles_n; t /= tiles_n;
  const int tm = t % tiles_m; t /= tiles_m;
  const int tap = t;
  const int r = tap / g.S, s = tap - r * g.S;
  const int ci0 = tm * TM, co0 = tn * TN;
  const int64_t Mg = (int64_t)g.N * g.Ho * g.Wo;
  // The slices differ by at most one 64-pixel chunk, and the longer ones are spread evenly over the
  // slice indices: consecutive slices run on the same XCD (and a compute unit there gets one block
  // of each of them), so with the longer slices first the first XCD would finish last.
  const int64_t p_begin = ((int64_t)split_idx * chunks / nsplit) * CH;
  int64_t p_end = ((int64_t)(split_idx + 1) * chunks / nsplit) * CH;
  if (p_end > Mg) p_end = Mg;

  const int a_cg = tid % GA;  // the thread's channel group is the same in every pass
  floatx4 acc[MT][NT];
#pragma unroll
  for (int i = 0; i < MT; ++i)
#pragma unroll
    for (int j = 0; j < NT; ++j) acc[i][j] = floatx4{0.f, 0.f, 0.f, 0.f};

  const int li = lane & 15, lk = lane >> 4;
  uint32_t wa[A_PASSES];
  bool oka[A_PASSES];
  float4 rb[B_PASSES];
  int rem_st = 0;  // pixel rows of the chunk in rb[] that lie inside the slice (the rest is zeroed when
                   // the chunk is staged, so that nothing waits for the loads before the MFMAs)
  // global loads of one 64-pixel chunk into registers
  // Output-pixel position (n, ho, wo) of each A pass, advanced by one chunk per fetch without
  // divisions; all loads are unconditional (clamped address, zeroed afterwards).
  int a_wo[A_PASSES], a_ho[A_PASSES], a_n[A_PASSES];
#pragma unroll
  for (int i = 0; i < A_PASSES; ++i) {
    const int64_t p = p_begin + (tid + kThreads * i) / GA;
    const int pp = p < Mg ? (int)p : 0;
    a_wo[i] = pp % g.Wo;
    const int q = pp / g.Wo;
    a_ho[i] = q % g.Ho;
    a_n[i] = q / g.Ho;
  }
  // one chunk ahead = (adv_n images, adv_h rows, adv_w columns), carried without a loop
  const int adv_n = CH / (g.Ho * g.Wo), adv_r = CH - adv_n * (g.Ho * g.Wo);
  const int adv_h = adv_r / g.Wo, adv_w = adv_r - adv_h * g.Wo;
  const bool flat = g.R == 1 && g.S == 1 && g.stride == 1 && g.pad == 0;  // input pixel = output pixel
  const bool a_lane_ok = (ci0 + a_cg * CPW) < g.Cin;
  // Addresses advance by a constant per chunk: every tensor has fewer than 2^31 elements, so
  // element offsets are 32-bit, computed once per pass and stepped (64-bit multiplies per load
  // and chunk took as long to issue as half the chunk's MFMAs).
  // dy: one base per chunk (uniform, kept in scalar registers) plus a constant offset per pass -
  // no vector arithmetic per load
  unsigned b_off[B_PASSES];  // byte offset of this pass from the chunk's first pixel, channel 0
  int b_row[B_PASSES];       // its pixel row within the chunk, CH if the pass never loads
#pragma unroll
  for (int j = 0; j < B_PASSES; ++j) {
    const int idx = tid + kThreads * j;
    const int pl = idx / GB, c = co0 + 4 * (idx % GB);
    const bool lane_ok = (CH * GB % kThreads == 0 || idx < CH * GB) && c < g.Cout;
    b_row[j] = lane_ok ? pl : CH;
    b_off[j] = (unsigned)(pl * g.Cout + c) * 4u;
  }
  unsigned a_off[A_PASSES];  // 1x1 stride-1 layers (pixel p itself): byte offset of the pass's word from
                             // the word of the chunk's first pixel, channel 0
  int a_row[A_PASSES];
#pragma unroll
  for (int i = 0; i < A_PASSES; ++i) {
    const int idx = tid + kThreads * i;
    const bool lane_ok = a_lane_ok && (CH * GA % kThreads == 0 || idx < CH * GA);
    a_row[i] = lane_ok ? idx / GA : CH;
    a_off[i] = (unsigned)(((idx / GA) * g.Cin + ci0) / CPW + a_cg) * 4u;
  }
  auto fetch = [&](int64_t pc) __attribute__((always_inline)) {
    const int rem = (int)(p_end - pc < CH ? p_end - pc : CH);  // rows of this chunk inside the slice
    const char* pkc = reinterpret_cast<const char*>(flat ? packed + pc * g.Cin / CPW : packed);
#pragma unroll
    for (int i = 0; i < A_PASSES; ++i) {
      // branch-free (a 1x1 stride-1 layer reads pixel p itself): a branch here would make the
      // compiler wait for the loads already in flight
      const int hi = a_ho[i] * g.stride + r - g.pad, wi = a_wo[i] * g.stride + s - g.pad;
      const bool inside = flat || (hi >= 0 && hi < g.H && wi >= 0 && wi < g.W);
      oka[i] = a_row[i] < rem && inside;
      const unsigned word =
          flat ? a_off[i] : (unsigned)((((a_n[i] * g.H + hi) * g.W + wi) * g.Cin + ci0) / CPW + a_cg) * 4u;
      wa[i] = *reinterpret_cast<const uint32_t*>(pkc + (oka[i] ? word : 0u));
      // advance to the same slot of the next chunk
      a_wo[i] += adv_w;
      a_ho[i] += adv_h;
      a_n[i] += adv_n;
      if (a_wo[i] >= g.Wo) { a_wo[i] -= g.Wo; ++a_ho[i]; }
      if (a_ho[i] >= g.Ho) { a_ho[i] -= g.Ho; ++a_n[i]; }
    }
    const char* dyc = reinterpret_cast<const char*>(dy + pc * g.Cout);  // rows outside the slice read its first element
#pragma unroll
    for (int j = 0; j < B_PASSES; ++j) rb[j] = *reinterpret_cast<const float4*>(dyc + (b_row[j] < rem ? b_off[j] : 0u));
    rem_st = rem;
  };
  if (p_begin < p_end) fetch(p_begin);
  // (the first chunk's loads are in flight while these constants arrive)
  // per-thread dequantization constants: the thread's channel group is the same in every pass
  // Eq. 10 as one multiply per element: step * ((code - 2^(K-1) + fb) + 0.5) = step * (code + offh)
  // with offh = fb - 2^(K-1) + 0.5, which fp32 holds exactly while |fb| < 2^22 (any layer whose
  // codes are not all saturated), as it does code + offh: the product is rounded once, as in the
  // formula.
  float step[CPW], offh[CPW];
  if constexpr (CPW % 4 == 0) {  // the thread's channels are CPW consecutive ones: 16-byte loads, all in flight at once
    const bool ok = a_lane_ok;   // channel counts are multiples of 16 here, so a group is inside or outside as a whole
    const int c = ok ? ci0 + a_cg * CPW : 0;
    float4 st4[CPW / 4];
    int4 fb4[CPW / 4];
#pragma unroll
    for (int v = 0; v < CPW / 4; ++v) {
      st4[v] = *reinterpret_cast<const float4*>(stats + P_STEP * g.Cin + c + 4 * v);
      fb4[v] = *reinterpret_cast<const int4*>(reinterpret_cast<const int32_t*>(stats) + P_FB * g.Cin + c + 4 * v);
    }
#pragma unroll
    for (int v = 0; v < CPW / 4; ++v) {
      const float sv[4] = {st4[v].x, st4[v].y, st4[v].z, st4[v].w};
      const int32_t fv[4] = {fb4[v].x, fb4[v].y, fb4[v].z, fb4[v].w};
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        step[4 * v + e] = ok ? sv[e] : 0.f;
        offh[4 * v + e] = (float)((ok ? fv[e] : 0) - (1 << (K % 32 - 1))) + 0.5f;
      }
    }
  } else {
#pragma unroll
    for (int v = 0; v < CPW; ++v) {
      const int c = ci0 + a_cg * CPW + v;
      const bool ok = K != 32 && c < g.Cin;
      step[v] = ok ? stats[P_STEP * g.Cin + c] : 0.f;
      const int32_t fb = ok ? reinterpret_cast<const int32_t*>(stats)[P_FB * g.Cin + c] : 0;
      offh[v] = (float)(fb - (K == 32 ? 0 : (1 << (K % 32 - 1)))) + 0.5f;
    }
  }

  for (int64_t pc = p_begin; pc < p_end; pc += CH) {
    __syncthreads();  // previous chunk fully consumed
#pragma unroll
    for (int i = 0; i < A_PASSES; ++i) {
      const int idx = tid + kThreads * i;
      if (CH * GA % kThreads == 0 || idx < CH * GA) {
        float* dst = &As[(idx / GA) * LDA + a_cg * CPW];
        float vals[CPW];
        // Vector instructions and matrix instructions do not overlap on a SIMD, so every one here
        // is matrix time lost: the codes are spread to one per byte (a byte converts to float in
        // one instruction), and the ReLU and the zeroing of pixels outside the slice or the image
        // are one median: med3(x, 0, inf) = max(x, 0), med3(x, 0, 0) = 0.
        const float lim = oka[i] ? __builtin_inff() : 0.f;
        uint32_t by[K == 4 ? 2 : 1];  // K == 4: codes 0,2,4,6 / 1,3,5,7 of the word, one per byte
        if constexpr (K == 4) {
          by[0] = wa[i] & 0x0F0F0F0Fu;
          by[1] = (wa[i] >> 4) & 0x0F0F0F0Fu;
        } else {
          by[0] = wa[i];
        }
#pragma unroll
        for (int v = 0; v < CPW; ++v) {
          if constexpr (K == 32) {
            const float f = __uint_as_float(wa[i]);
            vals[v] = (oka[i] && !(relu32 != 0 && f < 0.f)) ? f : 0.f;
          } else {
            const uint32_t src = K == 4 ? by[v & 1] : by[0];
            const int b = K == 4 ? v >> 1 : v;
            const float code = (float)((src >> (8 * b)) & 0xFFu);
            const float a2t = step[v] * (code + offh[v]);         // Eq. 10
            vals[v] = __builtin_amdgcn_fmed3f(a2t, 0.f, lim);     // Eq. 3
          }
        }
        // 16-byte writes: element-wise ones would land 64 lanes on four LDS banks
        if constexpr (CPW % 4 == 0) {
#pragma unroll
          for (int v = 0; v < CPW; v += 4)
            *reinterpret_cast<float4*>(dst + v) = make_float4(vals[v], vals[v + 1], vals[v + 2], vals[v + 3]);
        } else {
#pragma unroll
          for (int v = 0; v < CPW; ++v) dst[v] = vals[v];
        }
      }
    }
    if (rem_st == CH && co0 + TN <= g.Cout) {  // block-uniform: every pass holds real data
#pragma unroll
      for (int j = 0; j < B_PASSES; ++j) {
        const int idx = tid + kThreads * j;
        if (idx < CH * GB) *reinterpret_cast<float4*>(&Bs[(idx / GB) * LDB + 4 * (idx % GB)]) = rb[j];
      }
    } else {
#pragma unroll
      for (int j = 0; j < B_PASSES; ++j) {
        const int idx = tid + kThreads * j;
        if (idx < CH * GB)
          *reinterpret_cast<float4*>(&Bs[(idx / GB) * LDB + 4 * (idx % GB)]) = keep_if(b_row[j] < rem_st, rb[j]);
      }
    }
    __syncthreads();
    if (pc + CH < p_end) fetch(pc + CH);  // in flight while this chunk is contracted
    // wave w contracts pixels [16w, 16w+16) of the chunk.  Component e of the operand vectors is
    // pixel 4e + lk (fp32: k-step e, lane group = k) or 4lk + e (bf16: lane group owns 4 k).
    const int am0 = QUAD ? (wave >> 1) * (TM / 2) : 0, bn0 = QUAD ? (wave & 1) * (TN / 2) : 0;
    if constexpr (BF16 && QUAD) {
      // bf16 operands on the 32-deep matrix instruction: a lane supplies eight consecutive pixels
      // (k = 8 lk .. 8 lk + 7 of each half of the chunk), rounded by the hardware's packed convert
#pragma unroll
      for (int kh = 0; kh < 2; ++kh) {
        const int r0 = 32 * kh + 8 * lk;
        bf16x8_t a8[MT], b8[NT];
#pragma unroll
        for (int i = 0; i < MT; ++i) {
          float v[8];
#pragma unroll
          for (int e = 0; e < 8; ++e) v[e] = As[(r0 + e) * LDA + am0 + 16 * i + li];
          a8[i] = to_bf16x8(v);
        }
#pragma unroll
        for (int j = 0; j < NT; ++j) {
          float v[8];
#pragma unroll
          for (int e = 0; e < 8; ++e) v[e] = Bs[(r0 + e) * LDB + bn0 + 16 * j + li];
          b8[j] = to_bf16x8(v);
        }
#pragma unroll
        for (int i = 0; i < MT; ++i)
#pragma unroll
          for (int j = 0; j < NT; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a8[i], b8[j], acc[i][j], 0, 0, 0);
      }
    } else
#pragma unroll
    for (int kq = 0; kq < (QUAD ? 4 : 1); ++kq) {
      float4 af[MT], bf[NT];
      int row[4];
#pragma unroll
      for (int e = 0; e < 4; ++e) row[e] = 16 * (QUAD ? kq : wave) + (BF16 ? 4 * lk + e : 4 * e + lk);
#pragma unroll
      for (int i = 0; i < MT; ++i)
        af[i] = make_float4(As[row[0] * LDA + am0 + 16 * i + li], As[row[1] * LDA + am0 + 16 * i + li],
                            As[row[2] * LDA + am0 + 16 * i + li], As[row[3] * LDA + am0 + 16 * i + li]);
#pragma unroll
      for (int j = 0; j < NT; ++j)
        bf[j] = make_float4(Bs[row[0] * LDB + bn0 + 16 * j + li], Bs[row[1] * LDB + bn0 + 16 * j + li],
                            Bs[row[2] * LDB + bn0 + 16 * j + li], Bs[row[3] * LDB + bn0 + 16 * j + li]);
      mma_k4<BF16, MT, NT>(af, bf, acc);
    }
  }

  float* dst = partial + (int64_t)split_idx * g.R * g.S * g.Cin * g.Cout;
  if constexpr (QUAD) {  // each wave writes its own quadrant: nothing to sum
    const int am0 = (wave >> 1) * (TM / 2), bn0 = (wave & 1) * (TN / 2);
#pragma unroll
    for (int i = 0; i < MT; ++i)
#pragma unroll
      for (int j = 0; j < NT; ++j)
#pragma unroll
        for (int rr = 0; rr < 4; ++rr) {
          const int ci = ci0 + am0 + 16 * i + 4 * lk + rr, co = co0 + bn0 + 16 * j + li;
          if (ci < g.Cin && co < g.Cout) dst[((int64_t)tap * g.Cin + ci) * g.Cout + co] = acc[i][j][rr];
        }
    return;
  }

  // sum the four waves in order 0,1,2,3 through LDS, then write the tile
  for (int w = 0; w < 4; ++w) {
    __syncthreads();
    if (wave == w) {
#pragma unroll
      for (int i = 0; i < MT; ++i)
#pragma unroll
        for (int j = 0; j < NT; ++j)
#pragma unroll
          for (int rr = 0; rr < 4; ++rr) {
            float* d = &sm[(16 * i + 4 * lk + rr) * TN + 16 * j + li];
            *d = (w == 0) ? acc[i][j][rr] : *d + acc[i][j][rr];
          }
    }
  }
  __syncthreads();
  for (int idx = tid; idx < TM * TN / 4; idx += kThreads) {
    const int i = idx / (TN / 4), j = 4 * (idx % (TN / 4));
    const int ci = ci0 + i, co = co0 + j;
    if (ci < g.Cin && co < g.Cout)
      *reinterpret_cast<float4*>(dst + ((int64_t)tap * g.Cin + ci) * g.Cout + co) =
          *reinterpret_cast<const float4*>(&sm[i * TN + j]);
  }
}

// dW[i] = sum over the split-K partials, fixed order: 64 outputs x 4 interleaved parts per block.
__global__ __launch_bounds__(kThreads) void wgrad_reduce_kernel(const float* __restrict__ partial, int split,
                                                                int64_t n, float* __restrict__ dw) {
  __shared__ float sm[4][64];
  const int lane = threadIdx.x & 63, part = threadIdx.x >> 6;
  const int64_t i = (int64_t)blockIdx.x * 64 + lane;
  float s = 0.f;
  if (i < n) {
#pragma unroll 8
    for (int k = part; k < split; k += 4) s += partial[(int64_t)k * n + i];
  }
  sm[part][lane] = s;
  __syncthreads();
  if (part == 0 && i < n) dw[i] = ((sm[0][lane] + sm[1][lane]) + sm[2][lane]) + sm[3][lane];
}

// ------------------------------------------------------------------------------------------
// Fallbacks for channel counts that are not multiples of 16: one thread per output element.
__global__ __launch_bounds__(kThreads) void naive_fwd_kernel(const float* __restrict__ a3,
                                                             const float* __restrict__ w, const float* skip,
                                                             float* out, ConvGeom g) {
  const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
  const int64_t total = (int64_t)g.N * g.Ho * g.Wo * g.Cout;
  if (i >= total) return;
  const int co = (int)(i % g.Cout);
  int64_t p = i / g.Cout;
  const int wo = (int)(p % g.Wo); p /= g.Wo;
  const int ho = (int)(p % g.Ho);
  const int n = (int)(p / g.Ho);
  float acc = 0.f;
  for (int r = 0; r < g.R; ++r) {
    const int h = ho * g.stride + r - g.pad;
    if (h < 0 || h >= g.H) continue;
    for (int s = 0; s < g.S; ++s) {
      const int x = wo * g.stride + s - g.pad;
      if (x < 0 || x >= g.W) continue;
      const float* ap = a3 + (((int64_t)n * g.H + h) * g.W + x) * g.Cin;
      const float* wp = w + ((int64_t)(r * g.S + s) * g.Cin) * g.Cout + co;
      for (int ci = 0; ci < g.Cin; ++ci) acc += ap[ci] * wp[(int64_t)ci * g.Cout];
    }
  }
  if (skip != nullptr) acc += skip[i];
  out[i] = acc;
}

__global__ __launch_bounds__(kThreads) void naive_dgrad_kernel(const float* __restrict__ dy,
                                                               const float* __restrict__ w,
                                                               float* __restrict__ da3, ConvGeom g) {
  const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
  const int64_t total = (int64_t)g.N * g.H * g.W * g.Cin;
  if (i >= total) return;
  const int ci = (int)(i % g.Cin);
  int64_t p = i / g.Cin;
  const int x = (int)(p % g.W); p /= g.W;
  const int h = (int)(p % g.H);
  const int n = (int)(p / g.H);
  float acc = 0.f;
  for (int r = 0; r < g.R; ++r) {
    const int hh = h + g.pad - r;
    if (hh < 0 || hh % g.stride) continue;
    const int ho = hh / g.stride;
    if (ho >= g.Ho) continue;
    for (int s = 0; s < g.S; ++s) {
      const int ww = x + g.pad - s;
      if (ww < 0 || ww % g.stride) continue;
      const int wo = ww / g.stride;
      if (wo >= g.Wo) continue;
      const float* gp = dy + (((int64_t)n * g.Ho + ho) * g.Wo + wo) * g.Cout;
      const float* wp = w + ((int64_t)(r * g.S + s) * g.Cin + ci) * g.Cout;
      for (int co = 0; co < g.Cout; ++co) acc += gp[co] * wp[co];
    }
  }
  da3[i] = acc;
}

// One block per dW element; the 256 threads stride over the output pixels, fixed-order tree.
template <int K>
__global__ __launch_bounds__(kThreads) void naive_wgrad_kernel(const uint8_t* __restrict__ packed,
                                                               const float* __restrict__ stats,
                                                               const float* __restrict__ dy,
                                                               float* __restrict__ dw, ConvGeom g, int relu32) {
  __shared__ float red[kThreads];
  int t = blockIdx.x;
  const int co = t % g.Cout; t /= g.Cout;
  const int ci = t % g.Cin; t /= g.Cin;
  const int s = t % g.S, r = t / g.S;
  const float step = K == 32 ? 0.f : stats[P_STEP * g.Cin + ci];
  const int32_t fb = K == 32 ? 0 : reinterpret_cast<const int32_t*>(stats)[P_FB * g.Cin + ci];
  const int64_t Mg = (int64_t)g.N * g.Ho * g.Wo;
  float acc = 0.f;
  for (int64_t p = threadIdx.x; p < Mg; p += kThreads) {
    const int wo = (int)(p % g.Wo);
    const int64_t q = p / g.Wo;
    const int ho = (int)(q % g.Ho), n = (int)(q / g.Ho);
    const int hi = ho * g.stride + r - g.pad, wi = wo * g.stride + s - g.pad;
    if (hi < 0 || hi >= g.H || wi < 0 || wi >= g.W) continue;
    const int64_t e = (((int64_t)n * g.H + hi) * g.W + wi) * g.Cin + ci;
    if (K == 32) {
      const float f = reinterpret_cast<const float*>(packed)[e];
      if (!(relu32 != 0 && f < 0.f)) acc += f * dy[p * g.Cout + co];
      continue;
    }
    uint32_t code;
    if (K == 4) code = (packed[e >> 1] >> ((e & 1) * 4)) & 15u;
    else code = packed[e];
    const int32_t j = (int32_t)code - (K == 32 ? 0 : (1 << (K - 1))) + fb;
    const float a2t = step * ((float)j + 0.5f);
    if (a2t > 0.f) acc += a2t * dy[p * g.Cout + co];
  }
  red[threadIdx.x] = acc;
  __syncthreads();
  for (int h = kThreads / 2; h >= 1; h >>= 1) {
    if ((int)threadIdx.x < h) red[threadIdx.x] += red[threadIdx.x + h];
    __syncthreads();
  }
  if (threadIdx.x == 0) dw[blockIdx.x] = red[0];
}

inline bool mfma_ok(const ConvGeom& g) { return g.Cin % 16 == 0 && g.Cout % 16 == 0; }

// Tile choice, from timing the candidates on 1x1 and 3x3 layers at 56x56 and 14x14.  Blocks
// of one wave per SIMD spend much of their time at the two barriers of a chunk, so the tile
// that lets most blocks share a compute unit usually wins over the one with the fewest
// operand re-reads: 64x64 with 32-channel chunks (four blocks per unit) when the grid has
// at least two thousand of them, 128x64 (two per unit) below that; a contraction of at most
// 64 channels has too few chunks to fill the double buffer and takes 16-channel chunks.  With
// the normalize/quantize prologue the per-element work of staging is repeated by every block
// along the output channels, so that variant prefers 128 output channels per block.
template <int MODE, int FUSE>
int launch_igemm(hipStream_t st, const ConvGeom& g, bool bf16, const float* in, const float* w,
                 const float* skip, float* out, const float* stats, void* packed) {
  const int64_t raw = FUSE != 0 ? ((int64_t)g.N * g.H * g.W * g.Cin * FUSE + 7) / 8 : 0;
  const int pack_pad = (int)((raw + 127) / 128 * 128 - raw);
  const int Ng = MODE == 0 ? g.Cout : g.Cin;
  const int64_t Mg = MODE == 0 ? (int64_t)g.N * g.Ho * g.Wo : (int64_t)g.N * g.H * g.W;
  // dgrad of a strided convolution: pixel tiles per class of (h mod stride, w mod stride)
  constexpr bool CAN_CLS = MODE == 1 && FUSE == 0;
  const bool cls = CAN_CLS && g.stride > 1;
  auto mtiles = [&](int bm) __attribute__((always_inline)) {
    if (!cls) return (Mg + bm - 1) / bm;
    int64_t t = 0;
    for (int c = 0; c < g.stride * g.stride; ++c) {
      const int ph = c / g.stride, pw = c % g.stride;
      const int64_t hc = g.H > ph ? (g.H - ph + g.stride - 1) / g.stride : 0;
      const int64_t wc = g.W > pw ? (g.W - pw + g.stride - 1) / g.stride : 0;
      t += (g.N * hc * wc + bm - 1) / bm;
    }
    return t;
  };
  auto blocks = [&](int bm, int bn) __attribute__((always_inline)) { return mtiles(bm) * ((Ng + bn - 1) / bn); };
#define ABL_IGEMM(BM_, BN_, WM_, WN_, BK_)                                                     \
  do {                                                                                         \
    const int64_t mb8 = (mtiles(BM_) + 7) / 8 * 8;                                            \
    dim3 grid((unsigned)(mb8 * ((Ng + BN_ - 1) / BN_)));                                      \
    constexpr unsigned lds = 2u * (BM_ + BN_) * (BK_ + 4) * sizeof(float);                    \
    auto kern = cls ? (bf16 ? igemm_kernel<BM_, BN_, WM_, WN_, BK_, MODE, true, FUSE, CAN_CLS> \
                            : igemm_kernel<BM_, BN_, WM_, WN_, BK_, MODE, false, FUSE, CAN_CLS>) \
                    : (bf16 ? igemm_kernel<BM_, BN_, WM_, WN_, BK_, MODE, true, FUSE>          \
                            : igemm_kernel<BM_, BN_, WM_, WN_, BK_, MODE, false, FUSE>);       \
    if (lds > 64 * 1024 &&                                                                     \
        hipFuncSetAttribute(reinterpret_cast<const void*>(kern),                               \
                            hipFuncAttributeMaxDynamicSharedMemorySize, lds) != hipSuccess)    \
      return ABL_ERR_HIP;                                                                                          \
    kern<<<grid, kThreads, lds, st>>>(in, w, skip, out, g, stats, packed, pack_pad);           \
  } while (0)
  const int Cg = MODE == 0 ? g.Cin : g.Cout;
  const bool deep = (int64_t)Cg * g.R * g.S > 64;
  if (Ng > 32) {
    if (FUSE != 0 && Ng > 64) {
      if (Cg % 32 != 0) ABL_IGEMM(128, 128, 64, 64, 16);
      else if (blocks(128, 128) >= 512) ABL_IGEMM(128, 128, 64, 64, 32);
      else ABL_IGEMM(64, 128, 32, 64, 32);
    } else if (Cg % 32 != 0 || !deep) {
      if (Ng > 64 && blocks(128, 64) >= 1024) ABL_IGEMM(128, 64, 64, 32, 16);
      else ABL_IGEMM(64, 64, 32, 32, 16);
    } else if (blocks(64, 64) >= 2048 || blocks(128, 64) < 256) {
      ABL_IGEMM(64, 64, 32, 32, 32);
    } else {
      ABL_IGEMM(128, 64, 64, 32, 32);
    }
  } else if (Cg % 32 == 0) {  // 32-channel chunks: whole 128-byte lines per pixel row
    if (Ng > 16) ABL_IGEMM(256, 32, 64, 32, 32);
    else ABL_IGEMM(256, 16, 64, 16, 32);
  } else {
    if (Ng > 16) ABL_IGEMM(256, 32, 64, 32, 16);
    else ABL_IGEMM(256, 16, 64, 16, 16);
  }
#undef ABL_IGEMM
  return hip_status();
}

struct WgradPlan {
  int tm, tn, tiles, split, chunks;
};

WgradPlan wgrad_plan(const ConvGeom& g) {
  WgradPlan p;
  p.tm = g.Cin >= 64 ? 64 : (g.Cin >= 32 ? 32 : 16);
  p.tn = g.Cout >= 64 ? 64 : (g.Cout >= 32 ? 32 : 16);
  // 128 output channels per block where they divide evenly: the dequantization of the
  // activation chunk is shared by twice as many MFMAs
  if (p.tm == 64 && g.Cout % 128 == 0) p.tn = 128;
  p.tiles = g.R * g.S * ((g.Cin + p.tm - 1) / p.tm) * ((g.Cout + p.tn - 1) / p.tn);
  const int64_t Mg = (int64_t)g.N * g.Ho * g.Wo;
  const int64_t chunks = (Mg + 63) / 64;
  // three blocks share a compute unit: about 768 blocks in all (fewer only when the layer has
  // fewer than two chunks per block to give)
  int64_t split = 768 / p.tiles;
  if (split > 256) split = 256;
  if (split > chunks / 2) split = chunks / 2;
  if (split < 1) split = 1;
  p.chunks = (int)chunks;
  p.split = (int)split;
  return p;
}

}  // namespace

// Shapes for which the all-taps kernel is used instead of the per-tap one.
inline bool use_halo_wgrad(const ConvGeom& g) { return g.Cin <= 64 && halo_wgrad_partial_bytes(g) != 0; }

size_t wgrad_partial_bytes(const abl_shape& s) {
  const ConvGeom g = geom_of(s);
  if (!mfma_ok(g)) return 256;
  if (use_halo_wgrad(g)) {  // the per-tap kernel is still used when the activation is fp32
    const WgradPlan p = wgrad_plan(g);
    const size_t a = halo_wgrad_partial_bytes(g);
    const size_t b = ((size_t)p.split * g.R * g.S * g.Cin * g.Cout * sizeof(float) + 255) / 256 * 256;
    return a > b ? a : b;
  }
  const WgradPlan p = wgrad_plan(g);
  const size_t n = (size_t)g.R * g.S * g.Cin * g.Cout * sizeof(float);
  int img = image_wgrad_copies(g, 4);   // the register-resident kernels' copies (same count for K = 8)
  const int pw = rows_wgrad_copies(g, 4, false);
  if (pw > img) img = pw;
  return ((size_t)(p.split > img ? p.split : img) * n + 255) / 256 * 256;
}

int launch_conv_fwd(hipStream_t st, const abl_shape& s, bool bf16, const float* a3, const float* w,
                    const float* skip, float* y, double* sums, int* rows) {
  const ConvGeom g = geom_of(s);
  if (rows != nullptr) *rows = 0;
  if (!mfma_ok(g)) {
    const int64_t total = (int64_t)g.N * g.Ho * g.Wo * g.Cout;
    naive_fwd_kernel<<<(unsigned)((total + kThreads - 1) / kThreads), kThreads, 0, st>>>(a3, w, skip, y, g);
    return hip_status();
  }
  // bf16 operands: the 32-deep bf16 matrix instruction with bf16 tiles in LDS
  if (bf16 && image_bf16_supported(g, 0)) {
    const bool want = sums != nullptr && rows != nullptr && g.N <= kMaxPartialBlocks;
    if (want) *rows = g.N;
    return launch_image_bf16(st, g, 0, a3, w, skip, y, want ? sums : nullptr);
  }
  if (bf16 && bf16_gemm_supported(g, 0)) return launch_bf16_gemm(st, g, 0, a3, w, skip, y, sums, rows);
  // small images: the whole image resident in LDS, one row of sums per image
  if (!bf16 && image_f32_supported(g, 0)) {
    const bool want = sums != nullptr && rows != nullptr;
    if (want) *rows = g.N;
    return launch_image_f32(st, g, 0, a3, w, skip, y, want ? sums : nullptr);
  }
  if (halo_conv_supported(g)) {
    const int tiles = sums != nullptr && rows != nullptr ? halo_tile_count(g, 0) : 0;
    const bool want = tiles > 0 && tiles <= kMaxPartialBlocks;
    if (want) *rows = tiles;
    return launch_halo_conv(st, g, 0, bf16, a3, w, skip, y, want ? sums : nullptr);
  }
  // 1x1 layers that give about one block per compute unit: the output tile in registers, one row of sums
  // per row block
  if (const int nrb = !bf16 ? rows_f32_blocks(g, 0) : 0) {
    const bool want = sums != nullptr && rows != nullptr;
    if (want) *rows = nrb;
    return launch_rows_f32(st, g, 0, a3, w, skip, y, want ? sums : nullptr);
  }
  if (pointwise_supported(g, 0))
    return launch_pointwise_conv(st, g, 0, bf16, a3, w, skip, y, rows != nullptr ? sums : nullptr, rows);
  return launch_igemm<0, 0>(st, g, bf16, a3, w, skip, y, nullptr, nullptr);
}

bool igemm_fused_supported(const abl_shape& s) {
  const ConvGeom g = geom_of(s);
  return mfma_ok(g) && g.R == 1 && g.S == 1 && g.stride == 1 && g.pad == 0 &&
         (int64_t)g.N * g.H * g.W * g.Cin < (1ll << 31);
}

int launch_conv_fwd_fused(hipStream_t st, const abl_shape& s, int K, bool bf16, const float* x, const void* stats,
                          const float* w, const float* skip, float* y, void* packed, double* sums, int* rows) {
  if (!igemm_fused_supported(s)) return ABL_ERR_SHAPE;
  const ConvGeom g = geom_of(s);
  const float* sp = static_cast<const float*>(stats);
  if (rows != nullptr) *rows = 0;
  if (pointwise_supported(g, 0))
    return launch_pointwise_fwd_fused(st, g, K, bf16, x, sp, w, skip, y, packed, rows != nullptr ? sums : nullptr,
                                      rows);
  if (K == 4) return launch_igemm<0, 4>(st, g, bf16, x, w, skip, y, sp, packed);
  return launch_igemm<0, 8>(st, g, bf16, x, w, skip, y, sp, packed);
}

int launch_conv_dgrad(hipStream_t st, const abl_shape& s, bool bf16, const float* dy, const float* w,
                      float* da3) {
  const ConvGeom g = geom_of(s);
  if (!mfma_ok(g)) {
    const int64_t total = (int64_t)g.N * g.H * g.W * g.Cin;
    naive_dgrad_kernel<<<(unsigned)((total + kThreads - 1) / kThreads), kThreads, 0, st>>>(dy, w, da3, g);
    return hip_status();
  }
  if (bf16 && image_bf16_supported(g, 1)) return launch_image_bf16(st, g, 1, dy, w, nullptr, da3, nullptr);
  if (bf16 && bf16_gemm_supported(g, 1)) return launch_bf16_gemm(st, g, 1, dy, w, nullptr, da3);
  if (!bf16 && image_f32_supported(g, 1)) return launch_image_f32(st, g, 1, dy, w, nullptr, da3, nullptr);
  if (halo_conv_supported(g)) return launch_halo_conv(st, g, 1, bf16, dy, w, nullptr, da3);
  if (!bf16 && rows_f32_blocks(g, 1) > 0) return launch_rows_f32(st, g, 1, dy, w, nullptr, da3, nullptr);
  if (pointwise_supported(g, 1)) return launch_pointwise_conv(st, g, 1, bf16, dy, w, nullptr, da3);
  return launch_igemm<1, 0>(st, g, bf16, dy, w, nullptr, da3, nullptr, nullptr);
}

template <int TM, int TN>
static void launch_wgrad_tile(hipStream_t st, const ConvGeom& g, const WgradPlan& p, int K, bool bf16,
                              const void* packed, const float* stats, const float* dy, float* dst, int relu32) {
  dim3 grid((unsigned)(((int64_t)p.split * p.tiles + 7) / 8 * 8));
  const uint32_t* pk = static_cast<const uint32_t*>(packed);
  constexpr bool Q = TM == 64 && TN >= 64;
  auto kern = K == 4 ? (bf16 ? wgrad_kernel<TM, TN, 4, true, Q> : wgrad_kernel<TM, TN, 4, false, Q>)
            : K == 8 ? (bf16 ? wgrad_kernel<TM, TN, 8, true, Q> : wgrad_kernel<TM, TN, 8, false, Q>)
                     : (bf16 ? wgrad_kernel<TM, TN, 32, true, Q> : wgrad_kernel<TM, TN, 32, false, Q>);
  kern<<<grid, kThreads, 0, st>>>(pk, stats, dy, dst, g, p.chunks, p.split, relu32);
}

int launch_conv_wgrad_packed(hipStream_t st, const abl_shape& s, int K, bool bf16, const void* packed,
                             const void* stats, const float* dy, void* scratch, float* dw, bool relu32,
                             DwSum* defer) {
  const int r32 = relu32 ? 1 : 0;
  if (defer != nullptr) defer->copies = 0;
  const ConvGeom g = geom_of(s);
  const float* sp = static_cast<const float*>(stats);
  if (!mfma_ok(g)) {
    const unsigned blocks = (unsigned)(g.R * g.S * g.Cin * g.Cout);
    const uint8_t* pk = static_cast<const uint8_t*>(packed);
    if (K == 4) naive_wgrad_kernel<4><<<blocks, kThreads, 0, st>>>(pk, sp, dy, dw, g, 0);
    else if (K == 8) naive_wgrad_kernel<8><<<blocks, kThreads, 0, st>>>(pk, sp, dy, dw, g, 0);
    else naive_wgrad_kernel<32><<<blocks, kThreads, 0, st>>>(pk, sp, dy, dw, g, r32);
    return hip_status();
  }
  if (K != 32 && use_halo_wgrad(g)) return launch_halo_wgrad(st, g, K, bf16, packed, sp, dy, scratch, dw);
  // 3x3 layers on 14-pixel-wide images: the image-resident kernel, one copy of dW per share of the images
  if (const int copies = !relu32 ? image_wgrad_copies(g, K) : 0) {
    float* dst = copies == 1 ? dw : static_cast<float*>(scratch);
    if (int e = launch_image_wgrad(st, g, K, bf16, packed, sp, dy, dst)) return e;
    const int64_t n = (int64_t)g.R * g.S * g.Cin * g.Cout;
    if (copies > 1 && defer != nullptr) {
      *defer = DwSum{dst, copies, n, dw};
    } else if (copies > 1) {
      wgrad_reduce_kernel<<<(unsigned)((n + 63) / 64), kThreads, 0, st>>>(dst, copies, n, dw);
    }
    return hip_status();
  }
  // 1x1 layers with 64 x 256 channels and more: the kernel that keeps its tile of dW in registers
  if (const int copies = !relu32 ? rows_wgrad_copies(g, K, bf16) : 0) {
    float* dst = copies == 1 ? dw : static_cast<float*>(scratch);
    if (int e = launch_rows_wgrad(st, g, K, bf16, packed, sp, dy, dst)) return e;
    const int64_t n = (int64_t)g.Cin * g.Cout;
    if (copies > 1 && defer != nullptr) {
      *defer = DwSum{dst, copies, n, dw};
    } else if (copies > 1) {
      wgrad_reduce_kernel<<<(unsigned)((n + 63) / 64), kThreads, 0, st>>>(dst, copies, n, dw);
    }
    return hip_status();
  }
  const WgradPlan p = wgrad_plan(g);
  float* dst = p.split == 1 ? dw : static_cast<float*>(scratch);
  if (p.tm == 64 && p.tn == 128) launch_wgrad_tile<64, 128>(st, g, p, K, bf16, packed, sp, dy, dst, r32);
  else if (p.tm == 64 && p.tn == 64) launch_wgrad_tile<64, 64>(st, g, p, K, bf16, packed, sp, dy, dst, r32);
  else if (p.tm == 64 && p.tn == 32) launch_wgrad_tile<64, 32>(st, g, p, K, bf16, packed, sp, dy, dst, r32);
  else if (p.tm == 64 && p.tn == 16) launch_wgrad_tile<64, 16>(st, g, p, K, bf16, packed, sp, dy, dst, r32);
  else if (p.tm == 32 && p.tn == 64) launch_wgrad_tile<32, 64>(st, g, p, K, bf16, packed, sp, dy, dst, r32);
  else if (p.tm == 32 && p.tn == 32) launch_wgrad_tile<32, 32>(st, g, p, K, bf16, packed, sp, dy, dst, r32);
  else if (p.tm == 32 && p.tn == 16) launch_wgrad_tile<32, 16>(st, g, p, K, bf16, packed, sp, dy, dst, r32);
  else if (p.tm == 16 && p.tn == 64) launch_wgrad_tile<16, 64>(st, g, p, K, bf16, packed, sp, dy, dst, r32);
  else if (p.tm == 16 && p.tn == 32) launch_wgrad_tile<16, 32>(st, g, p, K, bf16, packed, sp, dy, dst, r32);
  else launch_wgrad_tile<16, 16>(st, g, p, K, bf16, packed, sp, dy, dst, r32);
  if (p.split > 1 && defer != nullptr) {  // the caller sums the copies in a launch of its own
    *defer = DwSum{dst, p.split, (int64_t)g.R * g.S * g.Cin * g.Cout, dw};
  } else if (p.split > 1) {
    const int64_t n = (int64_t)g.R * g.S * g.Cin * g.Cout;
    wgrad_reduce_kernel<<<(unsigned)((n + 63) / 64), kThreads, 0, st>>>(dst, p.split, n, dw);
  }
  return hip_status();
}

}  // namespace abl
