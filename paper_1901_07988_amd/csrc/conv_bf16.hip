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

template <int MODE, int BN>
__global__ __launch_bounds__(kThreads) void gemm_bf16_kernel(const float* __restrict__ in,
                                                             const float* __restrict__ wgt, const float* skip,
                                                             float* out, ConvGeom g) {
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

  // epilogue: the lane holds channels n0 + wn0 + 16 j + 4 lk .. +3 of pixel m0 + wm0 + 16 i + li
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
}

}  // namespace

bool bf16_gemm_supported(const ConvGeom& g, int mode) {
  const int Cg = mode == 0 ? g.Cin : g.Cout, Ng = mode == 0 ? g.Cout : g.Cin;
  if (Cg % BK != 0 || Ng % 64 != 0) return false;
  // 32-bit element offsets in the kernel
  const int64_t e_in = (int64_t)g.N * g.H * g.W * g.Cin, e_out = (int64_t)g.N * g.Ho * g.Wo * g.Cout;
  return e_in < ((int64_t)1 << 31) && e_out < ((int64_t)1 << 31);
}

int launch_bf16_gemm(hipStream_t st, const ConvGeom& g, int mode, const float* in, const float* w, const float* skip,
                     float* out) {
  if (!bf16_gemm_supported(g, mode)) return ABL_ERR_SHAPE;
  const int Ng = mode == 0 ? g.Cout : g.Cin;
  const int64_t Mg = mode == 0 ? (int64_t)g.N * g.Ho * g.Wo : (int64_t)g.N * g.H * g.W;
  const int64_t mblk = ((Mg + BM - 1) / BM + 7) / 8 * 8;  // whole XCD rounds; blocks past the end return
  // 128 output channels per block when that still leaves two blocks per compute unit
  const bool wide = Ng % 128 == 0 && mblk * (Ng / 128) >= 512;
  const unsigned grid = (unsigned)(mblk * (Ng / (wide ? 128 : 64)));
  if (mode == 0) {
    if (wide) gemm_bf16_kernel<0, 128><<<grid, kThreads, 0, st>>>(in, w, skip, out, g);
    else gemm_bf16_kernel<0, 64><<<grid, kThreads, 0, st>>>(in, w, skip, out, g);
  } else {
    if (wide) gemm_bf16_kernel<1, 128><<<grid, kThreads, 0, st>>>(in, w, nullptr, out, g);
    else gemm_bf16_kernel<1, 64><<<grid, kThreads, 0, st>>>(in, w, nullptr, out, g);
  }
  return hip_status();
}

}  // namespace abl
