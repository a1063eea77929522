// 3x3 'same' stride-1 convolutions on small images (up to 208 pixels: the 14x14 and 7x7 stages of
// an ImageNet network) in fp32: Eq. 4 (forward, mode 0) and the second half of Eq. 5 (gradient to
// the conv input, mode 1), the latter optionally with the Eq. 6-7 sums of the BN backward in its
// epilogue.
//
// One block = one image x 64 output channels, and the image stays in LDS, 64 contraction channels
// (one phase) at a time: (H+2)(W+2) positions of 64 floats with their zero border, 68 KB for 14x14,
// in two buffers that take turns - the next phase's channels are requested during this phase's
// MFMAs and written to the other buffer after them, so that only the first phase's loads are
// waited for.  That is what the 160 KB of LDS per compute unit are for: every input element is
// fetched once per block instead of once per tile of a pixel grid.  The four waves split the
// CONTRACTION: of the 9 taps x 4 sixteen-channel chunks of a phase each wave takes 9, and each
// keeps the block's whole output tile (up to 13 x 4 MFMA tiles = 208 accumulator registers) to
// itself.  So an activation fragment is read from LDS once per block and k-step (one 16-byte
// read feeds four MFMAs of each of the four channel tiles), no weights are shared (each wave
// streams its own k-steps' weights from the L2 straight into registers) and the main loop has no
// barrier and next to no vector-ALU work: per k-step 208 MFMAs against 13 LDS reads, 16 loads and
// some thirty other instructions.  The four partial tiles are added through the same LDS at the
// end in a fixed wave order; the wave that owns an output-channel tile adds the shortcut, stores,
// and takes the per-channel sums (of y for the next layer's Eq. 1, or Eq. 6-7 from the layer's
// codes).
//
// The file also holds the other kernels built for one block per compute unit with their results in
// accumulator registers, each described where it is defined: the weight gradient of the same 3x3 layers
// from the packed codes (image_wgrad_kernel, fp32 or bf16 operands), the 1x1 convolutions with long
// contractions (rows_f32_kernel) and the weight gradient of 1x1 layers (rows_wgrad_kernel,
// rows_wgrad_bf16_kernel).
//
// The MFMAs are written as inline assembly with the accumulator tied to the result: left to the
// register allocator, some tiles get a result register of their own and are copied back every
// k-step.  The compiler does not know these are matrix-core results, so the wait states they need
// before another kind of instruction reads them are inserted by hand after the loop.

#include <mutex>
#include <set>
#include <type_traits>
#include <utility>

#include "abl_internal.h"

namespace abl {
namespace {

constexpr int kThreads = 256;
constexpr int IMG_NB = 64;    // output channels per block
constexpr int IMG_PC = 64;    // contraction channels per phase; two phases' patches are resident

// More than the default 64 KB of LDS per block has to be asked for, once per kernel and device (the
// full 160 KB, so that the answer does not depend on the first shape seen).
int allow_full_lds(const void* kern) {
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

template <int MODE, int MT, int EPI>
__global__ __launch_bounds__(kThreads, 1) void image_f32_kernel(const float* __restrict__ in,
                                                                const float* __restrict__ wgt, const float* skip,
                                                                float* out, double* __restrict__ sums,
                                                                const uint8_t* __restrict__ codes,
                                                                const float* __restrict__ stats, ConvGeom g) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const int H = g.H, W = g.W, HW = H * W, PW = W + 2;
  const int Cg = MODE == 0 ? g.Cin : g.Cout;   // contraction channels: 16, 32, or a multiple of 64
  const int Ng = MODE == 0 ? g.Cout : g.Cin;   // output channels: a multiple of 64
  const int PC = Cg < IMG_PC ? Cg : IMG_PC;    // channels per phase (a power of two)
  const int pitch = 4 * PC + 16;               // bytes per patch position: the 16-byte fragments of 16
                                               // consecutive positions fall into different banks
  const int bufsz = (H + 2) * PW * pitch;      // one phase's patch; two of them take turns
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int li = lane & 15, lk = lane >> 4;
  // ids 8 apart share an XCD and its L2: the blocks of one image (same input) run there
  const int nblk = Ng / IMG_NB;
  const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
  const int img = (slot / nblk) * 8 + xcd;
  const int n0 = (slot % nblk) * IMG_NB;
  if (img >= g.N) return;

  // ---- the zero border of both patch buffers, once (the phases rewrite the interior only)
  {
    const int per = pitch >> 4;   // 16-byte pieces per position
    const int nz = (2 * PW + 2 * H) * per;
    for (int i0 = 0; i0 < nz; i0 += kThreads) {
      const int it = i0 + tid < nz ? i0 + tid : nz - 1;   // (a lane past the end repeats the last piece)
      const int bp = it / per, piece = it - bp * per;
      int pos;
      if (bp < PW) pos = bp;
      else if (bp < 2 * PW) pos = (H + 1) * PW + (bp - PW);
      else pos = (((bp - 2 * PW) >> 1) + 1) * PW + (((bp - 2 * PW) & 1) ? PW - 1 : 0);
      *reinterpret_cast<uint4*>(smem + pos * pitch + piece * 16) = make_uint4(0u, 0u, 0u, 0u);
      *reinterpret_cast<uint4*>(smem + bufsz + pos * pitch + piece * 16) = make_uint4(0u, 0u, 0u, 0u);
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
  const int cch_sh = __builtin_ctz((unsigned)PC) - 4;   // log2 of 16-channel chunks per phase
  const int T = 9 << cch_sh;
  const int ks_begin = wave * T / 4, ks_end = (wave + 1) * T / 4;
  auto a_offset = [&](int ks) __attribute__((always_inline)) {
    const int tap = ks >> cch_sh, cc = ks - (tap << cch_sh);
    const int r = tap / 3, s = tap - 3 * r;
    return (r * PW + s) * pitch + cc * 64;
  };
  // weights of one k-step: MFMA t of a chunk contracts channels 4 lk + t, so the lane's four
  // registers are four consecutive channels of its column (forward: four rows of W; gradient: 16
  // contiguous bytes).  Uniform part of the address in scalar registers, the lane's part a 32-bit
  // byte offset.
  uint32_t w_lane[4];
#pragma unroll
  for (int t = 0; t < 4; ++t)
    w_lane[t] = 4u * (MODE == 0 ? (uint32_t)((4 * lk + t) * g.Cout + li) : (uint32_t)(li * g.Cout + 4 * lk));
  int ph = 0;
  // part p of 8 (forward: two rows of one channel tile; gradient: parts 0, 2, 4, 6 a whole tile) or,
  // p < 0, everything
  auto load_w = [&](floatx4 (&dst)[4], int ks, int p) __attribute__((always_inline)) {
    const int tap = ks >> cch_sh, c0 = ph * PC + (ks - (tap << cch_sh)) * 16;
#pragma unroll
    for (int jj = 0; jj < 4; ++jj) {
      if (p >= 0 && (p >> 1) != jj) continue;
      const int nt = n0 + 16 * ((wave + jj) & 3);
      if (MODE == 0) {
        const char* wb = reinterpret_cast<const char*>(wgt + ((size_t)(tap * g.Cin + c0) * g.Cout + nt));
#pragma unroll
        for (int t = 0; t < 4; ++t) {
          if (p >= 0 && (t >> 1) != (p & 1)) continue;
          // (opaque to the optimizer: the 32-bit offset stays a register operand of the load beside
          // the scalar base instead of being widened to a 64-bit address outside the loop)
          asm volatile("" : "+v"(w_lane[t]));
          dst[jj][t] = *reinterpret_cast<const float*>(wb + w_lane[t]);
        }
      } else {
        // gradient to the input: tap (r', s') of the patch pairs with W[2 - r'][2 - s'][n][c]
        if (p >= 0 && (p & 1) != 0) continue;
        const char* wb = reinterpret_cast<const char*>(wgt + ((size_t)((8 - tap) * g.Cin + nt) * g.Cout + c0));
        asm volatile("" : "+v"(w_lane[0]));
        dst[jj] = *reinterpret_cast<const floatx4*>(wb + w_lane[0]);
      }
    }
  };

  floatx4 acc[4][MT];
#pragma unroll
  for (int jj = 0; jj < 4; ++jj)
#pragma unroll
    for (int i = 0; i < MT; ++i) acc[jj][i] = floatx4{0.f, 0.f, 0.f, 0.f};

  const int c4sh = __builtin_ctz((unsigned)PC) - 2;    // log2 of float4 per pixel and phase
  const int total = HW << c4sh;
  const uint32_t wmagic = 65536u / (unsigned)W + 1u;   // pix / W for pix * W < 65536
  const int nph = Cg / PC;
  // Staging of one phase, in two halves so that the next phase's loads can be in flight during
  // this phase's MFMAs: SU float4 per lane (13 for 14x14x64).  No branch anywhere (a guarded load
  // or store makes the compiler wait for everything in flight): a lane past the end repeats the
  // last item, which rewrites the same value.
  constexpr int SU = (16 * MT * (IMG_PC / 4) + kThreads - 1) / kThreads;
  floatx4 sv[SU];
  auto stage_load = [&](int p) __attribute__((always_inline)) {
    const float* src = in + (size_t)img * HW * Cg + p * PC;
#pragma unroll
    for (int u = 0; u < SU; ++u) {
      const int f = tid + kThreads * u;
      const int fi = f < total ? f : total - 1;
      const int pix = fi >> c4sh, c4 = fi - (pix << c4sh);
      sv[u] = *reinterpret_cast<const floatx4*>(src + (size_t)pix * Cg + 4 * c4);
    }
  };
  auto stage_store = [&](unsigned char* buf) __attribute__((always_inline)) {
#pragma unroll
    for (int u = 0; u < SU; ++u) {
      const int f = tid + kThreads * u;
      const int fi = f < total ? f : total - 1;
      const int pix = fi >> c4sh, c4 = fi - (pix << c4sh);
      const int h = (int)(((unsigned)pix * wmagic) >> 16), w = pix - h * W;
      *reinterpret_cast<floatx4*>(buf + ((h + 1) * PW + w + 1) * pitch + c4 * 16) = sv[u];
    }
  };
  stage_load(0);
  stage_store(smem);
  for (ph = 0; ph < nph; ++ph) {
    const unsigned char* cur = smem + (ph & 1) * bufsz;
    unsigned char* nxt = smem + ((ph + 1) & 1) * bufsz;
    const bool more_ph = ph + 1 < nph;
    // two sets of weight registers take turns by k-step; the next k-step's weights are requested in
    // eight parts behind the first eight tiles' MFMAs (every vector instruction between two MFMAs
    // costs the matrix pipe some cycles; a burst of them empties it)
    floatx4 w0[4], w1[4];
    load_w(w0, ks_begin, -1);
    __syncthreads();   // this phase's patch is complete; every wave is done with the other buffer
    // One set of activation fragments, refreshed in place: a tile's fragment of the next k-step
    // is requested as soon as its MFMAs of this k-step have been issued, a whole k-step ahead.
    floatx4 a[MT];
    {
      const int off = a_offset(ks_begin);
#pragma unroll
      for (int i = 0; i < MT; ++i) a[i] = *reinterpret_cast<const floatx4*>(cur + a_base[i] + off);
    }
    auto kstep = [&](const floatx4 (&wc)[4], floatx4 (&wn)[4], int ks) __attribute__((always_inline)) {
      const int kn = ks + 1 < ks_end ? ks + 1 : ks;   // the last k-step asks for its own operands again: no branch
      const int offn = a_offset(kn);
      __builtin_amdgcn_sched_barrier(0);
      // the order below is the schedule
#pragma unroll
      for (int i = 0; i < MT; ++i) {
#pragma unroll
        for (int t = 0; t < 4; ++t)
#pragma unroll
          for (int jj = 0; jj < 4; ++jj)
            asm volatile("v_mfma_f32_16x16x4_f32 %0, %1, %2, %0" : "+a"(acc[jj][i]) : "v"(wc[jj][t]), "v"(a[i][t]));
        a[i] = *reinterpret_cast<const floatx4*>(cur + a_base[i] + offn);
        constexpr int PP = (8 + MT - 1) / MT;   // parts per tile: all eight within the MT tiles
#pragma unroll
        for (int q = 0; q < PP; ++q)
          if (i * PP + q < 8) load_w(wn, kn, i * PP + q);
        __builtin_amdgcn_sched_barrier(0);
      }
    };
    // The next phase's channels are requested behind the first k-step's MFMAs and have the rest
    // of the phase to arrive (the load counter retires in order: requested any earlier, the first
    // k-step's wait for its weights would wait for them too); they go to the other buffer after
    // the last k-step.
    for (int ks = ks_begin; ks < ks_end; ks += 2) {
      kstep(w0, w1, ks);
      if (ks == ks_begin && more_ph) stage_load(ph + 1);
      __builtin_amdgcn_sched_barrier(0);
      if (ks + 1 < ks_end) kstep(w1, w0, ks + 1);
    }
    if (more_ph) stage_store(nxt);
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
  double s1[4] = {0.0, 0.0, 0.0, 0.0}, s2[4] = {0.0, 0.0, 0.0, 0.0};
  if (MODE == 0) {
    if (skip != nullptr) {
      // all the shortcut loads together, none of them guarded
      floatx4 sv[MT];
#pragma unroll
      for (int i = 0; i < MT; ++i) sv[i] = *reinterpret_cast<const floatx4*>(skip + o[i]);
#pragma unroll
      for (int i = 0; i < MT; ++i) {
        v[i][0] += sv[i][0]; v[i][1] += sv[i][1]; v[i][2] += sv[i][2]; v[i][3] += sv[i][3];
      }
    }
#pragma unroll
    for (int i = 0; i < MT; ++i) {
      if (16 * i + li < HW) {
        *reinterpret_cast<floatx4*>(out + o[i]) = v[i];
        if (sums != nullptr) {
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            s1[r] += (double)v[i][r];
            s2[r] += (double)v[i][r] * (double)v[i][r];
          }
        }
      }
    }
  } else {
    if constexpr (EPI != 0) {
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
            const int32_t j = (int32_t)code - (1 << (EPI - 1)) + fbv[r];
            const float a2t = st4[r] * ((float)j + 0.5f);        // Eq. 10
            const float da2 = a2t > 0.0f ? v[i][r] : 0.0f;       // Eq. 6
            const float a1t = (a2t - bt4[r]) * ig[r];            // inverse of Eq. 2
            s1[r] += (double)da2;
            s2[r] += (double)a1t * (double)da2;
          }
        }
      }
    }
#pragma unroll
    for (int i = 0; i < MT; ++i)
      if (16 * i + li < HW) *reinterpret_cast<floatx4*>(out + o[i]) = v[i];
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


// ---- weight gradient (first half of Eq. 5) of the same layers from the packed codes ----------------
// dW[tap][ci][co] = sum over images and pixels of A3~[pixel + tap][ci] * dy[pixel][co], A3~ = ReLU of Eq. 10.
// One block owns a 32 (ci) x 64 (co) tile of all nine taps and a share of the images; per image it
// dequantizes the tile's 32 channels of the image once into an LDS patch with its zero border (the nine
// taps are nine offsets into it) and stages the tile's 64 channels of dy beside it.  The contraction
// index of the MFMAs is the pixel (four per MFMA), the wave owns one 16-channel tile of ci and two of co for all 9
// taps (18 accumulator tiles), and per 4-pixel step it reads 2 fragments of dy and 9 of the patch
// - all at one address plus a constant (the image width is a template parameter) - for 18 MFMAs; the
// fragments of the next step are read while this step's MFMAs run.  The next image's dy and codes are
// requested at the start of an image's 49 steps and go to LDS after them.  Each share of the images
// leaves its own copy of dW, summed in a fixed order by the caller's launch.
constexpr int WG_CI = 32, WG_CO = 64;
constexpr int WG_AP = 4 * WG_CI + 64;   // bytes per patch position: the four pixel groups of a read hit
constexpr int WG_DP = 4 * WG_CO + 64;   // ... different quarters of the banks (48 resp. 80 words apart)

// BF16: operands rounded to bf16 on their way from LDS to the registers and contracted 16 at a time
// (v_mfma_f32_16x16x16_bf16); the tiles and the copies are the same.  Here the contraction runs over the
// positions of the PADDED rows (image width + 2 = 16 = one MFMA step per image row): dy is staged in the
// same 16-wide rows with zeros in the two border columns, so the patch address of every tap is the
// step's base plus a constant (no row wrap to track, 0 address instructions per read) and the two
// products with the border columns vanish.  The patch has one position of margin before and after it
// for the corner taps of the border columns.
template <int K, int IW, bool BF16 = false>
__global__ __launch_bounds__(kThreads, 1) void image_wgrad_kernel(const uint8_t* __restrict__ codes,
                                                                  const float* __restrict__ stats,
                                                                  const float* __restrict__ dy,
                                                                  float* __restrict__ dst, ConvGeom g, int splits) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  constexpr int PW = IW + 2;
  const int H = g.H, HW = H * IW;             // HW a multiple of 4
  unsigned char* const AL = smem + (BF16 ? WG_AP : 0);            // [(H+2) * PW][WG_AP] (BF16: a position of margin on either side)
  unsigned char* const DL = AL + ((H + 2) * PW + (BF16 ? 1 : 0)) * WG_AP;   // [HW][WG_DP]; BF16: [H * PW][WG_DP]
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int li = lane & 15, lk = lane >> 4;
  // ids 8 apart share an XCD and its L2: the blocks that stage the same dy (same co tile and share
  // of the images, different ci tiles) run there
  const int n_ci = g.Cin / WG_CI, n_co = g.Cout / WG_CO;
  int ci_blk, pair;
  if ((n_co * splits) % 8 == 0) {
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    pair = (slot / n_ci) * 8 + xcd;
    ci_blk = slot % n_ci;
  } else {
    pair = blockIdx.x / n_ci;
    ci_blk = blockIdx.x % n_ci;
  }
  const int co_blk = pair % n_co, split = pair / n_co;
  const int ci0 = ci_blk * WG_CI, co0 = co_blk * WG_CO;
  const int img_begin = split * g.N / splits, img_end = (split + 1) * g.N / splits;

  // ---- zero border of the patch, once
  {
    constexpr int per = WG_AP / 16;
    const int nz = (2 * PW + 2 * H) * per;
    for (int i0 = 0; i0 < nz; i0 += kThreads) {
      const int it = i0 + tid < nz ? i0 + tid : nz - 1;
      const int bp = it / per, piece = it - bp * per;
      int pos;
      if (bp < PW) pos = bp;
      else if (bp < 2 * PW) pos = (H + 1) * PW + (bp - PW);
      else pos = (((bp - 2 * PW) >> 1) + 1) * PW + (((bp - 2 * PW) & 1) ? PW - 1 : 0);
      *reinterpret_cast<uint4*>(AL + pos * WG_AP + piece * 16) = make_uint4(0u, 0u, 0u, 0u);
    }
    if constexpr (BF16) {
      // the two margin positions of the patch and the border columns of dy
      if (tid < 2 * per)
        *reinterpret_cast<uint4*>(AL + (tid < per ? -1 : (H + 2) * PW) * WG_AP + (tid % per) * 16) = make_uint4(0u, 0u, 0u, 0u);
      constexpr int perd = WG_DP / 16;
      for (int it = tid; it < 2 * H * perd; it += kThreads) {
        const int bp = it / perd, piece = it - bp * perd;
        *reinterpret_cast<uint4*>(DL + ((bp >> 1) * PW + ((bp & 1) ? PW - 1 : 0)) * WG_DP + piece * 16) = make_uint4(0u, 0u, 0u, 0u);
      }
    }
  }

  // ---- staging roles.  Codes: the thread dequantizes 8 channels (one 32- or 64-bit word) of pixels
  // tid/4 + 64 q.  Eq. 10 as one multiply per element: step * ((code - 2^(K-1) + fb) + 0.5) =
  // step * (code + offh), offh = fb - 2^(K-1) + 0.5 (exact in fp32 while |fb| < 2^22).
  const int cg = tid & 3, cpix = tid >> 2;
  constexpr int CQ = 4;                          // pixel rounds: 4 x 64 >= 196
  float stp[8], offh[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    const int c = ci0 + 8 * cg + e;
    stp[e] = stats[P_STEP * g.Cin + c];
    offh[e] = (float)(reinterpret_cast<const int32_t*>(stats)[P_FB * g.Cin + c] - (1 << (K - 1))) + 0.5f;
  }
  constexpr int DU = 13;                         // float4 of dy per thread: 13 x 256 >= 196 x 16
  floatx4 dyv[DU];
  uint32_t cw[CQ][K / 4];
  const int ndy = HW * (WG_CO / 4);
  auto stage_load = [&](int img) __attribute__((always_inline)) {
    const float* src = dy + ((size_t)img * HW) * g.Cout + co0;
#pragma unroll
    for (int u = 0; u < DU; ++u) {
      const int f = tid + kThreads * u;
      const int fi = f < ndy ? f : ndy - 1;   // (a lane past the end repeats the last item)
      dyv[u] = *reinterpret_cast<const floatx4*>(src + (size_t)(fi >> 4) * g.Cout + 4 * (fi & 15));
    }
    const uint8_t* cs = codes + (((size_t)img * HW) * g.Cin + ci0 + 8 * cg) * K / 8;
#pragma unroll
    for (int q = 0; q < CQ; ++q) {
      const int px = cpix + 64 * q;
      const int pc = px < HW ? px : HW - 1;
      const uint8_t* a = cs + (size_t)pc * g.Cin * K / 8;
      if (K == 4) cw[q][0] = *reinterpret_cast<const uint32_t*>(a);
      else {
        const uint2 t = *reinterpret_cast<const uint2*>(a);
        cw[q][0] = t.x;
        cw[q][K / 4 - 1] = t.y;
      }
    }
  };
  auto stage_store = [&]() __attribute__((always_inline)) {
#pragma unroll
    for (int u = 0; u < DU; ++u) {
      const int f = tid + kThreads * u;
      const int fi = f < ndy ? f : ndy - 1;
      int row = fi >> 4;                       // pixel h * IW + w
      if constexpr (BF16) {                    // ... to position h * PW + w + 1 of the padded rows
        const int h = (row * (65536 / IW + 1)) >> 16;   // row / IW for row < 4096
        row += h * (PW - IW) + 1;
      }
      *reinterpret_cast<floatx4*>(DL + row * WG_DP + (fi & 15) * 16) = dyv[u];
    }
#pragma unroll
    for (int q = 0; q < CQ; ++q) {
      const int px = cpix + 64 * q;
      const int pc = px < HW ? px : HW - 1;
      const int h = pc / IW, w = pc - h * IW;
      float v[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const uint32_t word = cw[q][(e * K) / 32];
        const uint32_t code = (word >> ((e * K) % 32)) & ((1u << K) - 1u);
        v[e] = fmaxf(stp[e] * ((float)code + offh[e]), 0.0f);   // Eq. 10, then the ReLU
      }
      unsigned char* d = AL + ((h + 1) * PW + w + 1) * WG_AP + cg * 32;
      *reinterpret_cast<floatx4*>(d) = floatx4{v[0], v[1], v[2], v[3]};
      *reinterpret_cast<floatx4*>(d + 16) = floatx4{v[4], v[5], v[6], v[7]};
    }
  };

  // the wave's tiles: ci tile wc, co tiles 2 wo and 2 wo + 1, all nine taps - 18 MFMAs per step
  // from 9 + 2 fragments
  const int wc = wave & 1, wo = wave >> 1;
  floatx4 acc[9][2];
#pragma unroll
  for (int t = 0; t < 9; ++t)
#pragma unroll
    for (int o = 0; o < 2; ++o) acc[t][o] = floatx4{0.f, 0.f, 0.f, 0.f};

  // fragments of one 4-pixel step: the lane's pixel is 4 j + lk
  struct Frag {
    float d[2];   // dy[pixel][co0 + 16 (2 wo + o) + li]
    float a[9];   // patch[pixel + tap][ci0 + 16 wc + li]
  };
  auto read_a = [&](Frag& f, int t, int abase) __attribute__((always_inline)) {
    f.a[t] = *reinterpret_cast<const float*>(AL + abase + ((t / 3) * PW + (t % 3)) * WG_AP);
  };
  auto read_d = [&](Frag& f, int o, int dbase) __attribute__((always_inline)) {
    f.d[o] = *reinterpret_cast<const float*>(DL + dbase + o * 64);
  };
  // One step: the 18 MFMAs on `cur` with the 11 reads of the next step's fragments spread between
  // them, one behind every pair of MFMAs.  Measured on 64 x 14 x 14 x 256 -> 256: all reads in a burst
  // between two steps 143 us, spread like this 136 us, the same reads as six two-address
  // instructions behind the first six pairs 141 us, no reads at all 120 us - every vector-memory or
  // vector-ALU instruction between two MFMAs costs the matrix pipe some 9 cycles, so what counts is
  // their number and an even spread.  The order below is the schedule.
  auto step = [&](const Frag& cur, Frag& nxt, int abase, int dbase) __attribute__((always_inline)) {
#pragma unroll
    for (int t = 0; t < 9; ++t) {
#pragma unroll
      for (int o = 0; o < 2; ++o)
        asm volatile("v_mfma_f32_16x16x4_f32 %0, %1, %2, %0" : "+a"(acc[t][o]) : "v"(cur.d[o]), "v"(cur.a[t]));
      read_a(nxt, t, abase);
      if (t < 2) read_d(nxt, t, dbase);
      __builtin_amdgcn_sched_barrier(0);
    }
  };
  auto mma = [&](const Frag& f) __attribute__((always_inline)) {
#pragma unroll
    for (int t = 0; t < 9; ++t)
#pragma unroll
      for (int o = 0; o < 2; ++o)
        asm volatile("v_mfma_f32_16x16x4_f32 %0, %1, %2, %0" : "+a"(acc[t][o]) : "v"(f.d[o]), "v"(f.a[t]));
  };

  if (img_begin < img_end) stage_load(img_begin);
  for (int img = img_begin; img < img_end; ++img) {
    __syncthreads();   // every wave is done with the previous image's patch and dy
    stage_store();
    __syncthreads();
    if (img + 1 < img_end) stage_load(img + 1);
    __builtin_amdgcn_sched_barrier(0);
    if constexpr (BF16) {
      // step j = image row j; the lane's positions are 4 i + lk of the padded row (element i of its operand:
      // any assignment of the step's 16 positions to the MFMA's 16 k will do, and with this one the four lane
      // groups of a read are at neighbouring positions - different banks, as in the fp32 loop).  Output
      // position P of row j reads the patch at P + (tap row) * PW + (tap column) - 1.
      static_assert(!BF16 || IW + 2 == 16, "one padded row per 16-deep MFMA");
      struct FragB {
        shortx4 d[2];   // four positions of dy[.][co0 + 16 (2 wo + o) + li]
        shortx4 a[9];   // four positions of patch[. + tap][ci0 + 16 wc + li]
      };
      auto pack4 = [](float x0, float x1, float x2, float x3) __attribute__((always_inline)) {
        typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
        const bf16x2_t lo = {(__bf16)x0, (__bf16)x1}, hi = {(__bf16)x2, (__bf16)x3};
        const uint2 u = make_uint2(__builtin_bit_cast(uint32_t, lo), __builtin_bit_cast(uint32_t, hi));
        return __builtin_bit_cast(shortx4, u);
      };
      auto read_frag = [&](FragB& f, int abase, int dbase) __attribute__((always_inline)) {
#pragma unroll
        for (int o = 0; o < 2; ++o)
          f.d[o] = pack4(*reinterpret_cast<const float*>(DL + dbase + o * 64),
                         *reinterpret_cast<const float*>(DL + dbase + 4 * WG_DP + o * 64),
                         *reinterpret_cast<const float*>(DL + dbase + 8 * WG_DP + o * 64),
                         *reinterpret_cast<const float*>(DL + dbase + 12 * WG_DP + o * 64));
#pragma unroll
        for (int t = 0; t < 9; ++t) {
          const int off = ((t / 3) * PW + (t % 3)) * WG_AP;
          f.a[t] = pack4(*reinterpret_cast<const float*>(AL + abase + off),
                         *reinterpret_cast<const float*>(AL + abase + 4 * WG_AP + off),
                         *reinterpret_cast<const float*>(AL + abase + 8 * WG_AP + off),
                         *reinterpret_cast<const float*>(AL + abase + 12 * WG_AP + off));
        }
      };
      auto mma16 = [&](const FragB& f) __attribute__((always_inline)) {
#pragma unroll
        for (int t = 0; t < 9; ++t)
#pragma unroll
          for (int o = 0; o < 2; ++o)
            acc[t][o] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(f.d[o], f.a[t], acc[t][o], 0, 0, 0);
      };
      int abase = (lk - 1) * WG_AP + (16 * wc + li) * 4;
      int dbase = lk * WG_DP + (32 * wo + li) * 4;
      FragB f0, f1;
      read_frag(f0, abase, dbase);
      for (int j = 0; j + 1 < H; j += 2) {
        abase += PW * WG_AP;
        dbase += PW * WG_DP;
        read_frag(f1, abase, dbase);
        mma16(f0);
        // (the last pair of an even count asks for one row past the image: the first row again, never used)
        const bool more = j + 2 < H;
        abase = more ? abase + PW * WG_AP : (lk - 1) * WG_AP + (16 * wc + li) * 4;
        dbase = more ? dbase + PW * WG_DP : lk * WG_DP + (32 * wo + li) * 4;
        read_frag(f0, abase, dbase);
        mma16(f1);
      }
      if (H & 1) mma16(f0);
      continue;
    }
    // The lane's pixel of step j is 4 j + lk.  Seven steps are 28 pixels = two image rows, so within such a
    // group the lane's patch positions are seven constants (the row wrap included) and from group to
    // group everything moves by two rows: one address add per step instead of tracking the column (six
    // vector instructions per step, each as dear as a third of an MFMA here).  H is even: H / 2 groups.
    static_assert(BF16 || (2 * IW) % 4 == 0, "two rows are a whole number of steps");
    constexpr int GS = 2 * IW / 4;   // steps per group: 7
    int off7[GS];
#pragma unroll
    for (int j = 0; j < GS; ++j) {
      const int p = lk + 4 * j, hh = p >= IW ? 1 : 0;
      off7[j] = (hh * PW + p - hh * IW) * WG_AP + (16 * wc + li) * 4;
    }
    int ag = 0;                                        // the group's first patch row, in bytes
    int dg = lk * WG_DP + (32 * wo + li) * 4;          // the lane's dy of the group's step 0
    Frag f0, f1;
#pragma unroll
    for (int t = 0; t < 9; ++t) read_a(f0, t, off7[0]);
#pragma unroll
    for (int o = 0; o < 2; ++o) read_d(f0, o, dg);
    // one group: fa holds the fragments of its step 0, the steps take fa, fb, fa, ... and leave the next
    // group's first fragments in fb (the image's last step asks for address 0 - never used)
    auto group = [&](Frag& fa, Frag& fb, bool last) __attribute__((always_inline)) {
#pragma unroll
      for (int j = 0; j < GS; ++j) {
        int an, dn;
        if (j + 1 < GS) {
          an = ag + off7[j + 1];
          dn = dg + (j + 1) * 4 * WG_DP;
        } else {
          an = last ? 0 : ag + 2 * PW * WG_AP + off7[0];
          dn = last ? 0 : dg + 2 * IW * WG_DP;
        }
        __builtin_amdgcn_sched_barrier(0);
        if (j & 1) step(fb, fa, an, dn);
        else step(fa, fb, an, dn);
      }
      ag += 2 * PW * WG_AP;
      dg += 2 * IW * WG_DP;
    };
    static_assert(BF16 || GS % 2 == 1, "an odd number of steps: the two fragment sets swap roles from group to group");
    const int groups = H / 2;
    for (int grp = 0; grp + 1 < groups; grp += 2) {
      group(f0, f1, false);
      group(f1, f0, grp + 2 >= groups);
    }
    if (groups & 1) group(f0, f1, true);
  }
  // the MFMAs' results are read below by instructions the compiler does not know to depend on a
  // matrix-core result: more wait states than the longest such hazard
  asm volatile("s_nop 15\n\ts_nop 15");
  float* out = dst + (size_t)split * 9 * g.Cin * g.Cout;
#pragma unroll
  for (int t = 0; t < 9; ++t)
#pragma unroll
    for (int o = 0; o < 2; ++o)
      *reinterpret_cast<floatx4*>(out + ((size_t)(t * g.Cin + ci0 + 16 * wc + li)) * g.Cout + co0 + 16 * (2 * wo + o) +
                                  4 * lk) = acc[t][o];
}

int image_wgrad_splits(const ConvGeom& g) {
  const int tiles = (g.Cin / WG_CI) * (g.Cout / WG_CO);
  int s = 256 / tiles;
  if (s > g.N) s = g.N;
  if (s > 16) s = 16;
  return s < 1 ? 1 : s;
}

// ---- weight gradient (first half of Eq. 5) of 1x1 stride-1 layers from the packed codes ------------
// dW[ci][co] = sum over the N H W pixels of A3~[pixel][ci] * dy[pixel][co], A3~ = ReLU of Eq. 10: one matrix
// product whose contraction index is the pixel (four per MFMA).  One block owns a 64 (ci) x 256 (co) tile
// and a share of the pixels; each wave keeps 64 x 64 of it (16 accumulator tiles) in registers.
// The rows and columns of an MFMA tile need not be neighbouring channels: lane li supplies, for its pixel,
// FOUR input channels (4 li .. 4 li + 3: one 16-byte LDS read) and FOUR output channels (4 li .. 4 li + 3
// of the wave's 64: one 16-byte load of dy straight from global memory, no LDS), and the 4 x 4 register
// pairs are the 16 MFMAs of a 4-pixel step - 2 operand instructions for 16 MFMAs instead of one 4-byte
// read per operand register.  Only the dequantized activation goes through LDS (shared by the four waves,
// dequantized once per block): 16 pixels at a time in two buffers, one 16- or 32-bit code word per thread
// and chunk, dequantized between the MFMAs of the chunk before.  The step of Eq. 10 is a factor per input
// channel and is applied to the sums at the end (max(step * x, 0) = step * max(x, 0), step > 0), so a
// dequantized element costs a convert, an add and a max.  Each share of the pixels leaves its own copy of
// dW, summed in a fixed order by the caller's launch: the chip's accumulators are 16 copies of a 1024 x 256
// dW.  (A 128 x 256 tile per block - eight input channels per lane, 32 MFMAs from 3 operand instructions,
// twice the accumulators and copies - measured 2-5 us slower on every shape tried.)
constexpr int PW_CI = 64, PW_CO = 256, PW_PX = 16;

template <int K>
__global__ __launch_bounds__(kThreads, 1) void rows_wgrad_kernel(const uint8_t* __restrict__ codes,
                                                                 const float* __restrict__ stats,
                                                                 const float* __restrict__ dy,
                                                                 float* __restrict__ dst, ConvGeom g, int splits) {
  __shared__ __attribute__((aligned(16))) float AL[2][PW_PX][PW_CI];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int li = lane & 15, lk = lane >> 4;
  // ids 8 apart share an XCD and its L2: the blocks that read the same dy (same co tile and share of
  // the pixels, different ci tiles) run there
  const int n_ci = g.Cin / PW_CI, n_co = g.Cout / PW_CO;
  int ci_blk, pair;
  if ((n_co * splits) % 8 == 0) {
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    pair = (slot / n_ci) * 8 + xcd;
    ci_blk = slot % n_ci;
  } else {
    pair = blockIdx.x / n_ci;
    ci_blk = blockIdx.x % n_ci;
  }
  const int co_blk = pair % n_co, split = pair / n_co;
  const int ci0 = ci_blk * PW_CI, co0 = co_blk * PW_CO + 64 * wave;
  const int chunks = (int)(((int64_t)g.N * g.H * g.W) / PW_PX);   // N H W is a multiple of 16
  const int c_begin = (int)((int64_t)split * chunks / splits), c_end = (int)((int64_t)(split + 1) * chunks / splits);

  // ---- staging role: the four channels ci0 + 4 cg .. of pixel px of a chunk.  Eq. 10 without its step:
  // (code - 2^(K-1) + fb) + 0.5 = code + offh, exact in fp32 while |fb| < 2^22.
  const int cg = tid & 15, px = tid >> 4;
  float offh[4];
#pragma unroll
  for (int e = 0; e < 4; ++e)
    offh[e] = (float)(reinterpret_cast<const int32_t*>(stats)[P_FB * g.Cin + ci0 + 4 * cg + e] - (1 << (K - 1))) + 0.5f;
  uint32_t c_lane = (uint32_t)((px * g.Cin + ci0 + 4 * cg) * K / 8);
  const size_t c_chunk = (size_t)PW_PX * g.Cin * K / 8;          // bytes of codes per chunk
  uint32_t cw[2];                                                 // code words of the chunks of either parity
  // (a chunk index past the tensor's last one asks for the last one again: never used)
  auto load_codes = [&](uint32_t& w, int c) __attribute__((always_inline)) {
    const uint8_t* cb = codes + (size_t)(c < chunks ? c : chunks - 1) * c_chunk;
    asm volatile("" : "+v"(c_lane));
    if constexpr (K == 4) w = *reinterpret_cast<const uint16_t*>(cb + c_lane);
    else w = *reinterpret_cast<const uint32_t*>(cb + c_lane);
  };
  float vals[4];
  uint32_t by[2];   // K = 4: the even and the odd codes of the word, one per byte (a byte converts in one instruction)
  auto dequant = [&](uint32_t w, int e) __attribute__((always_inline)) {
    uint32_t code;
    if constexpr (K == 4) {
      if (e == 0) {
        by[0] = w & 0x0F0Fu;
        by[1] = (w >> 4) & 0x0F0Fu;
        asm volatile("" : "+v"(by[0]), "+v"(by[1]));   // (kept as they are: not folded back into a field extract per code)
      }
      code = (by[e & 1] >> (8 * (e >> 1))) & 0xFFu;
    } else {
      code = (w >> (8 * e)) & 0xFFu;
    }
    vals[e] = fmaxf((float)code + offh[e], 0.0f);   // Eq. 10 over its step, then the ReLU
  };
  auto store_vals = [&](int buf) __attribute__((always_inline)) {
    *reinterpret_cast<floatx4*>(&AL[buf][px][4 * cg]) = floatx4{vals[0], vals[1], vals[2], vals[3]};
  };

  // ---- operands of the MFMAs.  dy: the lane's pixel of step s is 4 s + lk, its channels co0 + 4 li ..
  uint32_t d_lane[4];
#pragma unroll
  for (int s = 0; s < 4; ++s) d_lane[s] = 4u * (uint32_t)((4 * s + lk) * g.Cout + co0 + 4 * li);
  const size_t d_chunk = (size_t)PW_PX * g.Cout;                 // floats of dy per chunk
  floatx4 dyr[8];                                                // ring: slot 4 (chunk parity) + s, two chunks ahead
  auto load_dy = [&](int slot, int c, int s) __attribute__((always_inline)) {
    const char* db = reinterpret_cast<const char*>(dy + (size_t)(c < chunks ? c : chunks - 1) * d_chunk);
    asm volatile("" : "+v"(d_lane[s]));
    dyr[slot] = *reinterpret_cast<const floatx4*>(db + d_lane[s]);
  };
  floatx4 af[2];                                                 // two sets taking turns: channels 4 li .. + 3
  auto read_a = [&](int set, int buf, int s) __attribute__((always_inline)) {
    af[set] = *reinterpret_cast<const floatx4*>(&AL[buf][4 * s + lk][4 * li]);
  };

  floatx4 acc[4][4];   // [e][j]: rows = input channels 4 (4 lk + r) + e, column = output channel 4 li + j
#pragma unroll
  for (int e = 0; e < 4; ++e)
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[e][j] = floatx4{0.f, 0.f, 0.f, 0.f};

  // One chunk (four steps of 16 MFMAs) of parity PAR.  Between the MFMAs, one piece behind every group of
  // four: the reads of the next step's activation fragments, the dequantization of the next chunk (code
  // words in cw[PAR ^ 1], to buffer PAR ^ 1), the request for the code word of the chunk after that and,
  // behind a step's last MFMA, the request for dy of the same step two chunks ahead into the slot just
  // used.  The barrier sits behind step 2: the buffer written here was last read before the previous
  // chunk's barrier, and step 3 already reads the next chunk's first fragments from it.
  auto chunk = [&](auto par, int c) __attribute__((always_inline)) {
    constexpr int PAR = decltype(par)::value;
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      const int cur = s & 1, slot = 4 * PAR + s;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
#pragma unroll
        for (int j = 0; j < 4; ++j)
          asm volatile("v_mfma_f32_16x16x4_f32 %0, %1, %2, %0"
                       : "+a"(acc[e][j])
                       : "v"(af[cur][e]), "v"(dyr[slot][j]));
        if (e == 0) {
          if (s < 3) read_a(cur ^ 1, PAR, s + 1);
          else read_a(cur ^ 1, PAR ^ 1, 0);
        } else if (s == 0) {
          if (e == 1) load_codes(cw[PAR], c + 2);
          else dequant(cw[PAR ^ 1], e - 2);           // values 0, 1
        } else if (s == 1) {
          if (e >= 2) dequant(cw[PAR ^ 1], e);        // values 2, 3
        } else if (s == 2) {
          if (e == 1) store_vals(PAR ^ 1);
        }
        if (e == 3) load_dy(slot, c + 2, s);
        __builtin_amdgcn_sched_barrier(0);
      }
      if (s == 2) __syncthreads();
    }
  };

  if (c_begin < c_end) {
    load_codes(cw[0], c_begin);
    load_codes(cw[1], c_begin + 1);
#pragma unroll
    for (int s = 0; s < 4; ++s) load_dy(s, c_begin, s);
#pragma unroll
    for (int s = 0; s < 4; ++s) load_dy(4 + s, c_begin + 1, s);
#pragma unroll
    for (int e = 0; e < 4; ++e) dequant(cw[0], e);
    store_vals(0);
    __syncthreads();
    read_a(0, 0, 0);
    const int n = c_end - c_begin;
    for (int i = 0; i + 1 < n; i += 2) {
      chunk(std::integral_constant<int, 0>{}, c_begin + i);
      chunk(std::integral_constant<int, 1>{}, c_begin + i + 1);
    }
    // The MFMAs' results are read by instructions the compiler does not know to depend on a matrix-core
    // result - here already where it copies the accumulators around the conditional last chunk: more wait
    // states than the longest such hazard, tied to the accumulator written last (every other one is at
    // least one MFMA, 32 cycles, older), so that no read of it is placed above the wait.
    asm volatile("s_nop 15\n\ts_nop 15" : "+a"(acc[3][3]));
    if (n & 1) chunk(std::integral_constant<int, 0>{}, c_end - 1);
  }
  asm volatile("s_nop 15\n\ts_nop 15" : "+a"(acc[3][3]));
  float* out = dst + (size_t)split * g.Cin * g.Cout;
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    const int ci = ci0 + 4 * (4 * lk + r);
    const floatx4 st4 = *reinterpret_cast<const floatx4*>(stats + P_STEP * g.Cin + ci);
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const float st = st4[e];
      *reinterpret_cast<floatx4*>(out + (size_t)(ci + e) * g.Cout + co0 + 4 * li) =
          floatx4{st * acc[e][0][r], st * acc[e][1][r], st * acc[e][2][r], st * acc[e][3][r]};
    }
  }
}

// The same weight gradient with bf16 operands (v_mfma_f32_16x16x32_bf16: 32 pixels per MFMA, a lane
// supplies eight of them per operand register set).  The tile, the shares and the copies are those of the
// fp32 kernel; a chunk is 32 pixels = one step of 16 MFMAs.  Both operands are rounded to bf16 by the
// hardware's packed convert, which takes its two inputs from any two registers - so the regrouping from
// "four channels of one pixel" (what a 16-byte load delivers) to "eight pixels of one channel" (what
// the MFMA wants) costs nothing beyond the conversion itself: dy goes from eight 16-byte global loads
// (the lane's eight pixels) through 16 converts into the four operand sets; the activation is
// dequantized (Eq. 10 with its step, ReLU: the rounded value is that of the tiled bf16 kernel),
// converted in pairs of neighbouring pixels and written to LDS as [pixel group][e][li][8 pixels], from
// where a lane's operand set e is one 16-byte read.  dy runs four chunks ahead in a ring of 128 registers.
constexpr int PB_PX = 32;

template <int K>
__global__ __launch_bounds__(kThreads, 1) void rows_wgrad_bf16_kernel(const uint8_t* __restrict__ codes,
                                                                      const float* __restrict__ stats,
                                                                      const float* __restrict__ dy,
                                                                      float* __restrict__ dst, ConvGeom g,
                                                                      int splits) {
  __shared__ __attribute__((aligned(16))) uint32_t AL[2][4][4][16][4];   // [buffer][pixel group][e][li][4 pixel pairs]
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int li = lane & 15, lk = lane >> 4;
  const int n_ci = g.Cin / PW_CI, n_co = g.Cout / PW_CO;
  int ci_blk, pair;
  if ((n_co * splits) % 8 == 0) {
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    pair = (slot / n_ci) * 8 + xcd;
    ci_blk = slot % n_ci;
  } else {
    pair = blockIdx.x / n_ci;
    ci_blk = blockIdx.x % n_ci;
  }
  const int co_blk = pair % n_co, split = pair / n_co;
  const int ci0 = ci_blk * PW_CI, co0 = co_blk * PW_CO + 64 * wave;
  const int chunks = (int)(((int64_t)g.N * g.H * g.W) / PB_PX);   // N H W is a multiple of 32
  const int c_begin = (int)((int64_t)split * chunks / splits), c_end = (int)((int64_t)(split + 1) * chunks / splits);

  // ---- staging role: channels ci0 + 4 cg .., pixels 2 q and 2 q + 1 of a chunk (q = 4 wave + lk: wave w
  // stages pixel group w).  Eq. 10 as one add and one multiply: step * (code + offh), offh = fb - 2^(K-1) + 0.5.
  const int cg = tid & 15, q = tid >> 4;
  float stp[4], offh[4];
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const int c = ci0 + 4 * cg + e;
    stp[e] = stats[P_STEP * g.Cin + c];
    offh[e] = (float)(reinterpret_cast<const int32_t*>(stats)[P_FB * g.Cin + c] - (1 << (K - 1))) + 0.5f;
  }
  uint32_t c_lane = (uint32_t)((2 * q * g.Cin + ci0 + 4 * cg) * K / 8);
  const size_t c_chunk = (size_t)PB_PX * g.Cin * K / 8;          // bytes of codes per chunk
  const size_t c_pixel = (size_t)g.Cin * K / 8;                   // ... per pixel
  // the four codes of a pixel are 16 or 32 bits; kept in a word of their own size until they are
  // taken apart (widened on arrival they would have to be waited for at the top of the loop)
  using code_t = typename std::conditional<K == 4, uint16_t, uint32_t>::type;
  code_t cw[4][2];                                                // ring of four chunks: [slot][pixel]
  // (a chunk index past the tensor's last one asks for the last one again: never used)
  auto load_codes = [&](code_t (&w)[2], int c) __attribute__((always_inline)) {
    const uint8_t* cb = codes + (size_t)(c < chunks ? c : chunks - 1) * c_chunk;
#pragma unroll
    for (int p = 0; p < 2; ++p) {
      asm volatile("" : "+v"(c_lane));
      w[p] = *reinterpret_cast<const code_t*>(cb + p * c_pixel + c_lane);
    }
  };
  auto stage = [&](const code_t (&w)[2], int buf) __attribute__((always_inline)) {
    float v[2][4];
#pragma unroll
    for (int p = 0; p < 2; ++p)
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const uint32_t code = ((uint32_t)w[p] >> (K * e)) & ((1u << K) - 1u);
        v[p][e] = fmaxf(stp[e] * ((float)code + offh[e]), 0.0f);   // Eq. 10, then the ReLU
      }
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const __bf16 lo = (__bf16)v[0][e], hi = (__bf16)v[1][e];
      AL[buf][q >> 2][e][cg][q & 3] = (uint32_t)__builtin_bit_cast(uint16_t, lo) | ((uint32_t)__builtin_bit_cast(uint16_t, hi) << 16);
    }
  };

  // ---- operands.  dy: the lane's pixels are 8 lk .. 8 lk + 7 of the chunk, its channels co0 + 4 li ..
  uint32_t d_lane = 4u * (uint32_t)(8 * lk * g.Cout + co0 + 4 * li);
  const size_t d_chunk = (size_t)PB_PX * g.Cout;                 // floats of dy per chunk
  floatx4 dyr[4][8];                                             // ring of four chunks: [slot][pixel]
  auto load_dy = [&](int slot, int c) __attribute__((always_inline)) {
    const float* db = dy + (size_t)(c < chunks ? c : chunks - 1) * d_chunk;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      asm volatile("" : "+v"(d_lane));
      dyr[slot][i] = *reinterpret_cast<const floatx4*>(reinterpret_cast<const char*>(db + (size_t)i * g.Cout) + d_lane);
    }
  };
  // (one set: the next chunk's fragments are read after this chunk's MFMAs have been issued)
  bf16x8_t af[4];                                                // [e]: eight pixels of channel 4 li + e
  auto read_a = [&](int buf) __attribute__((always_inline)) {
#pragma unroll
    for (int e = 0; e < 4; ++e) af[e] = *reinterpret_cast<const bf16x8_t*>(&AL[buf][lk][e][li][0]);
  };

  floatx4 acc[4][4];   // [e][j]: rows = input channels 4 (4 lk + r) + e, column = output channel 4 li + j
#pragma unroll
  for (int e = 0; e < 4; ++e)
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[e][j] = floatx4{0.f, 0.f, 0.f, 0.f};

  // One chunk, ring slot SLOT (= chunk index mod 4 from the block's first): convert its dy, contract,
  // ask for dy of the chunk four ahead into the slot, dequantize the next chunk into the other buffer
  // and ask for the codes of the chunk four after that one.  One barrier per chunk: the buffer written here was
  // last read in the previous chunk, before that chunk's barrier.
  auto chunk = [&](auto slot_c, int c) __attribute__((always_inline)) {
    constexpr int SLOT = decltype(slot_c)::value, PAR = SLOT & 1;
    // (the fences keep the phases in this order: left alone, the scheduler starts on the code words of
    // later chunks at the top of the loop and waits for every load in flight to get at them)
    __builtin_amdgcn_sched_barrier(0);
    bf16x8_t d[4];
#pragma unroll
    for (int j = 0; j < 4; ++j)
      d[j] = bf16x8_t{(__bf16)dyr[SLOT][0][j], (__bf16)dyr[SLOT][1][j], (__bf16)dyr[SLOT][2][j], (__bf16)dyr[SLOT][3][j],
                      (__bf16)dyr[SLOT][4][j], (__bf16)dyr[SLOT][5][j], (__bf16)dyr[SLOT][6][j], (__bf16)dyr[SLOT][7][j]};
    // (the converted operands exist before the slot is asked for again: otherwise the conversions sink
    // below the loads and the old contents of the slot are copied out of their way first)
#pragma unroll
    for (int j = 0; j < 4; ++j) asm volatile("" : "+v"(d[j]));
    __builtin_amdgcn_sched_barrier(0);
    load_dy(SLOT, c + 4);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int e = 0; e < 4; ++e)
#pragma unroll
      for (int j = 0; j < 4; ++j)
        asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(acc[e][j]) : "v"(af[e]), "v"(d[j]));
    __builtin_amdgcn_sched_barrier(0);
    stage(cw[(SLOT + 1) & 3], PAR ^ 1);
    __builtin_amdgcn_sched_barrier(0);
    load_codes(cw[(SLOT + 1) & 3], c + 5);
    __syncthreads();
    read_a(PAR ^ 1);
    __builtin_amdgcn_sched_barrier(0);
  };

  if (c_begin < c_end) {
#pragma unroll
    for (int t = 0; t < 4; ++t) load_codes(cw[t], c_begin + t);
#pragma unroll
    for (int t = 0; t < 4; ++t) load_dy(t, c_begin + t);
    stage(cw[0], 0);
    load_codes(cw[0], c_begin + 4);
    __syncthreads();
    read_a(0);
    const int n = c_end - c_begin;
    int i = 0;
    for (; i + 3 < n; i += 4) {
      chunk(std::integral_constant<int, 0>{}, c_begin + i);
      chunk(std::integral_constant<int, 1>{}, c_begin + i + 1);
      chunk(std::integral_constant<int, 2>{}, c_begin + i + 2);
      chunk(std::integral_constant<int, 3>{}, c_begin + i + 3);
    }
    if (i < n) chunk(std::integral_constant<int, 0>{}, c_begin + i);
    if (i + 1 < n) chunk(std::integral_constant<int, 1>{}, c_begin + i + 1);
    if (i + 2 < n) chunk(std::integral_constant<int, 2>{}, c_begin + i + 2);
  }
  // the MFMAs' results are read below by instructions the compiler does not know to depend on a
  // matrix-core result: more wait states than the longest such hazard, tied to the accumulator written last
  asm volatile("s_nop 15\n\ts_nop 15" : "+a"(acc[3][3]));
  float* out = dst + (size_t)split * g.Cin * g.Cout;
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    const int ci = ci0 + 4 * (4 * lk + r);
#pragma unroll
    for (int e = 0; e < 4; ++e)
      *reinterpret_cast<floatx4*>(out + (size_t)(ci + e) * g.Cout + co0 + 4 * li) =
          floatx4{acc[e][0][r], acc[e][1][r], acc[e][2][r], acc[e][3][r]};
  }
}

int rows_wgrad_splits(const ConvGeom& g) {
  const int tiles = (g.Cin / PW_CI) * (g.Cout / PW_CO);
  return tiles <= 256 ? 256 / tiles : 0;
}

// ---- 1x1 stride-1 convolutions with everything but the weights' and activations' way in registers ----
// Eq. 4 (mode 0) and the second half of Eq. 5 (mode 1, optionally with the Eq. 6-7 sums) of a 1x1 layer
// are one matrix product of the [rows = N H W] x [Cg] activation with the weights.  One block takes up to
// 208 rows (13 MFMA tiles) and keeps its whole output tile in accumulator registers, as the image-resident
// kernels above do; with one filter tap no operand is used twice by a block, so nothing goes through LDS
// in the main loop: a wave loads its activation fragments (the lane's row, four consecutive channels: 16
// bytes) and weights straight from global memory into the registers the MFMAs read, a k-step (16 channels,
// 16 x MT MFMAs per wave) ahead.  The four waves split the contraction (which therefore has to be long:
// 512 channels and more) and add their partial tiles through LDS at the end in a fixed order; a block
// covers 64 output channels.  Per k-step MT + 16 (MT + 4 for the gradient) loads and a 16-register copy
// against 16 x MT MFMAs, no barrier.
template <int MODE, int MT, int EPI>
__global__ __launch_bounds__(kThreads, 1) void rows_f32_kernel(const float* __restrict__ in,
                                                               const float* __restrict__ wgt, const float* skip,
                                                               float* out, double* __restrict__ sums,
                                                               const uint8_t* __restrict__ codes,
                                                               const float* __restrict__ stats, ConvGeom g, int RB) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const int Cg = MODE == 0 ? g.Cin : g.Cout;   // contraction channels (multiple of 64)
  const int Ng = MODE == 0 ? g.Cout : g.Cin;   // output channels
  constexpr int NB = 64;                       // output channels per block
  const int64_t M = (int64_t)g.N * g.H * g.W;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int li = lane & 15, lk = lane >> 4;
  // ids 8 apart share an XCD and its L2: the blocks of one row block (same input) run there
  const int nblk = Ng / NB;
  const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
  const int rb = (slot / nblk) * 8 + xcd;
  const int n0 = (slot % nblk) * NB;
  const int64_t row0 = (int64_t)rb * RB;
  if (row0 >= M) return;
  const int rows = M - row0 < RB ? (int)(M - row0) : RB;

  // the lane's rows: byte offsets of (row, channels 4 lk ..) from the block's first row; rows past the
  // block repeat its last row and are never stored
  uint32_t a_lane[MT];
#pragma unroll
  for (int i = 0; i < MT; ++i) {
    const int m = 16 * i + li;
    a_lane[i] = 4u * (uint32_t)((m < rows ? m : rows - 1) * Cg + 4 * lk);
  }
  const char* const abase = reinterpret_cast<const char*>(in + row0 * Cg);
  uint32_t w_lane[4];
#pragma unroll
  for (int t = 0; t < 4; ++t)
    w_lane[t] = 4u * (MODE == 0 ? (uint32_t)((4 * lk + t) * g.Cout + li) : (uint32_t)(li * g.Cout + 4 * lk));
  // acc[jj]: the channel tile (wave + jj) % 4 of the block's 64, so that a wave's own tile (the one it
  // finishes) is acc[0] whatever the wave
  auto ntile = [&](int jj) __attribute__((always_inline)) { return n0 + 16 * ((wave + jj) & 3); };
  // k-steps of 16 channels; part p of 8 of a k-step's weights (forward: two rows of one channel tile;
  // gradient: parts 0, 2, 4, 6 a whole tile) or, p < 0, all of them
  auto load_w = [&](floatx4 (&dst)[4], int ks, int p) __attribute__((always_inline)) {
    const int c0 = 16 * ks;
#pragma unroll
    for (int jj = 0; jj < 4; ++jj) {
      if (p >= 0 && (p >> 1) != jj) continue;
      const int nt = ntile(jj);
      if (MODE == 0) {
        const char* wb = reinterpret_cast<const char*>(wgt + ((size_t)c0 * g.Cout + nt));
#pragma unroll
        for (int t = 0; t < 4; ++t) {
          if (p >= 0 && (t >> 1) != (p & 1)) continue;
          // (opaque to the optimizer: the 32-bit offset stays a register operand of the load beside
          // the scalar base instead of being widened to a 64-bit address outside the loop)
          asm volatile("" : "+v"(w_lane[t]));
          dst[jj][t] = *reinterpret_cast<const float*>(wb + w_lane[t]);
        }
      } else {
        if (p >= 0 && (p & 1) != 0) continue;
        const char* wb = reinterpret_cast<const char*>(wgt + ((size_t)nt * g.Cout + c0));
        asm volatile("" : "+v"(w_lane[0]));
        dst[jj] = *reinterpret_cast<const floatx4*>(wb + w_lane[0]);
      }
    }
  };
  auto load_a = [&](floatx4& dst, int i, int ks) __attribute__((always_inline)) {
    const char* ab = abase + (size_t)ks * 64;
    asm volatile("" : "+v"(a_lane[i]));
    dst = *reinterpret_cast<const floatx4*>(ab + a_lane[i]);
  };

  floatx4 acc[4][MT];
#pragma unroll
  for (int jj = 0; jj < 4; ++jj)
#pragma unroll
    for (int i = 0; i < MT; ++i) acc[jj][i] = floatx4{0.f, 0.f, 0.f, 0.f};

  const int nks = Cg / 16;
  const int ks_begin = wave * nks / 4, ks_end = (wave + 1) * nks / 4;
  floatx4 w0[4], w1[4], a[MT];
  load_w(w0, ks_begin, -1);
#pragma unroll
  for (int i = 0; i < MT; ++i) load_a(a[i], i, ks_begin);
  auto kstep = [&](const floatx4 (&wc)[4], floatx4 (&wn)[4], int ks) __attribute__((always_inline)) {
    const int kn = ks + 1 < ks_end ? ks + 1 : ks;   // the last k-step asks for its own operands again: no branch
    __builtin_amdgcn_sched_barrier(0);
    // the order below is the schedule: a tile's 16 MFMAs (MFMA t contracts channels 4 lk + t), then
    // the request for its next fragment and a part of the next k-step's weights
#pragma unroll
    for (int i = 0; i < MT; ++i) {
#pragma unroll
      for (int t = 0; t < 4; ++t)
#pragma unroll
        for (int jj = 0; jj < 4; ++jj)
          asm volatile("v_mfma_f32_16x16x4_f32 %0, %1, %2, %0" : "+a"(acc[jj][i]) : "v"(wc[jj][t]), "v"(a[i][t]));
      load_a(a[i], i, kn);
      constexpr int PP = (8 + MT - 1) / MT;   // parts per tile: all eight within the MT tiles
#pragma unroll
      for (int q = 0; q < PP; ++q)
        if (i * PP + q < 8) load_w(wn, kn, i * PP + q);
      __builtin_amdgcn_sched_barrier(0);
    }
  };
  // (one k-step per iteration and a copy of the 16 weight registers: with two k-steps per iteration
  // and the two sets taking turns the compiler keeps both iterations' fragments apart and spills)
  for (int ks = ks_begin; ks < ks_end; ++ks) {
    kstep(w0, w1, ks);
#pragma unroll
    for (int jj = 0; jj < 4; ++jj) w0[jj] = w1[jj];
  }
  // the last MFMAs' results are read below by instructions the compiler does not know to depend
  // on a matrix-core result: more wait states than the longest such hazard (18)
  asm volatile("s_nop 15\n\ts_nop 15");

  // ---- epilogue of one 16-channel tile: shortcut, store, per-channel sums (row rb of [blocks][2][Ng])
  auto finish = [&](floatx4 (&v)[MT], int nt) __attribute__((always_inline)) {
    const int nch = nt + 4 * lk;
    size_t o[MT];   // element offset of the lane's four channels; rows past the block: its last row's
#pragma unroll
    for (int i = 0; i < MT; ++i) {
      const int m = 16 * i + li;
      o[i] = (size_t)(row0 + (m < rows ? m : rows - 1)) * Ng + nch;
    }
    double s1[4] = {0.0, 0.0, 0.0, 0.0}, s2[4] = {0.0, 0.0, 0.0, 0.0};
    if (MODE == 0) {
      if (skip != nullptr) {
        floatx4 sv[MT];
#pragma unroll
        for (int i = 0; i < MT; ++i) sv[i] = *reinterpret_cast<const floatx4*>(skip + o[i]);
#pragma unroll
        for (int i = 0; i < MT; ++i) {
          v[i][0] += sv[i][0]; v[i][1] += sv[i][1]; v[i][2] += sv[i][2]; v[i][3] += sv[i][3];
        }
      }
#pragma unroll
      for (int i = 0; i < MT; ++i) {
        if (16 * i + li < rows) {
          *reinterpret_cast<floatx4*>(out + o[i]) = v[i];
          if (sums != nullptr) {
#pragma unroll
            for (int r = 0; r < 4; ++r) {
              s1[r] += (double)v[i][r];
              s2[r] += (double)v[i][r] * (double)v[i][r];
            }
          }
        }
      }
    } else {
      if constexpr (EPI != 0) {
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
          if (16 * i + li < rows) {
#pragma unroll
            for (int r = 0; r < 4; ++r) {
              const uint32_t code = (cw[i] >> (EPI * r)) & ((1u << EPI) - 1u);
              const int32_t j = (int32_t)code - (1 << (EPI - 1)) + fbv[r];
              const float a2t = st4[r] * ((float)j + 0.5f);        // Eq. 10
              const float da2 = a2t > 0.0f ? v[i][r] : 0.0f;       // Eq. 6
              const float a1t = (a2t - bt4[r]) * ig[r];            // inverse of Eq. 2
              s1[r] += (double)da2;
              s2[r] += (double)a1t * (double)da2;
            }
          }
        }
      }
#pragma unroll
      for (int i = 0; i < MT; ++i)
        if (16 * i + li < rows) *reinterpret_cast<floatx4*>(out + o[i]) = v[i];
    }
    if (sums != nullptr && (MODE == 0 || EPI != 0)) {
#pragma unroll
      for (int r = 0; r < 4; ++r) {
#pragma unroll
        for (int d = 1; d < 16; d <<= 1) {
          s1[r] += __shfl_xor(s1[r], d, 64);
          s2[r] += __shfl_xor(s2[r], d, 64);
        }
      }
      if (li == 0) {
        double* row = sums + (size_t)rb * 2 * Ng;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          row[nch + r] = s1[r];
          row[Ng + nch + r] = s2[r];
        }
      }
    }
  };

  // the four partial tiles -> one: wave w sends acc[jj], jj = 1..3, to the owner (w + jj) % 4, which
  // adds what it receives in the order jj = 1, 2, 3 of the senders
#pragma unroll
  for (int jj = 1; jj < 4; ++jj) {
    const int owner = (wave + jj) & 3;
    unsigned char* dst = smem + (size_t)((owner * 3 + (jj - 1)) * MT) * 1024 + lane * 16;
#pragma unroll
    for (int i = 0; i < MT; ++i) *reinterpret_cast<floatx4*>(dst + i * 1024) = acc[jj][i];
  }
  __syncthreads();
  floatx4 v[MT];
#pragma unroll
  for (int i = 0; i < MT; ++i) {
    v[i] = acc[0][i];
#pragma unroll
    for (int q = 0; q < 3; ++q) {
      const floatx4 t = *reinterpret_cast<const floatx4*>(smem + (size_t)((wave * 3 + q) * MT + i) * 1024 + lane * 16);
      v[i][0] += t[0]; v[i][1] += t[1]; v[i][2] += t[2]; v[i][3] += t[3];
    }
  }
  finish(v, ntile(0));
}

// rows per block and number of row blocks of the 1x1 kernel: whole images when one fits 13 tiles
// and the batch then fills the chip better (64 images x 4 channel blocks = 256), else 208 rows
struct RowsPlan {
  int RB, nrb, mt;
};
bool rows_plan(const ConvGeom& g, int mode, RowsPlan& p) {
  const int Cg = mode == 0 ? g.Cin : g.Cout, Ng = mode == 0 ? g.Cout : g.Cin;
  if (g.R != 1 || g.S != 1 || g.stride != 1 || g.pad != 0) return false;
  if (Cg % 64 != 0 || Ng % 64 != 0) return false;
  const int64_t M = (int64_t)g.N * g.H * g.W;
  const int64_t e_in = M * g.Cin, e_out = M * g.Cout;
  if (e_in >= ((int64_t)1 << 30) || e_out >= ((int64_t)1 << 30)) return false;   // 32-bit byte offsets
  // long contractions only (the waves split them): for 256 channels neither each wave reading every
  // fragment itself (256 output channels per block) nor a split in two (128 per block) measured
  // faster than the LDS-tiled kernel
  if (Cg < 512) return false;
  const int nb = 64;
  const int HW = g.H * g.W;
  p.mt = 13;
  p.RB = HW <= 208 && HW > 104 ? HW : 208;
  p.nrb = (int)((M + p.RB - 1) / p.RB);
  if (p.nrb > kMaxPartialBlocks) return false;
  // built for about one block per compute unit: with much fewer (or many more small ones) the tiled
  // kernels are faster
  const int64_t blocks = (int64_t)p.nrb * (Ng / nb);
  return blocks >= 224 && blocks <= 2048;
}

int image_mt(const ConvGeom& g) {
  const int tiles = (g.H * g.W + 15) / 16;
  return tiles <= 4 ? 4 : tiles <= 8 ? 8 : tiles <= 13 ? 13 : 0;
}

size_t image_lds_bytes(const ConvGeom& g, int mode) {
  const int Cg = mode == 0 ? g.Cin : g.Cout;
  const int PC = Cg < IMG_PC ? Cg : IMG_PC;
  const size_t patch = (size_t)2 * (g.H + 2) * (g.W + 2) * (4 * PC + 16);
  const size_t red = (size_t)12 * image_mt(g) * 1024;
  return patch > red ? patch : red;
}

template <int MODE, int EPI>
int launch_mt(hipStream_t st, const ConvGeom& g, const float* in, const float* w, const float* skip, float* out,
              double* sums, const uint8_t* codes, const float* stats) {
  const int Ng = MODE == 0 ? g.Cout : g.Cin;
  const int mt = image_mt(g);
  const size_t lds = image_lds_bytes(g, MODE);
  const unsigned grid = (unsigned)((g.N + 7) / 8 * 8 * (Ng / IMG_NB));
  auto kern = mt == 4 ? image_f32_kernel<MODE, 4, EPI> : mt == 8 ? image_f32_kernel<MODE, 8, EPI>
                                                                  : image_f32_kernel<MODE, 13, EPI>;
  if (int e = allow_full_lds(reinterpret_cast<const void*>(kern))) return e;
  kern<<<grid, kThreads, lds, st>>>(in, w, skip, out, sums, codes, stats, g);
  return hip_status();
}

}  // namespace

bool image_f32_supported(const ConvGeom& g, int mode) {
  const int Cg = mode == 0 ? g.Cin : g.Cout, Ng = mode == 0 ? g.Cout : g.Cin;
  if (g.R != 3 || g.S != 3 || g.stride != 1 || g.pad != 1) return false;
  if (Cg < 16 || (Cg < IMG_PC ? (Cg & (Cg - 1)) != 0 : Cg % IMG_PC != 0) || Ng % IMG_NB != 0) return false;
  if (image_mt(g) == 0 || g.N > kMaxPartialBlocks) return false;
  // one block per compute unit and round is what the kernel is built for: with fewer blocks than
  // most of a 256-unit round the tiled kernels are faster (measured: 64 images x 128 channels, 128
  // blocks, 64 us against 44)
  if ((int64_t)g.N * (Ng / IMG_NB) < 224) return false;
  if (image_lds_bytes(g, mode) > (size_t)160 * 1024) return false;
  const int64_t e_in = (int64_t)g.N * g.H * g.W * g.Cin, e_out = (int64_t)g.N * g.Ho * g.Wo * g.Cout;
  return e_in < ((int64_t)1 << 31) && e_out < ((int64_t)1 << 31);
}

int launch_image_f32(hipStream_t st, const ConvGeom& g, int mode, const float* in, const float* w,
                     const float* skip, float* out, double* sums) {
  if (!image_f32_supported(g, mode)) return ABL_ERR_SHAPE;
  if (mode == 0) return launch_mt<0, 0>(st, g, in, w, skip, out, sums, nullptr, nullptr);
  return launch_mt<1, 0>(st, g, in, w, nullptr, out, nullptr, nullptr, nullptr);
}

int launch_image_dgrad_reduce(hipStream_t st, const ConvGeom& g, int K, const float* dy, const float* w,
                              const void* packed, const void* stats, float* da3, double* partial) {
  if (!image_f32_supported(g, 1) || (K != 4 && K != 8)) return ABL_ERR_SHAPE;
  const uint8_t* codes = static_cast<const uint8_t*>(packed);
  const float* sp = static_cast<const float*>(stats);
  if (K == 4) return launch_mt<1, 4>(st, g, dy, w, nullptr, da3, partial, codes, sp);
  return launch_mt<1, 8>(st, g, dy, w, nullptr, da3, partial, codes, sp);
}

int image_wgrad_copies(const ConvGeom& g, int K) {
  if (g.R != 3 || g.S != 3 || g.stride != 1 || g.pad != 1 || (K != 4 && K != 8)) return 0;
  if (g.W != 14 || g.H < 2 || g.H > 14 || (g.H * g.W) % 4 != 0) return 0;
  if (g.Cin % WG_CI != 0 || g.Cout % WG_CO != 0) return 0;
  const int s = image_wgrad_splits(g);
  if ((int64_t)s * (g.Cin / WG_CI) * (g.Cout / WG_CO) < 224) return 0;   // built for one block per compute unit
  const int64_t e_in = (int64_t)g.N * g.H * g.W * g.Cin, e_out = (int64_t)g.N * g.Ho * g.Wo * g.Cout;
  if (e_in >= ((int64_t)1 << 31) || e_out >= ((int64_t)1 << 31)) return 0;
  return s;
}

int launch_image_wgrad(hipStream_t st, const ConvGeom& g, int K, bool bf16, const void* packed, const float* stats,
                       const float* dy, float* copies) {
  const int s = image_wgrad_copies(g, K);
  if (s == 0) return ABL_ERR_SHAPE;
  const size_t lds = bf16 ? (size_t)((g.H + 2) * (g.W + 2) + 2) * WG_AP + (size_t)g.H * (g.W + 2) * WG_DP
                          : (size_t)(g.H + 2) * (g.W + 2) * WG_AP + (size_t)g.H * g.W * WG_DP;
  const unsigned grid = (unsigned)(s * (g.Cin / WG_CI) * (g.Cout / WG_CO));
  auto kern = bf16 ? (K == 4 ? image_wgrad_kernel<4, 14, true> : image_wgrad_kernel<8, 14, true>)
                   : (K == 4 ? image_wgrad_kernel<4, 14> : image_wgrad_kernel<8, 14>);
  if (int e = allow_full_lds(reinterpret_cast<const void*>(kern))) return e;
  kern<<<grid, kThreads, lds, st>>>(static_cast<const uint8_t*>(packed), stats, dy, copies, g, s);
  return hip_status();
}

int rows_wgrad_copies(const ConvGeom& g, int K, bool bf16) {
  if (g.R != 1 || g.S != 1 || g.stride != 1 || g.pad != 0 || (K != 4 && K != 8)) return 0;
  if (g.Cin % PW_CI != 0 || g.Cout % PW_CO != 0) return 0;
  const int64_t M = (int64_t)g.N * g.H * g.W;
  if (M % (bf16 ? PB_PX : PW_PX) != 0) return 0;
  const int s = rows_wgrad_splits(g);
  if ((int64_t)s * (g.Cin / PW_CI) * (g.Cout / PW_CO) < 224) return 0;   // built for one block per compute unit
  if (M / PW_PX < (int64_t)16 * s) return 0;                             // ... with a long share of the pixels each
  if (M * g.Cin >= ((int64_t)1 << 30) || M * g.Cout >= ((int64_t)1 << 30)) return 0;   // 32-bit byte offsets
  return s;
}

int launch_rows_wgrad(hipStream_t st, const ConvGeom& g, int K, bool bf16, const void* packed, const float* stats,
                      const float* dy, float* copies) {
  const int s = rows_wgrad_copies(g, K, bf16);
  if (s == 0) return ABL_ERR_SHAPE;
  const unsigned grid = (unsigned)(s * (g.Cin / PW_CI) * (g.Cout / PW_CO));
  auto kern = bf16 ? (K == 4 ? rows_wgrad_bf16_kernel<4> : rows_wgrad_bf16_kernel<8>)
                   : (K == 4 ? rows_wgrad_kernel<4> : rows_wgrad_kernel<8>);
  kern<<<grid, kThreads, 0, st>>>(static_cast<const uint8_t*>(packed), stats, dy, copies, g, s);
  return hip_status();
}

namespace {
template <int MODE, int EPI>
int launch_rows(hipStream_t st, const ConvGeom& g, const float* in, const float* w, const float* skip, float* out,
                double* sums, const uint8_t* codes, const float* stats) {
  RowsPlan p;
  if (!rows_plan(g, MODE, p)) return ABL_ERR_SHAPE;
  const int Ng = MODE == 0 ? g.Cout : g.Cin;
  const unsigned grid = (unsigned)((p.nrb + 7) / 8 * 8 * (Ng / 64));
  auto kern = rows_f32_kernel<MODE, 13, EPI>;
  if (int e = allow_full_lds(reinterpret_cast<const void*>(kern))) return e;
  kern<<<grid, kThreads, (size_t)12 * 13 * 1024, st>>>(in, w, skip, out, sums, codes, stats, g, p.RB);
  return hip_status();
}
}  // namespace

int rows_f32_blocks(const ConvGeom& g, int mode) {
  RowsPlan p;
  return rows_plan(g, mode, p) ? p.nrb : 0;
}

int launch_rows_f32(hipStream_t st, const ConvGeom& g, int mode, const float* in, const float* w, const float* skip,
                    float* out, double* sums) {
  if (mode == 0) return launch_rows<0, 0>(st, g, in, w, skip, out, sums, nullptr, nullptr);
  return launch_rows<1, 0>(st, g, in, w, nullptr, out, nullptr, nullptr, nullptr);
}

int launch_rows_dgrad_reduce(hipStream_t st, const ConvGeom& g, int K, const float* dy, const float* w,
                             const void* packed, const void* stats, float* da3, double* partial) {
  const uint8_t* codes = static_cast<const uint8_t*>(packed);
  const float* sp = static_cast<const float*>(stats);
  if (K == 4) return launch_rows<1, 4>(st, g, dy, w, nullptr, da3, partial, codes, sp);
  if (K == 8) return launch_rows<1, 8>(st, g, dy, w, nullptr, da3, partial, codes, sp);
  return ABL_ERR_SHAPE;
}

}  // namespace abl
