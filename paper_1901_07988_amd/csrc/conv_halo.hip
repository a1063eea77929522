// Stride-1 convolutions (Eq. 4 forward, Eq. 5 gradient to the input) for filters larger than
// 1x1 on gfx950, with the input tile staged ONCE in LDS.
//
// An implicit GEMM that gathers its A operand tap by tap re-reads every input pixel R*S times
// from L2.  Here a block owns a tile of TI images x TH x TW output pixels; for each chunk of
// 16 input channels it stages the (TH+R-1) x (TW+S-1) input patch (zero filled outside the
// image) and the R*S*16 x BN slice of the weights, and every filter tap then reads its
// shifted view of that patch straight from LDS as the MFMA A operand
// (v_mfma_f32_16x16x4_f32; one ds_read_b128 = four k-steps).  An M-tile is 16 consecutive
// output pixels of the flattened tile, so tiles of any shape fill the matrix cores.
//
// MODE 0 forward : out[n,h,w,co] = sum in[n, h+r-pad, w+s-pad, ci] W[r,s,ci,co]
// MODE 1 dgrad   : out[n,h,w,ci] = sum in[n, h+pad-r, w+pad-s, co] W[r,s,ci,co]   (in = dy)

#include "abl_internal.h"

// the fused forward evaluates Eq. 1-3 and Eq. 9 here: one rounded fp32 operation at a time
#pragma clang fp contract(off)

// Scheduling fence that neither global memory nor matrix instructions may cross (vector, scalar and LDS ones may): keeps
// a prefetch where the source puts it, a whole tap or chunk of matrix work ahead of its use,
// instead of letting the scheduler sink it to the end of the loop body.
#define PIN_VMEM()                                      \
  do {                                                  \
    if (PIN) __builtin_amdgcn_sched_barrier(0x786);     \
  } while (0)

namespace abl {
namespace {


constexpr int kThreads = 256;
constexpr int PS = 20;     // floats per staged pixel: 16 channels + 4 pad (conflict-free b128 reads)
constexpr int AMAX = 6;    // float4 slots per thread for the input patch (<= 384 staged pixels)

// A step of a fixed number of cells through a [.. x height x width] box, split into digits
// (w < width, h < height), so that advancing a position carries at most once per digit.
struct BoxStep {
  int w, h, ti;
};

struct HaloPlan {
  int TI, TH, TW;                 // output tile: images, rows, cols
  int HH, HW;                     // staged patch rows, cols
  int tiles_i, tiles_h, tiles_w;  // tiles per batch / image height / image width
  int npix;                       // TI*TH*TW
  int mtiles;                     // ceil(npix / 16)
  int variant;                    // index into the instantiation table
  int threads;                    // threads per block of that variant (256 or 512)
  int bn;                         // output channels per block
  unsigned inv_HW, inv_HH, inv_TW, inv_TH;  // ceil(2^32 / d): exact quotient x/d while x*d < 2^32
  unsigned inv_tiles_w, inv_tiles_h;
  unsigned nblk_n, inv_nblk_n;    // blocks along the output channels
  BoxStep a_step;                 // threads/4 patch pixels further, as (cols, rows, images) of the patch
  BoxStep m_step;                 // 16 tile pixels further, as (cols, rows, images) of the tile
  unsigned lds_bytes;
  int pack_pad;                   // zero bytes after the last code (fused forward only)
};

// Optional per-channel reduction in the epilogue; one partial row [2][channels] per pixel tile.
//   forward (MODE 0): sum(y), sum(y^2) of the output          -> the next layer's Eq. 1 statistics
//   dgrad   (MODE 1): sum(dA2), sum(A1~ dA2) with the ReLU mask and A1~ rebuilt from the layer's
//                     K-bit codes (Eq. 6, Eq. 7)               -> first pass of the BN backward
struct EpiReduce {
  double* partial;        // nullptr: no reduction
  const uint8_t* codes;   // dgrad only: packed A2 of the layer
  int K;
};

// idx -> (ti, h, w) of a [.. x height x width] box, divisions by multiplication with
// inv = ceil(2^32 / d) (d = 1 has none).  EAGER: the products are formed unconditionally - as
// one arm of a conditional each drags the load of its `inv` from the argument block into a branch
// of its own, which the small 16-channel kernels pay for in set-up time; the larger variants
// measured faster with the conditional form.
template <bool EAGER = false>
__device__ inline void split3(int idx, int width, unsigned inv_w, int height, unsigned inv_h, int& ti, int& h,
                              int& w) {
  if constexpr (EAGER) {
    const int q0 = (int)__umulhi((unsigned)idx, inv_w);
    const int q = width == 1 ? idx : q0;
    w = idx - q * width;
    const int t0 = (int)__umulhi((unsigned)q, inv_h);
    ti = height == 1 ? q : t0;
    h = q - ti * height;
  } else {
    const int q = width == 1 ? idx : (int)__umulhi((unsigned)idx, inv_w);
    w = idx - q * width;
    ti = height == 1 ? q : (int)__umulhi((unsigned)q, inv_h);
    h = q - ti * height;
  }
}

template <bool EAGER = false>
__device__ inline unsigned udiv(unsigned x, unsigned d, unsigned inv) {
  if constexpr (EAGER) {
    const unsigned q = __umulhi(x, inv);
    return d == 1 ? x : q;
  } else {
    return d == 1 ? x : __umulhi(x, inv);
  }
}

__device__ inline void box_advance(int& w, int& h, int& ti, const BoxStep& s, int width, int height) {
  w += s.w;
  const int cw = w >= width ? 1 : 0;
  w -= cw ? width : 0;
  h += s.h + cw;
  const int ch = h >= height ? 1 : 0;
  h -= ch ? height : 0;
  ti += s.ti + ch;
}

// A block-uniform value held in a vector register.  The kernels below have more uniform state
// than scalar registers; what the unrolled per-lane index arithmetic uses again and again is
// moved to vector registers once, or the compiler re-loads it from the argument block (a
// scalar-cache round trip) at every use.
__device__ inline int in_vgpr(int x) {
  asm volatile("" : "+v"(x));
  return x;
}

// a * b + c for operands below 2^23 in magnitude (full-rate 24-bit multiplier)
__device__ inline int mad24(int a, int b, int c) { return __mul24(a, b) + c; }

// WAVES_N waves share the block's M-tiles and split its N-tiles; the other 4/WAVES_N groups
// split the M-tiles.  MT = M-tiles (16 pixels) per wave (upper bound, `mtiles` is the real
// count), NT = N-tiles (16 output channels) per wave.
// The MFMA computes the TRANSPOSED output tile: its first operand is the weight fragment (row =
// output channel), its second the pixel fragment (column = pixel), so a lane ends up with four
// consecutive channels of one pixel - one 16-byte store, one 16-byte shortcut load and one
// 16-/32-bit load of that pixel's codes in the epilogue.
// The weights are not staged: each lane fetches its fragment (four consecutive k of one output
// channel) straight from L2.  3x3 filters hold the fragments of all nine taps in registers: they
// are requested together with the first patch, and the registers of a tap are refilled for the
// next channel chunk right after its MFMAs (one tap of lookahead is about an L2 round trip: too
// little).  Other filter sizes fetch one tap ahead.  With more than 16 input channels the patch buffer is
// doubled and the next chunk's global loads are in flight during the MFMAs.
// FUSE = 0: `in` is the conv input.  FUSE = K (4 or 8, forward only): `in` is the layer input x;
// BatchNorm, scale & bias and ReLU (Eq. 1-3) are applied while the patch is staged, and the
// block that owns a pixel also writes its K-bit codes (Eq. 9).
// NW: waves per block (4 or 8).  Eight waves put two on every SIMD, so that one wave's waits (the
// LDS reads of a tap, the staging of the next chunk) are covered by the other's MFMAs where a
// shape yields only one block per compute unit (14x14 images: 64 tiles x 4 channel blocks).
template <int MODE, int WAVES_N, int MT, int NT, int TAPS9, bool BF16, int FUSE, int NW = 4>
__global__ __launch_bounds__(64 * NW) void halo_conv_kernel(const float* __restrict__ in,
                                                             const float* __restrict__ wgt, const float* skip,
                                                             float* out, ConvGeom g, HaloPlan p,
                                                             const float* __restrict__ stats,
                                                             void* __restrict__ packed, EpiReduce epi) {
  extern __shared__ __attribute__((aligned(16))) float lds[];
  // TAPS9 (3x3 filters only): 0 - weight fragments fetched one tap ahead; 1 - the fragments of all
  // nine taps held in registers and the epilogue's addresses and loads prepared during the first
  // wait (tiles of few M-tiles, where set-up and epilogue weigh most); 2 - fragments held only.
  constexpr bool HOLD9 = TAPS9 != 0, UNROLL_TAPS = TAPS9 == 1;
  // The pinned schedule of the widest unfused forward tile with held weights needs more than
  // 256 registers (one wave per SIMD instead of two): that variant keeps the free schedule.
  constexpr bool PIN = !(MODE == 0 && FUSE == 0 && MT >= 14 && TAPS9 == 2);
  constexpr int WAVES_M = NW / WAVES_N;
  constexpr int BN = WAVES_N * NT * 16;
  constexpr int TPB = 64 * NW;          // threads per block
  constexpr int AM = AMAX * 256 / TPB;  // patch slots per thread
  // Everything the set-up below reads from the argument block is requested here, in one batch
  // with one wait; left alone, the compiler fetches it field by field where it is first used and
  // the wave pays a scalar-cache round trip each time.
  asm volatile("" ::"s"(in), "s"(wgt), "s"(g.N), "s"(g.H), "s"(g.W), "s"(g.Cin), "s"(g.Cout), "s"(g.R), "s"(g.S),
               "s"(g.pad), "s"(g.Ho), "s"(g.Wo), "s"(p.TI), "s"(p.TH), "s"(p.TW), "s"(p.HH), "s"(p.HW),
               "s"(p.tiles_i), "s"(p.tiles_h), "s"(p.tiles_w), "s"(p.npix), "s"(p.inv_HW), "s"(p.inv_HH),
               "s"(p.inv_TW), "s"(p.inv_TH), "s"(p.inv_tiles_w), "s"(p.inv_tiles_h), "s"(p.nblk_n),
               "s"(p.inv_nblk_n));
  asm volatile("" ::"s"(p.a_step.w), "s"(p.a_step.h), "s"(p.a_step.ti), "s"(p.m_step.w), "s"(p.m_step.h),
               "s"(p.m_step.ti));
  const int taps = g.R * g.S;
  const int patch_floats = p.TI * p.HH * p.HW * PS;

  const int Hi = MODE == 0 ? g.H : g.Ho, Wi = MODE == 0 ? g.W : g.Wo;
  const int Hq = MODE == 0 ? g.Ho : g.H, Wq = MODE == 0 ? g.Wo : g.W;
  const int Cg = MODE == 0 ? g.Cin : g.Cout;
  const int Ng = MODE == 0 ? g.Cout : g.Cin;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int li = lane & 15, lk = lane >> 4;
  const int wave_m = wave / WAVES_N, wave_n = wave % WAVES_N;
  const int wn0 = wave_n * NT * 16;
  // M-tiles of this wave that hold pixels of the tile (wave-uniform): the others are skipped
  // where the variant has waves that would otherwise spend matrix-core time on padding (NW == 8)
  const int mt_left = p.mtiles - __builtin_amdgcn_readfirstlane(wave_m) * MT;
  const int mt_act = mt_left < 0 ? 0 : (mt_left < MT ? mt_left : MT);

  // ids 8 apart share an XCD (and its L2): the blocks that contract the same pixel tile against
  // different output-channel blocks run there back to back
  const unsigned slot = blockIdx.x >> 3;
  const unsigned sq = udiv<UNROLL_TAPS>(slot, p.nblk_n, p.inv_nblk_n);
  const int tile_id = sq * 8 + (blockIdx.x & 7);
  if (tile_id >= p.tiles_i * p.tiles_h * p.tiles_w) return;
  const unsigned t1 = udiv<UNROLL_TAPS>(tile_id, p.tiles_w, p.inv_tiles_w);
  const unsigned t2 = udiv<UNROLL_TAPS>(t1, p.tiles_h, p.inv_tiles_h);
  const int tw_i = tile_id - t1 * p.tiles_w, th_i = t1 - t2 * p.tiles_h;
  const int img0 = t2 * p.TI, h0 = th_i * p.TH, w0 = tw_i * p.TW;
  const int n0 = (slot - sq * p.nblk_n) * BN;
  // input coordinate of patch element (0,0)
  const int oh = h0 + (MODE == 0 ? -g.pad : g.pad - (g.R - 1));
  const int ow = w0 + (MODE == 0 ? -g.pad : g.pad - (g.S - 1));

  // global offsets (in floats, channel 0) of the patch elements this thread stages; -1 = zero
  // fill, -2 = past the end of the patch.  Kept as numbers in vector registers: per-slot
  // predicates would each occupy a pair of scalar registers for the whole kernel.
  const int totalA = p.TI * p.HH * p.HW * 4;
  int goff[AM];
  float4 ra[AM];
  // fused forward: bit j = slot j lies inside the block's pixel tile (not in its halo), where the
  // block writes codes
  unsigned ownbits = 0;
  {
    int ti, h, w;
    split3<UNROLL_TAPS>(tid >> 2, p.HW, p.inv_HW, p.HH, p.inv_HH, ti, h, w);
    // position in the input instead of in the patch
    ti += img0; h += oh; w += ow;
    const BoxStep step{in_vgpr(p.a_step.w), in_vgpr(p.a_step.h), in_vgpr(p.a_step.ti)};
    const int width = in_vgpr(p.HW), height = in_vgpr(p.HH);
    const int w_end = in_vgpr(ow + p.HW), h_end = in_vgpr(oh + p.HH);
    const int vN = in_vgpr(g.N), vHi = in_vgpr(Hi), vWi = in_vgpr(Wi), vCg = in_vgpr(Cg);
    const int vtotal = in_vgpr(totalA);
    const int vh0 = in_vgpr(h0), vw0 = in_vgpr(w0), vTH = in_vgpr(p.TH), vTW = in_vgpr(p.TW);
    const int c4 = 4 * (tid & 3);
#pragma unroll
    for (int j = 0; j < AM; ++j) {
      const int idx = tid + TPB * j;
      const bool ok = idx < vtotal && ti < vN && (unsigned)h < (unsigned)vHi && (unsigned)w < (unsigned)vWi;
      goff[j] = ok ? mad24(mad24(mad24(ti, vHi, h), vWi, w), vCg, c4) : (idx < vtotal ? -1 : -2);
      // the first chunk's load of a slot leaves as soon as its address is known, ahead of the
      // position arithmetic of the slots after it
      ra[j] = *reinterpret_cast<const float4*>(in + (ok ? goff[j] : 0));
      if (FUSE != 0) {
        const bool own = ok && (unsigned)(h - vh0) < (unsigned)vTH && (unsigned)(w - vw0) < (unsigned)vTW;
        ownbits |= (own ? 1u : 0u) << j;
      }
      // TPB/4 patch pixels further
      w += step.w;
      const bool cw = w >= w_end;
      w -= cw ? width : 0;
      h += step.h + (cw ? 1 : 0);
      const bool ch = h >= h_end;
      h -= ch ? height : 0;
      ti += step.ti + (ch ? 1 : 0);
    }
  }
  if (FUSE != 0 && blockIdx.x == 0 && tid < p.pack_pad)  // zero the tail of the last 128-byte row
    static_cast<uint8_t*>(packed)[((int64_t)g.N * g.H * g.W * g.Cin * FUSE) / 8 + tid] = 0;

  // per-channel constants of the 4 channels this thread stages (fused forward)
  float4 k_mean, k_rstd, k_gamma, k_beta, k_cq;
  int4 k_fb;
  int k_c0 = 0;
  auto fetch_a = [&](int c0, bool load_x) __attribute__((always_inline)) {
    // unconditional loads (lanes outside the image read element 0 and are zeroed): no branch
    // separates the loads, so all of them are in flight together
    if (load_x) {
#pragma unroll
      for (int j = 0; j < AM; ++j) {
        const bool ok = goff[j] >= 0;
        ra[j] = *reinterpret_cast<const float4*>(in + (ok ? goff[j] + c0 : 0));
      }
    }
    if (FUSE != 0) {
      const int c = c0 + 4 * (tid & 3);
      k_mean = *reinterpret_cast<const float4*>(stats + P_MEAN * g.Cin + c);
      k_rstd = *reinterpret_cast<const float4*>(stats + P_RSTD * g.Cin + c);
      k_gamma = *reinterpret_cast<const float4*>(stats + P_GAMMA * g.Cin + c);
      k_beta = *reinterpret_cast<const float4*>(stats + P_BETA * g.Cin + c);
      k_cq = *reinterpret_cast<const float4*>(stats + P_CQ * g.Cin + c);
      k_fb = *reinterpret_cast<const int4*>(reinterpret_cast<const int32_t*>(stats) + P_FB * g.Cin + c);
      k_c0 = c0;
    }
  };
  // Fused forward: all output-channel blocks of a pixel tile normalize the same patch; they take
  // turns over the 16-channel chunks in quantizing it and writing the codes, so that every block
  // has the same amount of vector work (were it all the first block's, the compute units holding
  // first blocks would finish last).
  const unsigned nblk_i = slot - sq * p.nblk_n;
  auto stage_a = [&](float* tileA) __attribute__((always_inline)) {
    const bool packs = FUSE != 0 && ((unsigned)k_c0 >> 4) % p.nblk_n == nblk_i;  // block-uniform
#pragma unroll
    for (int j = 0; j < AM; ++j) {
      const int idx = tid + TPB * j;
      if (goff[j] != -2) {
        const bool ok = goff[j] >= 0;
        float4 v = keep_if(ok, ra[j]);
        if (FUSE != 0) {
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
            a3[e] = (ok && a2[e] > 0.0f) ? a2[e] : 0.0f;  // Eq. 3; zero padding applies to A3
          }
          v = make_float4(a3[0], a3[1], a3[2], a3[3]);
          if (packs) {
            uint32_t word = 0;
#pragma unroll
            for (int e = 0; e < 4; ++e)
              word |= quant_code<(FUSE != 0 ? FUSE : 4)>(a2[e], cq[e], fb[e]) << ((FUSE != 0 ? FUSE : 4) * e);  // Eq. 9
            if ((ownbits >> j) & 1u) {
              const int64_t e0 = (int64_t)goff[j] + k_c0;  // flat element index of the first of 4 codes
              if (FUSE == 4) reinterpret_cast<uint16_t*>(packed)[e0 >> 2] = (uint16_t)word;
              else reinterpret_cast<uint32_t*>(packed)[e0 >> 2] = word;
            }
          }
        }
        *reinterpret_cast<float4*>(&tileA[(idx >> 2) * PS + 4 * (idx & 3)]) = v;
      }
    }
  };
  // Weight fragment of this lane for chunk c0, tap t: k = c0 + 4*lk .. +3 of output channel
  // n0 + wn0 + 16j + li.  Channels past the last one re-read the last one (never stored), so the
  // loaded registers go to the MFMAs untouched and no wait has to precede them.
  int boff[NT];  // lane part of the fragment address: (k = 4lk, its channel) of chunk 0, tap 0
#pragma unroll
  for (int j = 0; j < NT; ++j) {
    int n = n0 + wn0 + 16 * j + li;
    n = n < Ng ? n : Ng - 1;
    boff[j] = MODE == 0 ? mad24(4 * lk, g.Cout, n) : mad24(n, g.Cout, 4 * lk);
  }
  auto fetch_b = [&](int c0, int t, float4 (&bf)[NT]) __attribute__((always_inline)) {
    // uniform part: tap t, chunk c0
    const float* src = wgt + (int64_t)t * g.Cin * g.Cout + (MODE == 0 ? (int64_t)c0 * g.Cout : c0);
#pragma unroll
    for (int j = 0; j < NT; ++j) {
      if (MODE == 0) {
        const float* q = src + boff[j];
        bf[j] = make_float4(q[0], q[g.Cout], q[2 * g.Cout], q[3 * g.Cout]);
      } else {
        bf[j] = *reinterpret_cast<const float4*>(src + boff[j]);
      }
    }
  };

  constexpr int HELD = HOLD9 ? 9 : 1;
  float4 bw[HELD][NT], bnext[NT];
  fetch_a(0, false);  // chunk 0 of the patch was requested while the offsets were computed
#pragma unroll
  for (int t = 0; t < HELD; ++t) fetch_b(0, t, bw[t]);

  // LDS base of this lane's pixel in each of the wave's M-tiles
  int base[MT];
  const BoxStep mstep{in_vgpr(p.m_step.w), in_vgpr(p.m_step.h), in_vgpr(p.m_step.ti)};
  const int vTW = in_vgpr(p.TW), vTH = in_vgpr(p.TH), vnpix = in_vgpr(p.npix);
  {
    const int m0 = wave_m * MT * 16 + li;
    int ti, h, w;
    split3<UNROLL_TAPS>(m0, p.TW, p.inv_TW, p.TH, p.inv_TH, ti, h, w);
    const int vHH = in_vgpr(p.HH), vHW = in_vgpr(p.HW);
#pragma unroll
    for (int i = 0; i < MT; ++i) {
      // lanes past the last pixel read the first one (their results are not stored)
      base[i] = m0 + 16 * i < vnpix ? mad24(mad24(mad24(ti, vHH, h), vHW, w), PS, 4 * lk) : 4 * lk;
      box_advance(w, h, ti, mstep, vTW, vTH);
    }
  }

  floatx4 acc[NT][MT];  // acc[j][i][r]: pixel 16i + li of the wave, channel 16j + 4lk + r
#pragma unroll
  for (int j = 0; j < NT; ++j)
#pragma unroll
    for (int i = 0; i < MT; ++i) acc[j][i] = floatx4{0.f, 0.f, 0.f, 0.f};

  // The small (all-taps-in-registers) variants spend the wait for their first loads on the
  // epilogue's index arithmetic and request the shortcut values now: in the epilogue itself a
  // memory round trip would be exposed in every block.
  int eoff[UNROLL_TAPS ? MT : 1];
  unsigned epix = 0;
  float4 esv[UNROLL_TAPS ? MT : 1][NT];
  uint32_t ecw[UNROLL_TAPS ? MT : 1][NT];
  float4 r_step[NT], r_beta[NT], r_gm[NT];  // per-channel constants of the Eq. 6-7 epilogue
  int4 r_fb[NT];
  if constexpr (UNROLL_TAPS) {
    int e_ti, e_h, e_w;
    split3<true>(wave_m * MT * 16 + li, p.TW, p.inv_TW, p.TH, p.inv_TH, e_ti, e_h, e_w);
    const int vN = in_vgpr(g.N), vHq = in_vgpr(Hq), vWq = in_vgpr(Wq), vNg = in_vgpr(Ng);
    const int vimg0 = in_vgpr(img0), vh0 = in_vgpr(h0), vw0 = in_vgpr(w0);
    const int cb = n0 + wn0 + 4 * lk;
#pragma unroll
    for (int i = 0; i < MT; ++i) {
      const int m = wave_m * MT * 16 + 16 * i + li;
      const int n = vimg0 + e_ti, hq = vh0 + e_h, wq = vw0 + e_w;
      const bool pix_ok = m < vnpix && n < vN && hq < vHq && wq < vWq;
      eoff[i] = mad24(mad24(mad24(n, vHq, hq), vWq, wq), vNg, cb);  // element (pixel, channel cb)
      epix |= (pix_ok ? 1u : 0u) << i;
      box_advance(e_w, e_h, e_ti, mstep, vTW, vTH);
      if (skip != nullptr) {
#pragma unroll
        for (int j = 0; j < NT; ++j)
          esv[i][j] = *reinterpret_cast<const float4*>(skip + (pix_ok && cb + 16 * j < Ng ? eoff[i] + 16 * j : 0));
      }
      if (MODE == 1 && epi.partial != nullptr) {  // the codes behind the Eq. 6-7 sums
#pragma unroll
        for (int j = 0; j < NT; ++j) {
          const int el = pix_ok && cb + 16 * j < Ng ? eoff[i] + 16 * j : 0;
          ecw[i][j] = epi.K == 4 ? (uint32_t) * reinterpret_cast<const uint16_t*>(epi.codes + (el >> 1))
                                 : *reinterpret_cast<const uint32_t*>(epi.codes + el);
        }
      }
    }
    if (MODE == 1 && epi.partial != nullptr) {
#pragma unroll
      for (int j = 0; j < NT; ++j) {
        const int c = cb + 16 * j < Ng ? cb + 16 * j : 0;
        r_step[j] = *reinterpret_cast<const float4*>(stats + P_STEP * Ng + c);
        r_beta[j] = *reinterpret_cast<const float4*>(stats + P_BETA * Ng + c);
        r_gm[j] = *reinterpret_cast<const float4*>(stats + P_GAMMA * Ng + c);
        r_fb[j] = *reinterpret_cast<const int4*>(reinterpret_cast<const int32_t*>(stats) + P_FB * Ng + c);
      }
    }
  }

  stage_a(lds);
  __syncthreads();
  int buf = 0;
  for (int c0 = 0; c0 < Cg; c0 += 16) {
    const float* tileA = lds + buf * patch_floats;
    const bool more = c0 + 16 < Cg;
    // Loads for the next chunk are issued without a branch (the last chunk re-reads itself and
    // drops the result): the compiler can then count the loads in flight and wait only for the
    // ones a tap needs, instead of draining all of them at every branch target.
    const int cn = more ? c0 + 16 : c0;
    fetch_a(cn, true);
    PIN_VMEM();
    if (HOLD9) {
#pragma unroll
      for (int t = 0; t < 9; ++t) {
        const int r = t / 3, s = t % 3;
        const int rr = MODE == 0 ? r : 2 - r, ss = MODE == 0 ? s : 2 - s;
        const int aoff = (rr * p.HW + ss) * PS;
        float4 af[MT];
        if (NW == 8 && mt_act == MT - 1) {
          // the wave's last M-tile lies past the tile's pixels: neither read nor contracted
#pragma unroll
          for (int i = 0; i < MT - 1; ++i) af[i] = *reinterpret_cast<const float4*>(&tileA[base[i] + aoff]);
          af[MT - 1] = make_float4(0.f, 0.f, 0.f, 0.f);
          mma_k4_first<BF16, NT, MT, MT - 1>(bw[t], af, acc);
        } else {
#pragma unroll
          for (int i = 0; i < MT; ++i) af[i] = *reinterpret_cast<const float4*>(&tileA[base[i] + aoff]);
          mma_k4<BF16, NT, MT>(bw[t], af, acc);
        }
        // the same tap of the next chunk: a whole chunk of matrix work ahead of its use
        fetch_b(cn, t, bw[t]);
        PIN_VMEM();
      }
    } else {
      int r = 0, s = 0;
      for (int t = 0; t < taps; ++t) {
        {
          const bool last = t + 1 == taps;
          fetch_b(last ? cn : c0, last ? 0 : t + 1, bnext);
          PIN_VMEM();
        }
        const int rr = MODE == 0 ? r : g.R - 1 - r, ss = MODE == 0 ? s : g.S - 1 - s;
        const int aoff = (rr * p.HW + ss) * PS;
        float4 af[MT];
        if (NW == 8 && mt_act == MT - 1) {
          // the wave's last M-tile lies past the tile's pixels: neither read nor contracted
#pragma unroll
          for (int i = 0; i < MT - 1; ++i) af[i] = *reinterpret_cast<const float4*>(&tileA[base[i] + aoff]);
          af[MT - 1] = make_float4(0.f, 0.f, 0.f, 0.f);
          mma_k4_first<BF16, NT, MT, MT - 1>(bw[0], af, acc);
        } else {
#pragma unroll
          for (int i = 0; i < MT; ++i) af[i] = *reinterpret_cast<const float4*>(&tileA[base[i] + aoff]);
          mma_k4<BF16, NT, MT>(bw[0], af, acc);
        }
#pragma unroll
        for (int j = 0; j < NT; ++j) bw[0][j] = bnext[j];
        if (++s == g.S) { s = 0; ++r; }
      }
    }
    if (more) {
      stage_a(lds + (buf ^ 1) * patch_floats);
      __syncthreads();
      buf ^= 1;
    }
  }

  // epilogue: the lane holds channels cb + 16j .. +3 (cb = n0 + wn0 + 4lk) of pixel 16i + li
  const bool reduce = epi.partial != nullptr;
  const int cb = n0 + wn0 + 4 * lk;
  double s1[NT][4], s2[NT][4];
  float4 r_ig[NT];
#pragma unroll
  for (int j = 0; j < NT; ++j) {
#pragma unroll
    for (int r = 0; r < 4; ++r) s1[j][r] = s2[j][r] = 0.0;
    if (MODE == 1 && reduce) {
      if constexpr (!UNROLL_TAPS) {
        const int c = cb + 16 * j < Ng ? cb + 16 * j : 0;
        r_step[j] = *reinterpret_cast<const float4*>(stats + P_STEP * Ng + c);
        r_beta[j] = *reinterpret_cast<const float4*>(stats + P_BETA * Ng + c);
        r_gm[j] = *reinterpret_cast<const float4*>(stats + P_GAMMA * Ng + c);
        r_fb[j] = *reinterpret_cast<const int4*>(reinterpret_cast<const int32_t*>(stats) + P_FB * Ng + c);
      }
      r_ig[j] = make_float4(1.0f / r_gm[j].x, 1.0f / r_gm[j].y, 1.0f / r_gm[j].z, 1.0f / r_gm[j].w);
    }
  }
  int e_ti, e_h, e_w;
  split3<UNROLL_TAPS>(wave_m * MT * 16 + li, p.TW, p.inv_TW, p.TH, p.inv_TH, e_ti, e_h, e_w);
  const int vN = in_vgpr(g.N), vHq = in_vgpr(Hq), vWq = in_vgpr(Wq), vNg = in_vgpr(Ng);
  const int vimg0 = in_vgpr(img0), vh0 = in_vgpr(h0), vw0 = in_vgpr(w0);
#pragma unroll
  for (int i = 0; i < MT; ++i) {
    bool pix_ok;
    int off;
    if constexpr (UNROLL_TAPS) {
      pix_ok = ((epix >> i) & 1u) != 0;
      off = eoff[i];
    } else {
      const int m = wave_m * MT * 16 + 16 * i + li;
      const int n = vimg0 + e_ti, hq = vh0 + e_h, wq = vw0 + e_w;
      pix_ok = m < vnpix && n < vN && hq < vHq && wq < vWq;
      off = mad24(mad24(mad24(n, vHq, hq), vWq, wq), vNg, cb);  // element (pixel, channel cb)
      box_advance(e_w, e_h, e_ti, mstep, vTW, vTH);
    }
    bool ok[NT];
#pragma unroll
    for (int j = 0; j < NT; ++j) ok[j] = pix_ok && cb + 16 * j < Ng;
    if (skip != nullptr) {
      float4 sv[NT];
#pragma unroll
      for (int j = 0; j < NT; ++j) {
        if constexpr (UNROLL_TAPS) sv[j] = esv[i][j];
        else sv[j] = *reinterpret_cast<const float4*>(skip + (ok[j] ? off + 16 * j : 0));
      }
#pragma unroll
      for (int j = 0; j < NT; ++j) {
        acc[j][i][0] += sv[j].x; acc[j][i][1] += sv[j].y; acc[j][i][2] += sv[j].z; acc[j][i][3] += sv[j].w;
      }
    }
    if (reduce) {
      if (MODE == 0) {
#pragma unroll
        for (int j = 0; j < NT; ++j)
          if (ok[j]) {
#pragma unroll
            for (int r = 0; r < 4; ++r) {
              const double v = (double)acc[j][i][r];
              s1[j][r] += v;
              s2[j][r] += v * v;
            }
          }
      } else {
        uint32_t cw[NT];  // the K-bit codes of the lane's 4 channels
#pragma unroll
        for (int j = 0; j < NT; ++j) {
          if constexpr (UNROLL_TAPS) {
            cw[j] = ecw[i][j];
          } else {
            const int el = ok[j] ? off + 16 * j : 0;
            cw[j] = epi.K == 4 ? (uint32_t) * reinterpret_cast<const uint16_t*>(epi.codes + (el >> 1))
                               : *reinterpret_cast<const uint32_t*>(epi.codes + el);
          }
        }
#pragma unroll
        for (int j = 0; j < NT; ++j)
          if (ok[j]) {
            const float st4[4] = {r_step[j].x, r_step[j].y, r_step[j].z, r_step[j].w};
            const float bt4[4] = {r_beta[j].x, r_beta[j].y, r_beta[j].z, r_beta[j].w};
            const float ig4[4] = {r_ig[j].x, r_ig[j].y, r_ig[j].z, r_ig[j].w};
            const int32_t fb4[4] = {r_fb[j].x, r_fb[j].y, r_fb[j].z, r_fb[j].w};
#pragma unroll
            for (int r = 0; r < 4; ++r) {
              const uint32_t code = (cw[j] >> (epi.K * r)) & ((1u << epi.K) - 1u);
              const int32_t jj = (int32_t)code - (1 << (epi.K - 1)) + fb4[r];
              const float a2t = st4[r] * ((float)jj + 0.5f);                   // Eq. 10
              const float da2 = a2t > 0.0f ? acc[j][i][r] : 0.0f;             // Eq. 6
              const float a1t = (a2t - bt4[r]) * ig4[r];                      // inverse of Eq. 2
              s1[j][r] += (double)da2;
              s2[j][r] += (double)a1t * (double)da2;
            }
          }
      }
    }
#pragma unroll
    for (int j = 0; j < NT; ++j)
      if (ok[j])
        *reinterpret_cast<float4*>(out + off + 16 * j) =
            make_float4(acc[j][i][0], acc[j][i][1], acc[j][i][2], acc[j][i][3]);
  }
  if (reduce) {
    // fixed order: the 16 pixels of a row of lanes by a butterfly, then the waves that share a
    // channel through LDS
    __syncthreads();  // every wave is done with the patch
    double* red = reinterpret_cast<double*>(lds);  // [2][WAVES_M][BN]
#pragma unroll
    for (int j = 0; j < NT; ++j)
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const double t1 = row16_sum(s1[j][r]), t2 = row16_sum(s2[j][r]);
        if (li == 0) {
          red[(0 * WAVES_M + wave_m) * BN + wn0 + 16 * j + 4 * lk + r] = t1;
          red[(1 * WAVES_M + wave_m) * BN + wn0 + 16 * j + 4 * lk + r] = t2;
        }
      }
    __syncthreads();
    for (int c = tid; c < 2 * BN; c += TPB) {
      const int qv = c / BN, ch = c % BN;
      double t = 0.0;
#pragma unroll
      for (int k = 0; k < WAVES_M; ++k) t += red[(qv * WAVES_M + k) * BN + ch];
      if (n0 + ch < Ng) epi.partial[((int64_t)tile_id * 2 + qv) * Ng + n0 + ch] = t;
    }
  }
}

// ---- host side ----------------------------------------------------------------------------
struct Variant {
  int waves_n, mt, nt, nw;
};
// instantiation table; `variant` in the plan indexes it
constexpr Variant kVariants[] = {
    {1, 4, 1, 4},   // 0: 256 px x 16 ch   (16-channel CIFAR layers)
    {1, 2, 2, 4},   // 1: 128 px x 32 ch
    {1, 4, 2, 4},   // 2: 256 px x 32 ch
    {4, 4, 1, 4},   // 3: 64 px x 64 ch
    {4, 8, 1, 4},   // 4: 128 px x 64 ch
    {4, 14, 1, 4},  // 5: 224 px x 64 ch   (56x56 ImageNet layers)
    {4, 7, 1, 8},   // 6: 224 px x 64 ch in eight waves, two halves of the pixels (14x14 ImageNet layers)
};
constexpr int kNumVariants = sizeof(kVariants) / sizeof(kVariants[0]);
constexpr int kPatchSlots = AMAX * kThreads;  // float4 patch elements a block can stage, whatever its size

inline int cdiv(int a, int b) { return (a + b - 1) / b; }

// Choose the tile shape with at most `maxpix` output pixels that minimises staged patch
// elements plus padded M-tile work over the whole image.
void choose_tile(int Hq, int Wq, int N, int R, int S, int maxpix, HaloPlan& p, int threads = kThreads) {
  if (Hq * Wq <= maxpix) {
    p.TH = Hq; p.TW = Wq;
    p.TI = maxpix / (Hq * Wq);
    if (p.TI > N) p.TI = N;
    while (p.TI > 1 && p.TI * (Hq + R - 1) * (Wq + S - 1) * 4 > kPatchSlots) --p.TI;
  } else {
    p.TI = 1;
    p.TH = p.TW = 0;
    long best = -1;
    for (int kw = 1; kw <= 16; ++kw) {
      const int tw = cdiv(Wq, kw);
      if (tw > maxpix) continue;
      for (int kh = 1; kh <= Hq; ++kh) {
        const int th = cdiv(Hq, kh);
        if (th * tw > maxpix) continue;
        if ((th + R - 1) * (tw + S - 1) * 4 > kPatchSlots) continue;
        const long tiles = (long)cdiv(Hq, th) * cdiv(Wq, tw);
        const long cost = tiles * ((long)(th + R - 1) * (tw + S - 1) + 2L * 16 * cdiv(th * tw, 16));
        if (best < 0 || cost < best) {
          best = cost;
          p.TH = th; p.TW = tw;
        }
        break;  // larger kh only shrinks the tile further
      }
    }
  }
  p.HH = p.TH + R - 1;
  p.HW = p.TW + S - 1;
  p.tiles_i = cdiv(N, p.TI);
  p.tiles_h = cdiv(Hq, p.TH);
  p.tiles_w = cdiv(Wq, p.TW);
  p.npix = p.TI * p.TH * p.TW;
  p.mtiles = cdiv(p.npix, 16);
  auto inv = [](int d) { return (unsigned)(((1ull << 32) + d - 1) / d); };  // unused for d == 1
  p.inv_HW = inv(p.HW); p.inv_HH = inv(p.HH);
  p.inv_TW = inv(p.TW); p.inv_TH = inv(p.TH);
  p.inv_tiles_w = inv(p.tiles_w); p.inv_tiles_h = inv(p.tiles_h);
  auto digits = [](int cells, int width, int height) {
    BoxStep b;
    b.w = cells % width;
    b.h = (cells / width) % height;
    b.ti = cells / width / height;
    return b;
  };
  p.threads = threads;
  p.a_step = digits(threads / 4, p.HW, p.HH);
  p.m_step = digits(16, p.TW, p.TH);
}

bool make_plan(const ConvGeom& g, int mode, HaloPlan& p) {
  const int Hq = mode == 0 ? g.Ho : g.H, Wq = mode == 0 ? g.Wo : g.W;
  const int Ng = mode == 0 ? g.Cout : g.Cin;
  int v;
  if (Ng <= 16) v = 0;
  else if (Ng <= 32) v = (int64_t)g.N * Hq * Wq >= 256 * 512 ? 2 : 1;
  else {
    // 64 output channels per block and 224, 128 or 64 pixels: the largest tile whose blocks
    // fill whole rounds of the 256 compute units to 85 % (measured on the 14x14, 28x28 and 56x56
    // ImageNet layers: an even spread matters more than the tile), else the fullest
    double best = -1.0;
    v = 3;
    for (int cand = 5; cand >= 3; --cand) {
      HaloPlan t;
      choose_tile(Hq, Wq, g.N, g.R, g.S, kVariants[cand].mt * 16, t);
      if (t.TH <= 0) continue;
      const int64_t blocks = (int64_t)t.tiles_i * t.tiles_h * t.tiles_w * cdiv(Ng, 64);
      const double eff = (double)blocks / (double)((blocks + 255) / 256 * 256);
      if (eff >= 0.85) {
        v = cand;
        break;
      }
      if (eff > best) {
        best = eff;
        v = cand;
      }
    }
  }
#ifndef ABL_HALO_NO_8WAVES
  if (v == 5) {
    // the 224-pixel tile with fewer than two blocks per compute unit: eight waves per block
    HaloPlan t;
    choose_tile(Hq, Wq, g.N, g.R, g.S, kVariants[5].mt * 16, t);
    if ((int64_t)t.tiles_i * t.tiles_h * t.tiles_w * cdiv(Ng, 64) < 2 * 256) v = 6;
  }
#endif
  const Variant& var = kVariants[v];
  const int waves_m = var.nw / var.waves_n;
  choose_tile(Hq, Wq, g.N, g.R, g.S, waves_m * var.mt * 16, p, 64 * var.nw);
  p.variant = v;
  p.bn = var.waves_n * var.nt * 16;
  p.nblk_n = (unsigned)cdiv(Ng, p.bn);
  p.inv_nblk_n = (unsigned)(((1ull << 32) + p.nblk_n - 1) / p.nblk_n);
  // 24-bit index arithmetic and multiply-high divisions in the kernel
  const int64_t pixels = (int64_t)g.N * (g.H > g.Ho ? g.H : g.Ho) * (g.W > g.Wo ? g.W : g.Wo);
  if (pixels >= (1 << 23) || pixels * (g.Cin > g.Cout ? g.Cin : g.Cout) >= (1ll << 31)) return false;
  const int Cg = mode == 0 ? g.Cin : g.Cout;
  const size_t fl = (size_t)p.TI * p.HH * p.HW * PS * (Cg > 16 ? 2 : 1);
  p.lds_bytes = (unsigned)(fl * sizeof(float));
  return p.lds_bytes <= 64 * 1024 && p.TI * p.HH * p.HW * 4 <= kPatchSlots && p.TH > 0;
}

template <int MODE, int V, int FUSE>
void launch_variant(hipStream_t st, const ConvGeom& g, const HaloPlan& p, bool bf16, const float* in, const float* w,
                    const float* skip, float* out, const float* stats, void* packed, const EpiReduce& epi) {
  constexpr Variant var = kVariants[V];
  const int Ng = MODE == 0 ? g.Cout : g.Cin;
  dim3 grid(cdiv(p.tiles_i * p.tiles_h * p.tiles_w, 8) * 8 * p.nblk_n);
  const bool taps9 = g.R == 3 && g.S == 3;
  if constexpr (var.nw == 8) {
    auto kern = taps9 ? (bf16 ? halo_conv_kernel<MODE, var.waves_n, var.mt, var.nt, 2, true, FUSE, 8>
                              : halo_conv_kernel<MODE, var.waves_n, var.mt, var.nt, 2, false, FUSE, 8>)
                      : (bf16 ? halo_conv_kernel<MODE, var.waves_n, var.mt, var.nt, 0, true, FUSE, 8>
                              : halo_conv_kernel<MODE, var.waves_n, var.mt, var.nt, 0, false, FUSE, 8>);
    kern<<<grid, 512, p.lds_bytes, st>>>(in, w, skip, out, g, p, stats, packed, epi);
  } else {
    // 3x3 filters: the weight fragments of all nine taps stay in registers; tiles of few M-tiles
    // also prepare their epilogue early
    // (the fused forward of the 14-M-tile variant would pass 256 registers with the held
    // fragments and lose its second wave per SIMD: it keeps the one-tap lookahead)
    constexpr int T9 = var.mt * var.nt <= 4 ? 1 : (FUSE != 0 && var.mt >= 14 ? 0 : 2);
    auto kern = taps9 ? (bf16 ? halo_conv_kernel<MODE, var.waves_n, var.mt, var.nt, T9, true, FUSE>
                              : halo_conv_kernel<MODE, var.waves_n, var.mt, var.nt, T9, false, FUSE>)
                      : (bf16 ? halo_conv_kernel<MODE, var.waves_n, var.mt, var.nt, 0, true, FUSE>
                              : halo_conv_kernel<MODE, var.waves_n, var.mt, var.nt, 0, false, FUSE>);
    kern<<<grid, kThreads, p.lds_bytes, st>>>(in, w, skip, out, g, p, stats, packed, epi);
  }
}

template <int MODE, int FUSE>
void launch_mode(hipStream_t st, const ConvGeom& g, const HaloPlan& p, bool bf16, const float* in, const float* w,
                 const float* skip, float* out, const float* stats, void* packed, const EpiReduce& epi) {
  switch (p.variant) {
    case 0: launch_variant<MODE, 0, FUSE>(st, g, p, bf16, in, w, skip, out, stats, packed, epi); break;
    case 1: launch_variant<MODE, 1, FUSE>(st, g, p, bf16, in, w, skip, out, stats, packed, epi); break;
    case 2: launch_variant<MODE, 2, FUSE>(st, g, p, bf16, in, w, skip, out, stats, packed, epi); break;
    case 3: launch_variant<MODE, 3, FUSE>(st, g, p, bf16, in, w, skip, out, stats, packed, epi); break;
    case 4: launch_variant<MODE, 4, FUSE>(st, g, p, bf16, in, w, skip, out, stats, packed, epi); break;
    case 5: launch_variant<MODE, 5, FUSE>(st, g, p, bf16, in, w, skip, out, stats, packed, epi); break;
    default: launch_variant<MODE, 6, FUSE>(st, g, p, bf16, in, w, skip, out, stats, packed, epi); break;
  }
}

// ------------------------------------------------------------------------------------------
// Weight gradient (Eq. 5) of a stride-1 RxS convolution from the packed activation, all taps
// in one pass.  A block owns 16 input channels x 16*NT output channels and walks over pixel
// tiles; per tile it stages the dequantized + ReLU'd activation patch (Eq. 10, Eq. 3) and the
// dy tile in LDS once, and every group of 4 output pixels then feeds R*S MFMAs (one per tap,
// A = activation at the shifted pixel, B = dy).  dy is read once per block instead of once per
// tap.  The four waves take interleaved pixel groups and are summed in a fixed order at the
// end.  partial layout: [gridDim.x][R][S][Cin][Cout].
template <int K, int NT, int R, int S, bool BF16>
__global__ __launch_bounds__(kThreads) void halo_wgrad_kernel(const uint32_t* __restrict__ packed,
                                                              const float* __restrict__ stats,
                                                              const float* __restrict__ dy,
                                                              float* __restrict__ partial, ConvGeom g,
                                                              HaloPlan p) {
  extern __shared__ __attribute__((aligned(16))) float lds[];
  constexpr int TAPS = R * S;
  constexpr int BNW = 16 * NT;
  constexpr int PSB = (BNW % 32 == 0) ? BNW + 16 : BNW;
  constexpr int WPP = 16 * K / 32;  // packed 32-bit words per pixel for 16 channels
  const int patch = p.TI * p.HH * p.HW;
  const int npix4 = (p.npix + 15) & ~15;     // pixel rows of the dy tile, padded to whole groups of 16
  float* tileA = lds;                       // [patch][16]
  float* tileB = tileA + patch * 16;        // [npix4][PSB]
  int* pixbase = reinterpret_cast<int*>(tileB + npix4 * PSB);  // [npix4] LDS offset of pixel m in tileA
  int* pixloc = pixbase + npix4;                               // [npix4] (ti<<16)|(h<<8)|w, -1 = padding

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int li = lane & 15, lk = lane >> 4;
  const int cout_blocks = (g.Cout + BNW - 1) / BNW;
  const int ci0 = (blockIdx.y / cout_blocks) * 16, co0 = (blockIdx.y % cout_blocks) * BNW;

  for (int m = tid; m < npix4; m += kThreads) {
    if (m < p.npix) {
      const int w = m % p.TW, q = m / p.TW;
      const int h = q % p.TH, ti = q / p.TH;
      pixbase[m] = ((ti * p.HH + h) * p.HW + w) * 16;
      pixloc[m] = (ti << 16) | (h << 8) | w;
    } else {
      pixbase[m] = 0;
      pixloc[m] = -1;
    }
  }

  float step[16];
  int32_t fb[16];
#pragma unroll
  for (int v = 0; v < 16; ++v) {
    step[v] = stats[P_STEP * g.Cin + ci0 + v];
    fb[v] = reinterpret_cast<const int32_t*>(stats)[P_FB * g.Cin + ci0 + v];
  }

  floatx4 acc[TAPS][NT];
#pragma unroll
  for (int t = 0; t < TAPS; ++t)
#pragma unroll
    for (int j = 0; j < NT; ++j) acc[t][j] = floatx4{0.f, 0.f, 0.f, 0.f};

  const int ntiles = p.tiles_i * p.tiles_h * p.tiles_w;
  for (int tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
    int b = tile;
    const int tw_i = b % p.tiles_w; b /= p.tiles_w;
    const int th_i = b % p.tiles_h; b /= p.tiles_h;
    const int img0 = b * p.TI, h0 = th_i * p.TH, w0 = tw_i * p.TW;
    __syncthreads();  // previous tile consumed (and the lookup tables written)
    for (int idx = tid; idx < patch; idx += kThreads) {
      int pix = idx;
      const int ww = pix % p.HW; pix /= p.HW;
      const int hh = pix % p.HH;
      const int ti = pix / p.HH;
      const int n = img0 + ti, hi = h0 - g.pad + hh, wi = w0 - g.pad + ww;
      uint32_t wd[WPP];
      const bool ok = n < g.N && hi >= 0 && hi < g.H && wi >= 0 && wi < g.W;
      if (ok) {
        const uint32_t* src = packed + ((((int64_t)n * g.H + hi) * g.W + wi) * g.Cin + ci0) * K / 32;
        if (WPP == 2) {
          const uint2 t = *reinterpret_cast<const uint2*>(src);
          wd[0] = t.x; wd[1] = t.y;
        } else {
          const uint4 t = *reinterpret_cast<const uint4*>(src);
          wd[0] = t.x; wd[1] = t.y; wd[2 % WPP] = t.z; wd[3 % WPP] = t.w;
        }
      }
      float v[16];
#pragma unroll
      for (int c = 0; c < 16; ++c) {
        const uint32_t code = ok ? (wd[c * K / 32] >> ((c * K) % 32)) & ((1u << K) - 1) : 0u;
        const int32_t j = (int32_t)code - (1 << (K - 1)) + fb[c];
        const float a2t = step[c] * ((float)j + 0.5f);  // Eq. 10
        v[c] = (ok && a2t > 0.f) ? a2t : 0.f;           // Eq. 3
      }
      float4* dst = reinterpret_cast<float4*>(&tileA[idx * 16]);
      dst[0] = make_float4(v[0], v[1], v[2], v[3]);
      dst[1] = make_float4(v[4], v[5], v[6], v[7]);
      dst[2] = make_float4(v[8], v[9], v[10], v[11]);
      dst[3] = make_float4(v[12], v[13], v[14], v[15]);
    }
    for (int idx = tid; idx < npix4 * (BNW / 4); idx += kThreads) {
      const int m = idx / (BNW / 4), c4 = 4 * (idx % (BNW / 4));
      const int loc = pixloc[m];
      float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
      if (loc >= 0) {
        const int n = img0 + (loc >> 16), ho = h0 + ((loc >> 8) & 255), wo = w0 + (loc & 255);
        if (n < g.N && ho < g.Ho && wo < g.Wo && co0 + c4 < g.Cout)
          v = *reinterpret_cast<const float4*>(dy + (((int64_t)n * g.Ho + ho) * g.Wo + wo) * g.Cout + co0 + c4);
      }
      *reinterpret_cast<float4*>(&tileB[m * PSB + c4]) = v;
    }
    __syncthreads();
    // 16 pixels per step.  Component e of the operand vectors is pixel 4e + lk (fp32: k-step e,
    // lane group = k) or 4lk + e (bf16: the lane group owns 4 consecutive k).
    for (int q = wave; q < npix4 / 16; q += 4) {
      int pb[4];
      float4 bf[NT];
      {
        int m[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          m[e] = 16 * q + (BF16 ? 4 * lk + e : 4 * e + lk);
          pb[e] = pixbase[m[e]] + li;
        }
#pragma unroll
        for (int j = 0; j < NT; ++j)
          bf[j] = make_float4(tileB[m[0] * PSB + 16 * j + li], tileB[m[1] * PSB + 16 * j + li],
                              tileB[m[2] * PSB + 16 * j + li], tileB[m[3] * PSB + 16 * j + li]);
      }
#pragma unroll
      for (int t = 0; t < TAPS; ++t) {
        const int toff = ((t / S) * p.HW + (t % S)) * 16;
        float4 a[1];
        a[0] = make_float4(tileA[pb[0] + toff], tileA[pb[1] + toff], tileA[pb[2] + toff], tileA[pb[3] + toff]);
        mma_k4<BF16, 1, NT>(a, bf, reinterpret_cast<floatx4(&)[1][NT]>(acc[t]));
      }
    }
  }

  // sum the four waves in order through LDS: red[tap][ci][co]
  float* red = lds;
  for (int w = 0; w < 4; ++w) {
    __syncthreads();
    if (wave == w) {
#pragma unroll
      for (int t = 0; t < TAPS; ++t)
#pragma unroll
        for (int j = 0; j < NT; ++j)
#pragma unroll
          for (int rr = 0; rr < 4; ++rr) {
            float* d = &red[(t * 16 + 4 * lk + rr) * BNW + 16 * j + li];
            *d = (w == 0) ? acc[t][j][rr] : *d + acc[t][j][rr];
          }
    }
  }
  __syncthreads();
  float* dst = partial + (int64_t)blockIdx.x * TAPS * g.Cin * g.Cout;
  for (int idx = tid; idx < TAPS * 16 * (BNW / 4); idx += kThreads) {
    const int row = idx / (BNW / 4), c4 = 4 * (idx % (BNW / 4));
    const int t = row >> 4, ci = ci0 + (row & 15);
    if (co0 + c4 < g.Cout)
      *reinterpret_cast<float4*>(dst + ((int64_t)t * g.Cin + ci) * g.Cout + co0 + c4) =
          *reinterpret_cast<const float4*>(&red[row * BNW + c4]);
  }
}

// dW[i] = sum of nb partial copies, fixed order: 16 outputs x 16 interleaved parts per block.
__global__ __launch_bounds__(kThreads) void partial_sum_kernel(const float* __restrict__ partial, int nb,
                                                               int64_t n, float* __restrict__ dw) {
  __shared__ float sm[16][17];
  const int o = threadIdx.x & 15, part = threadIdx.x >> 4;
  const int64_t i = (int64_t)blockIdx.x * 16 + o;
  float s = 0.f;
  if (i < n) {
#pragma unroll 8
    for (int k = part; k < nb; k += 16) s += partial[(int64_t)k * n + i];
  }
  sm[part][o] = s;
  __syncthreads();
  for (int h = 8; h >= 1; h >>= 1) {
    if (part < h) sm[part][o] += sm[part + h][o];
    __syncthreads();
  }
  if (part == 0 && i < n) dw[i] = sm[0][o];
}

struct WgradHaloPlan {
  HaloPlan tile;
  int nt;        // 16-wide output-channel tiles per block
  int nblk;      // blocks along the pixel tiles (= number of partial copies)
  int gridy;     // cin chunks x cout blocks
};

bool make_wgrad_plan(const ConvGeom& g, WgradHaloPlan& wp) {
  if (g.stride != 1 || g.R != 3 || g.S != 3 || g.Cin % 16 != 0 || g.Cout % 16 != 0 || g.pad > 2) return false;
  wp.nt = g.Cout >= 64 ? 4 : (g.Cout >= 32 ? 2 : 1);
  HaloPlan& p = wp.tile;
  choose_tile(g.Ho, g.Wo, g.N, g.R, g.S, 256, p);
  if (p.TH <= 0 || p.TH > 255 || p.TW > 255) return false;
  const int bnw = 16 * wp.nt, psb = (bnw % 32 == 0) ? bnw + 16 : bnw;
  const int npix4 = (p.npix + 15) & ~15;
  size_t fl = (size_t)p.TI * p.HH * p.HW * 16 + (size_t)npix4 * psb + 2 * (size_t)npix4;
  const size_t red = (size_t)g.R * g.S * 16 * bnw;
  if (fl < red) fl = red;
  p.lds_bytes = (unsigned)(fl * sizeof(float));
  if (p.lds_bytes > 64 * 1024) return false;
  wp.gridy = (g.Cin / 16) * ((g.Cout + bnw - 1) / bnw);
  const int ntiles = p.tiles_i * p.tiles_h * p.tiles_w;
  int nblk = 512 / wp.gridy;
  if (nblk < 16) nblk = 16;
  if (nblk > ntiles) nblk = ntiles;
  // even share of tiles per block
  const int per = cdiv(ntiles, nblk);
  wp.nblk = cdiv(ntiles, per);
  return true;
}


// ------------------------------------------------------------------------------------------
// Backward of a 3x3 'same' stride-1 layer with 16 input and 16 output channels in ONE kernel:
// the gradient to the conv input (Eq. 5) with its Eq. 6-7 sums, and the weight gradient (Eq. 5)
// from the packed activation.  Both contractions consume dy; a block stages the dy patch of its
// pixel tile and the dequantized, ReLU'd activation patch (Eq. 10, Eq. 3) once, in the same
// geometry, and runs the two sets of MFMAs from them:
//   dA3[p, ci]      = sum_t sum_co dy[p + pad - t, co] W[t, ci, co]    (A = W, B = dy patch)
//   dW[t, ci, co]  += sum_p A3~[p + t - pad, ci] dy[p, co]              (A = A3~ patch, B = dy)
// The Eq. 6-7 sums take the mask and A1~ from the staged activation, so the codes are read from
// memory once.  At 16 channels the per-block fixed costs (index set-up, the first loads, the
// epilogues) outweigh the MFMAs; sharing them between the two contractions halves them.
// Outputs per pixel tile: partial[tile][2][16] doubles, wpartial[tile][3][3][16][16] floats.
template <int K, bool BF16>
__global__ __launch_bounds__(kThreads) void halo_bwd16_kernel(const float* __restrict__ dy,
                                                              const float* __restrict__ wgt,
                                                              const uint8_t* __restrict__ packed,
                                                              const float* __restrict__ stats,
                                                              float* __restrict__ da3, double* __restrict__ partial,
                                                              float* __restrict__ wpartial, ConvGeom g, HaloPlan p) {
  extern __shared__ __attribute__((aligned(16))) float lds[];
  constexpr int C = 16;
  asm volatile("" ::"s"(dy), "s"(wgt), "s"(packed), "s"(stats), "s"(g.N), "s"(g.H), "s"(g.W), "s"(p.TI), "s"(p.TH),
               "s"(p.TW), "s"(p.HH), "s"(p.HW), "s"(p.tiles_h), "s"(p.tiles_w), "s"(p.npix), "s"(p.inv_HW),
               "s"(p.inv_HH), "s"(p.inv_TW), "s"(p.inv_TH), "s"(p.inv_tiles_w), "s"(p.inv_tiles_h),
               "s"(p.a_step.w), "s"(p.a_step.h), "s"(p.a_step.ti));
  const int patch = p.TI * p.HH * p.HW;
  float* tdy = lds;                                       // [patch][PS] dy
  float* tact = lds + patch * PS;                         // [patch][PS] A3~
  // the two patches are reused for the cross-wave sum of dW (4 x 9 x 256 floats) at the end
  // (+ one spare pixel row behind the activation patch: the target of staging slots past its end)
  const int region = (2 * patch + 1) * PS > 4 * 9 * 256 ? (2 * patch + 1) * PS : 4 * 9 * 256;
  int* pixbase = reinterpret_cast<int*>(lds + region);    // [256] LDS offset of tile pixel m, tap (0,0)
  int* pixoff = pixbase + kThreads;                       // [256] global offset of (pixel m, channel 0), -1 outside
  double* red = reinterpret_cast<double*>(pixoff + kThreads);  // [2][4][16]

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int li = lane & 15, lk = lane >> 4;
  const int tile = blockIdx.x;
  const unsigned t1 = udiv<true>(tile, p.tiles_w, p.inv_tiles_w);
  const unsigned t2 = udiv<true>(t1, p.tiles_h, p.inv_tiles_h);
  const int img0 = t2 * p.TI, h0 = (t1 - t2 * p.tiles_h) * p.TH, w0 = (tile - t1 * p.tiles_w) * p.TW;
  const int oh = h0 - 1, ow = w0 - 1;  // image coordinate of patch element (0,0), both patches

  // table entry of tile pixel m = tid
  {
    int ti, h, w;
    split3<true>(tid, p.TW, p.inv_TW, p.TH, p.inv_TH, ti, h, w);
    const bool in_tile = tid < p.npix;
    const int n = img0 + ti, hq = h0 + h, wq = w0 + w;
    pixbase[tid] = in_tile ? mad24(mad24(mad24(ti, p.HH, h), p.HW, w), PS, 0) : 0;
    pixoff[tid] = in_tile && n < g.N && hq < g.H && wq < g.W ? mad24(mad24(mad24(n, g.H, hq), g.W, wq), C, 0) : -1;
  }

  // global element offsets of the patch elements this thread stages (4 channels each); -1 = zero
  // fill, -2 = past the end of the patch
  const int totalA = patch * 4;
  int goff[AMAX];
  // dy and the codes of the same elements: each slot's loads leave as soon as its address is known
  float4 rd[AMAX];
  uint32_t rc[AMAX];
  {
    int ti, h, w;
    split3<true>(tid >> 2, p.HW, p.inv_HW, p.HH, p.inv_HH, ti, h, w);
    ti += img0; h += oh; w += ow;
    const BoxStep step{in_vgpr(p.a_step.w), in_vgpr(p.a_step.h), in_vgpr(p.a_step.ti)};
    const int width = in_vgpr(p.HW), height = in_vgpr(p.HH);
    const int w_end = in_vgpr(ow + p.HW), h_end = in_vgpr(oh + p.HH);
    const int vN = in_vgpr(g.N), vH = in_vgpr(g.H), vW = in_vgpr(g.W), vtotal = in_vgpr(totalA);
    const int c4 = 4 * (tid & 3);
#pragma unroll
    for (int j = 0; j < AMAX; ++j) {
      const int idx = tid + kThreads * j;
      const bool ok = idx < vtotal && ti < vN && (unsigned)h < (unsigned)vH && (unsigned)w < (unsigned)vW;
      goff[j] = ok ? mad24(mad24(mad24(ti, vH, h), vW, w), C, c4) : (idx < vtotal ? -1 : -2);
      {
        const int e0 = ok ? goff[j] : 0;
        rd[j] = *reinterpret_cast<const float4*>(dy + e0);
        rc[j] = K == 4 ? (uint32_t) * reinterpret_cast<const uint16_t*>(packed + (e0 >> 1))
                       : *reinterpret_cast<const uint32_t*>(packed + e0);
      }
      w += step.w;
      const bool cw = w >= w_end;
      w -= cw ? width : 0;
      h += step.h + (cw ? 1 : 0);
      const bool ch = h >= h_end;
      h -= ch ? height : 0;
      ti += step.ti + (ch ? 1 : 0);
    }
  }

  // the rest of the block's loads in one batch: quantizer constants and the weight fragments
  const int c4 = 4 * (tid & 3);
  const float4 q_step = *reinterpret_cast<const float4*>(stats + P_STEP * C + c4);
  const int4 q_fb = *reinterpret_cast<const int4*>(reinterpret_cast<const int32_t*>(stats) + P_FB * C + c4);
  // (the epilogue's constants too: requested there, their round trip would be exposed)
  const float4 e_beta = *reinterpret_cast<const float4*>(stats + P_BETA * C + 4 * lk);
  const float4 e_gm = *reinterpret_cast<const float4*>(stats + P_GAMMA * C + 4 * lk);
  // dgrad weight fragment: k = co = 4lk .. +3, row = ci = li
  float4 bw[9][1];
#pragma unroll
  for (int t = 0; t < 9; ++t)
    bw[t][0] = *reinterpret_cast<const float4*>(wgt + (t * C + li) * C + 4 * lk);

  // Both patches are staged before the first MFMA (the activation one branch-free: slots past the
  // end of the patch write the spare row).  dy and the codes of a slot are requested together,
  // so neither patch has to wait for the other, and dequantizing between the taps of the dA3
  // contraction instead gained nothing: fp32 MFMAs and vector ALU instructions share the SIMD's
  // issue slots on this chip (measured: their times add up, across waves too), and the staging
  // stores between the taps kept every fragment read right in front of its MFMAs.
#pragma unroll
  for (int j = 0; j < AMAX; ++j) {
    const int idx = tid + kThreads * j;
    if (goff[j] != -2) *reinterpret_cast<float4*>(&tdy[(idx >> 2) * PS + 4 * (idx & 3)]) = keep_if(goff[j] >= 0, rd[j]);
  }
  auto stage_act = [&](int j) __attribute__((always_inline)) {
    const int idx = tid + kThreads * j;
    const bool ok = goff[j] >= 0;
    const float st4[4] = {q_step.x, q_step.y, q_step.z, q_step.w};
    const int32_t fb4[4] = {q_fb.x, q_fb.y, q_fb.z, q_fb.w};
    float a[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const float a2t = dequant<K>((rc[j] >> (K * e)) & ((1u << K) - 1u), st4[e], fb4[e]);  // Eq. 10
      a[e] = (ok && a2t > 0.0f) ? a2t : 0.0f;                                              // Eq. 3
    }
    const int o = goff[j] != -2 ? (idx >> 2) * PS + 4 * (idx & 3) : patch * PS + 4 * (idx & 3);
    *reinterpret_cast<float4*>(&tact[o]) = make_float4(a[0], a[1], a[2], a[3]);
  };
#pragma unroll
  for (int j = 0; j < AMAX; ++j) stage_act(j);
  __syncthreads();

  const int ctr = (p.HW + 1) * PS;  // from tap (0,0) to the pixel itself
  // ---- dA3 tile: 4 M-tiles of 16 pixels per wave, transposed output (lane = pixel li, channels 4lk..) ----
  floatx4 accd[1][4];
  int mbase[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    accd[0][i] = floatx4{0.f, 0.f, 0.f, 0.f};
    mbase[i] = pixbase[wave * 64 + 16 * i + li];
  }
#pragma unroll
  for (int t = 0; t < 9; ++t) {
    const int aoff = ((2 - t / 3) * p.HW + (2 - t % 3)) * PS + 4 * lk;
    float4 af[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) af[i] = *reinterpret_cast<const float4*>(&tdy[mbase[i] + aoff]);
    mma_k4<BF16, 1, 4>(bw[t], af, accd);
  }

  // ---- dW: the wave's 64 pixels, 16 per step; component e of the operand vectors is pixel
  // 4e + lk of the step (fp32: k-step e, lane group = k) or 4lk + e (bf16) ----
  // The operands of a step (9 taps x 4 pixels of A3~, 4 pixels of dy per lane) are read into
  // registers one step ahead of the MFMAs that use them.
  floatx4 accw[9];
#pragma unroll
  for (int t = 0; t < 9; ++t) accw[t] = floatx4{0.f, 0.f, 0.f, 0.f};
  float av[2][9][4], bv[2][4];
  auto read_step = [&](int q, float (&a)[9][4], float (&b)[4]) __attribute__((always_inline)) {
    int pb[4];
    bool in[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const int m = wave * 64 + 16 * q + (BF16 ? 4 * lk + e : 4 * e + lk);
      pb[e] = pixbase[m] + li;
      in[e] = pixoff[m] >= 0;
    }
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      // pixels that are not part of the tile or the image contribute nothing
      const float v = tdy[pb[e] + ctr];
      b[e] = in[e] ? v : 0.0f;
    }
#pragma unroll
    for (int t = 0; t < 9; ++t)
#pragma unroll
      for (int e = 0; e < 4; ++e) a[t][e] = tact[pb[e] + ((t / 3) * p.HW + (t % 3)) * PS];
  };
  read_step(0, av[0], bv[0]);
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    // the scheduler would otherwise sink every read to just before its MFMA and wait for it there
    if (q + 1 < 4) read_step(q + 1, av[(q + 1) & 1], bv[(q + 1) & 1]);
    __builtin_amdgcn_sched_barrier(0);
    const float(&a)[9][4] = av[q & 1];
    const float(&b)[4] = bv[q & 1];
    if constexpr (BF16) {
      const shortx4 bb = to_bf16x4(make_float4(b[0], b[1], b[2], b[3]));
#pragma unroll
      for (int t = 0; t < 9; ++t)
        accw[t] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(to_bf16x4(make_float4(a[t][0], a[t][1], a[t][2], a[t][3])),
                                                            bb, accw[t], 0, 0, 0);
    } else {
      // k-step outermost: consecutive MFMAs write different accumulators
#pragma unroll
      for (int e = 0; e < 4; ++e)
#pragma unroll
        for (int t = 0; t < 9; ++t) accw[t] = mfma16(a[t][e], b[e], accw[t]);
    }
  }

  // ---- epilogue of dA3: store, and the Eq. 6-7 sums with mask and A1~ from the staged activation ----
  {
    const float bt4[4] = {e_beta.x, e_beta.y, e_beta.z, e_beta.w};
    const float ig4[4] = {1.0f / e_gm.x, 1.0f / e_gm.y, 1.0f / e_gm.z, 1.0f / e_gm.w};
    double s1[4] = {0.0, 0.0, 0.0, 0.0}, s2[4] = {0.0, 0.0, 0.0, 0.0};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int off = pixoff[wave * 64 + 16 * i + li];
      const float4 a3 = *reinterpret_cast<const float4*>(&tact[mbase[i] + ctr + 4 * lk]);
      const float a3t[4] = {a3.x, a3.y, a3.z, a3.w};
      if (off >= 0) {
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const float da2 = a3t[r] > 0.0f ? accd[0][i][r] : 0.0f;  // Eq. 6
          const float a1t = (a3t[r] - bt4[r]) * ig4[r];             // inverse of Eq. 2
          s1[r] += (double)da2;
          s2[r] += (double)a1t * (double)da2;
        }
        *reinterpret_cast<float4*>(da3 + off + 4 * lk) =
            make_float4(accd[0][i][0], accd[0][i][1], accd[0][i][2], accd[0][i][3]);
      }
    }
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const double u1 = row16_sum(s1[r]), u2 = row16_sum(s2[r]);
      if (li == 0) {
        red[(0 * 4 + wave) * C + 4 * lk + r] = u1;
        red[(1 * 4 + wave) * C + 4 * lk + r] = u2;
      }
    }
  }
  __syncthreads();  // every wave is done with the patches
  if (tid < 2 * C) {
    const int qv = tid / C, ch = tid % C;
    const double t = ((red[(qv * 4 + 0) * C + ch] + red[(qv * 4 + 1) * C + ch]) + red[(qv * 4 + 2) * C + ch]) +
                     red[(qv * 4 + 3) * C + ch];
    partial[((int64_t)tile * 2 + qv) * C + ch] = t;
  }
  // ---- dW: the four waves are summed in order through LDS; wred[wave][t][ci][co] ----
  float* wred = lds;
#pragma unroll
  for (int t = 0; t < 9; ++t)
#pragma unroll
    for (int r = 0; r < 4; ++r) wred[(wave * 9 + t) * 256 + (4 * lk + r) * C + li] = accw[t][r];
  __syncthreads();
  float* dst = wpartial + (int64_t)tile * (9 * C * C);
#pragma unroll
  for (int k = 0; k < 9; ++k) {
    const int idx = tid + kThreads * k;
    dst[idx] = ((wred[idx] + wred[2304 + idx]) + wred[2 * 2304 + idx]) + wred[3 * 2304 + idx];
  }
}

bool make_bwd16_plan(const ConvGeom& g, HaloPlan& p) {
  if (g.stride != 1 || g.R != 3 || g.S != 3 || g.pad != 1 || g.Cin != 16 || g.Cout != 16) return false;
  const int64_t pixels = (int64_t)g.N * g.H * g.W;
  if (pixels >= (1 << 23)) return false;  // 24-bit index arithmetic
  choose_tile(g.H, g.W, g.N, 3, 3, 256, p);
  if (p.TH <= 0) return false;
  const int tiles = p.tiles_i * p.tiles_h * p.tiles_w;
  if (tiles > kMaxPartialBlocks) return false;
  size_t bytes = (size_t)2 * p.TI * p.HH * p.HW * PS * sizeof(float);
  const size_t wred = (size_t)4 * 9 * 256 * sizeof(float);
  if (bytes < wred) bytes = wred;
  bytes += PS * sizeof(float);  // spare pixel row
  bytes += 2 * kThreads * sizeof(int) + 2 * 4 * 16 * sizeof(double);
  p.lds_bytes = (unsigned)bytes;
  return bytes <= 64 * 1024;
}

}  // namespace

bool halo_conv_supported(const ConvGeom& g) {
  if (g.stride != 1 || g.R * g.S < 2 || g.R > 7 || g.S > 7) return false;
  if (g.Cin % 16 != 0 || g.Cout % 16 != 0) return false;
  if (g.pad > g.R - 1 || g.pad > g.S - 1) return false;
  HaloPlan p;
  return make_plan(g, 0, p) && make_plan(g, 1, p);
}

int launch_halo_conv(hipStream_t st, const ConvGeom& g, int mode, bool bf16, const float* in, const float* w,
                     const float* skip, float* out, double* out_partial) {
  HaloPlan p;
  if (!make_plan(g, mode, p)) return ABL_ERR_SHAPE;
  p.pack_pad = 0;
  const EpiReduce none{nullptr, nullptr, 0};
  const EpiReduce sums{out_partial, nullptr, 0};  // forward only: sums of y for the next layer's Eq. 1
  if (mode == 0) launch_mode<0, 0>(st, g, p, bf16, in, w, skip, out, nullptr, nullptr, sums);
  else launch_mode<1, 0>(st, g, p, bf16, in, w, nullptr, out, nullptr, nullptr, none);
  return hip_status();
}

bool halo_fused_supported(const ConvGeom& g) {
  return halo_conv_supported(g) && g.Ho == g.H && g.Wo == g.W;
}

int halo_tile_count(const ConvGeom& g, int mode) {
  HaloPlan p;
  if (!make_plan(g, mode, p)) return 0;
  return p.tiles_i * p.tiles_h * p.tiles_w;
}

int launch_halo_fwd_fused(hipStream_t st, const ConvGeom& g, int K, bool bf16, const float* x,
                          const void* stats, const float* w, const float* skip, float* y, void* packed,
                          double* out_partial) {
  HaloPlan p;
  if (!make_plan(g, 0, p)) return ABL_ERR_SHAPE;
  const int64_t raw = ((int64_t)g.N * g.H * g.W * g.Cin * K + 7) / 8;
  p.pack_pad = (int)((raw + 127) / 128 * 128 - raw);
  const float* sp = static_cast<const float*>(stats);
  const EpiReduce epi{out_partial, nullptr, 0};
  if (K == 4) launch_mode<0, 4>(st, g, p, bf16, x, w, skip, y, sp, packed, epi);
  else launch_mode<0, 8>(st, g, p, bf16, x, w, skip, y, sp, packed, epi);
  return hip_status();
}

int launch_halo_dgrad_reduce(hipStream_t st, const ConvGeom& g, int K, bool bf16, const float* dy,
                             const float* w, const void* packed, const void* stats, float* da3,
                             double* partial) {
  HaloPlan p;
  if (!make_plan(g, 1, p)) return ABL_ERR_SHAPE;
  p.pack_pad = 0;
  const EpiReduce epi{partial, static_cast<const uint8_t*>(packed), K};
  launch_mode<1, 0>(st, g, p, bf16, dy, w, nullptr, da3, static_cast<const float*>(stats), nullptr, epi);
  return hip_status();
}

}  // namespace abl

namespace abl {

size_t halo_wgrad_partial_bytes(const ConvGeom& g) {
  WgradHaloPlan wp;
  if (!make_wgrad_plan(g, wp)) return 0;
  size_t copies = (size_t)wp.nblk;
  HaloPlan p;  // the fused backward kernel keeps one copy per pixel tile
  if (make_bwd16_plan(g, p) && (size_t)p.tiles_i * p.tiles_h * p.tiles_w > copies)
    copies = (size_t)p.tiles_i * p.tiles_h * p.tiles_w;
  return (copies * g.R * g.S * g.Cin * g.Cout * sizeof(float) + 255) / 256 * 256;
}

int launch_halo_wgrad(hipStream_t st, const ConvGeom& g, int K, bool bf16, const void* packed, const float* stats,
                      const float* dy, void* scratch, float* dw) {
  WgradHaloPlan wp;
  if (!make_wgrad_plan(g, wp)) return ABL_ERR_SHAPE;
  const uint32_t* pk = static_cast<const uint32_t*>(packed);
  float* part = wp.nblk == 1 ? dw : static_cast<float*>(scratch);
  dim3 grid(wp.nblk, wp.gridy);
  const unsigned lds = wp.tile.lds_bytes;
#define ABL_WG(KK, NN)                                                                          \
  do {                                                                                          \
    auto kern = bf16 ? halo_wgrad_kernel<KK, NN, 3, 3, true> : halo_wgrad_kernel<KK, NN, 3, 3, false>; \
    kern<<<grid, kThreads, lds, st>>>(pk, stats, dy, part, g, wp.tile);                         \
  } while (0)
  if (K == 4) {
    if (wp.nt == 1) ABL_WG(4, 1); else if (wp.nt == 2) ABL_WG(4, 2); else ABL_WG(4, 4);
  } else {
    if (wp.nt == 1) ABL_WG(8, 1); else if (wp.nt == 2) ABL_WG(8, 2); else ABL_WG(8, 4);
  }
#undef ABL_WG
  if (wp.nblk > 1) {
    const int64_t n = (int64_t)g.R * g.S * g.Cin * g.Cout;
    partial_sum_kernel<<<(unsigned)((n + 15) / 16), kThreads, 0, st>>>(part, wp.nblk, n, dw);
  }
  return hip_status();
}

int halo_bwd16_tiles(const ConvGeom& g) {
  HaloPlan p;
  if (!make_bwd16_plan(g, p)) return 0;
  return p.tiles_i * p.tiles_h * p.tiles_w;
}

int launch_halo_bwd16(hipStream_t st, const ConvGeom& g, int K, bool bf16, const float* dy, const float* w,
                      const void* packed, const void* stats, float* da3, double* partial, void* wscratch,
                      float* dw) {
  HaloPlan p;
  if (!make_bwd16_plan(g, p)) return ABL_ERR_SHAPE;
  const int tiles = p.tiles_i * p.tiles_h * p.tiles_w;
  const uint8_t* pk = static_cast<const uint8_t*>(packed);
  const float* sp = static_cast<const float*>(stats);
  float* wpart = static_cast<float*>(wscratch);
  auto kern = K == 4 ? (bf16 ? halo_bwd16_kernel<4, true> : halo_bwd16_kernel<4, false>)
                     : (bf16 ? halo_bwd16_kernel<8, true> : halo_bwd16_kernel<8, false>);
  kern<<<tiles, kThreads, p.lds_bytes, st>>>(dy, w, pk, sp, da3, partial, wpart, g, p);
  if (dw != nullptr) {
    const int64_t n = 9 * 16 * 16;
    partial_sum_kernel<<<(unsigned)((n + 15) / 16), kThreads, 0, st>>>(wpart, tiles, n, dw);
  }
  return hip_status();
}

}  // namespace abl
