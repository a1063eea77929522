// Pointwise (1x1, stride 1, no padding) convolutions of the approximate-activation layer as
// plain GEMMs for gfx950 (CDNA4):
//   forward  Eq. 4           y[p][co]   = sum_ci A3[p][ci] W[ci][co]     (+ identity shortcut)
//   dgrad    Eq. 5, 2nd half dA3[p][ci] = sum_co dy[p][co] W[ci][co]
// and the forward with Eq. 1-3 and Eq. 9 applied to the input on its way to the matrix cores
// (A3 never reaches memory; the output-channel blocks share the writing of the K-bit codes).
//
// A pixel's channels are contiguous in NHWC, which is exactly what a lane of
// v_mfma_f32_16x16x4_f32 needs of the activation operand: four consecutive k of one row.  So
// the activations go from global memory straight into registers in MFMA layout - no LDS
// staging and no barrier for them - with a ring of four 16-channel groups in flight per wave
// that runs on from one pixel tile into the next.  A wave owns 16 pixels x 16*NT output
// channels: few accumulators, so many waves share a compute unit, and tiles small enough to
// spread evenly (measured: occupancy and an even spread decide here, larger tiles lose).
// Only the weights (shared by all waves, and needed with k contiguous, i.e. transposed in
// the forward) sit in LDS:
//   contraction of at most 256 channels: the whole slice, written once per block;
//   longer: 64- or 128-channel chunks in two buffers, the next chunk's global loads in flight while
//           the current one is contracted, one barrier per chunk.
// Every block walks over a run of consecutive pixel tiles; the runs differ by at most one tile.
// A long contraction makes a tile a long piece of work, and the tile count of the ImageNet
// shapes is an awkward multiple of the compute-unit count (12544 pixels x 256 channels are 3.06
// tiles per SIMD: with whole tiles some SIMDs would do four, a quarter of the chip's time lost).
// There the grid is cut in two: whole rounds of one tile per SIMD, and the pixel rows left over
// in blocks whose four waves share one 16-pixel row group and take a quarter of the contraction
// each - a quarter of a tile's time.
#include <mutex>
#include <type_traits>
#include <unordered_map>

#include "abl_internal.h"

// Eq. 1-3 and Eq. 9 are evaluated here: one rounded fp32 operation at a time
#pragma clang fp contract(off)

namespace abl {
namespace {

constexpr int KC = 256;    // longest contraction whose weights stay in LDS for the whole block
constexpr int CHC_N = 64;   // chunk length beyond that: four-wave blocks (the balanced grid, see below)
constexpr int CHC_W = 128;  // ... eight-wave blocks
constexpr int CHC_U8 = -1;  // template code: whole contraction in LDS, eight-wave blocks
constexpr int PF = 4;      // 16-channel groups in flight per wave
constexpr int NCONST = 6;  // per-channel constants of the fused prologue: mean rstd gamma beta cq fb

inline int pointwise_chunk(int Kd, bool wide) { return Kd <= KC ? Kd : (wide ? CHC_W : CHC_N); }
inline unsigned pointwise_lds_bytes(int Kd, int nt, bool fuse, bool wide) {
  const int ch = pointwise_chunk(Kd, wide), nbuf = Kd <= KC ? 1 : 2;
  return (unsigned)(nbuf * (16 * nt * (ch + 4) + (fuse ? NCONST * ch : 0)) * sizeof(float));
}

// MODE 0: in = A3 (or x with FUSE) [M][Kd = Cin], out = y [M][N = Cout], weight(k, n) = wgt[k * ldw + n]
// MODE 1: in = dy [M][Kd = Cout], out = dA3 [M][N = Cin],                weight(k, n) = wgt[n * ldw + k]
// ldw = Cout.  Kd is a multiple of 64 (and of CHC when chunked), N a multiple of 16 * NT.
// Pixel tiles of 16 * WAVES rows; block `r` of an output-channel block takes run_base tiles, one
// more if r < run_rem, in order.
// CHUNKED blocks past `main_grid` are the split ones: block main_grid + i has row group
// rem_sub0 + i / (N / BN) (16 pixels) and output-channel block i % (N / BN).
// SUMS: the block also leaves per-channel fp64 sums of what it holds in registers (row `run`,
// layout [rows][2][N]) - forward: of its outputs and their squares, for the statistics of the
// next layer's Eq. 1; dgrad: of dA2 = dA3 where the dequantized activation is positive (Eq. 6)
// and of A1~ * dA2 (Eq. 7), with the layer's codes read here (`packed`, code_bits wide, and the
// layer's `stats`), which saves the separate reduce pass over dA3.
template <int MODE, int NT, int CHC, bool BF16, int FUSE, bool SUMS>
__global__ __launch_bounds__((CHC == CHC_W || CHC == CHC_U8) ? 512 : 256, (CHC == CHC_N || CHC == CHC_U8) ? 4 : 1) void pointwise_kernel(
    const float* __restrict__ in, const float* __restrict__ wgt, const float* skip, float* out, int64_t M, int Kd,
    int N, int ldw, int run_base, int run_rem, const float* __restrict__ stats, void* __restrict__ packed,
    int pack_pad, double* __restrict__ sums, int code_bits, int main_grid, int rem_sub0) {
  static_assert(FUSE == 0 || MODE == 0, "the prologue belongs to the forward");
  constexpr bool CHUNKED = CHC > 0;  // CHC: 0 or CHC_U8 (the whole contraction in LDS), CHC_N or CHC_W
  constexpr int WAVES = (CHC == CHC_W || CHC == CHC_U8) ? 8 : 4;
  constexpr int CQ4 = CHUNKED ? CHC / 4 : 1;  // 16-byte items of a chunk row
  static_assert(!(CHUNKED && SUMS), "the sums are kept by the unchunked kernels only");
  constexpr int kThreads = 64 * WAVES;
  constexpr int BN = 16 * NT, BM = 16 * WAVES;
  constexpr int KB = FUSE != 0 ? FUSE : 4;
  extern __shared__ __attribute__((aligned(16))) float lds[];
  const int CH = CHUNKED ? CHC : Kd;  // contraction channels per weight chunk
  const int LDW = CH + 4;             // row stride: 16-byte aligned rows, each shifted by 4 banks
  constexpr int NBUF = CHUNKED ? 2 : 1;
  float* const Ws = lds;                    // [NBUF][BN][LDW]  weight(k, n) at [n * LDW + k - chunk start]
  float* const Cs = lds + NBUF * BN * LDW;  // [NBUF][NCONST][CH]  (fused prologue only)

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int li = lane & 15, lk = lane >> 4;
  // ids 8 apart share an XCD (and its L2): the blocks that read the same pixel rows for
  // different output-channel blocks run there back to back
  const int nblk_n = N / BN;
  const bool split = CHUNKED && (int)blockIdx.x >= main_grid;  // block-uniform
  const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
  const int run = (slot / nblk_n) * 8 + xcd;
  const int rem_i = (int)blockIdx.x - main_grid;
  const int nblk_i = split ? rem_i % nblk_n : slot % nblk_n;
  const int n0 = nblk_i * BN;
  if (FUSE != 0 && blockIdx.x == 0 && tid < pack_pad)  // tail of the last 128-byte row of codes
    static_cast<uint8_t*>(packed)[(M * Kd * FUSE) / 8 + tid] = 0;
  // tiles of BM pixels, or (split blocks) of one 16-pixel row group
  // Eight-wave unchunked blocks (DEAL): nothing ties the waves of a block to each other inside
  // the tile loop, so the 16-pixel row groups are dealt to the waves directly - wave w of all
  // (run_base blocks x 8) takes groups [w * groups / waves, (w + 1) * groups / waves) - and no
  // wave has more than one group above the average (128-pixel tiles per block: 3.06 tiles per
  // block meant 4 for some).
  constexpr bool DEAL = CHC == CHC_U8;
  int64_t t_begin, t_end;
  if (!DEAL) {
    t_begin = split ? rem_sub0 + rem_i / nblk_n : (int64_t)run * run_base + (run < run_rem ? run : run_rem);
    t_end = split ? t_begin + 1 : t_begin + run_base + (run < run_rem ? 1 : 0);
    if (t_end == t_begin) return;
  } else {  // (a wave without groups still takes part in the barriers)
    const int64_t groups = (M + 15) >> 4, waves = (int64_t)run_base * WAVES;
    const int64_t gw = (int64_t)run * WAVES + __builtin_amdgcn_readfirstlane(tid >> 6);
    t_begin = gw * groups / waves;
    t_end = (gw + 1) * groups / waves;
  }

  constexpr int planes[NCONST] = {P_MEAN, P_RSTD, P_GAMMA, P_BETA, P_CQ, P_FB};
  if (!CHUNKED) {  // the whole slice of the weights (and the prologue constants), once
    const int q4 = Kd >> 2;
    if (MODE == 0) {
      // transposed on the way: 16-byte loads along the output channels (the tensor's contiguous
      // direction), element-wise LDS writes.  A wave takes 16 k x 16 channels per step: its
      // writes of one element each land 4 banks apart per channel and one apart per k, on all 32
      // banks.
      for (int idx = tid; idx < BN * q4; idx += kThreads) {
        const int l = idx & 63, up = idx >> 6;
        const int k = 16 * (up / NT) + (l & 15), n = 16 * (up % NT) + 4 * (l >> 4);
        const float4 v = *reinterpret_cast<const float4*>(wgt + (int64_t)k * ldw + n0 + n);
        Ws[(n + 0) * LDW + k] = v.x;
        Ws[(n + 1) * LDW + k] = v.y;
        Ws[(n + 2) * LDW + k] = v.z;
        Ws[(n + 3) * LDW + k] = v.w;
      }
    } else {
      for (int idx = tid; idx < BN * q4; idx += kThreads) {
        const int n = idx / q4, q = idx - n * q4;
        *reinterpret_cast<float4*>(&Ws[n * LDW + 4 * q]) =
            *reinterpret_cast<const float4*>(wgt + (int64_t)(n0 + n) * ldw + 4 * q);
      }
    }
    if (FUSE != 0) {
      for (int idx = tid; idx < NCONST * q4; idx += kThreads) {
        const int pl = idx / q4, q = idx - pl * q4;
        *reinterpret_cast<float4*>(&Cs[pl * CH + 4 * q]) =
            *reinterpret_cast<const float4*>(stats + (int64_t)planes[pl] * Kd + 4 * q);
      }
    }
  }
  // chunked: this thread's share of a 128-channel chunk, held in registers between its global
  // loads and its LDS writes
  constexpr int WITEMS = CHUNKED ? BN * CQ4 / kThreads : 1;
  static_assert(!CHUNKED || BN * CQ4 % kThreads == 0, "whole staging items per thread");
  static_assert(!CHUNKED || (CHC == 16 * WAVES && WITEMS == NT), "forward staging: a wave per 16 k, an item per 16 channels");
  // (first-class vector values: as HIP's float4 structs this array was left in scratch memory by
  // the dgrad instantiation, with a full wait before every spill)
  floatx4 wreg[WITEMS];
  floatx4 creg = floatx4{0.f, 0.f, 0.f, 0.f};
  auto load_chunk = [&](int c0) __attribute__((always_inline)) {
#pragma unroll
    for (int it = 0; it < WITEMS; ++it) {
      const int idx = tid + it * kThreads;
      if (MODE == 0) {
        // four consecutive output channels of one k (the tensor's contiguous direction); the
        // transposition happens on the way into LDS.  A wave takes 16 k x 16 channels.
        const int k = 16 * wave + (lane & 15), n = 16 * it + 4 * (lane >> 4);
        wreg[it] = *reinterpret_cast<const floatx4*>(wgt + (int64_t)(c0 + k) * ldw + n0 + n);
      } else {
        const int n = idx / CQ4, q = idx % CQ4;
        wreg[it] = *reinterpret_cast<const floatx4*>(wgt + (int64_t)(n0 + n) * ldw + c0 + 4 * q);
      }
    }
    if (FUSE != 0 && tid < NCONST * CQ4) {
      const int pl = tid / CQ4, q = tid % CQ4;
      creg = *reinterpret_cast<const floatx4*>(stats + (int64_t)planes[pl] * Kd + c0 + 4 * q);
    }
  };
  auto store_chunk = [&](int buf) __attribute__((always_inline)) {
    float* W = Ws + buf * BN * LDW;
#pragma unroll
    for (int it = 0; it < WITEMS; ++it) {
      if (MODE == 0) {
        // (rows 4 banks apart: the 64 lanes of one of these writes spread over all 32 banks)
        const int k = 16 * wave + (lane & 15), n = 16 * it + 4 * (lane >> 4);
#pragma unroll
        for (int e = 0; e < 4; ++e) W[(n + e) * LDW + k] = wreg[it][e];
      } else {
        const int idx = tid + it * kThreads;
        const int n = idx / CQ4, q = idx % CQ4;
        *reinterpret_cast<floatx4*>(&W[n * LDW + 4 * q]) = wreg[it];
      }
    }
    if (FUSE != 0 && tid < NCONST * CQ4) {
      const int pl = tid / CQ4, q = tid % CQ4;
      *reinterpret_cast<floatx4*>(&Cs[buf * NCONST * CH + pl * CH + 4 * q]) = creg;
    }
  };
  if (CHUNKED) {
    load_chunk(0);
    store_chunk(0);
  }
  __syncthreads();

  const int KG = Kd >> 4;        // 16-channel groups of the contraction
  const int GPC = CH >> 4;       // ... per weight chunk
  const int NC = CHUNKED ? Kd / CHC : 1;

  // Eq. 1-3 on the four channels kl + 4lk .. +3 (of chunk constants Cc) of pixel prow, and Eq. 9
  // with the codes written for the block's share of the channel groups: all output-channel
  // blocks of a pixel tile normalize the same values, and they take turns over the groups in
  // quantizing them, so that every block has the same amount of vector work (were it all the
  // first block's, the compute units holding first blocks would finish last).  kg = 16-channel
  // group of the whole contraction.
  auto bn_relu_quant = [&](float4& av, const float* Cc, int kl, int kg, int64_t prow, bool pok)
                           __attribute__((always_inline)) {
    const float4 c_mean = *reinterpret_cast<const float4*>(&Cc[0 * CH + kl + 4 * lk]);
    const float4 c_rstd = *reinterpret_cast<const float4*>(&Cc[1 * CH + kl + 4 * lk]);
    const float4 c_gm = *reinterpret_cast<const float4*>(&Cc[2 * CH + kl + 4 * lk]);
    const float4 c_bt = *reinterpret_cast<const float4*>(&Cc[3 * CH + kl + 4 * lk]);
    const float xs[4] = {av.x, av.y, av.z, av.w};
    const float mean[4] = {c_mean.x, c_mean.y, c_mean.z, c_mean.w};
    const float rstd[4] = {c_rstd.x, c_rstd.y, c_rstd.z, c_rstd.w};
    const float gm[4] = {c_gm.x, c_gm.y, c_gm.z, c_gm.w};
    const float bt[4] = {c_bt.x, c_bt.y, c_bt.z, c_bt.w};
    float a2[4], a3[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const float d = xs[e] - mean[e];
      const float a1 = d * rstd[e];  // Eq. 1
      const float t = gm[e] * a1;
      a2[e] = t + bt[e];             // Eq. 2
      a3[e] = a2[e] > 0.0f ? a2[e] : 0.0f;  // Eq. 3
    }
    av = make_float4(a3[0], a3[1], a3[2], a3[3]);
    if (kg % nblk_n == nblk_i) {  // wave-uniform
      const float4 c_cq = *reinterpret_cast<const float4*>(&Cc[4 * CH + kl + 4 * lk]);
      const int4 c_fb = *reinterpret_cast<const int4*>(&Cc[5 * CH + kl + 4 * lk]);
      const float cq[4] = {c_cq.x, c_cq.y, c_cq.z, c_cq.w};
      const int32_t fb[4] = {c_fb.x, c_fb.y, c_fb.z, c_fb.w};
      uint32_t word = 0;
#pragma unroll
      for (int e = 0; e < 4; ++e) word |= quant_code<KB>(a2[e], cq[e], fb[e]) << (KB * e);  // Eq. 9
      if (pok) {
        const int64_t e0 = prow * Kd + kg * 16 + 4 * lk;  // flat index of the first of 4 codes
        if (KB == 4) reinterpret_cast<uint16_t*>(packed)[e0 >> 2] = (uint16_t)word;
        else reinterpret_cast<uint32_t*>(packed)[e0 >> 2] = word;
      }
    }
  };

  // Whole tiles: a wave has 16 pixels x all BN channels of each tile of the block's run.
  auto walk = [&]() __attribute__((always_inline)) {
    // The ring of loads runs on across pixel tiles: while a tile's last groups are contracted
    // and its results stored, the first groups of the block's next tile are already in flight.
    auto row_ptr = [&](int64_t tile) __attribute__((always_inline)) {
      const int64_t p = DEAL ? tile * 16 + li : tile * BM + wave * 16 + li;
      return in + (p < M ? p : 0) * Kd + 4 * lk;  // rows past the end read row 0 and are never stored
    };
    const float* xp = row_ptr(t_begin);
    float4 ring[PF];
#pragma unroll
    for (int s = 0; s < PF; ++s) ring[s] = *reinterpret_cast<const float4*>(xp + 16 * s);
    // (the same explicit wait as after a tile's stores, see below: the contraction loop is then
    // entered with nothing pending on every path, and the compiler can count the ring's loads)
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0)

    // SUMS: this lane's pixels (at most a few dozen), its four channels of every tile column.
    // The forward sums feed a variance (sum of squares minus square of the sum): fp64 from the
    // first addition.  The gradient sums have no such cancellation: fp32 per lane, fp64 from the
    // reduction over lanes on.
    using sum_t = typename std::conditional<MODE == 0, double, float>::type;
    sum_t s1[NT][4], s2[NT][4];
#pragma unroll
    for (int j = 0; j < NT; ++j)
#pragma unroll
      for (int r = 0; r < 4; ++r) s1[j][r] = s2[j][r] = (sum_t)0;
    // dgrad sums: Eq. 10 constants of the lane's channels n0 + 16j + 4lk .. +3.  Eq. 10 is one add
    // and one multiply: step * ((code - 2^(K-1) + fb) + 0.5) = step * (code + offh), offh exact in
    // fp32 while |fb| < 2^22.
    float4 r_step[NT], r_offh[NT];
    if (SUMS && MODE == 1) {
#pragma unroll
      for (int j = 0; j < NT; ++j) {
        const int c = n0 + 16 * j + 4 * lk;
        r_step[j] = *reinterpret_cast<const float4*>(stats + P_STEP * N + c);
        const int4 fb = *reinterpret_cast<const int4*>(reinterpret_cast<const int32_t*>(stats) + P_FB * N + c);
        const float half = 0.5f - (float)(1 << (code_bits - 1));
        r_offh[j] = make_float4((float)fb.x + half, (float)fb.y + half, (float)fb.z + half, (float)fb.w + half);
      }
    }

    int step = 0;  // (tile, chunk) pairs done so far: chunk buffers alternate with it
    for (int64_t tile = t_begin; tile < t_end; ++tile) {
      const bool has_next = tile + 1 < t_end;
      const float* xpn = row_ptr(has_next ? tile + 1 : tile);
      const int64_t prow = DEAL ? tile * 16 + li : tile * BM + wave * 16 + li;
      const bool pok = prow < M;
      floatx4 acc[NT][1];  // acc[j][0][r]: pixel prow, channel n0 + 16j + 4lk + r
#pragma unroll
      for (int j = 0; j < NT; ++j) acc[j][0] = floatx4{0.f, 0.f, 0.f, 0.f};
      // What the epilogue reads from memory is requested now, without branches on the lane: asked
      // for between the tile's stores, each value would cost a wait for the store before it as
      // well (a load's wait covers everything older), four memory round trips in a row per tile.
      float4 skv[NT];
      uint32_t cwv[NT];
      {
        const int64_t o0 = (pok ? prow : 0) * N + n0 + 4 * lk;
        if (skip != nullptr) {
#pragma unroll
          for (int j = 0; j < NT; ++j) skv[j] = *reinterpret_cast<const float4*>(skip + o0 + 16 * j);
        }
        if (SUMS && MODE == 1) {
          const uint8_t* codes = static_cast<const uint8_t*>(packed);
#pragma unroll
          for (int j = 0; j < NT; ++j)
            cwv[j] = code_bits == 4 ? (uint32_t) * reinterpret_cast<const uint16_t*>(codes + ((o0 + 16 * j) >> 1))
                                    : *reinterpret_cast<const uint32_t*>(codes + o0 + 16 * j);
        }
      }

      for (int c = 0; c < NC; ++c, ++step) {
        const int buf = CHUNKED ? (step & 1) : 0;
        const bool more = CHUNKED && (has_next || c + 1 < NC);  // another chunk follows: fetch it now
        if (more) load_chunk(c + 1 < NC ? (c + 1) * CHC : 0);
        const float* W = Ws + buf * BN * LDW;
        const float* Cc = Cs + buf * NCONST * CH;
        for (int g0 = 0; g0 < GPC; g0 += PF) {
#pragma unroll
          for (int s = 0; s < PF; ++s) {
            const int kl = (g0 + s) * 16;     // offset inside the chunk
            const int kg = c * GPC + g0 + s;  // group of the whole contraction
            float4 a[1] = {ring[s]};
            if (FUSE != 0) bn_relu_quant(a[0], Cc, kl, kg, prow, pok);
            float4 wf[NT];
#pragma unroll
            for (int j = 0; j < NT; ++j)
              wf[j] = *reinterpret_cast<const float4*>(&W[(16 * j + li) * LDW + kl + 4 * lk]);
            mma_k4<BF16, NT, 1>(wf, a, acc);
            // Refill the slot AFTER the MFMAs that read it (no copy of the old value is needed, so
            // nothing has to wait for a younger load), without a branch (past the block's last tile
            // the loads re-read that tile and are never used: behind a branch the compiler cannot
            // count the loads in flight and waits for all of them), and pinned here (left alone, the
            // scheduler sinks all PF refills to the end of the loop body, right in front of their use).
            {
              const bool same = kg + PF < KG;
              const float* src = (same ? xp : xpn) + 16 * (same ? kg + PF : kg + PF - KG);
              ring[s] = *reinterpret_cast<const float4*>(src);
              __builtin_amdgcn_sched_barrier(0);
            }
          }
        }
        if (CHUNKED) {
          // the other buffer was last read in the previous step, which every wave left at that
          // step's barrier
          if (more) store_chunk(buf ^ 1);
          __syncthreads();
        }
      }

      // 16-byte stores (and shortcut loads) of four consecutive channels of the pixel
      if (pok) {
#pragma unroll
        for (int j = 0; j < NT; ++j) {
          const int64_t o = prow * N + n0 + 16 * j + 4 * lk;
          float4 v = make_float4(acc[j][0][0], acc[j][0][1], acc[j][0][2], acc[j][0][3]);
          if (skip != nullptr) {
            const float4 sv = skv[j];
            v.x += sv.x; v.y += sv.y; v.z += sv.z; v.w += sv.w;
          }
          *reinterpret_cast<float4*>(out + o) = v;
          if (SUMS && MODE == 0) {
            const float vs[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
            for (int r = 0; r < 4; ++r) {
              const double d = (double)vs[r];
              s1[j][r] += d;
              s2[j][r] += d * d;
            }
          }
          if (SUMS && MODE == 1) {
            // Eq. 6 and the sum of Eq. 7 by linearity: sum A1~ dA2 = (sum A2~ dA2 - beta sum dA2) / gamma,
            // so a lane adds up dA2 and A2~ dA2 (a handful of pixels in fp32, fp64 from the reduction
            // over lanes on) and beta, gamma enter once per block - vector instructions cost matrix
            // time here, and this epilogue runs once per 16 x 64 outputs.
            const uint32_t cw = cwv[j];
            // one code per byte (a byte at a fixed position converts to float in one instruction); K = 4:
            // codes 0, 2 in the bytes of one word, codes 1, 3 in those of the other
            float code[4];
            if (code_bits == 4) {  // uniform
              const uint32_t ce = cw & 0x0F0Fu, co = (cw >> 4) & 0x0F0Fu;
              code[0] = (float)(ce & 0xFFu);
              code[1] = (float)(co & 0xFFu);
              code[2] = (float)((ce >> 8) & 0xFFu);
              code[3] = (float)((co >> 8) & 0xFFu);
            } else {
#pragma unroll
              for (int r = 0; r < 4; ++r) code[r] = (float)((cw >> (8 * r)) & 0xFFu);
            }
            const float vs[4] = {v.x, v.y, v.z, v.w};
            const float st4[4] = {r_step[j].x, r_step[j].y, r_step[j].z, r_step[j].w};
            const float oh4[4] = {r_offh[j].x, r_offh[j].y, r_offh[j].z, r_offh[j].w};
#pragma unroll
            for (int r = 0; r < 4; ++r) {
              const float a2t = st4[r] * (code[r] + oh4[r]);       // Eq. 10
              const float da2 = a2t > 0.0f ? vs[r] : 0.0f;         // Eq. 6
              s1[j][r] += da2;
              s2[j][r] = __builtin_fmaf(a2t, da2, s2[j][r]);
            }
          }
        }
      }
      // The tile's stores share the counter of the loads and may complete out of order with them:
      // while one is pending the compiler must wait for everything before it may read a loaded
      // register, and it would do so at the head of the contraction loop in every iteration.  One
      // explicit wait here (the next tile's first groups have been in flight for a while) lets it
      // count the ring's loads instead.
      __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0)
      xp = xpn;
    }
    if constexpr (SUMS) {
      // fixed order: the 16 pixels of a row of lanes by a butterfly, then the waves through LDS
      __syncthreads();  // every wave is done with the weights
      double* red = reinterpret_cast<double*>(lds);  // [2][WAVES][BN]
#pragma unroll
      for (int j = 0; j < NT; ++j)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const double t1 = row16_sum((double)s1[j][r]), t2 = row16_sum((double)s2[j][r]);
          if (li == 0) {
            red[(0 * WAVES + wave) * BN + 16 * j + 4 * lk + r] = t1;
            red[(1 * WAVES + wave) * BN + 16 * j + 4 * lk + r] = t2;
          }
        }
      __syncthreads();
      for (int ch = tid; ch < BN; ch += kThreads) {
        double t1 = 0.0, t2 = 0.0;
#pragma unroll
        for (int k = 0; k < WAVES; ++k) {
          t1 += red[(0 * WAVES + k) * BN + ch];
          t2 += red[(1 * WAVES + k) * BN + ch];
        }
        if (MODE == 1)  // the lanes added up A2~ dA2: A1~ = (A2~ - beta) / gamma (inverse of Eq. 2)
          t2 = (t2 - (double)stats[P_BETA * N + n0 + ch] * t1) / (double)stats[P_GAMMA * N + n0 + ch];
        sums[((int64_t)run * 2 + 0) * N + n0 + ch] = t1;
        sums[((int64_t)run * 2 + 1) * N + n0 + ch] = t2;
      }
    }
  };

  // A split row group: the block has 16 pixels x BN channels, wave w contracts the w-th
  // 16-channel group of every weight chunk (a quarter of the contraction, so a quarter of a whole
  // tile's time on each SIMD), and the four partial results are added through LDS in wave order.
  auto walk_split = [&]() __attribute__((always_inline)) {
    const int64_t prow = t_begin * 16 + li;
    const bool pok = prow < M;
    const float* xp = in + (pok ? prow : 0) * Kd + 16 * wave + 4 * lk;  // rows past the end read row 0
    // (one chunk of lookahead: a split block shares its compute unit with whole-tile blocks that
    // keep the matrix cores busy, so its own latency is hidden by them and a ring is not needed)
    float4 a_next = *reinterpret_cast<const float4*>(xp);
    floatx4 acc[NT][1];
#pragma unroll
    for (int j = 0; j < NT; ++j) acc[j][0] = floatx4{0.f, 0.f, 0.f, 0.f};
    const int kl = 16 * wave;
    for (int c = 0; c < NC; ++c) {
      const int buf = c & 1;
      const bool more = c + 1 < NC;
      if (more) load_chunk((c + 1) * CHC);
      const float* W = Ws + buf * BN * LDW;
      const float* Cc = Cs + buf * NCONST * CH;
      float4 a[1] = {a_next};
      a_next = *reinterpret_cast<const float4*>(xp + CHC * (more ? c + 1 : c));  // (last: re-read, unused)
      if (FUSE != 0) bn_relu_quant(a[0], Cc, kl, c * GPC + wave, prow, pok);
      float4 wf[NT];
#pragma unroll
      for (int j = 0; j < NT; ++j)
        wf[j] = *reinterpret_cast<const float4*>(&W[(16 * j + li) * LDW + kl + 4 * lk]);
      mma_k4<BF16, NT, 1>(wf, a, acc);
      if (more) store_chunk(buf ^ 1);
      __syncthreads();
    }
    // every wave has left the last chunk: the weights' LDS now carries the partial results
    float* red = lds;  // [WAVES][NT][4][64]
#pragma unroll
    for (int j = 0; j < NT; ++j)
#pragma unroll
      for (int r = 0; r < 4; ++r) red[((wave * NT + j) * 4 + r) * 64 + lane] = acc[j][0][r];
    __syncthreads();
    if constexpr (NT == WAVES) {  // wave w finishes the w-th 16-channel column
      float v[4];
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        float t = red[((0 * NT + wave) * 4 + r) * 64 + lane];
#pragma unroll
        for (int k = 1; k < WAVES; ++k) t += red[((k * NT + wave) * 4 + r) * 64 + lane];
        v[r] = t;
      }
      if (pok) {
        const int64_t o = prow * N + n0 + 16 * wave + 4 * lk;
        float4 vv = make_float4(v[0], v[1], v[2], v[3]);
        if (skip != nullptr) {
          const float4 sv = *reinterpret_cast<const float4*>(skip + o);
          vv.x += sv.x; vv.y += sv.y; vv.z += sv.z; vv.w += sv.w;
        }
        *reinterpret_cast<float4*>(out + o) = vv;
      }
    }
  };
  if (CHUNKED && split) {
    if constexpr (CHUNKED && NT == WAVES) walk_split();
  } else {
    walk();
  }
}

struct PointwisePlan {
  int nt;
  bool chunked;
  bool wide;  // chunked with eight-wave blocks and CHC_W-channel chunks
  bool u8;    // unchunked with eight-wave blocks
  int run_base, run_rem;
  int rows;  // blocks per output-channel block that have tiles (= rows of sums)
  unsigned grid;
  int main_grid;  // blocks that walk whole tiles; the ones after them take one split row group each
  int rem_sub0;   // first 16-pixel row group of the split part
};

// Blocks of a kernel that its registers allow on one compute unit (asked of the runtime once per
// kernel).  The grid is sized to what is resident at once: a plan that counts on four blocks per
// unit where the registers admit three leaves a quarter of the blocks for a second, mostly empty
// round.
int resident_blocks(const void* kern, int threads) {
  static std::mutex mu;
  static std::unordered_map<const void*, int> cache;
  std::lock_guard<std::mutex> lock(mu);
  auto it = cache.find(kern);
  if (it != cache.end()) return it->second;
  int n = 0;
  if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, kern, threads, 0) != hipSuccess || n < 1) {
    (void)hipGetLastError();
    n = 1;
  }
  cache.emplace(kern, n);
  return n;
}

bool make_pointwise_plan(const ConvGeom& g, int mode, bool fuse, bool sums, PointwisePlan& p, int occ_regs = 4) {
  if (g.R != 1 || g.S != 1 || g.stride != 1 || g.pad != 0) return false;
  const int Kd = mode == 0 ? g.Cin : g.Cout, N = mode == 0 ? g.Cout : g.Cin;
  if (Kd % 64 != 0 || N % 16 != 0) return false;
  p.chunked = Kd > KC;
  p.wide = false;
  const int64_t M = (int64_t)g.N * g.H * g.W;
  if (M * Kd >= ((int64_t)1 << 31) || M * N >= ((int64_t)1 << 31)) return false;
  p.nt = N % 64 == 0 ? 4 : (N % 32 == 0 ? 2 : 1);
  const int nblk_n = N / (16 * p.nt);
  // Chunked: whole rounds of one 64-pixel tile per SIMD (a block's four waves sit on the four
  // SIMDs of a compute unit) and the row groups left over split four ways over the contraction.
  // A split block goes through the same chain of chunk loads and barriers as a whole tile with a
  // quarter of the matrix work: with fewer than two rounds beside it, it would be what the grid
  // waits for, and eight-wave blocks on 128-pixel tiles (half the weight staging per pixel) do
  // better.
  const int64_t sub = (M + 15) / 16;
  const int64_t rounds = (sub / 4) * nblk_n / 256;
  const bool balanced = p.chunked && p.nt == 4 && rounds >= 2;
  p.wide = p.chunked && !balanced && Kd % CHC_W == 0;
  // as many blocks as fit the compute units at once (the weights' LDS; four waves per SIMD)
  const unsigned lds = pointwise_lds_bytes(Kd, p.nt, fuse, p.wide);
  int occ = (int)((160u * 1024u) / lds);
  // a long unchunked contraction leaves LDS for two blocks: eight waves each, or a SIMD would
  // have only two waves to hide its loads and stores with
  // (not where the kernel also keeps per-channel sums - their registers do not fit four waves per
  // SIMD - and, measured, no gain where a single output-channel block does all of the quantizing)
  p.u8 = !p.chunked && occ <= 2 && !sums && !(fuse && nblk_n < 4);
  const int occ_max = p.wide || p.u8 ? 2 : 4;
  if (occ > occ_max) occ = occ_max;
  if (occ > occ_regs) occ = occ_regs;
  if (occ < 1) occ = 1;
  const int bm = p.wide || p.u8 ? 128 : 64;
  int64_t mtiles = (M + bm - 1) / bm;
  int64_t rem_sub = 0;
  if (balanced) {
    mtiles = rounds * 256 / nblk_n;
    rem_sub = sub - 4 * mtiles;
  }
  int64_t runs = (int64_t)256 * occ / nblk_n / 8 * 8;  // blocks per output-channel block, whole XCD rounds
  if (runs > kMaxPartialBlocks) runs = kMaxPartialBlocks;  // one row of sums per block
  if (runs < 8) runs = 8;
  if (runs > (mtiles + 7) / 8 * 8) runs = (mtiles + 7) / 8 * 8;
  if (p.u8) {  // the kernel deals the row groups to the waves of `runs` blocks itself
    p.run_base = (int)runs;
    p.run_rem = 0;
    p.rows = (int)runs;
  } else {
    p.run_base = runs > 0 ? (int)(mtiles / runs) : 0;
    p.run_rem = runs > 0 ? (int)(mtiles % runs) : 0;
    p.rows = p.run_base > 0 ? (int)runs : p.run_rem;
  }
  p.main_grid = (int)(runs * nblk_n);
  p.rem_sub0 = (int)(4 * mtiles);
  p.grid = (unsigned)(p.main_grid + rem_sub * nblk_n);
  return true;
}

template <int MODE, int FUSE>
int launch_pointwise(hipStream_t st, const ConvGeom& g, bool bf16, const float* in, const float* w, const float* skip,
                     float* out, const float* stats, void* packed, double* sums, int* rows, int code_bits = 0) {
  PointwisePlan p;
  if (!make_pointwise_plan(g, MODE, FUSE != 0, sums != nullptr, p)) return ABL_ERR_SHAPE;
  const int64_t M = (int64_t)g.N * g.H * g.W;
  const int Kd = MODE == 0 ? g.Cin : g.Cout, N = MODE == 0 ? g.Cout : g.Cin;
  const int64_t raw = FUSE != 0 ? (M * Kd * FUSE + 7) / 8 : 0;
  const int pack_pad = (int)((raw + 127) / 128 * 128 - raw);
  const unsigned lds = pointwise_lds_bytes(Kd, p.nt, FUSE != 0, p.wide);
  // (the chunked kernels keep no sums: their registers cost more than the pass they save)
  if (p.chunked) sums = nullptr;
  if (rows != nullptr) *rows = sums != nullptr ? p.rows : 0;
#define ABL_PW(NT_, CHC_)                                                                                    \
  do {                                                                                                       \
    if (sums != nullptr) ABL_PW_S(NT_, CHC_, true);                                                          \
    else ABL_PW_S(NT_, CHC_, false);                                                                         \
  } while (0)
#define ABL_PW_S(NT_, CHC_, SUMS_)                                                                           \
  do {                                                                                                       \
    auto kern = bf16 ? pointwise_kernel<MODE, NT_, CHC_, true, FUSE, (SUMS_) && (CHC_) <= 0>                 \
                     : pointwise_kernel<MODE, NT_, CHC_, false, FUSE, (SUMS_) && (CHC_) <= 0>;               \
    if (lds > 64 * 1024 &&                                                                                   \
        hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, \
                            lds) != hipSuccess)                                                              \
      return ABL_ERR_HIP;                                                                                    \
    /* same variant, grid sized to the blocks the kernel's registers allow per compute unit */              \
    make_pointwise_plan(g, MODE, FUSE != 0, sums != nullptr, p,                                              \
                        resident_blocks(reinterpret_cast<const void*>(kern),                                 \
                                        (CHC_) == CHC_W || (CHC_) == CHC_U8 ? 512 : 256));                   \
    if (rows != nullptr) *rows = sums != nullptr ? p.rows : 0;                                               \
    kern<<<p.grid, (CHC_) == CHC_W || (CHC_) == CHC_U8 ? 512 : 256, lds, st>>>(in, w, skip, out, M, Kd, N, g.Cout, p.run_base,   \
                                                           p.run_rem, stats, packed, pack_pad, sums,         \
                                                           code_bits, p.main_grid, p.rem_sub0);              \
  } while (0)
#define ABL_PW_C(NT_)                      \
  do {                                     \
    if (p.wide) ABL_PW(NT_, CHC_W);        \
    else if (p.chunked) ABL_PW(NT_, CHC_N); \
    else if (p.u8) ABL_PW(NT_, CHC_U8);    \
    else ABL_PW(NT_, 0);                   \
  } while (0)
  if (p.nt == 4) ABL_PW_C(4);
  else if (p.nt == 2) ABL_PW_C(2);
  else ABL_PW_C(1);
#undef ABL_PW_C
#undef ABL_PW
#undef ABL_PW_S
  return hip_status();
}

}  // namespace

int launch_pointwise_dgrad_reduce(hipStream_t st, const ConvGeom& g, int K, bool bf16, const float* dy, const float* w,
                                  const void* packed, const void* stats, float* da3, double* sums, int* rows) {
  if ((K != 4 && K != 8) || sums == nullptr || rows == nullptr) return ABL_ERR_ARG;
  return launch_pointwise<1, 0>(st, g, bf16, dy, w, nullptr, da3, static_cast<const float*>(stats),
                                const_cast<void*>(packed), sums, rows, K);
}

bool pointwise_supported(const ConvGeom& g, int mode) {
  PointwisePlan p;
  return make_pointwise_plan(g, mode, false, false, p);
}

int launch_pointwise_conv(hipStream_t st, const ConvGeom& g, int mode, bool bf16, const float* in, const float* w,
                          const float* skip, float* out, double* sums, int* rows) {
  if (mode == 0) return launch_pointwise<0, 0>(st, g, bf16, in, w, skip, out, nullptr, nullptr, sums, rows);
  if (rows != nullptr) *rows = 0;
  return launch_pointwise<1, 0>(st, g, bf16, in, w, nullptr, out, nullptr, nullptr, nullptr, nullptr);
}

int launch_pointwise_fwd_fused(hipStream_t st, const ConvGeom& g, int K, bool bf16, const float* x, const float* stats,
                               const float* w, const float* skip, float* y, void* packed, double* sums, int* rows) {
  if (K == 4) return launch_pointwise<0, 4>(st, g, bf16, x, w, skip, y, stats, packed, sums, rows);
  if (K == 8) return launch_pointwise<0, 8>(st, g, bf16, x, w, skip, y, stats, packed, sums, rows);
  return ABL_ERR_ARG;
}

}  // namespace abl
