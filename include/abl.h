/* abl - approximate-activation backprop layer for AMD MI355X (gfx950).
 *
 * C ABI of the hot path of "Backprop with Approximate Activations for
 * Memory-efficient Network Training" (Chakrabarti & Moseley, arXiv 1901.07988):
 * one pre-activation layer  BatchNorm -> scale & bias -> ReLU -> convolution
 * (Sec. 3.1, Eq. 1-4) whose forward pass is exact and keeps only a K-bit copy of
 * the pre-ReLU activation A2 plus per-channel vectors (Sec. 3.2, Eq. 9), and whose
 * backward pass (Eq. 5-8) is computed from that copy alone (Eq. 10).
 *
 * General rules, valid for every entry point unless it says otherwise:
 *   - every tensor pointer is a DEVICE pointer owned by the caller, 16-byte
 *     aligned; the library allocates nothing, keeps no state (abl_backward_noalloc apart:
 *     it remembers where its fixed workspace lives), enqueues its
 *     kernels on `stream` (a hipStream_t passed as void*, NULL = default stream)
 *     and never synchronises.  Shapes and sizes are host values.
 *   - activations are fp32, NHWC ("first dim = sample, last dim = channel",
 *     Sec. 3.1); conv weights are fp32 [R][S][Cin][Cout]; the linear transform of
 *     Eq. 4 is a zero-padded cross-correlation without bias.
 *   - the BN tensor of a layer is its input: M = N*H*W rows of Cin channels,
 *     E = M*Cin elements.  Batch statistics use the biased variance, eps = 1e-5.
 *   - K is 4 or 8, or 32 for exact storage (the paper's baseline, Sec. 4: one full-precision
 *     copy of A2 per layer, alpha = 1): the "codes" are then the fp32 values themselves, the
 *     quantizer planes of `stats` are zero, and the backward pass is exact back-propagation.
 *     The fused-kernel entry points (abl_bn_conv_fwd, abl_conv_dgrad_bn_reduce,
 *     abl_conv_bwd_bn_reduce) and the abl_postact_* grouping take K = 4 or 8 only.
 *   - `flags` is a bit set of the ABL_* flags an entry point documents; unknown bits are an
 *     ABL_ERR_ARG.
 *   - return value: ABL_OK or an ABL_ERR_* code; on error nothing was enqueued
 *     (ABL_ERR_HIP: a launch failed, earlier launches of the call may have run).  The stack
 *     calls validate every layer's shape and pointers before their first launch.
 *   - preconditions that are NOT checked: finite inputs, gamma != 0.
 *
 * Packed store (opaque to callers, specified because parity is on bytes):
 * codes in flat NHWC element order; K=8: byte e = code e; K=4: byte e/2 holds
 * code 2j in bits 0-3 and code 2j+1 in bits 4-7; zero padded to a multiple of
 * 128 bytes.  `stats` = 8 planes of Cin 4-byte values:
 * mean, var, rstd, gamma, beta, cq = 2^K/(6 gamma), step = 6 gamma/2^K (fp32) and
 * fb = floor(beta*cq) (int32).
 */
#ifndef ABL_H_
#define ABL_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct abl_shape {
  int32_t N, H, W;      /* input batch, height, width                        */
  int32_t Cin, Cout;    /* input (= BN) channels, output channels            */
  int32_t R, S;         /* filter height, width                              */
  int32_t stride, pad;  /* same in both spatial dims; Ho=(H+2pad-R)/stride+1 */
} abl_shape;

enum {
  ABL_OK = 0,
  ABL_ERR_ARG = 1,      /* null / misaligned pointer, unsupported K, bad flag       */
  ABL_ERR_SHAPE = 2,    /* non-positive dim, empty output, more than 2^31-1 elements */
  ABL_ERR_SCRATCH = 3,  /* scratch buffer smaller than abl_scratch_bytes            */
  ABL_ERR_HIP = 4       /* kernel launch failed                                     */
};

enum {
  ABL_ACCUM_DX = 1u << 0, /* abl_backward / abl_bn_bwd: dx += result (residual-stream gradient, Sec. 3.4) */
  ABL_MATH_BF16 = 1u << 1, /* contractions (Eq. 4, Eq. 5): operands rounded to bf16 on the way into the
                             matrix cores, fp32 accumulation; everything else (statistics, codes,
                             BN forward/backward) is unchanged.  Default: fp32 operands. */
  ABL_XIN_F32 = 1u << 3,   /* abl_postact_backward: xin is the exact fp32 conv input            */
  ABL_NAIVE_FWD = 1u << 5, /* abl_forward / abl_stack_forward: the comparison baseline of Sec. 4 - the
                              convolution consumes the ReLU of the DEQUANTIZED copy (Eq. 10) instead
                              of the exact A3, so the approximation error enters the forward pass and
                              compounds from layer to layer; for error studies, not for speed */
  ABL_XIN_PACKED = 1u << 4 /* abl_postact_backward: xin / xin_stats are the previous layer's
                              packed store and stats (its ReLU output is rebuilt on the fly)   */
};

#define ABL_BN_EPS 1e-5f
#define ABL_STATS_PLANES 8

const char* abl_error_string(int code);

/* Bytes of the K-bit store of one layer's A2 (Sec. 3.4: alpha = K/32 of the fp32
 * tensor): ceil(E*K/8) rounded up to 128.  0 on invalid arguments. */
size_t abl_packed_bytes(const abl_shape* shape, int K);
/* Bytes of the per-channel vectors kept with the store (Sec. 3.2): 32*Cin. */
size_t abl_stats_bytes(const abl_shape* shape);
/* Bytes of reusable workspace that abl_forward / abl_backward need for this
 * shape: one fp32 tensor for A3 (forward) or its gradient (backward) - the
 * "+1" buffer of Sec. 3.4 - plus reduction partials. */
size_t abl_scratch_bytes(const abl_shape* shape, int K);
/* Which kernels abl_forward uses for this shape when y does not alias x (for tools that report the
 * launches of a layer step): 1 = one kernel applies Eq. 1-3 and Eq. 9 while it stages the input of
 * the contraction (abl_bn_conv_fwd), 0 = the normalise-ReLU-pack pass followed by the plain
 * contraction (abl_bn_relu_pack, abl_conv_fwd).  Negative (an ABL_ERR_ code, negated) on invalid
 * arguments.  flags as for abl_forward. */
int abl_forward_is_fused(const abl_shape* shape, int K, uint32_t flags);

/* Forward of one layer (Sec. 3.2; Eq. 1-4 and Eq. 9).
 *   x      [N,H,W,Cin]      in
 *   W      [R,S,Cin,Cout]   in
 *   gamma, beta [Cin]       in
 *   skip   [N,Ho,Wo,Cout]   in, may be NULL; y = conv(...) + skip (identity
 *                           shortcut, Sec. 3.4).  May alias y.
 *   y      [N,Ho,Wo,Cout]   out.  May alias x (x is consumed before y is written).
 *   packed abl_packed_bytes out: K-bit codes of A2
 *   stats  abl_stats_bytes  out
 *   scratch                 workspace, contents undefined afterwards
 * y is computed from the full-precision A3 and does not depend on K.  flags: ABL_MATH_BF16. */
int abl_forward(void* stream, const abl_shape* shape, int K, uint32_t flags,
                const float* x, const float* W, const float* gamma, const float* beta,
                const float* skip, void* scratch, size_t scratch_bytes,
                float* y, void* packed, void* stats);

/* Backward of one layer from the stored copy only (Sec. 3.2; Eq. 10, Eq. 5-8).
 *   packed, stats           in, as written by abl_forward (gamma and beta are
 *                           taken from the snapshot in `stats`)
 *   dy     [N,Ho,Wo,Cout]   in
 *   W      [R,S,Cin,Cout]   in
 *   dx     [N,H,W,Cin]      out (or accumulated into with ABL_ACCUM_DX).  May alias dy.
 *   dW     [R,S,Cin,Cout]   out: approximate (uses the dequantized A3)
 *   dgamma, dbeta [Cin]     out: dgamma approximate, dbeta exact (Sec. 3.3)
 * flags: ABL_ACCUM_DX, ABL_MATH_BF16. */
int abl_backward(void* stream, const abl_shape* shape, int K, uint32_t flags,
                 const void* packed, const void* stats, const float* dy, const float* W,
                 void* scratch, size_t scratch_bytes,
                 float* dx, float* dW, float* dgamma, float* dbeta);

/* abl_backward for callers that cannot allocate device memory or pass a workspace: code under
 * HIP graph capture, tight serving or training loops, harnesses that forbid hipMalloc.  Same
 * arguments, outputs, aliasing rules and flags as abl_backward, without `scratch`: the workspace is
 * a fixed array of ABL_NOALLOC_SCRATCH_BYTES in device memory that the library itself holds (one
 * copy on every GPU that loads the library, kept until the process ends).  The call allocates and
 * frees nothing; its first use on a device looks up that device's address of the array.
 *   - shapes whose abl_scratch_bytes(shape, K) exceeds the array give ABL_ERR_SCRATCH and enqueue
 *     nothing (abl_noalloc_scratch_limit() returns the limit); a failed address lookup gives
 *     ABL_ERR_HIP; other errors as abl_backward.
 *   - all calls on one GPU share the one array and it keeps the previous call's contents (nothing
 *     in it needs clearing: whatever a kernel reads there an earlier kernel of the same call has
 *     written).  Two calls that overlap in time on one GPU - different streams, or graphs replayed
 *     concurrently - race on it; calls on one stream are ordered and safe. */
#define ABL_NOALLOC_SCRATCH_BYTES (32u << 20)
size_t abl_noalloc_scratch_limit(void);
int abl_backward_noalloc(void* stream, const abl_shape* shape, int K, uint32_t flags,
                         const void* packed, const void* stats, const float* dy, const float* W,
                         float* dx, float* dW, float* dgamma, float* dbeta);

/* The same layer with a leaky ReLU in place of Eq. 3 (Sec. 3.4: the method carries over to
 * non-linearities whose gradient depends on the sign of the activation only):
 * A3 = A2 where A2 > 0, slope * A2 elsewhere; Eq. 6 becomes dA2 = dA3 resp. slope * dA3, taken
 * from the sign of the dequantized copy (Eq. 10), and the weight gradient contracts the leaky
 * ReLU of that copy.  What is stored is unchanged (the K-bit codes of A2, Eq. 9), so packed,
 * stats and scratch have the sizes of abl_forward / abl_backward and all arguments the same
 * meaning, layout and aliasing rules.  slope in [0, 1] (0 = the ReLU; else ABL_ERR_ARG); the
 * backward must be given the slope of the forward.  These calls run the unfused stages.
 * flags: ABL_MATH_BF16; backward also ABL_ACCUM_DX. */
int abl_leaky_forward(void* stream, const abl_shape* shape, int K, uint32_t flags, float slope,
                      const float* x, const float* W, const float* gamma, const float* beta,
                      const float* skip, void* scratch, size_t scratch_bytes,
                      float* y, void* packed, void* stats);
int abl_leaky_backward(void* stream, const abl_shape* shape, int K, uint32_t flags, float slope,
                       const void* packed, const void* stats, const float* dy, const float* W,
                       void* scratch, size_t scratch_bytes,
                       float* dx, float* dW, float* dgamma, float* dbeta);

/* ---- stage-level entry points (the steps the two calls above are made of) ---- */

/* Eq. 1 statistics of x [M,C] and the per-channel constants of Eq. 9/10 -> stats.
 * scratch: abl_bn_scratch_bytes(M, C). */
size_t abl_bn_scratch_bytes(int64_t M, int32_t C);
int abl_bn_stats(void* stream, const float* x, int64_t M, int32_t C, const float* gamma,
                 const float* beta, int K, void* scratch, size_t scratch_bytes, void* stats);
/* Eq. 1-3 and Eq. 9 in one pass over x: writes A3 = max(0, A2) (fp32 [M,C]) and the
 * packed codes of A2. */
int abl_bn_relu_pack(void* stream, const float* x, int64_t M, int32_t C, int K,
                     const void* stats, float* a3, void* packed);
/* Eq. 9 alone: a2 fp32 [M,C] -> packed codes (gamma, beta, cq, fb from stats). */
int abl_pack(void* stream, const float* a2, int64_t M, int32_t C, int K, const void* stats,
             void* packed);
/* Eq. 10 alone: packed codes -> fp32 [M,C] reconstruction of A2. */
int abl_unpack(void* stream, const void* packed, int64_t M, int32_t C, int K,
               const void* stats, float* a2t);
/* Eq. 6-8 from the packed copy: da3 [M,C] -> dx [M,C] (+= with ABL_ACCUM_DX), dgamma, dbeta.
 * dx may alias da3.  scratch: abl_bn_scratch_bytes(M, C). */
int abl_bn_bwd(void* stream, const void* packed, const void* stats, const float* da3,
               int64_t M, int32_t C, int K, uint32_t flags, void* scratch, size_t scratch_bytes,
               float* dx, float* dgamma, float* dbeta);
/* Eq. 4: y = a3 (*) W (+ skip).  skip may be NULL or alias y.  flags: ABL_MATH_BF16. */
int abl_conv_fwd(void* stream, const abl_shape* shape, uint32_t flags, const float* a3, const float* W,
                 const float* skip, float* y);
/* Eq. 5, gradient to the conv input: da3 [N,H,W,Cin] from dy [N,Ho,Wo,Cout].  flags: ABL_MATH_BF16. */
int abl_conv_dgrad(void* stream, const abl_shape* shape, uint32_t flags, const float* dy, const float* W,
                   float* da3);
/* Eq. 5, gradient to the weights, with A3 rebuilt on the fly from the packed codes
 * (Eq. 10 then Eq. 3); no full-precision copy of the activation is written to memory.
 * scratch: abl_wgrad_scratch_bytes(shape).  flags: ABL_MATH_BF16. */
size_t abl_wgrad_scratch_bytes(const abl_shape* shape);
int abl_conv_wgrad_packed(void* stream, const abl_shape* shape, int K, uint32_t flags, const void* packed,
                          const void* stats, const float* dy, void* scratch,
                          size_t scratch_bytes, float* dW);

/* ---- the two fused kernels that abl_forward / abl_backward use where they can ----
 * Both exist for stride-1 convolutions with channel counts that are multiples of 16: filters
 * larger than 1x1 (abl_bn_conv_fwd also needs Ho == H, Wo == W), and 1x1 filters without padding
 * (abl_conv_dgrad_bn_reduce: Cout a multiple of 64 and at most 256).  Other shapes give
 * ABL_ERR_SHAPE and the layer calls fall back to the separate stages.
 *
 * abl_bn_conv_fwd: Eq. 1-3, Eq. 9 and Eq. 4 in one kernel - x is normalised, ReLU'd, quantized
 * and packed while the convolution stages its input patch; A3 is never written to memory.
 * stats must hold the statistics of x (abl_bn_stats).  y must not alias x; skip may alias y. */
int abl_bn_conv_fwd(void* stream, const abl_shape* shape, int K, uint32_t flags, const float* x,
                    const void* stats, const float* W, const float* skip, float* y, void* packed);
/* abl_conv_dgrad_bn_reduce: Eq. 5 (gradient to the conv input) with the sums of Eq. 7 taken in
 * the epilogue from the layer's packed codes (Eq. 10, Eq. 6): writes da3 and `*rows` partial rows
 * [rows][2][Cin] of doubles (sum dA2, sum A1~ dA2) at the start of scratch
 * (abl_bn_scratch_bytes(N*H*W, Cin)); `*rows` is a host value set by the call. */
int abl_conv_dgrad_bn_reduce(void* stream, const abl_shape* shape, int K, uint32_t flags,
                             const float* dy, const float* W, const void* packed, const void* stats,
                             void* scratch, size_t scratch_bytes, float* da3, int32_t* rows);

/* abl_conv_bwd_bn_reduce: both contractions of Eq. 5 and the sums of Eq. 7 in one pass over dy
 * and the packed codes, for 3x3 'same' stride-1 layers with 16 input and 16 output channels
 * (ABL_ERR_SHAPE otherwise): writes da3 (gradient to the conv input), dW (from the dequantized
 * activation, Eq. 10 and Eq. 3) and `*rows` partial rows [rows][2][16] of doubles (sum dA2,
 * sum A1~ dA2) at the start of scratch.  scratch: abl_bn_scratch_bytes(N*H*W, 16) rounded up to
 * 256 + abl_wgrad_scratch_bytes(shape) bytes; `*rows` is a host value set by the call.
 * dW may be NULL: the weight gradient is then left as `*rows` unsummed copies [rows][3][3][16][16]
 * behind the partial rows (at scratch + the rounded abl_bn_scratch_bytes) and the call is a
 * single kernel launch. */
int abl_conv_bwd_bn_reduce(void* stream, const abl_shape* shape, int K, uint32_t flags, const float* dy,
                           const float* W, const void* packed, const void* stats, void* scratch,
                           size_t scratch_bytes, float* da3, float* dW, int32_t* rows);

/* ---- the layer grouped as conv -> BN -> ReLU ----
 * The paper groups a convolution with the non-linearities that PRECEDE it (Sec. 3.1) and that
 * is what abl_forward / abl_backward implement.  These entry points run the same kernels with
 * the convolution first:  y = ReLU(gamma * BN(conv(x, W)) + beta).  The BN tensor is then the
 * conv OUTPUT: M' = N*Ho*Wo rows of Cout channels (gamma, beta, stats, packed are sized for it),
 * and what is packed is still the pre-ReLU BN output A2 (Sec. 3.2).  For plain chains without
 * shortcuts.
 *   forward : x [N,H,W,Cin], W, gamma/beta [Cout] -> y [N,Ho,Wo,Cout], packed, stats
 *   backward: dy [N,Ho,Wo,Cout] -> dx [N,H,W,Cin] (NULL: not wanted), dW, dgamma/dbeta [Cout].
 *             Eq. 5's weight gradient needs the conv input, which this layer does not store:
 *             ABL_XIN_F32    xin = the exact fp32 input (bottom of a network);
 *             ABL_XIN_PACKED xin, xin_stats = packed store and stats of the previous layer of
 *                            the chain (its channel count is Cin, its resolution H x W, same K);
 *                            the input ReLU(dequantized A2) is rebuilt on the fly (Eq. 10, Eq. 3).
 * flags: ABL_MATH_BF16, and for the backward exactly one of ABL_XIN_F32 / ABL_XIN_PACKED. */
size_t abl_postact_packed_bytes(const abl_shape* shape, int K);
size_t abl_postact_stats_bytes(const abl_shape* shape);
size_t abl_postact_scratch_bytes(const abl_shape* shape, int K);
int abl_postact_forward(void* stream, const abl_shape* shape, int K, uint32_t flags,
                        const float* x, const float* W, const float* gamma, const float* beta,
                        void* scratch, size_t scratch_bytes, float* y, void* packed, void* stats);
int abl_postact_backward(void* stream, const abl_shape* shape, int K, uint32_t flags,
                         const void* packed, const void* stats, const float* dy, const float* W,
                         const void* xin, const void* xin_stats, void* scratch, size_t scratch_bytes,
                         float* dx, float* dW, float* dgamma, float* dbeta);

/* ---- residual stack (Sec. 3.4; Fig. 2; Sec. 4 first paragraph) ----
 * A chain of layers with an identity shortcut around every group of `skip_every`
 * layers whose input and output shapes agree (0: plain chain).  Two caller-owned
 * fp32 buffers hold the residual stream and the straight path; they are reused for
 * the gradients in the backward pass.  Each must hold the largest layer input or
 * output of the stack.  Per layer the caller provides parameters, the packed store
 * and stats (written by the forward, read by the backward) and gradient outputs. */
typedef struct abl_layer {
  abl_shape shape;
  const float* W;
  const float* gamma;
  const float* beta;
  void* packed;   /* abl_packed_bytes(&shape, K) */
  void* stats;    /* abl_stats_bytes(&shape)     */
  float* dW;      /* backward outputs            */
  float* dgamma;
  float* dbeta;
} abl_layer;

/* Largest abl_scratch_bytes over the layers / largest activation in bytes. */
size_t abl_stack_scratch_bytes(const abl_layer* layers, int32_t L, int K);
size_t abl_stack_buffer_bytes(const abl_layer* layers, int32_t L);
/* Forward: the input batch must already be in buf_s.  On return the stack output is
 * in buf_s. */
int abl_stack_forward(void* stream, const abl_layer* layers, int32_t L, int K, uint32_t flags,
                      int32_t skip_every, float* buf_s, float* buf_t,
                      void* scratch, size_t scratch_bytes);
/* Backward: the gradient of the stack output must already be in buf_s.  On return
 * the gradient of the stack input is in buf_s and every layer's dW, dgamma, dbeta
 * are written. */
int abl_stack_backward(void* stream, const abl_layer* layers, int32_t L, int K, uint32_t flags,
                       int32_t skip_every, float* buf_s, float* buf_t,
                       void* scratch, size_t scratch_bytes);

/* The same two calls with an inspection hook, for parity tests that check every layer against a
 * reference on the layer's own inputs: before layer i runs, its input x_i [N,H,W,Cin] (forward)
 * resp. its incoming gradient dy_i [N,Ho,Wo,Cout] (backward) is copied to trace[i].  `trace` is a
 * host array of L device pointers (caller-owned, 16-byte aligned, each large enough for that
 * tensor); NULL entries, or trace == NULL, copy nothing.  Results are those of the plain calls bit
 * for bit (the copies only read).  With an identity shortcut around a group, the value added to
 * the group's output is the input of its first layer, and the gradient its first layer
 * accumulates into is the incoming gradient of its last layer. */
int abl_stack_forward_traced(void* stream, const abl_layer* layers, int32_t L, int K, uint32_t flags,
                             int32_t skip_every, float* buf_s, float* buf_t,
                             void* scratch, size_t scratch_bytes, float* const* trace);
int abl_stack_backward_traced(void* stream, const abl_layer* layers, int32_t L, int K, uint32_t flags,
                              int32_t skip_every, float* buf_s, float* buf_t,
                              void* scratch, size_t scratch_bytes, float* const* trace);

/* ---- parameter update -----------------------------------------------------------
 * SGD with momentum and weight decay, the update rule of the paper's experiments
 * (Sec. 4: momentum 0.9, weight decay 2e-4 on CIFAR and 1e-4 on ImageNet), applied to
 * one parameter tensor of n floats in place:
 *     v <- momentum * v + (grad + weight_decay * w);   w <- w - lr * v
 * every operation rounded to fp32 on its own, in this order.  w, grad, v: device
 * pointers, 16-byte aligned, caller-owned; grad is read only; n >= 0 (n = 0 is a
 * no-op that does not look at the pointers).  Errors: ABL_ERR_ARG (null / misaligned
 * pointer, n < 0), ABL_ERR_SHAPE (n >= 2^40), ABL_ERR_HIP. */
int abl_sgd_momentum(void* stream, int64_t n, float lr, float momentum, float weight_decay,
                     float* w, const float* grad, float* v);

/* ---- measurement aid ---------------------------------------------------------------
 * Not a step of the method: plain streaming kernels that show what this device's memory system
 * delivers, the ceiling that the HBM-bound passes (Eq. 1-3, Eq. 8-10) are reported against.
 *   mode 0: read `bytes` from src (dst: at least 16 writable bytes, normally left untouched)
 *   mode 1: write `bytes` to dst (src ignored)
 *   mode 2: copy `bytes` from src to dst (no overlap)
 * src, dst: device pointers, 16-byte aligned, caller-owned; bytes a positive multiple of 16.
 * Errors: ABL_ERR_ARG (mode, null / misaligned pointer), ABL_ERR_SHAPE (bytes), ABL_ERR_HIP. */
int abl_hbm_probe(void* stream, int mode, const void* src, void* dst, size_t bytes);
/* The matrix-core counterpart, the ceiling that the contractions (Eq. 4, Eq. 5) are reported
 * against: every wave of a fixed grid issues `iters` rounds of eight independent matrix
 * instructions on register operands - mode 0: fp32 16x16x4 (the instruction of the default
 * path), mode 1: bf16 16x16x32 with fp32 accumulation (ABL_MATH_BF16).  abl_mfma_probe_flops
 * returns the floating-point operations one such launch performs (0 on invalid arguments);
 * `out` receives abl_mfma_probe_out_bytes() bytes of sums that only keep the work alive.
 * Errors: ABL_ERR_ARG (mode, iters outside [1, 2^24], null / misaligned out), ABL_ERR_SCRATCH
 * (out_bytes too small), ABL_ERR_HIP. */
size_t abl_mfma_probe_out_bytes(void);
double abl_mfma_probe_flops(int mode, int iters);
int abl_mfma_probe(void* stream, int mode, int iters, void* out, size_t out_bytes);

#ifdef __cplusplus
}
#endif
#endif /* ABL_H_ */
