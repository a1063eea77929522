"""Oracle for approximate-activation backprop (arXiv 1901.07988) - TEST INFRASTRUCTURE ONLY.

Thin numpy front end over ``abl_oracle.cpp`` (plain CPU loops, compiled with
``g++ -O2 -ffp-contract=off``) plus the composition of those steps into a layer
forward (Sec. 3.1 Eq. 1-4, Sec. 3.2 Eq. 9), a layer backward (Eq. 10, Eq. 5-8) and
a residual stack (Sec. 3.4; Fig. 2).  Nothing here is shared with, or imported
by, the GPU library; only tests, the smoke check and the benchmark's CPU-baseline
leg may import this module.

Layouts: activations NHWC, weights [R][S][Cin][Cout].  ``dtype`` is the storage /
elementwise type (float32 = what the GPU path decides codes in; float64 = for
finite-difference checks); sums are always accumulated in double.

Parity status of each function is listed in the design notes; every function
here is pinned by the CPU tests except the *size* of the training-accuracy
effect of the approximation (needs the paper's datasets): parity unpinned.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "abl_oracle.cpp")
_LIB = os.path.join(_HERE, "liboracle.so")

EPS = 1e-5  # batch-norm epsilon; the paper leaves it symbolic (Eq. 1)


def build(force: bool = False) -> str:
    """Compile the C++ oracle (host only)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["g++", "-O2", "-fopenmp", "-ffp-contract=off", "-fno-fast-math", "-std=c++17",
               "-shared", "-fPIC", "-o", _LIB, _SRC]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def _L():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
    return _lib


def _suf(dtype):
    dtype = np.dtype(dtype)
    if dtype == np.float32:
        return "f32", ctypes.c_float
    if dtype == np.float64:
        return "f64", ctypes.c_double
    raise TypeError(dtype)


def _p(a):
    return a.ctypes.data_as(ctypes.c_void_p)


def _c(a, dtype):
    return np.ascontiguousarray(a, dtype=dtype)


@dataclass
class Shape:
    """One layer: input [N,H,W,Cin] -> output [N,Ho,Wo,Cout], filter R x S."""
    N: int
    H: int
    W: int
    Cin: int
    Cout: int
    R: int = 3
    S: int = 3
    stride: int = 1
    pad: int = 1

    @property
    def Ho(self):
        return (self.H + 2 * self.pad - self.R) // self.stride + 1

    @property
    def Wo(self):
        return (self.W + 2 * self.pad - self.S) // self.stride + 1

    @property
    def M(self):
        return self.N * self.H * self.W

    @property
    def E(self):
        return self.M * self.Cin


# --------------------------------------------------------------------------- steps
def bn_stats(x, dtype=np.float32):
    """Eq. 1: per-channel mean and biased variance over all but the last dim."""
    suf, _ = _suf(dtype)
    x = _c(x, dtype)
    C = x.shape[-1]
    M = x.size // C
    mean = np.empty(C, dtype)
    var = np.empty(C, dtype)
    getattr(_L(), f"orc_bn_stats_{suf}")(_p(x), ctypes.c_int64(M), C, _p(mean), _p(var))
    return mean, var


def bn_rstd(var, eps=EPS, dtype=np.float32):
    """Eq. 1: (sigma^2 + eps)^(-1/2)."""
    suf, ct = _suf(dtype)
    var = _c(var, dtype)
    rstd = np.empty_like(var)
    getattr(_L(), f"orc_bn_rstd_{suf}")(_p(var), var.size, ct(np.dtype(dtype).type(eps)), _p(rstd))
    return rstd


def bn_relu(x, mean, rstd, gamma, beta, dtype=np.float32, slope=0.0):
    """Eq. 1-3: returns (A2, A3).  ``slope`` > 0: leaky ReLU (Sec. 3.4), A3 = slope * A2 where A2 <= 0."""
    suf, ct = _suf(dtype)
    x = _c(x, dtype)
    C = x.shape[-1]
    M = x.size // C
    a2 = np.empty_like(x)
    a3 = np.empty_like(x)
    getattr(_L(), f"orc_bn_relu_{suf}")(_p(x), ctypes.c_int64(M), C, _p(_c(mean, dtype)),
                                        _p(_c(rstd, dtype)), _p(_c(gamma, dtype)),
                                        _p(_c(beta, dtype)), ct(np.dtype(dtype).type(slope)), _p(a2), _p(a3))
    return a2, a3


def quant_consts(gamma, beta, K, dtype=np.float32):
    """Per-channel constants of Eq. 9/10: (2^K/(6 gamma), 6 gamma/2^K, floor(beta 2^K/(6 gamma)))."""
    suf, _ = _suf(dtype)
    gamma = _c(gamma, dtype)
    beta = _c(beta, dtype)
    C = gamma.size
    cq = np.empty(C, dtype)
    step = np.empty(C, dtype)
    fb = np.empty(C, np.int32)
    getattr(_L(), f"orc_quant_consts_{suf}")(_p(gamma), _p(beta), C, int(K), _p(cq), _p(step), _p(fb))
    return cq, step, fb


def quantize(a2, gamma, beta, K, dtype=np.float32):
    """Eq. 9: int32 codes in [0, 2^K-1], same shape as a2."""
    suf, _ = _suf(dtype)
    a2 = _c(a2, dtype)
    C = a2.shape[-1]
    M = a2.size // C
    cq, _, fb = quant_consts(gamma, beta, K, dtype)
    q = np.empty(a2.shape, np.int32)
    getattr(_L(), f"orc_quantize_{suf}")(_p(a2), ctypes.c_int64(M), C, _p(cq), _p(fb), int(K), _p(q))
    return q


def dequantize(q, gamma, beta, K, dtype=np.float32):
    """Eq. 10: bin-midpoint reconstruction of A2 from the codes."""
    suf, _ = _suf(dtype)
    q = _c(q, np.int32)
    C = q.shape[-1]
    M = q.size // C
    _, step, fb = quant_consts(gamma, beta, K, dtype)
    out = np.empty(q.shape, dtype)
    getattr(_L(), f"orc_dequantize_{suf}")(_p(q), ctypes.c_int64(M), C, _p(step), _p(fb), int(K), _p(out))
    return out


def packed_bytes(E, K):
    """Size of the stored K-bit tensor: ceil(E*K/8) rounded up to 128-byte rows (Sec. 3.4: alpha = K/32)."""
    if K == 32:
        return 4 * E
    return (-(-E * K // 8) + 127) // 128 * 128


def pack_codes(q, K):
    """Codes -> bytes, flat element order, LSB first, zero padded to 128-byte rows."""
    q = _c(q, np.int32).ravel()
    nb = packed_bytes(q.size, K)
    out = np.empty(nb, np.uint8)
    _L().orc_pack_codes(_p(q), ctypes.c_int64(q.size), int(K), _p(out), ctypes.c_int64(nb))
    return out


def unpack_codes(buf, shape, K):
    buf = _c(buf, np.uint8)
    E = int(np.prod(shape))
    q = np.empty(E, np.int32)
    _L().orc_unpack_codes(_p(buf), ctypes.c_int64(E), int(K), _p(q))
    return q.reshape(shape)


def _conv_args(s: Shape):
    return (s.N, s.H, s.W, s.Cin, s.Cout, s.R, s.S, s.stride, s.pad)


def conv_fwd(a3, w, s: Shape, dtype=np.float32):
    """Eq. 4 as a zero-padded cross-correlation."""
    suf, _ = _suf(dtype)
    a3 = _c(a3, dtype)
    w = _c(w, dtype)
    assert a3.shape == (s.N, s.H, s.W, s.Cin) and w.shape == (s.R, s.S, s.Cin, s.Cout)
    y = np.empty((s.N, s.Ho, s.Wo, s.Cout), dtype)
    getattr(_L(), f"orc_conv_fwd_{suf}")(_p(a3), _p(w), *_conv_args(s), _p(y))
    return y


def conv_dgrad(dy, w, s: Shape, dtype=np.float32):
    """Eq. 5 (second half): gradient to the conv input."""
    suf, _ = _suf(dtype)
    dy = _c(dy, dtype)
    w = _c(w, dtype)
    assert dy.shape == (s.N, s.Ho, s.Wo, s.Cout)
    da3 = np.empty((s.N, s.H, s.W, s.Cin), dtype)
    getattr(_L(), f"orc_conv_dgrad_{suf}")(_p(dy), _p(w), *_conv_args(s), _p(da3))
    return da3


def conv_wgrad(a3, dy, s: Shape, dtype=np.float32):
    """Eq. 5 (first half): gradient to the weights."""
    suf, _ = _suf(dtype)
    a3 = _c(a3, dtype)
    dy = _c(dy, dtype)
    dw = np.empty((s.R, s.S, s.Cin, s.Cout), dtype)
    getattr(_L(), f"orc_conv_wgrad_{suf}")(_p(a3), _p(dy), *_conv_args(s), _p(dw))
    return dw


def bn_relu_bwd(a2t, da3, rstd, gamma, beta, dtype=np.float32, slope=0.0):
    """Eq. 6-8 from a (possibly approximate) copy of A2: returns (dx, dgamma, dbeta).
    ``slope`` > 0: leaky ReLU, dA2 = slope * dA3 where the copy of A2 is <= 0."""
    suf, ct = _suf(dtype)
    a2t = _c(a2t, dtype)
    da3 = _c(da3, dtype)
    C = a2t.shape[-1]
    M = a2t.size // C
    dx = np.empty_like(a2t)
    dg = np.empty(C, dtype)
    db = np.empty(C, dtype)
    getattr(_L(), f"orc_bn_relu_bwd_{suf}")(_p(a2t), _p(da3), ctypes.c_int64(M), C,
                                            _p(_c(rstd, dtype)), _p(_c(gamma, dtype)),
                                            _p(_c(beta, dtype)), ct(np.dtype(dtype).type(slope)),
                                            _p(dx), _p(dg), _p(db))
    return dx, dg, db


# --------------------------------------------------------------------------- one layer
@dataclass
class Saved:
    """What a layer keeps for its backward pass (Sec. 3.2): the K-bit copy of A2 and the
    per-channel vectors.  With K == 32 ``store`` is A2 itself (exact storage, Sec. 3.2 first
    paragraph / the "exact" baseline of Sec. 4)."""
    K: int
    shape: Shape
    store: np.ndarray  # uint8 packed codes, or A2 when K == 32
    mean: np.ndarray
    var: np.ndarray
    rstd: np.ndarray
    gamma: np.ndarray
    beta: np.ndarray
    slope: float = 0.0  # 0: ReLU; > 0: leaky ReLU (Sec. 3.4)

    @property
    def nbytes(self):
        return self.store.nbytes


def layer_forward(x, w, gamma, beta, K, s: Shape, skip=None, dtype=np.float32, eps=EPS,
                  stats=None, keep=False, naive=False, slope=0.0):
    """Forward of one pre-activation layer.  The output never sees the codes: it is computed
    from the full-precision A3 (Sec. 3.2), so it is the same for every K.

    ``stats`` = (mean, var) overrides the batch statistics (used to feed the GPU's own
    statistics to the quantizer in the two-tier code-parity test).
    Returns (y, Saved) and, with ``keep``, also a dict of the intermediates.

    ``naive``: the comparison baseline of Sec. 4 - the convolution consumes the ReLU of the
    dequantized copy instead of the exact A3, so the approximation also enters the forward pass.

    ``slope`` > 0: the non-linearity is a leaky ReLU (Sec. 3.4 admits any whose gradient depends
    on the sign of the activation only); what is stored is unchanged - the K-bit copy of A2.
    """
    x = _c(x, dtype)
    mean, var = bn_stats(x, dtype) if stats is None else (_c(stats[0], dtype), _c(stats[1], dtype))
    rstd = bn_rstd(var, eps, dtype)
    if naive and slope != 0.0:
        raise ValueError("the naive baseline is defined for the plain ReLU only")
    a2, a3 = bn_relu(x, mean, rstd, gamma, beta, dtype, slope)
    if K == 32:
        store, q = a2.copy(), None
    else:
        q = quantize(a2, gamma, beta, K, dtype)
        store = pack_codes(q, K)
        if naive:
            a3 = np.maximum(dequantize(q, gamma, beta, K, dtype), np.dtype(dtype).type(0))
    y = conv_fwd(a3, w, s, dtype)
    if skip is not None:
        y = y + _c(skip, dtype)
    saved = Saved(K, s, store, mean, var, rstd, _c(gamma, dtype).copy(), _c(beta, dtype).copy(), float(slope))
    if keep:
        return y, saved, dict(a2=a2, a3=a3, q=q)
    return y, saved


def recover_a2(saved: Saved, dtype=np.float32):
    """Eq. 10 applied to the stored copy (identity for exact storage)."""
    s = saved.shape
    if saved.K == 32:
        return saved.store
    q = unpack_codes(saved.store, (s.N, s.H, s.W, s.Cin), saved.K)
    return dequantize(q, saved.gamma, saved.beta, saved.K, dtype)


def layer_backward(saved: Saved, dy, w, dtype=np.float32, keep=False):
    """Backward of one layer from the stored copy only (Sec. 3.2; Eq. 5-8).
    Returns (dx, dW, dgamma, dbeta)."""
    s = saved.shape
    a2t = recover_a2(saved, dtype)
    if saved.slope == 0.0:
        a3t = np.maximum(a2t, np.dtype(dtype).type(0))  # Eq. 3 on the approximate copy
    else:                                               # ... or its leaky version (Sec. 3.4)
        a3t = np.where(a2t > 0, a2t, np.dtype(dtype).type(saved.slope) * a2t).astype(dtype)
    dw = conv_wgrad(a3t, dy, s, dtype)                  # Eq. 5, approximate
    da3 = conv_dgrad(dy, w, s, dtype)                   # Eq. 5, exact
    dx, dg, db = bn_relu_bwd(a2t, da3, saved.rstd, saved.gamma, saved.beta, dtype, saved.slope)
    if keep:
        return dx, dw, dg, db, dict(a2t=a2t, a3t=a3t, da3=da3)
    return dx, dw, dg, db


# --------------------------------------------------------------------------- residual stack
def stack_forward(x, layers, K, dtype=np.float32, skip_every=2, naive=False):
    """Chain of pre-activation layers with identity skips (Sec. 3.4, Fig. 2).

    ``layers`` is a list of (Shape, W, gamma, beta).  The residual stream enters a group of
    ``skip_every`` layers and is added to that group's output when the shapes agree
    (skip_every == 0: plain feed-forward chain).  Returns (output, [Saved per layer])."""
    s_stream = _c(x, dtype)
    t = s_stream
    saved = []
    for i, (sh, w, g, b) in enumerate(layers):
        last_of_group = skip_every > 0 and (i + 1) % skip_every == 0
        y, sv = layer_forward(t, w, g, b, K, sh, dtype=dtype, naive=naive)
        if last_of_group and y.shape == s_stream.shape:
            y = y + s_stream
        saved.append(sv)
        t = y
        if skip_every == 0 or last_of_group:
            s_stream = y
    return t, saved


def stack_backward(saved, layers, dy, dtype=np.float32, skip_every=2):
    """Backward through ``stack_forward``: gradients through a skip are copied and added
    (Sec. 3.4).  Returns (dx, [(dW, dgamma, dbeta) per layer])."""
    L = len(layers)
    grads = [None] * L
    g = _c(dy, dtype)
    g_stream = None  # gradient w.r.t. the residual stream leaving the current group
    for i in range(L - 1, -1, -1):
        sh, w, _, _ = layers[i]
        last_of_group = skip_every > 0 and (i + 1) % skip_every == 0
        first_of_group = skip_every > 0 and i % skip_every == 0
        if last_of_group:
            in_shape = (layers[i - skip_every + 1][0].N, layers[i - skip_every + 1][0].H,
                        layers[i - skip_every + 1][0].W, layers[i - skip_every + 1][0].Cin)
            g_stream = g if g.shape == in_shape else None
        dx, dw, dg, db = layer_backward(saved[i], g, w, dtype)
        grads[i] = (dw, dg, db)
        if first_of_group and g_stream is not None:
            dx = dx + g_stream
            g_stream = None
        g = dx
    return g, grads


# --------------------------------------------------------------------------- sampled outputs
# Eq. 4 / Eq. 5 evaluated output by output in double, for tensors too large to run the full
# loops on in a test.  Same definitions as conv_fwd / conv_dgrad / conv_wgrad above.
def conv_fwd_at(a3, w, s: Shape, pts):
    """y[n, ho, wo, :] for each (n, ho, wo) in pts."""
    out = np.zeros((len(pts), s.Cout), np.float64)
    w64 = np.asarray(w, np.float64)
    for i, (n, ho, wo) in enumerate(pts):
        for r in range(s.R):
            h = ho * s.stride + r - s.pad
            if h < 0 or h >= s.H:
                continue
            for q in range(s.S):
                x = wo * s.stride + q - s.pad
                if x < 0 or x >= s.W:
                    continue
                out[i] += np.asarray(a3[n, h, x], np.float64) @ w64[r, q]
    return out


def conv_dgrad_at(dy, w, s: Shape, pts):
    """da3[n, h, x, :] for each (n, h, x) in pts."""
    out = np.zeros((len(pts), s.Cin), np.float64)
    w64 = np.asarray(w, np.float64)
    for i, (n, h, x) in enumerate(pts):
        for r in range(s.R):
            hh = h + s.pad - r
            if hh < 0 or hh % s.stride or hh // s.stride >= s.Ho:
                continue
            for q in range(s.S):
                ww = x + s.pad - q
                if ww < 0 or ww % s.stride or ww // s.stride >= s.Wo:
                    continue
                out[i] += w64[r, q] @ np.asarray(dy[n, hh // s.stride, ww // s.stride], np.float64)
    return out


def conv_wgrad_at(a3, dy, s: Shape, entries):
    """dW[r, q, ci, :] for each (r, q, ci) in entries."""
    out = np.zeros((len(entries), s.Cout), np.float64)
    for i, (r, q, ci) in enumerate(entries):
        ho = np.arange(s.Ho)
        wo = np.arange(s.Wo)
        h = ho * s.stride + r - s.pad
        x = wo * s.stride + q - s.pad
        hv = (h >= 0) & (h < s.H)
        xv = (x >= 0) & (x < s.W)
        a = np.asarray(a3[:, h[hv]][:, :, x[xv], ci], np.float64)          # [N, ho', wo']
        g = np.asarray(dy[:, ho[hv]][:, :, wo[xv], :], np.float64)         # [N, ho', wo', Cout]
        out[i] = np.einsum("nhw,nhwc->c", a, g)
    return out


# --------------------------------------------------------------------------- conv -> BN -> ReLU grouping
# The paper groups a convolution with the non-linearities that precede it (Sec. 3.1).  The same
# three operations grouped with the convolution FIRST give y = ReLU(gamma * BN(conv(x)) + beta);
# what is stored is still the K-bit copy of the pre-ReLU BN output A2 (Sec. 3.2), which now has
# the conv output's shape.  A chain of such layers is conv_0, then pre-activation layers, then a
# trailing BN-ReLU - the CPU tests assert that identity bit for bit.
def postact_forward(x, w, gamma, beta, K, s: Shape, dtype=np.float32, eps=EPS, keep=False):
    """Returns (y, Saved); Saved.shape describes the BN tensor [N,Ho,Wo,Cout]."""
    t = conv_fwd(x, w, s, dtype)                                 # Eq. 4
    mean, var = bn_stats(t, dtype)
    rstd = bn_rstd(var, eps, dtype)
    a2, a3 = bn_relu(t, mean, rstd, gamma, beta, dtype)          # Eq. 1-3
    bn_shape = Shape(s.N, s.Ho, s.Wo, s.Cout, s.Cout, 1, 1, 1, 0)
    store = a2.copy() if K == 32 else pack_codes(quantize(a2, gamma, beta, K, dtype), K)   # Eq. 9
    saved = Saved(K, bn_shape, store, mean, var, rstd, _c(gamma, dtype).copy(), _c(beta, dtype).copy())
    if keep:
        return a3, saved, dict(t=t, a2=a2)
    return a3, saved


def postact_backward(saved: Saved, dy, w, s: Shape, xin, dtype=np.float32):
    """dy is the gradient of y = A3.  ``xin`` is the conv input: an fp32 array, or the Saved of the
    previous layer of the chain, whose ReLU(dequantized A2) (Eq. 10, Eq. 3) was this layer's input.
    Returns (dx, dW, dgamma, dbeta)."""
    a2t = recover_a2(saved, dtype)
    dt, dg, db = bn_relu_bwd(a2t, dy, saved.rstd, saved.gamma, saved.beta, dtype)   # Eq. 6-8
    if isinstance(xin, Saved):
        xa = np.maximum(recover_a2(xin, dtype), np.dtype(dtype).type(0))
    else:
        xa = _c(xin, dtype)
    dw = conv_wgrad(xa, dt, s, dtype)      # Eq. 5
    dx = conv_dgrad(dt, w, s, dtype)       # Eq. 5
    return dx, dw, dg, db


def sgd_momentum(w, grad, v, lr, momentum, weight_decay, dtype=np.float32):
    """SGD with momentum and weight decay, the update rule of the paper's experiments (Sec. 4):
    v <- momentum * v + (grad + weight_decay * w);  w <- w - lr * v, each operation rounded to
    ``dtype``.  Returns (w_new, v_new)."""
    t = np.dtype(dtype).type
    w, grad, v = _c(w, dtype), _c(grad, dtype), _c(v, dtype)
    d = grad + t(weight_decay) * w
    v_new = t(momentum) * v + d
    return w - t(lr) * v_new, v_new
