"""Helpers for the GPU parity tests: run the C-ABI entry points on numpy inputs and bring the
results back as numpy arrays.  Allocation and copies only - no arithmetic of the method."""
import numpy as np
import torch

from paper_1901_07988_amd import binding as B

PLANES = ("mean", "var", "rstd", "gamma", "beta", "cq", "step", "fb")


def dev(a, dtype=None):
    t = torch.from_numpy(np.ascontiguousarray(a))
    if dtype is not None:
        t = t.to(dtype)
    return t.cuda()


def zeros_bytes(n):
    return torch.zeros(max(int(n), 16), dtype=torch.uint8, device="cuda")


def stats_to_dict(stats_t, C):
    raw = stats_t.cpu().numpy().view(np.float32).reshape(B.STATS_PLANES, C)
    d = {k: raw[i].copy() for i, k in enumerate(PLANES)}
    d["fb"] = raw[7].view(np.int32).copy()
    return d


def stats_from_arrays(mean, var, rstd, gamma, beta, cq, step, fb):
    """Build a device stats block from numpy vectors (used to inject reference statistics)."""
    C = len(mean)
    raw = np.empty((B.STATS_PLANES, C), np.float32)
    for i, v in enumerate((mean, var, rstd, gamma, beta, cq, step)):
        raw[i] = np.asarray(v, np.float32)
    raw[7] = np.asarray(fb, np.int32).view(np.float32)
    return dev(raw.view(np.uint8).reshape(-1))


def run_bn_stats(x, gamma, beta, K):
    C = x.shape[-1]
    M = x.size // C
    scratch = zeros_bytes(B.abl_bn_scratch_bytes(M, C))
    stats = zeros_bytes(B.STATS_PLANES * 4 * C)
    B.abl_bn_stats(dev(x), M, C, dev(gamma), dev(beta), K, scratch, stats)
    torch.cuda.synchronize()
    return stats


def run_bn_relu_pack(x, stats_t, K):
    C = x.shape[-1]
    M = x.size // C
    nb = (-(-M * C * K // 8) + 127) // 128 * 128
    packed = torch.full((nb,), 0xAB, dtype=torch.uint8, device="cuda")
    a3 = torch.empty(x.shape, dtype=torch.float32, device="cuda")
    B.abl_bn_relu_pack(dev(x), M, C, K, stats_t, a3, packed)
    torch.cuda.synchronize()
    return a3.cpu().numpy(), packed.cpu().numpy()


def run_pack(a2, stats_t, K):
    C = a2.shape[-1]
    M = a2.size // C
    nb = (-(-M * C * K // 8) + 127) // 128 * 128
    packed = torch.full((nb,), 0xCD, dtype=torch.uint8, device="cuda")
    B.abl_pack(dev(a2), M, C, K, stats_t, packed)
    torch.cuda.synchronize()
    return packed.cpu().numpy()


def run_unpack(packed, shape, stats_t, K):
    C = shape[-1]
    M = int(np.prod(shape)) // C
    out = torch.empty(tuple(shape), dtype=torch.float32, device="cuda")
    B.abl_unpack(dev(packed), M, C, K, stats_t, out)
    torch.cuda.synchronize()
    return out.cpu().numpy()


def run_bn_bwd(packed, stats_t, da3, K, accum_into=None, alias=False):
    C = da3.shape[-1]
    M = da3.size // C
    scratch = zeros_bytes(B.abl_bn_scratch_bytes(M, C))
    g = dev(da3)
    if alias:
        dx = g
    elif accum_into is not None:
        dx = dev(accum_into)
    else:
        dx = torch.empty(da3.shape, dtype=torch.float32, device="cuda")
    dg = torch.empty(C, dtype=torch.float32, device="cuda")
    db = torch.empty(C, dtype=torch.float32, device="cuda")
    B.abl_bn_bwd(dev(packed), stats_t, g, M, C, K, scratch, dx, dg, db,
                 flags=B.ABL_ACCUM_DX if accum_into is not None else 0)
    torch.cuda.synchronize()
    return dx.cpu().numpy(), dg.cpu().numpy(), db.cpu().numpy()


def out_shape(s):
    return (s.N, s.Ho, s.Wo, s.Cout)


def run_conv_fwd(s, a3, w, skip=None, alias_skip=False, flags=0):
    y = torch.empty(out_shape(s), dtype=torch.float32, device="cuda")
    sk = None
    if skip is not None:
        sk = dev(skip)
        if alias_skip:
            y = sk
    B.abl_conv_fwd(s.as_tuple(), dev(a3), dev(w), sk, y, flags=flags)
    torch.cuda.synchronize()
    return y.cpu().numpy()


def run_conv_dgrad(s, dy, w, flags=0):
    da3 = torch.empty((s.N, s.H, s.W, s.Cin), dtype=torch.float32, device="cuda")
    B.abl_conv_dgrad(s.as_tuple(), dev(dy), dev(w), da3, flags=flags)
    torch.cuda.synchronize()
    return da3.cpu().numpy()


def run_conv_wgrad(s, K, packed, stats_t, dy, flags=0):
    scratch = zeros_bytes(B.abl_wgrad_scratch_bytes(s.as_tuple()))
    dw = torch.empty((s.R, s.S, s.Cin, s.Cout), dtype=torch.float32, device="cuda")
    B.abl_conv_wgrad_packed(s.as_tuple(), K, dev(packed), stats_t, dev(dy), scratch, dw, flags=flags)
    torch.cuda.synchronize()
    return dw.cpu().numpy()


class LayerRun:
    """One abl_forward (+ abl_backward) on the device; with `slope` the leaky-ReLU calls."""

    def __init__(self, s, K, flags=0, slope=None):
        self.s, self.K, self.flags, self.slope = s, K, flags, slope
        t = s.as_tuple()
        self.scratch = zeros_bytes(B.abl_scratch_bytes(t, K))
        self.packed = torch.full((B.abl_packed_bytes(t, K),), 0xEE, dtype=torch.uint8, device="cuda")
        self.stats = zeros_bytes(B.abl_stats_bytes(t))

    def forward(self, x, w, gamma, beta, skip=None, in_place=False):
        s = self.s
        xd = dev(x)
        if in_place:
            assert x.size >= int(np.prod(out_shape(s)))
            y = xd.view(-1)[: int(np.prod(out_shape(s)))].view(out_shape(s))
        else:
            y = torch.empty(out_shape(s), dtype=torch.float32, device="cuda")
        args = (xd, dev(w), dev(gamma), dev(beta), None if skip is None else dev(skip), self.scratch, y,
                self.packed, self.stats)
        if self.slope is None:
            B.abl_forward(s.as_tuple(), self.K, *args, flags=self.flags)
        else:
            B.abl_leaky_forward(s.as_tuple(), self.K, self.slope, *args, flags=self.flags)
        torch.cuda.synchronize()
        return y.cpu().numpy()

    def backward(self, dy, w, accum_into=None):
        s = self.s
        dx = dev(accum_into) if accum_into is not None else torch.empty((s.N, s.H, s.W, s.Cin), dtype=torch.float32, device="cuda")
        dw = torch.empty((s.R, s.S, s.Cin, s.Cout), dtype=torch.float32, device="cuda")
        dg = torch.empty(s.Cin, dtype=torch.float32, device="cuda")
        db = torch.empty(s.Cin, dtype=torch.float32, device="cuda")
        flags = (self.flags & ~B.ABL_NAIVE_FWD) | (B.ABL_ACCUM_DX if accum_into is not None else 0)
        args = (self.packed, self.stats, dev(dy), dev(w), self.scratch, dx, dw, dg, db)
        if self.slope is None:
            B.abl_backward(s.as_tuple(), self.K, *args, flags=flags)
        else:
            B.abl_leaky_backward(s.as_tuple(), self.K, self.slope, *args, flags=flags)
        torch.cuda.synchronize()
        return dx.cpu().numpy(), dw.cpu().numpy(), dg.cpu().numpy(), db.cpu().numpy()


class StackRun:
    """A residual stack on the device: owns the two activation buffers, the workspace and the
    per-layer stores."""

    def __init__(self, layers, K, skip_every, flags=0):
        self.K, self.skip_every, self.flags = K, skip_every, flags
        self.descs = []
        for s, w, g, b in layers:
            t = s.as_tuple()
            self.descs.append(dict(
                shape=t, W=dev(w), gamma=dev(g), beta=dev(b),
                packed=zeros_bytes(B.abl_packed_bytes(t, K)), stats=zeros_bytes(B.abl_stats_bytes(t)),
                dW=torch.empty(w.shape, dtype=torch.float32, device="cuda"),
                dgamma=torch.empty(s.Cin, dtype=torch.float32, device="cuda"),
                dbeta=torch.empty(s.Cin, dtype=torch.float32, device="cuda")))
        self.layers = B.make_layers(self.descs)
        self.scratch = zeros_bytes(B.abl_stack_scratch_bytes(self.layers, K))
        nb = B.abl_stack_buffer_bytes(self.layers)
        self.buf_s = torch.zeros(nb // 4, dtype=torch.float32, device="cuda")
        self.buf_t = torch.zeros(nb // 4, dtype=torch.float32, device="cuda")
        self.first, self.last = layers[0][0], layers[-1][0]

    def load(self, a):
        self.buf_s[: a.size].copy_(torch.from_numpy(np.ascontiguousarray(a)).view(-1))

    def forward(self):
        B.abl_stack_forward(self.layers, self.K, self.skip_every, self.buf_s, self.buf_t, self.scratch,
                            flags=self.flags)

    def backward(self):
        B.abl_stack_backward(self.layers, self.K, self.skip_every, self.buf_s, self.buf_t, self.scratch,
                             flags=self.flags & ~B.ABL_NAIVE_FWD)

    def output(self):
        n = int(np.prod(out_shape(self.last)))
        return self.buf_s[:n].cpu().numpy().reshape(out_shape(self.last))

    def input_grad(self):
        f = self.first
        n = f.N * f.H * f.W * f.Cin
        return self.buf_s[:n].cpu().numpy().reshape(f.N, f.H, f.W, f.Cin)

    def stored_bytes(self):
        return sum(d["packed"].numel() + d["stats"].numel() for d in self.descs)


class PostactRun:
    """One conv -> BN -> ReLU layer on the device (abl_postact_forward / abl_postact_backward)."""

    def __init__(self, s, K, flags=0):
        self.s, self.K, self.flags = s, K, flags
        t = s.as_tuple()
        self.scratch = zeros_bytes(B.abl_postact_scratch_bytes(t, K))
        self.packed = torch.full((B.abl_postact_packed_bytes(t, K),), 0xEE, dtype=torch.uint8, device="cuda")
        self.stats = zeros_bytes(B.abl_postact_stats_bytes(t))

    def forward(self, x, w, gamma, beta):
        s = self.s
        self.y = torch.empty(out_shape(s), dtype=torch.float32, device="cuda")
        B.abl_postact_forward(s.as_tuple(), self.K, dev(x), dev(w), dev(gamma), dev(beta), self.scratch, self.y,
                              self.packed, self.stats, flags=self.flags)
        torch.cuda.synchronize()
        return self.y.cpu().numpy()

    def backward(self, dy, w, xin=None, prev=None, want_dx=True):
        """xin: fp32 conv input (numpy) or prev: the PostactRun of the previous layer."""
        s = self.s
        dx = torch.empty((s.N, s.H, s.W, s.Cin), dtype=torch.float32, device="cuda") if want_dx else None
        dw = torch.empty((s.R, s.S, s.Cin, s.Cout), dtype=torch.float32, device="cuda")
        dg = torch.empty(s.Cout, dtype=torch.float32, device="cuda")
        db = torch.empty(s.Cout, dtype=torch.float32, device="cuda")
        if prev is not None:
            B.abl_postact_backward(s.as_tuple(), self.K, self.packed, self.stats, dev(dy), dev(w), prev.packed,
                                   prev.stats, self.scratch, dx, dw, dg, db, self.flags | B.ABL_XIN_PACKED)
        else:
            B.abl_postact_backward(s.as_tuple(), self.K, self.packed, self.stats, dev(dy), dev(w), dev(xin), None,
                                   self.scratch, dx, dw, dg, db, self.flags | B.ABL_XIN_F32)
        torch.cuda.synchronize()
        return (None if dx is None else dx.cpu().numpy()), dw.cpu().numpy(), dg.cpu().numpy(), db.cpu().numpy()
