"""Device-side holders for the layer and stack calls: they own the device buffers a call needs
(workspace, packed store, statistics, the two shared activation buffers of a stack) and pass them to
the C-ABI entry points.  Allocation and copies only - every step of the method runs in libabl."""
import numpy as np
import torch

from . import binding as B


def dev(a, dtype=None):
    """numpy array -> contiguous device tensor."""
    t = torch.from_numpy(np.ascontiguousarray(a))
    if dtype is not None:
        t = t.to(dtype)
    return t.cuda()


def zeros_bytes(n):
    """n zero bytes on the device (at least 16, so that the pointer is never null)."""
    return torch.zeros(max(int(n), 16), dtype=torch.uint8, device="cuda")


def out_shape(s):
    return (s.N, s.Ho, s.Wo, s.Cout)


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
        self.shapes = [l[0] for l in layers]

    def load(self, a):
        self.buf_s[: a.size].copy_(torch.from_numpy(np.ascontiguousarray(a)).view(-1))

    def forward(self, trace=False):
        """trace=True: returns one device tensor per layer holding that layer's input (inspection
        hook of the library; results are unchanged)."""
        if not trace:
            B.abl_stack_forward(self.layers, self.K, self.skip_every, self.buf_s, self.buf_t, self.scratch,
                                flags=self.flags)
            return None
        tr = [torch.empty(d["shape"][0] * d["shape"][1] * d["shape"][2] * d["shape"][3], dtype=torch.float32,
                          device="cuda") for d in self.descs]
        B.abl_stack_forward_traced(self.layers, self.K, self.skip_every, self.buf_s, self.buf_t, self.scratch, tr,
                                   flags=self.flags)
        return tr

    def backward(self, trace=False):
        """trace=True: returns one device tensor per layer holding that layer's incoming gradient."""
        flags = self.flags & ~B.ABL_NAIVE_FWD
        if not trace:
            B.abl_stack_backward(self.layers, self.K, self.skip_every, self.buf_s, self.buf_t, self.scratch,
                                 flags=flags)
            return None
        tr = [torch.empty(int(np.prod(out_shape(s))), dtype=torch.float32, device="cuda") for s in self.shapes]
        B.abl_stack_backward_traced(self.layers, self.K, self.skip_every, self.buf_s, self.buf_t, self.scratch, tr,
                                    flags=flags)
        return tr

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
