"""Helpers for the GPU parity tests: run the C-ABI entry points on numpy inputs and bring the
results back as numpy arrays.  Allocation and copies only - no arithmetic of the method."""
import numpy as np
import torch

from paper_1901_07988_amd import binding as B
from paper_1901_07988_amd.runtime import (LayerRun, PostactRun, StackRun, dev, out_shape,  # noqa: F401
                                          zeros_bytes)

PLANES = ("mean", "var", "rstd", "gamma", "beta", "cq", "step", "fb")



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
