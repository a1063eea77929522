"""ctypes binding of libabl.so: the same entry points as include/abl.h, taking torch
tensors that live on the GPU.  Argument marshalling only - every step of the path runs in
the HIP kernels behind the C ABI.  Importing this module fails loudly when the library has
not been built (python -m paper_1901_07988_amd.build)."""
from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libabl.so")

ABL_OK, ABL_ERR_ARG, ABL_ERR_SHAPE, ABL_ERR_SCRATCH, ABL_ERR_HIP = range(5)
ABL_ACCUM_DX = 1
ABL_MATH_BF16 = 2
ABL_XIN_F32 = 8
ABL_NAIVE_FWD = 32
ABL_XIN_PACKED = 16
STATS_PLANES = 8


class AblError(RuntimeError):
    def __init__(self, code, where):
        self.code = code
        super().__init__("%s: %s (code %d)" % (where, lib.abl_error_string(code).decode(), code))


class abl_shape(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in ("N", "H", "W", "Cin", "Cout", "R", "S", "stride", "pad")]


class abl_layer(ctypes.Structure):
    _fields_ = [("shape", abl_shape), ("W", ctypes.c_void_p), ("gamma", ctypes.c_void_p),
                ("beta", ctypes.c_void_p), ("packed", ctypes.c_void_p), ("stats", ctypes.c_void_p),
                ("dW", ctypes.c_void_p), ("dgamma", ctypes.c_void_p), ("dbeta", ctypes.c_void_p)]


if not os.path.exists(LIB_PATH):
    raise ImportError("libabl.so is not built: run `python -m paper_1901_07988_amd.build` "
                      "(there is no CPU fallback)")
lib = ctypes.CDLL(LIB_PATH)

_vp, _sz, _i32, _i64, _u32 = ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int32, ctypes.c_int64, ctypes.c_uint32
_shp = ctypes.POINTER(abl_shape)
_lay = ctypes.POINTER(abl_layer)
_SIGS = {
    "abl_error_string": (ctypes.c_char_p, [ctypes.c_int]),
    "abl_packed_bytes": (_sz, [_shp, ctypes.c_int]),
    "abl_stats_bytes": (_sz, [_shp]),
    "abl_scratch_bytes": (_sz, [_shp, ctypes.c_int]),
    "abl_forward_is_fused": (ctypes.c_int, [_shp, ctypes.c_int, ctypes.c_uint32]),
    "abl_bn_scratch_bytes": (_sz, [_i64, _i32]),
    "abl_wgrad_scratch_bytes": (_sz, [_shp]),
    "abl_forward": (ctypes.c_int, [_vp, _shp, ctypes.c_int, _u32, _vp, _vp, _vp, _vp, _vp, _vp, _sz, _vp, _vp, _vp]),
    "abl_backward": (ctypes.c_int, [_vp, _shp, ctypes.c_int, _u32, _vp, _vp, _vp, _vp, _vp, _sz, _vp, _vp, _vp, _vp]),
    "abl_noalloc_scratch_limit": (_sz, []),
    "abl_backward_noalloc": (ctypes.c_int, [_vp, _shp, ctypes.c_int, _u32, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp]),
    "abl_leaky_forward": (ctypes.c_int, [_vp, _shp, ctypes.c_int, _u32, ctypes.c_float, _vp, _vp, _vp, _vp, _vp, _vp,
                                         _sz, _vp, _vp, _vp]),
    "abl_leaky_backward": (ctypes.c_int, [_vp, _shp, ctypes.c_int, _u32, ctypes.c_float, _vp, _vp, _vp, _vp, _vp, _sz,
                                          _vp, _vp, _vp, _vp]),
    "abl_bn_stats": (ctypes.c_int, [_vp, _vp, _i64, _i32, _vp, _vp, ctypes.c_int, _vp, _sz, _vp]),
    "abl_bn_relu_pack": (ctypes.c_int, [_vp, _vp, _i64, _i32, ctypes.c_int, _vp, _vp, _vp]),
    "abl_pack": (ctypes.c_int, [_vp, _vp, _i64, _i32, ctypes.c_int, _vp, _vp]),
    "abl_unpack": (ctypes.c_int, [_vp, _vp, _i64, _i32, ctypes.c_int, _vp, _vp]),
    "abl_bn_bwd": (ctypes.c_int, [_vp, _vp, _vp, _vp, _i64, _i32, ctypes.c_int, _u32, _vp, _sz, _vp, _vp, _vp]),
    "abl_conv_fwd": (ctypes.c_int, [_vp, _shp, _u32, _vp, _vp, _vp, _vp]),
    "abl_conv_dgrad": (ctypes.c_int, [_vp, _shp, _u32, _vp, _vp, _vp]),
    "abl_conv_wgrad_packed": (ctypes.c_int, [_vp, _shp, ctypes.c_int, _u32, _vp, _vp, _vp, _vp, _sz, _vp]),
    "abl_bn_conv_fwd": (ctypes.c_int, [_vp, _shp, ctypes.c_int, _u32, _vp, _vp, _vp, _vp, _vp, _vp]),
    "abl_conv_dgrad_bn_reduce": (ctypes.c_int, [_vp, _shp, ctypes.c_int, _u32, _vp, _vp, _vp, _vp, _vp, _sz, _vp,
                                                ctypes.POINTER(ctypes.c_int32)]),
    "abl_conv_bwd_bn_reduce": (ctypes.c_int, [_vp, _shp, ctypes.c_int, _u32, _vp, _vp, _vp, _vp, _vp, _sz, _vp, _vp,
                                              ctypes.POINTER(ctypes.c_int32)]),
    "abl_postact_packed_bytes": (_sz, [_shp, ctypes.c_int]),
    "abl_postact_stats_bytes": (_sz, [_shp]),
    "abl_postact_scratch_bytes": (_sz, [_shp, ctypes.c_int]),
    "abl_postact_forward": (ctypes.c_int, [_vp, _shp, ctypes.c_int, _u32, _vp, _vp, _vp, _vp, _vp, _sz, _vp, _vp, _vp]),
    "abl_postact_backward": (ctypes.c_int, [_vp, _shp, ctypes.c_int, _u32, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _sz,
                                            _vp, _vp, _vp, _vp]),
    "abl_stack_scratch_bytes": (_sz, [_lay, _i32, ctypes.c_int]),
    "abl_stack_buffer_bytes": (_sz, [_lay, _i32]),
    "abl_stack_forward": (ctypes.c_int, [_vp, _lay, _i32, ctypes.c_int, _u32, _i32, _vp, _vp, _vp, _sz]),
    "abl_stack_backward": (ctypes.c_int, [_vp, _lay, _i32, ctypes.c_int, _u32, _i32, _vp, _vp, _vp, _sz]),
    "abl_stack_forward_traced": (ctypes.c_int, [_vp, _lay, _i32, ctypes.c_int, _u32, _i32, _vp, _vp, _vp, _sz,
                                                ctypes.POINTER(_vp)]),
    "abl_stack_backward_traced": (ctypes.c_int, [_vp, _lay, _i32, ctypes.c_int, _u32, _i32, _vp, _vp, _vp, _sz,
                                                 ctypes.POINTER(_vp)]),
    "abl_sgd_momentum": (ctypes.c_int, [_vp, _i64, ctypes.c_float, ctypes.c_float, ctypes.c_float, _vp, _vp, _vp]),
    "abl_hbm_probe": (ctypes.c_int, [_vp, ctypes.c_int, _vp, _vp, _sz]),
    "abl_mfma_probe_out_bytes": (_sz, []),
    "abl_mfma_probe_flops": (ctypes.c_double, [ctypes.c_int, ctypes.c_int]),
    "abl_mfma_probe": (ctypes.c_int, [_vp, ctypes.c_int, ctypes.c_int, _vp, _sz]),
}
for _name, (_res, _args) in _SIGS.items():
    _fn = getattr(lib, _name)
    _fn.restype = _res
    _fn.argtypes = _args

EXPORTS = tuple(_SIGS)


def shape_struct(s) -> abl_shape:
    """Accepts an abl_shape, a 9-tuple or anything with N,H,W,Cin,Cout,R,S,stride,pad."""
    if isinstance(s, abl_shape):
        return s
    if isinstance(s, (tuple, list)):
        return abl_shape(*[int(v) for v in s])
    return abl_shape(int(s.N), int(s.H), int(s.W), int(s.Cin), int(s.Cout), int(s.R), int(s.S),
                     int(s.stride), int(s.pad))


def _ptr(t):
    if t is None:
        return None
    if isinstance(t, int):
        return t
    assert t.is_cuda and t.is_contiguous(), "device, contiguous tensors only"
    return t.data_ptr()


def _stream():
    return torch.cuda.current_stream().cuda_stream


def _check(code, where):
    if code != ABL_OK:
        raise AblError(code, where)


# ---- sizes ---------------------------------------------------------------------------------
def abl_packed_bytes(shape, K):
    return lib.abl_packed_bytes(ctypes.byref(shape_struct(shape)), K)


def abl_stats_bytes(shape):
    return lib.abl_stats_bytes(ctypes.byref(shape_struct(shape)))


def abl_scratch_bytes(shape, K):
    return lib.abl_scratch_bytes(ctypes.byref(shape_struct(shape)), K)


def abl_forward_is_fused(shape, K, flags=0):
    r = lib.abl_forward_is_fused(ctypes.byref(shape_struct(shape)), K, flags)
    if r < 0:
        raise AblError(-r, "abl_forward_is_fused")
    return r == 1


def abl_bn_scratch_bytes(M, C):
    return lib.abl_bn_scratch_bytes(M, C)


def abl_wgrad_scratch_bytes(shape):
    return lib.abl_wgrad_scratch_bytes(ctypes.byref(shape_struct(shape)))


# ---- layer ---------------------------------------------------------------------------------
def abl_forward(shape, K, x, W, gamma, beta, skip, scratch, y, packed, stats, flags=0):
    s = shape_struct(shape)
    _check(lib.abl_forward(_stream(), ctypes.byref(s), K, flags, _ptr(x), _ptr(W), _ptr(gamma), _ptr(beta),
                           _ptr(skip), _ptr(scratch), scratch.numel() * scratch.element_size(), _ptr(y),
                           _ptr(packed), _ptr(stats)), "abl_forward")


def abl_backward(shape, K, packed, stats, dy, W, scratch, dx, dW, dgamma, dbeta, flags=0):
    s = shape_struct(shape)
    _check(lib.abl_backward(_stream(), ctypes.byref(s), K, flags, _ptr(packed), _ptr(stats), _ptr(dy), _ptr(W),
                            _ptr(scratch), scratch.numel() * scratch.element_size(), _ptr(dx), _ptr(dW),
                            _ptr(dgamma), _ptr(dbeta)), "abl_backward")


def abl_noalloc_scratch_limit():
    return lib.abl_noalloc_scratch_limit()


def abl_backward_noalloc(shape, K, packed, stats, dy, W, dx, dW, dgamma, dbeta, flags=0):
    s = shape_struct(shape)
    _check(lib.abl_backward_noalloc(_stream(), ctypes.byref(s), K, flags, _ptr(packed), _ptr(stats), _ptr(dy),
                                    _ptr(W), _ptr(dx), _ptr(dW), _ptr(dgamma), _ptr(dbeta)), "abl_backward_noalloc")


def abl_leaky_forward(shape, K, slope, x, W, gamma, beta, skip, scratch, y, packed, stats, flags=0):
    s = shape_struct(shape)
    _check(lib.abl_leaky_forward(_stream(), ctypes.byref(s), K, flags, slope, _ptr(x), _ptr(W), _ptr(gamma),
                                 _ptr(beta), _ptr(skip), _ptr(scratch), scratch.numel() * scratch.element_size(),
                                 _ptr(y), _ptr(packed), _ptr(stats)), "abl_leaky_forward")


def abl_leaky_backward(shape, K, slope, packed, stats, dy, W, scratch, dx, dW, dgamma, dbeta, flags=0):
    s = shape_struct(shape)
    _check(lib.abl_leaky_backward(_stream(), ctypes.byref(s), K, flags, slope, _ptr(packed), _ptr(stats), _ptr(dy),
                                  _ptr(W), _ptr(scratch), scratch.numel() * scratch.element_size(), _ptr(dx),
                                  _ptr(dW), _ptr(dgamma), _ptr(dbeta)), "abl_leaky_backward")


# ---- fused kernels -------------------------------------------------------------------------------
def abl_bn_conv_fwd(shape, K, x, stats, W, skip, y, packed, flags=0):
    s = shape_struct(shape)
    _check(lib.abl_bn_conv_fwd(_stream(), ctypes.byref(s), K, flags, _ptr(x), _ptr(stats), _ptr(W), _ptr(skip),
                               _ptr(y), _ptr(packed)), "abl_bn_conv_fwd")


def abl_conv_dgrad_bn_reduce(shape, K, dy, W, packed, stats, scratch, da3, flags=0):
    """Returns the number of partial rows written to the start of scratch."""
    s = shape_struct(shape)
    rows = ctypes.c_int32(0)
    _check(lib.abl_conv_dgrad_bn_reduce(_stream(), ctypes.byref(s), K, flags, _ptr(dy), _ptr(W), _ptr(packed),
                                        _ptr(stats), _ptr(scratch), scratch.numel() * scratch.element_size(),
                                        _ptr(da3), ctypes.byref(rows)), "abl_conv_dgrad_bn_reduce")
    return rows.value


def abl_conv_bwd_bn_reduce(shape, K, dy, W, packed, stats, scratch, da3, dW, flags=0):
    """Returns the number of partial rows written to the start of scratch."""
    s = shape_struct(shape)
    rows = ctypes.c_int32(0)
    _check(lib.abl_conv_bwd_bn_reduce(_stream(), ctypes.byref(s), K, flags, _ptr(dy), _ptr(W), _ptr(packed),
                                      _ptr(stats), _ptr(scratch), scratch.numel() * scratch.element_size(),
                                      _ptr(da3), _ptr(dW), ctypes.byref(rows)), "abl_conv_bwd_bn_reduce")
    return rows.value


# ---- conv -> BN -> ReLU grouping -----------------------------------------------------------------
def abl_postact_packed_bytes(shape, K):
    return lib.abl_postact_packed_bytes(ctypes.byref(shape_struct(shape)), K)


def abl_postact_stats_bytes(shape):
    return lib.abl_postact_stats_bytes(ctypes.byref(shape_struct(shape)))


def abl_postact_scratch_bytes(shape, K):
    return lib.abl_postact_scratch_bytes(ctypes.byref(shape_struct(shape)), K)


def abl_postact_forward(shape, K, x, W, gamma, beta, scratch, y, packed, stats, flags=0):
    s = shape_struct(shape)
    _check(lib.abl_postact_forward(_stream(), ctypes.byref(s), K, flags, _ptr(x), _ptr(W), _ptr(gamma), _ptr(beta),
                                   _ptr(scratch), scratch.numel() * scratch.element_size(), _ptr(y), _ptr(packed),
                                   _ptr(stats)), "abl_postact_forward")


def abl_postact_backward(shape, K, packed, stats, dy, W, xin, xin_stats, scratch, dx, dW, dgamma, dbeta, flags):
    s = shape_struct(shape)
    _check(lib.abl_postact_backward(_stream(), ctypes.byref(s), K, flags, _ptr(packed), _ptr(stats), _ptr(dy),
                                    _ptr(W), _ptr(xin), _ptr(xin_stats), _ptr(scratch),
                                    scratch.numel() * scratch.element_size(), _ptr(dx), _ptr(dW), _ptr(dgamma),
                                    _ptr(dbeta)), "abl_postact_backward")


# ---- stages --------------------------------------------------------------------------------
def abl_bn_stats(x, M, C, gamma, beta, K, scratch, stats):
    _check(lib.abl_bn_stats(_stream(), _ptr(x), M, C, _ptr(gamma), _ptr(beta), K, _ptr(scratch),
                            scratch.numel() * scratch.element_size(), _ptr(stats)), "abl_bn_stats")


def abl_bn_relu_pack(x, M, C, K, stats, a3, packed):
    _check(lib.abl_bn_relu_pack(_stream(), _ptr(x), M, C, K, _ptr(stats), _ptr(a3), _ptr(packed)),
           "abl_bn_relu_pack")


def abl_pack(a2, M, C, K, stats, packed):
    _check(lib.abl_pack(_stream(), _ptr(a2), M, C, K, _ptr(stats), _ptr(packed)), "abl_pack")


def abl_unpack(packed, M, C, K, stats, a2t):
    _check(lib.abl_unpack(_stream(), _ptr(packed), M, C, K, _ptr(stats), _ptr(a2t)), "abl_unpack")


def abl_bn_bwd(packed, stats, da3, M, C, K, scratch, dx, dgamma, dbeta, flags=0):
    _check(lib.abl_bn_bwd(_stream(), _ptr(packed), _ptr(stats), _ptr(da3), M, C, K, flags, _ptr(scratch),
                          scratch.numel() * scratch.element_size(), _ptr(dx), _ptr(dgamma), _ptr(dbeta)),
           "abl_bn_bwd")


def abl_conv_fwd(shape, a3, W, skip, y, flags=0):
    s = shape_struct(shape)
    _check(lib.abl_conv_fwd(_stream(), ctypes.byref(s), flags, _ptr(a3), _ptr(W), _ptr(skip), _ptr(y)),
           "abl_conv_fwd")


def abl_conv_dgrad(shape, dy, W, da3, flags=0):
    s = shape_struct(shape)
    _check(lib.abl_conv_dgrad(_stream(), ctypes.byref(s), flags, _ptr(dy), _ptr(W), _ptr(da3)), "abl_conv_dgrad")


def abl_conv_wgrad_packed(shape, K, packed, stats, dy, scratch, dW, flags=0):
    s = shape_struct(shape)
    _check(lib.abl_conv_wgrad_packed(_stream(), ctypes.byref(s), K, flags, _ptr(packed), _ptr(stats), _ptr(dy),
                                     _ptr(scratch), scratch.numel() * scratch.element_size(), _ptr(dW)),
           "abl_conv_wgrad_packed")


# ---- stack ---------------------------------------------------------------------------------
def make_layers(descs):
    """descs: list of dicts with shape, W, gamma, beta, packed, stats, dW, dgamma, dbeta (tensors)."""
    arr = (abl_layer * len(descs))()
    for i, d in enumerate(descs):
        arr[i].shape = shape_struct(d["shape"])
        for k in ("W", "gamma", "beta", "packed", "stats", "dW", "dgamma", "dbeta"):
            setattr(arr[i], k, _ptr(d.get(k)))
    return arr


def abl_stack_scratch_bytes(layers, K):
    return lib.abl_stack_scratch_bytes(layers, len(layers), K)


def abl_stack_buffer_bytes(layers):
    return lib.abl_stack_buffer_bytes(layers, len(layers))


def abl_stack_forward(layers, K, skip_every, buf_s, buf_t, scratch, flags=0):
    _check(lib.abl_stack_forward(_stream(), layers, len(layers), K, flags, skip_every, _ptr(buf_s), _ptr(buf_t),
                                 _ptr(scratch), scratch.numel() * scratch.element_size()), "abl_stack_forward")


def abl_stack_backward(layers, K, skip_every, buf_s, buf_t, scratch, flags=0):
    _check(lib.abl_stack_backward(_stream(), layers, len(layers), K, flags, skip_every, _ptr(buf_s), _ptr(buf_t),
                                  _ptr(scratch), scratch.numel() * scratch.element_size()), "abl_stack_backward")


def _trace_array(trace, n):
    arr = (_vp * n)()
    for i in range(n):
        arr[i] = _ptr(trace[i]) if trace is not None and trace[i] is not None else None
    return arr


def abl_stack_forward_traced(layers, K, skip_every, buf_s, buf_t, scratch, trace, flags=0):
    """trace: list of len(layers) device tensors (or None entries) that receive each layer's input."""
    _check(lib.abl_stack_forward_traced(_stream(), layers, len(layers), K, flags, skip_every, _ptr(buf_s),
                                        _ptr(buf_t), _ptr(scratch), scratch.numel() * scratch.element_size(),
                                        _trace_array(trace, len(layers))), "abl_stack_forward_traced")


def abl_stack_backward_traced(layers, K, skip_every, buf_s, buf_t, scratch, trace, flags=0):
    """trace: list of len(layers) device tensors (or None entries) that receive each layer's incoming gradient."""
    _check(lib.abl_stack_backward_traced(_stream(), layers, len(layers), K, flags, skip_every, _ptr(buf_s),
                                         _ptr(buf_t), _ptr(scratch), scratch.numel() * scratch.element_size(),
                                         _trace_array(trace, len(layers))), "abl_stack_backward_traced")


def abl_sgd_momentum(w, grad, v, lr, momentum, weight_decay):
    _check(lib.abl_sgd_momentum(_stream(), w.numel(), lr, momentum, weight_decay, _ptr(w), _ptr(grad), _ptr(v)),
           "abl_sgd_momentum")


# ---- measurement aid -------------------------------------------------------------------------
def abl_hbm_probe(mode, src, dst, nbytes):
    """mode 0 read src, 1 write dst, 2 copy src -> dst; nbytes a multiple of 16."""
    _check(lib.abl_hbm_probe(_stream(), mode, _ptr(src), _ptr(dst), nbytes), "abl_hbm_probe")


def abl_mfma_probe_out_bytes():
    return lib.abl_mfma_probe_out_bytes()


def abl_mfma_probe_flops(mode, iters):
    return lib.abl_mfma_probe_flops(mode, iters)


def abl_mfma_probe(mode, iters, out):
    """mode 0 fp32 16x16x4, mode 1 bf16 16x16x32; out: abl_mfma_probe_out_bytes() bytes."""
    _check(lib.abl_mfma_probe(_stream(), mode, iters, _ptr(out), out.numel() * out.element_size()), "abl_mfma_probe")
