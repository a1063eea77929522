"""Host-side checks that need no GPU: the C-ABI library loads, exports every symbol that
include/abl.h declares, and its size queries and argument validation behave as documented."""
import ctypes
import os
import re

import pytest

from paper_1901_07988_amd import synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def B():
    lib = os.path.join(ROOT, "paper_1901_07988_amd", "libabl.so")
    if not os.path.exists(lib):
        from paper_1901_07988_amd import build
        build.build(verbose=False)
    from paper_1901_07988_amd import binding
    return binding


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "abl.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(abl_[a-z_0-9]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(B):
    names = declared_symbols()
    assert len(names) >= 18
    for n in names:
        assert hasattr(B.lib, n), n
    assert set(names) == set(B.EXPORTS)


def test_packed_and_stats_sizes(B, oracle):
    wls = [synth.config1(), synth.config2(), *synth.config3(), synth.config4(), synth.config5()]
    for wl in wls:
        for s in wl.shapes:
            for K in (4, 8):
                pb = B.abl_packed_bytes(s.as_tuple(), K)
                assert pb == oracle.packed_bytes(s.E, K) == 4 * s.E * K // 32       # alpha = K/32
                meta = B.abl_stats_bytes(s.as_tuple())
                assert meta == 32 * s.Cin
                assert pb + meta <= (K / 32 + 0.01) * 4 * s.E
                assert B.abl_scratch_bytes(s.as_tuple(), K) >= 4 * s.E
    assert B.abl_packed_bytes((1, 1, 1, 3, 4, 1, 1, 1, 0), 4) == 128      # ragged tail is padded
    assert B.abl_packed_bytes((1, 3, 3, 43, 4, 1, 1, 1, 0), 8) == 512


def test_invalid_arguments_are_rejected_before_any_launch(B):
    s = B.shape_struct((2, 8, 8, 16, 16, 3, 3, 1, 1))
    ref = ctypes.byref(s)
    assert B.lib.abl_packed_bytes(ref, 5) == 0
    assert B.lib.abl_packed_bytes(None, 4) == 0
    bad = B.shape_struct((2, 2, 2, 16, 16, 5, 5, 1, 0))                   # filter larger than input
    assert B.lib.abl_packed_bytes(ctypes.byref(bad), 4) == 0
    assert B.lib.abl_forward(None, ref, 4, 0, None, None, None, None, None, None, 0, None, None, None) == B.ABL_ERR_ARG
    assert B.lib.abl_forward(None, ref, 3, 0, 16, 16, 16, 16, None, 16, 0, 16, 16, 16) == B.ABL_ERR_ARG
    assert B.lib.abl_forward(None, ref, 4, 0, 16, 16, 16, 16, None, 16, 0, 16, 16, 16) == B.ABL_ERR_SCRATCH
    assert B.lib.abl_forward(None, ref, 4, 0, 20, 16, 16, 16, None, 16, 1 << 30, 16, 16, 16) == B.ABL_ERR_ARG
    assert B.lib.abl_backward(None, ctypes.byref(bad), 4, 0, 16, 16, 16, 16, 16, 1 << 30, 16, 16, 16, 16) == B.ABL_ERR_SHAPE
    assert B.lib.abl_bn_stats(None, 16, 0, 16, 16, 16, 4, 16, 1 << 20, 16) == B.ABL_ERR_SHAPE
    assert B.lib.abl_bn_bwd(None, 16, 16, 16, 10, 16, 4, 8, 16, 1 << 20, 16, 16, 16) == B.ABL_ERR_ARG  # unknown flag
    assert b"scratch" in B.lib.abl_error_string(B.ABL_ERR_SCRATCH)


def test_stack_plan_validation(B):
    mk = lambda t: dict(shape=t)
    ok = B.make_layers([mk((2, 8, 8, 16, 32, 3, 3, 2, 1)), mk((2, 4, 4, 32, 32, 3, 3, 1, 1))])
    assert B.abl_stack_buffer_bytes(ok) == 2 * 8 * 8 * 16 * 4
    assert B.abl_stack_scratch_bytes(ok, 4) >= 2 * 8 * 8 * 16 * 4
    broken = B.make_layers([mk((2, 8, 8, 16, 32, 3, 3, 2, 1)), mk((2, 8, 8, 32, 32, 3, 3, 1, 1))])
    assert B.lib.abl_stack_forward(None, broken, 2, 4, 0, 0, 16, 32, 48, 1 << 30) == B.ABL_ERR_SHAPE


def test_stack_calls_validate_every_layer_before_the_first_launch(B):
    """A null or misaligned pointer in the LAST layer is reported as an argument error: had the
    layers before it been enqueued first, the call would have launched kernels on the made-up
    addresses of this test (and, on a machine without a GPU, returned a launch failure instead)."""
    shapes = [(2, 8, 8, 16, 16, 3, 3, 1, 1)] * 3
    full = dict(W=16, gamma=32, beta=48, packed=64, stats=80, dW=96, dgamma=112, dbeta=128)
    for direction, fields in (("forward", ("W", "gamma", "beta", "packed", "stats")),
                              ("backward", ("W", "packed", "stats", "dW", "dgamma", "dbeta"))):
        fn = getattr(B.lib, "abl_stack_" + direction)
        for name in fields:
            for bad in (None, 24):                       # null, not 16-byte aligned
                descs = [dict(shape=t, **full) for t in shapes]
                descs[-1][name] = bad
                layers = B.make_layers(descs)
                assert fn(None, layers, 3, 4, 0, 0, 16, 32, 48, 1 << 30) == B.ABL_ERR_ARG, (direction, name, bad)
    # a workspace that is too small is reported before any launch as well
    layers = B.make_layers([dict(shape=t, **full) for t in shapes])
    assert B.lib.abl_stack_forward(None, layers, 3, 4, 0, 0, 16, 32, 48, 1024) == B.ABL_ERR_SCRATCH
    trace = (ctypes.c_void_p * 3)(16, 32, 40)            # misaligned inspection pointer
    assert B.lib.abl_stack_forward_traced(None, layers, 3, 4, 0, 0, 16, 32, 48, 1 << 30, trace) == B.ABL_ERR_ARG
    assert B.lib.abl_stack_backward_traced(None, layers, 3, 4, 0, 0, 16, 32, 48, 1 << 30, trace) == B.ABL_ERR_ARG


def test_exact_storage_sizes_and_k_validation(B):
    """K = 32 keeps the fp32 tensor (alpha = 1, Sec. 3.4); the fused entry points refuse it."""
    t = (4, 32, 32, 16, 16, 3, 3, 1, 1)
    E = 4 * 32 * 32 * 16
    assert B.abl_packed_bytes(t, 32) == 4 * E
    assert B.abl_packed_bytes(t, 8) * 4 == B.abl_packed_bytes(t, 32)
    assert B.abl_scratch_bytes(t, 32) > 0
    ref = ctypes.byref(B.shape_struct(t))
    assert B.lib.abl_packed_bytes(ref, 16) == 0
    assert B.lib.abl_bn_conv_fwd(None, ref, 32, 0, 16, 16, 16, None, 32, 16) == B.ABL_ERR_ARG
    assert B.lib.abl_postact_packed_bytes(ref, 32) == 0


def test_bench_refuses_more_than_one_gpu():
    """bench.py measures one GPU's share; a larger --gpus exits with a message and a non-zero code
    before anything touches a device."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True,
                       text=True, timeout=120)
    assert r.returncode != 0
    assert "one GPU" in r.stderr and r.stdout.strip() == ""


def test_forward_path_query(B):
    """abl_forward_is_fused answers from the shape alone (no launch): the 56x56 bottleneck layers take
    the kernel with the Eq. 1-3 / Eq. 9 prologue, the 14x14 layers that the register-resident kernels
    cover take the pack pass plus the plain contraction, exact storage never fuses."""
    assert B.abl_forward_is_fused((64, 56, 56, 256, 64, 1, 1, 1, 0), 4) is True
    assert B.abl_forward_is_fused((64, 56, 56, 64, 64, 3, 3, 1, 1), 4) is True
    assert B.abl_forward_is_fused((64, 14, 14, 1024, 256, 1, 1, 1, 0), 4) is False
    assert B.abl_forward_is_fused((64, 14, 14, 256, 256, 3, 3, 1, 1), 8) is False
    assert B.abl_forward_is_fused((2, 14, 14, 256, 256, 3, 3, 1, 1), 4) is True      # too few blocks for them
    assert B.abl_forward_is_fused((64, 56, 56, 64, 64, 3, 3, 1, 1), 32) is False
    with pytest.raises(B.AblError) as e:
        B.abl_forward_is_fused((64, 56, 56, 64, 64, 3, 3, 1, 1), 5)
    assert e.value.code == B.ABL_ERR_ARG
