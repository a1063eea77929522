"""abl_backward_noalloc (the entry point for callers that cannot allocate) against abl_backward:
same inputs, bit-identical outputs, on two calls in a row, the second on a smaller layer, so that
what the first call left in the library's fixed workspace cannot leak into the second."""
import ctypes

import numpy as np
import pytest
import torch

from paper_1901_07988_amd import binding as B
from paper_1901_07988_amd import synth
from paper_1901_07988_amd.runtime import LayerRun, dev

pytestmark = pytest.mark.gpu


def backward_both_ways(s, K, seed):
    x, w, gamma, beta, dy = synth.draw_layer(s, seed=seed)
    run = LayerRun(s, K)
    run.forward(x, w, gamma, beta)
    want = run.backward(dy, w)
    f32 = dict(dtype=torch.float32, device="cuda")
    dx = torch.full((s.N, s.H, s.W, s.Cin), 7.0, **f32)
    dw = torch.full((s.R, s.S, s.Cin, s.Cout), 7.0, **f32)
    dg, db = torch.full((s.Cin,), 7.0, **f32), torch.full((s.Cin,), 7.0, **f32)
    B.abl_backward_noalloc(s.as_tuple(), K, run.packed, run.stats, dev(dy), dev(w), dx, dw, dg, db)
    torch.cuda.synchronize()
    got = tuple(t.cpu().numpy() for t in (dx, dw, dg, db))
    return want, got


@pytest.mark.parametrize("K", [4, 8])
def test_noalloc_backward_matches_backward_twice_in_a_row(K):
    # first a layer that takes the one-kernel backward (workspace: dA3, partial rows, dW copies),
    # then a smaller one of another shape that takes the separate kernels
    big = synth.LayerShape(16, 32, 32, 16, 16)
    small = synth.LayerShape(3, 9, 11, 32, 48)
    assert B.abl_scratch_bytes(big.as_tuple(), K) <= B.abl_noalloc_scratch_limit()
    for s, seed in ((big, 11), (small, 12)):
        want, got = backward_both_ways(s, K, seed)
        for name, a, b in zip(("dx", "dW", "dgamma", "dbeta"), want, got):
            np.testing.assert_array_equal(a, b, err_msg="%s K=%d %s" % (name, K, s))


def test_noalloc_backward_rejects_what_does_not_fit():
    s = synth.LayerShape(64, 56, 56, 256, 64, 1, 1, 1, 0)       # needs far more than the fixed workspace
    assert B.abl_scratch_bytes(s.as_tuple(), 4) > B.abl_noalloc_scratch_limit()
    t = torch.zeros(64, device="cuda")
    p = t.data_ptr()
    ss = B.shape_struct(s.as_tuple())
    code = B.lib.abl_backward_noalloc(None, ctypes.byref(ss), 4, 0, p, p, p, p, p, p, p, p)
    assert code == B.ABL_ERR_SCRATCH
    bad = B.shape_struct((2, 2, 2, 16, 16, 5, 5, 1, 0))
    assert B.lib.abl_backward_noalloc(None, ctypes.byref(bad), 4, 0, p, p, p, p, p, p, p, p) == B.ABL_ERR_SHAPE
    assert B.lib.abl_backward_noalloc(None, ctypes.byref(ss), 5, 0, p, p, p, p, p, p, p, p) == B.ABL_ERR_ARG
