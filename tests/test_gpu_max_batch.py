"""Max-batch probe on the GPU (Sec. 4, Table 2 analogue): the bottleneck network it runs is
checked against the oracle at a small size, and what it allocates against its own accounting."""
import numpy as np
import pytest

from paper_1901_07988_amd import max_batch as MB
from paper_1901_07988_amd import synth

from tests.stack_check import teacher_forced
from tests.test_gpu_parity import TOL, oshape, rel, G  # noqa: F401  (G is a fixture)

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("K", [4, 32])
def test_bottleneck_network_matches_oracle(G, oracle, K):
    o = oracle
    print("case bottleneck network depth 20, N=2, K=%d" % K, flush=True)
    wl = synth.Workload("resnet body, depth 20", MB.resnet_body(2, 20), MB.SKIP_EVERY, "normal", "random")
    x, layers, dy = synth.draw_stack(wl, synth.DEFAULT_SEED)
    run = G.StackRun(layers, K, wl.skip_every)
    run.load(x)
    run.forward()
    olayers = [(oshape(o, s), w, g, b) for s, w, g, b in layers]
    y_ref, saved = o.stack_forward(x, olayers, K, np.float32, wl.skip_every)
    assert rel(run.output(), y_ref) < TOL
    teacher_forced(G, o, wl, K, verbose=False)


def test_probe_allocates_what_it_accounts_for(G):
    budget = 192 << 20
    got = {}
    for K in (32, 4):
        N = MB.max_batch(29, K, budget)
        print("case max-batch probe depth 29, K=%d, N=%d" % (K, N), flush=True)
        assert N >= 1
        want = MB.step_bytes(MB.resnet_body(N, 29), K)["total"]
        r = MB.measure(29, K, N, steps=2, warmup=1)
        assert r["finite"]
        # torch's caching allocator rounds each of the 27 x 8 + 3 tensors up (a few per cent here)
        assert want <= r["allocated_bytes"] <= 1.06 * want + (1 << 20)
        # nothing else is allocated while the steps run (two event objects aside)
        assert r["peak_bytes"] <= r["allocated_bytes"] + (1 << 20)
        assert r["ms_per_sample"] > 0
        got[K] = N
    assert got[4] > 2 * got[32]   # a shallow network: the two full-precision buffers dominate
