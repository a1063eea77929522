"""The library's calls can be recorded into a HIP graph (they allocate nothing, never synchronise
and enqueue kernels only - no memset nodes): a training step of a residual stack captured once and
replayed on fresh inputs, with eager work and synchronisations between the replays, gives the
bits of the eager step every time."""
import numpy as np
import pytest
import torch

from paper_1901_07988_amd import synth

from tests.test_gpu_parity import G  # noqa: F401  (fixture)

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("workload", ["config2", "bottleneck"])
def test_graph_replays_match_the_eager_step(G, workload):
    if workload == "config2":
        wl = synth.config2(N=8, layers=6)
    else:
        s = [synth.LayerShape(4, 14, 14, 128, 64, 1, 1, 1, 0), synth.LayerShape(4, 14, 14, 64, 64),
             synth.LayerShape(4, 14, 14, 64, 128, 1, 1, 1, 0)]
        wl = synth.Workload("bottleneck", s, 3, "normal", "random")
    print("case graph", workload, flush=True)
    x, layers, dy = synth.draw_stack(wl, 3)
    run = G.StackRun(layers, 4, wl.skip_every)
    n_in, n_out = x.size, dy.size
    xin = torch.empty(n_in, dtype=torch.float32, device="cuda")
    gin = torch.empty(n_out, dtype=torch.float32, device="cuda")
    out = torch.empty(n_out, dtype=torch.float32, device="cuda")

    def step():
        run.buf_s[:n_in].copy_(xin)
        run.forward()
        out.copy_(run.buf_s[:n_out])
        run.buf_s[:n_out].copy_(gin)
        run.backward()

    def results():
        torch.cuda.synchronize()
        r = [out.cpu().numpy().copy(), run.buf_s[:n_in].cpu().numpy().copy()]
        for d in run.descs:
            r += [d["dW"].cpu().numpy().copy(), d["dgamma"].cpu().numpy().copy(), d["dbeta"].cpu().numpy().copy(),
                  d["packed"].cpu().numpy().copy()]
        return r

    rng = np.random.default_rng(9)
    batches = [(rng.standard_normal(n_in).astype(np.float32), rng.standard_normal(n_out).astype(np.float32))
               for _ in range(3)]
    eager = []
    for xb, gb in batches:
        xin.copy_(torch.from_numpy(xb))
        gin.copy_(torch.from_numpy(gb))
        step()
        eager.append(results())

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()                                   # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        step()
    for rep in range(2):
        for (xb, gb), want in zip(batches, eager):
            xin.copy_(torch.from_numpy(xb))
            gin.copy_(torch.from_numpy(gb))
            run.buf_t.normal_()                  # eager work between the replays
            torch.cuda.synchronize()
            graph.replay()
            got = results()
            for a, b in zip(got, want):
                assert a.tobytes() == b.tobytes()
