"""Stack parity, layer by layer, on the GPU's own layer inputs (teacher forcing).

Below the first layer of a stack the two sides quantize activations that differ by the fp32
rounding of the convolutions above, so an end-to-end comparison of codes can only be statistical.
Here every layer of the GPU stack is checked on its own: the library's inspection hook hands out
the input x_i the layer really saw (and, backward, the gradient dy_i it really received), the
oracle runs that one layer on exactly those tensors, and the bars are the single-layer ones:
statistics within one ulp, packed bytes bit for bit, y, dx, dW, dgamma, dbeta within 1e-4.
Run at the full sizes of the workloads, in the launch configuration bench.py times."""
import numpy as np
import pytest

from paper_1901_07988_amd import synth

pytestmark = pytest.mark.gpu

TOL = 1e-4


@pytest.fixture(scope="module")
def G():
    torch = pytest.importorskip("torch")
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from tests import gpu_util
    return gpu_util


def rel(a, b):
    return float(np.max(np.abs(np.asarray(a, np.float64) - np.asarray(b, np.float64))) /
                 max(float(np.max(np.abs(b))), 1e-30))


def ulps(a, b):
    """Largest distance in units of the last place between two fp32 vectors of equal sign pattern."""
    ia, ib = a.view(np.int32).astype(np.int64), b.view(np.int32).astype(np.int64)
    return int(np.max(np.abs(ia - ib)))


def group_of(i, L, g):
    """(first, last, in_group) of layer i's shortcut group of g layers (the library's rule)."""
    if g <= 0:
        return i, i, False
    g0 = (i // g) * g
    if g0 + g > L:
        return i, i, False
    return g0, g0 + g - 1, True


def teacher_forced(G, o, wl, K, seed=synth.DEFAULT_SEED):
    x, layers, dy = synth.draw_stack(wl, seed)
    L, g = len(layers), wl.skip_every
    run = G.StackRun(layers, K, g)
    run.load(x)
    xin = run.forward(trace=True)
    y_top = run.output()
    run.load(dy)
    dyin = run.backward(trace=True)
    dx_bottom = run.input_grad()
    worst = dict(y=0.0, dx=0.0, dW=0.0, dgamma=0.0, dbeta=0.0, stat_ulps=0)

    def shortcut(i):
        g0, g1, ing = group_of(i, L, g)
        if not ing:
            return False
        a, b = layers[g0][0], layers[g1][0]
        return (a.N, a.H, a.W, a.Cin) == (b.N, b.Ho, b.Wo, b.Cout)

    for i, (s, w, gamma, beta) in enumerate(layers):
        os_ = o.Shape(*s.as_tuple())
        g0, g1, _ = group_of(i, L, g)
        xi = xin[i].cpu().numpy().reshape(s.N, s.H, s.W, s.Cin)
        # ---- forward of layer i on the GPU's own input
        mean, var = o.bn_stats(xi)
        rstd = o.bn_rstd(var)
        sd = G.stats_to_dict(run.descs[i]["stats"], s.Cin)
        worst["stat_ulps"] = max(worst["stat_ulps"], ulps(sd["mean"], mean), ulps(sd["var"], var),
                                 ulps(sd["rstd"], rstd))
        assert worst["stat_ulps"] <= 1, (i, "statistics")
        np.testing.assert_array_equal(sd["gamma"], gamma)
        np.testing.assert_array_equal(sd["beta"], beta)
        # codes: the oracle's Eq. 1-3 and Eq. 9 with the statistics the GPU used
        a2, a3 = o.bn_relu(xi, sd["mean"], sd["rstd"], gamma, beta)
        q = o.quantize(a2, gamma, beta, K)
        assert run.descs[i]["packed"].cpu().numpy().tobytes() == o.pack_codes(q, K).tobytes(), (i, "packed bytes")
        y_ref = o.conv_fwd(a3, w, os_)
        if shortcut(i) and i == g1:
            y_ref = y_ref + xin[g0].cpu().numpy().reshape(y_ref.shape)
        y_gpu = (xin[i + 1].cpu().numpy() if i + 1 < L else y_top).reshape(y_ref.shape)
        worst["y"] = max(worst["y"], rel(y_gpu, y_ref))
        assert worst["y"] < TOL, (i, "y")
        del a3, y_ref, y_gpu
        # ---- backward of layer i on the gradient the GPU layer received
        dyi = dyin[i].cpu().numpy().reshape(s.N, s.Ho, s.Wo, s.Cout)
        a2t = o.dequantize(q, gamma, beta, K)
        da3 = o.conv_dgrad(dyi, w, os_)
        dw_ref = o.conv_wgrad(np.maximum(a2t, np.float32(0)), dyi, os_)
        dx_ref, dg_ref, db_ref = o.bn_relu_bwd(a2t, da3, sd["rstd"], gamma, beta)
        if shortcut(i) and i == g0:      # the gradient of the residual stream is accumulated into
            dx_ref = dx_ref + dyin[g1].cpu().numpy().reshape(dx_ref.shape)
        dx_gpu = (dyin[i - 1].cpu().numpy() if i > 0 else dx_bottom).reshape(dx_ref.shape)
        d = run.descs[i]
        for name, got, ref in (("dx", dx_gpu, dx_ref), ("dW", d["dW"].cpu().numpy(), dw_ref),
                               ("dgamma", d["dgamma"].cpu().numpy(), dg_ref),
                               ("dbeta", d["dbeta"].cpu().numpy(), db_ref)):
            worst[name] = max(worst[name], rel(got, ref))
            assert worst[name] < TOL, (i, name, worst[name])
        print("layer %2d/%d ok  %s" % (i + 1, L, {k: (v if k == "stat_ulps" else float("%.2g" % v))
                                                 for k, v in worst.items()}), flush=True)
    exact = sum(4 * s.E for s, *_ in layers)
    assert run.stored_bytes() <= (K / 32 + 0.01) * exact
    return worst


@pytest.mark.parametrize("K", [4, 8])
def test_config2_stack_layer_by_layer(G, oracle, K):
    """18 x [3x3 16->16 @32x32], N=128, identity shortcut every 2 layers."""
    teacher_forced(G, oracle, synth.config2(), K)


@pytest.mark.parametrize("K", [4, 8])
def test_config5_stack_layer_by_layer(G, oracle, K):
    """12 bottlenecks 1024-256-256-1024 @14x14, N=64 (36 layers), random gamma / beta."""
    teacher_forced(G, oracle, synth.config5(), K)


@pytest.mark.parametrize("K", [4, 8])
def test_config4_block_layer_by_layer(G, oracle, K):
    """Bottleneck 256-64-64-256 @56x56, N=64: the 205 MB activations."""
    teacher_forced(G, oracle, synth.config4(), K)


@pytest.mark.parametrize("which", [0, 1], ids=["32ch@16x16", "64ch@8x8"])
def test_config3_stages_layer_by_layer(G, oracle, which):
    """Stride-2 transition + 17 stride-1 layers, N=128."""
    teacher_forced(G, oracle, synth.config3()[which], 4)
