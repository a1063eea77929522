"""Layer-by-layer ("teacher-forced") parity of a GPU stack or conv-first layer against the oracle.

Below the first layer of a stack the two sides quantize activations that differ by the fp32
rounding of the convolutions above, so an end-to-end comparison of codes could only be
statistical.  Instead every layer is checked on its own: the library's inspection hook hands out
the input x_i the layer really saw (and, backward, the gradient dy_i it really received), the
oracle runs that one layer on exactly those tensors, and the bars are the single-layer ones:
statistics within one ulp, packed bytes bit for bit, y, dx, dW, dgamma, dbeta within 1e-4."""
import numpy as np

from paper_1901_07988_amd import synth

TOL = 1e-4


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


def teacher_forced(G, o, wl, K, seed=synth.DEFAULT_SEED, verbose=True, flags=0, tol=TOL):
    """Runs the workload's stack on the GPU (forward and backward, traced) and checks every layer
    against the oracle on the GPU's own tensors.  K = 32 is exact storage: the store is the fp32 A2.
    flags / tol: the library flags of the run and the bar on y and the gradients (statistics and
    packed bytes keep their exact bars whatever the flags).
    Returns the worst relative error per quantity."""
    x, layers, dy = synth.draw_stack(wl, seed)
    L, g = len(layers), wl.skip_every
    run = G.StackRun(layers, K, g, flags=flags)
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
        got_store = run.descs[i]["packed"].cpu().numpy()
        if K == 32:
            assert got_store[: a2.nbytes].tobytes() == a2.tobytes(), (i, "stored A2")
        else:
            q = o.quantize(a2, gamma, beta, K)
            want_store = o.pack_codes(q, K)
            assert got_store[: want_store.size].tobytes() == want_store.tobytes(), (i, "packed bytes")
            assert not got_store[want_store.size:].any(), (i, "padding of the last 128-byte row")
        y_ref = o.conv_fwd(a3, w, os_)
        if shortcut(i) and i == g1:
            y_ref = y_ref + xin[g0].cpu().numpy().reshape(y_ref.shape)
        y_gpu = (xin[i + 1].cpu().numpy() if i + 1 < L else y_top).reshape(y_ref.shape)
        worst["y"] = max(worst["y"], rel(y_gpu, y_ref))
        assert worst["y"] < tol, (i, "y")
        del a3, y_ref, y_gpu
        # ---- backward of layer i on the gradient the GPU layer received
        dyi = dyin[i].cpu().numpy().reshape(s.N, s.Ho, s.Wo, s.Cout)
        a2t = a2 if K == 32 else o.dequantize(q, gamma, beta, K)
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
            assert worst[name] < tol, (i, name, worst[name])
        if verbose:
            print("layer %2d/%d ok  %s" % (i + 1, L, {k: (v if k == "stat_ulps" else float("%.2g" % v))
                                                     for k, v in worst.items()}), flush=True)
    return worst


def postact_teacher_forced(G, o, run, s, K, x, w, gamma, beta, dy, prev=None):
    """One conv -> BN -> ReLU layer (PostactRun `run`) forward and backward, every stage against the
    oracle on the GPU's own intermediate tensors: the conv output t and the gradient dt that the
    BN backward hands to the two contractions both sit in the layer's workspace after the calls.
    x: the fp32 conv input; prev = (PostactRun, q, gamma, beta) of the layer below when the weight
    gradient is to be taken from that layer's packed store instead.  Returns (y, dx) of the GPU."""
    import torch
    os_ = o.Shape(*s.as_tuple())
    Eo = s.N * s.Ho * s.Wo * s.Cout
    y = run.forward(x, w, gamma, beta)
    t_gpu = run.scratch[: 4 * Eo].view(torch.float32).cpu().numpy().reshape(s.N, s.Ho, s.Wo, s.Cout)
    assert rel(t_gpu, o.conv_fwd(x, w, os_)) < TOL
    mean, var = o.bn_stats(t_gpu)
    rstd = o.bn_rstd(var)
    sd = G.stats_to_dict(run.stats, s.Cout)
    assert max(ulps(sd["mean"], mean), ulps(sd["var"], var), ulps(sd["rstd"], rstd)) <= 1
    a2, a3 = o.bn_relu(t_gpu, sd["mean"], sd["rstd"], gamma, beta)
    assert y.tobytes() == a3.tobytes()                       # Eq. 1-3 element by element: bit-exact
    q = o.quantize(a2, gamma, beta, K)
    want = o.pack_codes(q, K)
    got = run.packed.cpu().numpy()
    assert got[: want.size].tobytes() == want.tobytes() and not got[want.size:].any()
    if prev is None:
        dx, dw, dg, db = run.backward(dy, w, xin=x)
        conv_in = x
    else:
        prun, pq, pgamma, pbeta = prev
        dx, dw, dg, db = run.backward(dy, w, prev=prun)
        conv_in = np.maximum(o.dequantize(pq, pgamma, pbeta, K), np.float32(0))   # what the store holds of x
    dt_gpu = run.scratch[: 4 * Eo].view(torch.float32).cpu().numpy().reshape(t_gpu.shape)
    dt_ref, dg_ref, db_ref = o.bn_relu_bwd(o.dequantize(q, gamma, beta, K), dy, sd["rstd"], gamma, beta)
    assert rel(dt_gpu, dt_ref) < TOL and rel(dg, dg_ref) < TOL and rel(db, db_ref) < TOL
    assert rel(dw, o.conv_wgrad(conv_in, dt_gpu, os_)) < TOL
    assert rel(dx, o.conv_dgrad(dt_gpu, w, os_)) < TOL
    return y, dx, dw, q


