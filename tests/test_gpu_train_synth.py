"""Synthetic teacher-student training through the library (Sec. 4, Fig. 3-4 analogue): the loss
of the K-bit runs follows the exact run, and the approximation error of dW stays far below the
batch-to-batch variance of the exact dW."""
import pytest

from paper_1901_07988_amd import train_synth as T

from tests.test_gpu_parity import G  # noqa: F401  (fixture)

pytestmark = pytest.mark.gpu


def test_training_with_approximate_activations_follows_exact(G):
    print("case train_synth 6 layers, batch 16, 40 steps", flush=True)
    curves, nets = {}, {}
    for mode in ("exact", "proposed8", "proposed4"):
        curves[mode], nets[mode] = T.train(mode, steps=40, layers_n=6, batch=16, lr=0.05)
    e = curves["exact"]
    assert e[-1] < 0.5 * e[0]                     # it trains
    assert sum(e[-5:]) < sum(e[10:15]) < sum(e[:5])          # and keeps falling (batches are fresh: noisy)
    # the forward pass is exact, so the first loss is the same number in every mode
    assert curves["proposed4"][0] == e[0] and curves["proposed8"][0] == e[0]
    # Fig. 3: the approximate runs stay on top of the exact one
    assert abs(curves["proposed8"][-1] - e[-1]) < 0.005 * e[-1]
    assert abs(curves["proposed4"][-1] - e[-1]) < 0.02 * e[-1]
    # Fig. 4: approximation error of dW at least an order of magnitude below the SGD noise
    for err, noise in T.gradient_noise(nets["exact"], 4, nbatches=6):
        assert noise > 0 and err < 0.1 * noise
    for err8, (err4, _) in zip((x[0] for x in T.gradient_noise(nets["exact"], 8, nbatches=2)),
                               T.gradient_noise(nets["exact"], 4, nbatches=2)):
        assert err8 < err4                         # more bits, smaller error (Sec. 3.3)
