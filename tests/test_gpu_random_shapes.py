"""Seeded random layer shapes and stacks through the C ABI against the oracle: every kernel
family (patch, pointwise, tiled implicit GEMM, element-wise fallbacks) with shapes nobody chose
by hand - odd channel counts, 1x1 / 3x3 / 5x5 filters, stride 2, with and without padding or a
shortcut."""
import numpy as np
import pytest

from paper_1901_07988_amd import synth
from paper_1901_07988_amd.synth import LayerShape

from tests.stack_check import teacher_forced
from tests.test_gpu_parity import TOL, oshape, rel, G  # noqa: F401  (G is a fixture)

pytestmark = pytest.mark.gpu

CHANNELS = [16, 32, 48, 64, 80, 96, 128, 192, 256, 320, 384, 512, 12, 20]


def _random_layer(rng):
    while True:
        R = int(rng.choice([1, 1, 3, 3, 5]))
        stride = int(rng.choice([1, 1, 1, 2]))
        pad = int(rng.choice([0, R // 2]))
        lo = max(1, R - 2 * pad)
        s = LayerShape(int(rng.integers(1, 6)), int(rng.integers(lo, 21)), int(rng.integers(lo, 21)),
                       int(rng.choice(CHANNELS)), int(rng.choice(CHANNELS)), R, R, stride, pad)
        if s.Ho >= 1 and s.Wo >= 1:
            return s


@pytest.mark.parametrize("seed", range(6))
def test_random_layers(G, oracle, seed):
    o = oracle
    rng = np.random.default_rng(1000 + seed)
    for _ in range(12):
        s = _random_layer(rng)
        K = int(rng.choice([4, 8]))
        print("case random layer", s.as_tuple(), K, flush=True)
        x, w, gamma, beta, dy = synth.draw_layer(s, int(rng.integers(1 << 30)), "normal", "random")
        skip = rng.standard_normal((s.N, s.Ho, s.Wo, s.Cout)).astype(np.float32) if rng.random() < 0.3 else None
        run = G.LayerRun(s, K)
        y = run.forward(x, w, gamma, beta, skip=skip)
        y_ref, saved = o.layer_forward(x, w, gamma, beta, K, oshape(o, s), skip=skip)
        assert run.packed.cpu().numpy().tobytes() == saved.store.tobytes()
        assert rel(y, y_ref) < TOL
        dx, dw, dg, db = run.backward(dy, w)
        dx_ref, dw_ref, dg_ref, db_ref = o.layer_backward(saved, dy, w)
        assert rel(dx, dx_ref) < TOL and rel(dw, dw_ref) < TOL
        assert rel(dg, dg_ref) < TOL and rel(db, db_ref) < TOL


@pytest.mark.parametrize("seed", range(4))
def test_random_stacks(G, oracle, seed):
    o = oracle
    rng = np.random.default_rng(2000 + seed)
    for _ in range(5):
        L, skip_every = int(rng.integers(2, 8)), int(rng.choice([0, 2, 3]))
        N, h, w_ = int(rng.integers(1, 5)), int(rng.integers(4, 17)), int(rng.integers(4, 17))
        c = int(rng.choice([16, 32, 64, 128, 256]))
        shapes = []
        for _i in range(L):
            R = int(rng.choice([1, 3]))
            stride = 2 if (rng.random() < 0.12 and h >= 4 and w_ >= 4) else 1
            co = int(rng.choice([16, 32, 64, 128, 256])) if rng.random() < 0.5 else c
            sh = LayerShape(N, h, w_, c, co, R, R, stride, R // 2)
            shapes.append(sh)
            h, w_, c = sh.Ho, sh.Wo, co
        K = int(rng.choice([4, 8]))
        print("case random stack", [s.as_tuple() for s in shapes], "skip", skip_every, "K", K, flush=True)
        wl = synth.Workload("random stack", shapes, skip_every, "normal", "random")
        seed = int(rng.integers(1 << 30))
        x, layers, dy = synth.draw_stack(wl, seed)
        run = G.StackRun(layers, K, skip_every)
        run.load(x)
        run.forward()
        ol = [(oshape(o, s), w, g, b) for s, w, g, b in layers]
        y_ref, saved = o.stack_forward(x, ol, K, np.float32, skip_every)
        assert rel(run.output(), y_ref) < TOL
        # codes and gradients: every layer on the GPU's own tensors
        teacher_forced(G, o, wl, K, seed=seed, verbose=False)


def _random_resident_layer(rng):
    """A layer that one of the register-resident kernels takes in at least one direction: enough
    images (or rows) for 224 blocks of 64 output channels."""
    kind = int(rng.integers(0, 4))
    if kind == 3:      # 1x1 with 64 x 256 channel tiles: rows_wgrad_kernel (tiles x shares of the pixels >= 224, >= 16 chunks each)
        cin, cout = int(rng.choice([64, 128, 192, 320])), int(rng.choice([256, 512]))
        shares = 256 // ((cin // 64) * (cout // 256))
        return LayerShape(1, 16, 16 * shares + int(rng.integers(0, 40)), cin, cout, 1, 1, 1, 0)
    if kind == 0:      # 3x3 'same' on a small image: image_f32_kernel forward and / or data gradient
        H, W = int(rng.integers(2, 15)), int(rng.integers(2, 15))
        while H * W > 208:
            H -= 1
        cin, cout = int(rng.choice([16, 32, 64, 128, 192])), int(rng.choice([64, 128, 256]))
        N = -(-224 // (cout // 64)) + int(rng.integers(0, 5))
        return LayerShape(N, H, W, cin, cout)
    if kind == 1:      # 3x3 'same', 14 pixels wide: image_wgrad_kernel (32 x 64 channel tiles x shares of the images >= 224)
        H = int(rng.choice([2, 4, 6, 10, 14]))
        cin, cout = [(160, 320), (256, 128), (64, 512), (96, 320)][int(rng.integers(0, 4))]
        return LayerShape(16 + int(rng.integers(0, 3)), H, 14, cin, cout)
    # 1x1 with a long contraction: rows_f32_kernel forward (Cin >= 512) or data gradient (Cout >= 512)
    big, small = int(rng.choice([512, 576, 1024])), int(rng.choice([64, 128]))
    rows = -(-224 // (small // 64)) * 208 + int(rng.integers(1, 400))
    H = int(rng.integers(20, 60))
    Wd = -(-rows // H)
    return LayerShape(1, H, Wd, big, small, 1, 1, 1, 0) if rng.random() < 0.5 else LayerShape(1, H, Wd, small, big, 1, 1, 1, 0)


@pytest.mark.parametrize("seed", range(3))
def test_random_layers_on_the_register_resident_kernels(G, oracle, seed):
    """Seeded random shapes large enough for the one-block-per-compute-unit kernels (whole image or
    row block resident, output tile or a tile of dW in accumulator registers): image sizes that leave
    ragged pixel tiles, batches that are not multiples of eight, single-phase and multi-phase
    contractions, tile counts that do not divide the 256 blocks."""
    o = oracle
    rng = np.random.default_rng(3000 + seed)
    for _ in range(5):
        s = _random_resident_layer(rng)
        K = int(rng.choice([4, 8]))
        print("case random resident layer", s.as_tuple(), K, flush=True)
        x, w, gamma, beta, dy = synth.draw_layer(s, int(rng.integers(1 << 30)), "normal", "random")
        skip = rng.standard_normal((s.N, s.Ho, s.Wo, s.Cout)).astype(np.float32) if rng.random() < 0.3 else None
        run = G.LayerRun(s, K)
        y = run.forward(x, w, gamma, beta, skip=skip)
        y_ref, saved = o.layer_forward(x, w, gamma, beta, K, oshape(o, s), skip=skip)
        assert run.packed.cpu().numpy().tobytes() == saved.store.tobytes()
        assert rel(y, y_ref) < TOL
        dx, dw, dg, db = run.backward(dy, w)
        dx_ref, dw_ref, dg_ref, db_ref = o.layer_backward(saved, dy, w)
        assert rel(dx, dx_ref) < TOL and rel(dw, dw_ref) < TOL
        assert rel(dg, dg_ref) < TOL and rel(db, db_ref) < TOL
