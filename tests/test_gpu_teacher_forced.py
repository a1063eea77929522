"""Stack parity, layer by layer, on the GPU's own layer inputs (teacher forcing).

Below the first layer of a stack the two sides quantize activations that differ by the fp32
rounding of the convolutions above, so an end-to-end comparison of codes can only be statistical.
Here every layer of the GPU stack is checked on its own: the library's inspection hook hands out
the input x_i the layer really saw (and, backward, the gradient dy_i it really received), the
oracle runs that one layer on exactly those tensors, and the bars are the single-layer ones:
statistics within one ulp, packed bytes bit for bit, y, dx, dW, dgamma, dbeta within 1e-4.
Run at the full sizes of the workloads, in the launch configuration bench.py times."""
import pytest

from paper_1901_07988_amd import synth
from tests.stack_check import teacher_forced

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def G():
    torch = pytest.importorskip("torch")
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from tests import gpu_util
    return gpu_util


@pytest.mark.parametrize("K", [4, 8])
def test_config2_stack_layer_by_layer(G, oracle, K):
    """18 x [3x3 16->16 @32x32], N=128, identity shortcut every 2 layers."""
    wl = synth.config2()
    teacher_forced(G, oracle, wl, K)


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


def test_bf16_stack_layer_by_layer(G, oracle):
    """ABL_MATH_BF16 on three bottlenecks 1024-256-256-1024 @14x14, N=9: the contractions round their
    operands to bf16 (bar 2e-2), while every layer's statistics - taken from the sums that the
    convolution above left in its epilogue - and its packed bytes stay exact on the GPU's own
    tensors."""
    from paper_1901_07988_amd import binding as B
    wl = synth.config5(N=9, blocks=3)
    teacher_forced(G, oracle, wl, 4, flags=B.ABL_MATH_BF16, tol=2e-2)
