"""Host logic of the max-batch probe (Sec. 4, Table 2 analogue): the network builder and the
memory accounting, from the library's size queries only - no GPU."""
import pytest

from paper_1901_07988_amd import binding as B
from paper_1901_07988_amd import max_batch as MB


@pytest.mark.parametrize("depth", [11, 29, 164])
def test_network_body_chains(depth):
    n = (depth - 2) // 9
    shapes = MB.resnet_body(3, depth)
    assert len(shapes) == 9 * n == depth - 2
    for a, b in zip(shapes, shapes[1:]):
        assert (a.N, a.Ho, a.Wo, a.Cout) == (b.N, b.H, b.W, b.Cin)
    # three stages at 32, 16, 8 pixels; 16/32/64 bottleneck channels; output 256 channels at 8x8
    assert [s.H for s in shapes[::3 * n]] == [32, 32, 16]
    assert [s.Cout for s in shapes[1::3 * n]] == [16, 32, 64]
    last = shapes[-1]
    assert (last.Ho, last.Wo, last.Cout) == (8, 8, 256)
    # blocks other than the first of a stage keep their shape: the identity shortcut applies
    for g in range(0, len(shapes), 3):
        first, lastb = shapes[g], shapes[g + 2]
        same = (first.H, first.W, first.Cin) == (lastb.Ho, lastb.Wo, lastb.Cout)
        assert same == ((g // 3) % n != 0)
    with pytest.raises(ValueError):
        MB.resnet_body(1, 100)


def test_stored_bytes_follow_the_bit_width():
    shapes = MB.resnet_body(64, 29)
    exact, k8, k4 = (MB.step_bytes(shapes, K) for K in (32, 8, 4))
    E = sum(s.E for s in shapes)
    assert exact["stored"] >= 4 * E and exact["stored"] <= 4 * E + 256 * len(shapes)
    # Sec. 3.4: alpha = 1/4 and 1/8 of the exact copy (up to padding of each layer's rows)
    assert k8["stored"] <= exact["stored"] / 4 * 1.01 + 256 * len(shapes)
    assert k4["stored"] <= exact["stored"] / 8 * 1.01 + 256 * len(shapes)
    assert k4["stored"] >= E // 2
    # everything that is not a stored copy is the same in the three modes, up to the workspace
    for key in ("stats", "params", "buffers"):
        assert exact[key] == k8[key] == k4[key]
    assert exact["total"] == sum(v for k, v in exact.items() if k != "total")


def test_bytes_grow_with_the_batch():
    prev = 0
    for N in (1, 2, 5, 16, 64):
        t = MB.step_bytes(MB.resnet_body(N, 20), 4)["total"]
        assert t > prev
        prev = t


@pytest.mark.parametrize("K", [4, 8, 32])
def test_max_batch_is_the_largest_that_fits(K):
    budget = 256 << 20
    N = MB.max_batch(29, K, budget)
    assert N >= 1
    assert MB.step_bytes(MB.resnet_body(N, 29), K)["total"] <= budget
    assert MB.step_bytes(MB.resnet_body(N + 1, 29), K)["total"] > budget
    assert MB.max_batch(29, K, 1 << 10) == 0


def test_gain_grows_with_depth_and_stays_below_the_storage_ratio():
    """Sec. 3.4: memory is O(W + 1 + alpha L) against O(L): the batch gain approaches 1/alpha = 8
    from below as the network gets deeper (Table 2 shows the same trend)."""
    budget = int(MB.BUDGET_GB * (1 << 30))
    ratios = []
    for depth in (29, 164, 1001):
        e, k = MB.max_batch(depth, 32, budget), MB.max_batch(depth, 4, budget)
        assert e >= 1
        ratios.append(k / e)
    assert ratios[0] < ratios[1] < ratios[2] < 8.0
    assert ratios[2] > 6.0


def test_batch_limit_respects_the_index_ranges():
    lim = MB.batch_limit(164)
    assert lim * 32 * 32 < MB.PIXEL_LIMIT <= (lim + 1) * 32 * 32
    # a budget larger than any GPU: the probe stops at the index limit instead
    assert MB.max_batch(11, 4, 1 << 50) == MB.batch_limit(11)
    assert B.abl_packed_bytes(MB.resnet_body(lim, 11)[0].as_tuple(), 4) > 0
