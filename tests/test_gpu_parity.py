"""GPU parity: the HIP path (through the C ABI) against the CPU oracle on the same seeded inputs.

Bars: K-bit codes, packed bytes and every integer are bit-exact; fp32 tensors are within
1e-4 of the oracle, measured per tensor as max|a-b| / max|b|.  A3 and the dequantized A2 are
the same chain of individually rounded fp32 operations on both sides, so they are compared
bit for bit as well."""
import numpy as np
import pytest

from paper_1901_07988_amd import synth
from paper_1901_07988_amd.synth import LayerShape
from tests.stack_check import postact_teacher_forced, teacher_forced

pytestmark = pytest.mark.gpu

TOL = 1e-4
TOL_BF16 = 2e-2        # contractions with operands rounded to bf16 (8 mantissa bits), fp32 accumulation


@pytest.fixture(scope="module")
def G():
    torch = pytest.importorskip("torch")
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from tests import gpu_util
    return gpu_util


def rel(a, b):
    return float(np.max(np.abs(a.astype(np.float64) - b.astype(np.float64))) / max(float(np.max(np.abs(b))), 1e-30))


def oshape(o, s):
    return o.Shape(*s.as_tuple())


def rand_affine(rng, C):
    return rng.uniform(0.5, 1.5, C).astype(np.float32), (rng.standard_normal(C) * 0.2).astype(np.float32)


# (M, C): several row tiles with ragged tails; C = 16/64/256/1024 take the vector path,
# 12/20 the 4-wide path, 7/3 the any-C fallback
BN_CASES = [(8192, 16), (1000, 16), (4099, 64), (777, 256), (131, 1024), (515, 12), (333, 20), (513, 7),
            (1, 16), (3, 3), (100, 1)]


@pytest.mark.parametrize("M,C", BN_CASES)
@pytest.mark.parametrize("K", [4, 8])
def test_stats_codes_and_a3(G, oracle, M, C, K):
    o = oracle
    print("case bn M=%d C=%d K=%d" % (M, C, K), flush=True)
    rng = np.random.default_rng(1000 * M + C + K)
    x = (rng.standard_normal((M, C)) * rng.uniform(0.5, 3, C) + rng.standard_normal(C)).astype(np.float32)
    gamma, beta = rand_affine(rng, C)
    if C > 2:
        gamma[1] = -gamma[1]                      # a negative scale reverses the bins
    st = G.run_bn_stats(x, gamma, beta, K)
    sd = G.stats_to_dict(st, C)
    mean, var = o.bn_stats(x)
    rstd = o.bn_rstd(var)
    cq, step, fb = o.quant_consts(gamma, beta, K)
    # tier 2: the statistics themselves (fp64 accumulation on both sides -> same fp32 values)
    for name, ref in (("mean", mean), ("var", var), ("rstd", rstd)):
        ulp = np.abs(sd[name].view(np.int32).astype(np.int64) - ref.view(np.int32).astype(np.int64))
        assert ulp.max() <= 1, (name, ulp.max())
    np.testing.assert_array_equal(sd["gamma"], gamma)
    np.testing.assert_array_equal(sd["beta"], beta)
    np.testing.assert_array_equal(sd["cq"], cq)
    np.testing.assert_array_equal(sd["step"], step)
    np.testing.assert_array_equal(sd["fb"], fb)
    # tier 1: codes and A3 with the GPU's statistics fed to the oracle -> bit-exact
    a3, packed = G.run_bn_relu_pack(x, st, K)
    rstd_g = o.bn_rstd(sd["var"])
    np.testing.assert_array_equal(rstd_g, sd["rstd"])
    a2_ref, a3_ref = o.bn_relu(x, sd["mean"], sd["rstd"], gamma, beta)
    packed_ref = o.pack_codes(o.quantize(a2_ref, gamma, beta, K), K)
    assert a3.tobytes() == a3_ref.tobytes()
    assert packed.tobytes() == packed_ref.tobytes()
    # and against the oracle's own statistics
    _, a3_own = o.bn_relu(x, mean, rstd, gamma, beta)
    a2_own, _ = o.bn_relu(x, mean, rstd, gamma, beta)
    own = o.pack_codes(o.quantize(a2_own, gamma, beta, K), K)
    assert int(np.count_nonzero(own != packed)) == 0
    assert a3.tobytes() == a3_own.tobytes()


@pytest.mark.parametrize("M,C", BN_CASES)
@pytest.mark.parametrize("K", [4, 8])
def test_pack_unpack_round_trip(G, oracle, M, C, K):
    o = oracle
    print("case pack M=%d C=%d K=%d" % (M, C, K), flush=True)
    rng = np.random.default_rng(7 * M + C + K)
    gamma, beta = rand_affine(rng, C)
    a2 = (gamma * rng.standard_normal((M, C)) * 1.2 + beta).astype(np.float32)
    a2.reshape(-1)[:: max(1, a2.size // 50)] *= 40          # some far outside the clip range
    cq, step, fb = o.quant_consts(gamma, beta, K)
    z = np.zeros(C, np.float32)
    st = G.stats_from_arrays(z, z + 1, z + 1, gamma, beta, cq, step, fb)
    q_ref = o.quantize(a2, gamma, beta, K)
    packed = G.run_pack(a2, st, K)
    assert packed.tobytes() == o.pack_codes(q_ref, K).tobytes()
    a2t = G.run_unpack(packed, a2.shape, st, K)
    assert a2t.tobytes() == o.dequantize(q_ref, gamma, beta, K).tobytes()
    # pack -> unpack -> pack leaves the store unchanged, unpack again gives the same tensor
    packed2 = G.run_pack(a2t, st, K)
    assert packed2.tobytes() == packed.tobytes()
    assert G.run_unpack(packed2, a2.shape, st, K).tobytes() == a2t.tobytes()


@pytest.mark.parametrize("M,C", BN_CASES)
@pytest.mark.parametrize("K", [4, 8])
def test_bn_backward(G, oracle, M, C, K):
    o = oracle
    print("case bnbwd M=%d C=%d K=%d" % (M, C, K), flush=True)
    rng = np.random.default_rng(13 * M + C + K)
    x = rng.standard_normal((M, C)).astype(np.float32)
    gamma, beta = rand_affine(rng, C)
    mean, var = o.bn_stats(x)
    rstd = o.bn_rstd(var)
    a2, _ = o.bn_relu(x, mean, rstd, gamma, beta)
    q = o.quantize(a2, gamma, beta, K)
    packed = o.pack_codes(q, K)
    cq, step, fb = o.quant_consts(gamma, beta, K)
    st = G.stats_from_arrays(mean, var, rstd, gamma, beta, cq, step, fb)
    da3 = rng.standard_normal((M, C)).astype(np.float32)
    dx_ref, dg_ref, db_ref = o.bn_relu_bwd(o.dequantize(q, gamma, beta, K), da3, rstd, gamma, beta)
    dx, dg, db = G.run_bn_bwd(packed, st, da3, K)
    scale = max(1.0, float(np.abs(da3).sum(0).max()))
    assert rel(dx, dx_ref) < TOL
    assert np.max(np.abs(dg - dg_ref)) < TOL * scale and np.max(np.abs(db - db_ref)) < TOL * scale
    # in place (dx aliases da3) and accumulate
    dx2, _, _ = G.run_bn_bwd(packed, st, da3, K, alias=True)
    assert dx2.tobytes() == dx.tobytes()
    base = rng.standard_normal((M, C)).astype(np.float32)
    dx3, _, _ = G.run_bn_bwd(packed, st, da3, K, accum_into=base)
    assert rel(dx3, base + dx_ref) < TOL


CONV_CASES = [
    LayerShape(2, 32, 32, 16, 16),                     # config-1/2 layer, small batch
    LayerShape(3, 9, 7, 16, 16),                       # ragged pixel tail
    LayerShape(2, 16, 16, 32, 32),
    LayerShape(2, 8, 8, 64, 64),
    LayerShape(2, 32, 32, 16, 32, stride=2),           # config-3 transitions
    LayerShape(2, 16, 16, 32, 64, stride=2),
    LayerShape(2, 14, 14, 256, 64, 1, 1, 1, 0),        # bottleneck 1x1s
    LayerShape(1, 14, 14, 64, 256, 1, 1, 1, 0),
    LayerShape(1, 7, 7, 1024, 256, 1, 1, 1, 0),
    LayerShape(1, 14, 14, 256, 256),
    LayerShape(2, 12, 12, 64, 64),
    LayerShape(1, 10, 10, 48, 80),                     # channel counts that are not tile multiples
    LayerShape(2, 9, 9, 96, 144, stride=2),
    LayerShape(2, 7, 6, 5, 3),                         # fallback kernels (channels not multiple of 16)
    LayerShape(1, 6, 6, 8, 12, 3, 3, 2, 0),
    LayerShape(1, 5, 5, 16, 16, 5, 5, 1, 2),           # 5x5 filter
    LayerShape(1, 56, 56, 64, 64),                     # ImageNet 3x3 at full resolution, one image
    LayerShape(3, 20, 33, 16, 16),                     # tiles that do not divide the image
    LayerShape(5, 8, 8, 64, 64),                       # several images per tile, ragged batch
    LayerShape(2, 16, 16, 32, 32, 3, 3, 1, 0),         # no padding
    LayerShape(1, 12, 12, 16, 32, 3, 3, 1, 2),         # padding larger than 'same'
    LayerShape(2, 9, 11, 32, 16, 1, 3, 1, 1),          # 1x3 filter
    LayerShape(3, 13, 11, 64, 128, stride=2),          # strided, channel counts of the bf16 GEMM kernels
    LayerShape(2, 10, 10, 128, 64, 5, 5, 1, 2),
    LayerShape(2, 14, 14, 64, 128, 1, 1, 2, 0),        # strided 1x1 (projection shortcut): three input pixels in four get no tap
    LayerShape(1, 7, 9, 32, 48, 1, 1, 2, 0),           # ... odd image sizes
    LayerShape(1, 10, 11, 16, 32, 3, 3, 3, 1),         # stride 3: nine classes of input pixels in the data gradient
    LayerShape(2, 15, 13, 32, 32, 5, 5, 2, 2),         # 5x5 stride 2
    LayerShape(9, 14, 14, 64, 128),                    # bf16: whole image in LDS, more images than XCDs
    LayerShape(2, 14, 14, 256, 256),                   # ... the 135 KB patch of the 14x14 bottlenecks
    LayerShape(2, 10, 11, 32, 64),                     # ... 7 pixel tiles
    LayerShape(1, 13, 16, 128, 64),                    # ... 208 pixels: the largest image
    LayerShape(56, 3, 3, 256, 256),                    # fp32: whole image in LDS (grids of 224 blocks and more), two channel phases
    LayerShape(28, 9, 9, 128, 512),                    # ... one phase, 6 pixel tiles
    LayerShape(57, 14, 13, 64, 256),                   # ... 12 pixel tiles, ragged last tile, batch not a multiple of 8
    LayerShape(8, 14, 14, 256, 256),                   # ... weight gradient with the image in LDS: 49 pixel steps, 8 shares of the images
    LayerShape(7, 6, 14, 64, 1024),                    # ... 21 steps, one image per share
    LayerShape(9, 12, 14, 128, 512),                   # ... 42 steps, shares of one and two images
]


@pytest.mark.parametrize("s", CONV_CASES, ids=lambda s: "x".join(map(str, s.as_tuple())))
def test_conv_forward_and_dgrad(G, oracle, s):
    o = oracle
    print("case conv", s.as_tuple(), flush=True)
    rng = np.random.default_rng(sum(s.as_tuple()))
    a3 = np.maximum(rng.standard_normal((s.N, s.H, s.W, s.Cin)), 0).astype(np.float32)
    w = synth.he_normal(rng, s)
    dy = rng.standard_normal((s.N, s.Ho, s.Wo, s.Cout)).astype(np.float32)
    y_ref = o.conv_fwd(a3, w, oshape(o, s))
    assert rel(G.run_conv_fwd(s, a3, w), y_ref) < TOL
    skip = rng.standard_normal(y_ref.shape).astype(np.float32)
    assert rel(G.run_conv_fwd(s, a3, w, skip), y_ref + skip) < TOL
    assert rel(G.run_conv_fwd(s, a3, w, skip, alias_skip=True), y_ref + skip) < TOL
    assert rel(G.run_conv_dgrad(s, dy, w), o.conv_dgrad(dy, w, oshape(o, s))) < TOL


def to_bf16(a):
    """fp32 array rounded to the nearest bf16 (ties to even), returned as fp32."""
    u = np.ascontiguousarray(a, np.float32).view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32).reshape(np.shape(a))


@pytest.mark.parametrize("s", CONV_CASES, ids=lambda s: "x".join(map(str, s.as_tuple())))
def test_conv_bf16_variant(G, oracle, s):
    """ABL_MATH_BF16: same contractions with operands rounded to bf16; the oracle stays fp32/fp64
    and the bar is the looser 2e-2.  The result must differ from the fp32 path (the flag is live)
    wherever the matrix-core kernels are used."""
    from paper_1901_07988_amd import binding as B
    o = oracle
    print("case conv bf16", s.as_tuple(), flush=True)
    rng = np.random.default_rng(sum(s.as_tuple()) + 99)
    a3 = np.maximum(rng.standard_normal((s.N, s.H, s.W, s.Cin)), 0).astype(np.float32)
    w = synth.he_normal(rng, s)
    dy = rng.standard_normal((s.N, s.Ho, s.Wo, s.Cout)).astype(np.float32)
    skip = rng.standard_normal(dy.shape).astype(np.float32)
    y_ref = o.conv_fwd(a3, w, oshape(o, s))
    y = G.run_conv_fwd(s, a3, w, skip, flags=B.ABL_MATH_BF16)
    assert rel(y, y_ref + skip) < TOL_BF16
    da = G.run_conv_dgrad(s, dy, w, flags=B.ABL_MATH_BF16)
    assert rel(da, o.conv_dgrad(dy, w, oshape(o, s))) < TOL_BF16
    gamma, beta = rand_affine(rng, s.Cin)
    a2 = (gamma * rng.standard_normal((s.N, s.H, s.W, s.Cin)) + beta).astype(np.float32)
    K = 4
    q = o.quantize(a2, gamma, beta, K)
    cq, step, fb = o.quant_consts(gamma, beta, K)
    z = np.zeros(s.Cin, np.float32)
    st = G.stats_from_arrays(z, z + 1, z + 1, gamma, beta, cq, step, fb)
    dw_ref = o.conv_wgrad(np.maximum(o.dequantize(q, gamma, beta, K), 0), dy, oshape(o, s))
    dw = G.run_conv_wgrad(s, K, o.pack_codes(q, K), st, dy, flags=B.ABL_MATH_BF16)
    assert rel(dw, dw_ref) < TOL_BF16
    if s.Cin % 16 == 0 and s.Cout % 16 == 0:
        assert rel(y, y_ref + skip) > 1e-5 and rel(da, o.conv_dgrad(dy, w, oshape(o, s))) > 1e-5
        # the same precision on both sides: the oracle on operands rounded to bf16 (round to nearest
        # even) differs from the kernels by the order of the fp32 accumulation only
        assert rel(y, o.conv_fwd(to_bf16(a3), to_bf16(w), oshape(o, s)) + skip) < TOL
        assert rel(da, o.conv_dgrad(to_bf16(dy), to_bf16(w), oshape(o, s))) < TOL
        a3t = np.maximum(o.dequantize(q, gamma, beta, K), np.float32(0))
        assert rel(dw, o.conv_wgrad(to_bf16(a3t), to_bf16(dy), oshape(o, s))) < TOL


@pytest.mark.parametrize("s", CONV_CASES, ids=lambda s: "x".join(map(str, s.as_tuple())))
@pytest.mark.parametrize("K", [4, 8])
def test_conv_wgrad_from_packed(G, oracle, s, K):
    o = oracle
    print("case wgrad", s.as_tuple(), K, flush=True)
    rng = np.random.default_rng(sum(s.as_tuple()) + K)
    gamma, beta = rand_affine(rng, s.Cin)
    a2 = (gamma * rng.standard_normal((s.N, s.H, s.W, s.Cin)) + beta).astype(np.float32)
    q = o.quantize(a2, gamma, beta, K)
    cq, step, fb = o.quant_consts(gamma, beta, K)
    z = np.zeros(s.Cin, np.float32)
    st = G.stats_from_arrays(z, z + 1, z + 1, gamma, beta, cq, step, fb)
    dy = rng.standard_normal((s.N, s.Ho, s.Wo, s.Cout)).astype(np.float32)
    a3t = np.maximum(o.dequantize(q, gamma, beta, K), 0)
    dw_ref = o.conv_wgrad(a3t, dy, oshape(o, s))
    dw = G.run_conv_wgrad(s, K, o.pack_codes(q, K), st, dy)
    assert rel(dw, dw_ref) < TOL


PW_WGRAD_CASES = [
    LayerShape(16, 32, 32, 256, 256, 1, 1, 1, 0),      # 4 tiles x 64 shares of exactly 16 chunks
    LayerShape(41, 40, 20, 128, 256, 1, 1, 1, 0),      # 2 tiles x 128 shares of 16 or 17 chunks
    LayerShape(9, 48, 48, 384, 256, 1, 1, 1, 0),       # 6 tiles x 42 shares (not a multiple of 8) of 30 or 31
    LayerShape(64, 14, 14, 1024, 256, 1, 1, 1, 0),     # config 5: 16 tiles x 16 shares of 49
    LayerShape(64, 14, 14, 256, 1024, 1, 1, 1, 0),
]


@pytest.mark.parametrize("s", PW_WGRAD_CASES, ids=lambda s: "x".join(map(str, s.as_tuple())))
@pytest.mark.parametrize("K", [4, 8])
def test_pointwise_wgrad_in_registers(G, oracle, s, K):
    """Weight gradient of 1x1 layers with at least 64 x 256 channels and 16 chunks of 16 pixels per
    block: the kernel that keeps a 64 x 256 tile of dW in registers and applies the step of Eq. 10
    to the sums.  Even and odd chunk counts per block, block counts that do and do not fill the
    eight-way block mapping, a folded bias that moves the ReLU threshold between codes."""
    o = oracle
    print("case pointwise wgrad", s.as_tuple(), K, flush=True)
    rng = np.random.default_rng(sum(s.as_tuple()) + K)
    gamma, beta = rand_affine(rng, s.Cin)
    a2 = (gamma * rng.standard_normal((s.N, s.H, s.W, s.Cin)) + beta).astype(np.float32)
    q = o.quantize(a2, gamma, beta, K)
    cq, step, fb = o.quant_consts(gamma, beta, K)
    z = np.zeros(s.Cin, np.float32)
    st = G.stats_from_arrays(z, z + 1, z + 1, gamma, beta, cq, step, fb)
    dy = rng.standard_normal((s.N, s.Ho, s.Wo, s.Cout)).astype(np.float32)
    a3t = np.maximum(o.dequantize(q, gamma, beta, K), 0)
    dw_ref = o.conv_wgrad(a3t, dy, oshape(o, s))
    dw = G.run_conv_wgrad(s, K, o.pack_codes(q, K), st, dy)
    assert rel(dw, dw_ref) < TOL


@pytest.mark.parametrize("s", PW_WGRAD_CASES, ids=lambda s: "x".join(map(str, s.as_tuple())))
@pytest.mark.parametrize("K", [4, 8])
def test_pointwise_wgrad_in_registers_bf16(G, oracle, s, K):
    """The same shapes with ABL_MATH_BF16: operands rounded to bf16 (the dequantized activation with its
    step, as in the tiled kernel) and contracted 32 pixels per MFMA.  Against the oracle on operands
    rounded the same way the difference is the order of the fp32 accumulation only."""
    from paper_1901_07988_amd import binding as B
    o = oracle
    print("case pointwise wgrad bf16", s.as_tuple(), K, flush=True)
    rng = np.random.default_rng(sum(s.as_tuple()) + K + 1)
    gamma, beta = rand_affine(rng, s.Cin)
    a2 = (gamma * rng.standard_normal((s.N, s.H, s.W, s.Cin)) + beta).astype(np.float32)
    q = o.quantize(a2, gamma, beta, K)
    cq, step, fb = o.quant_consts(gamma, beta, K)
    z = np.zeros(s.Cin, np.float32)
    st = G.stats_from_arrays(z, z + 1, z + 1, gamma, beta, cq, step, fb)
    dy = rng.standard_normal((s.N, s.Ho, s.Wo, s.Cout)).astype(np.float32)
    a3t = np.maximum(o.dequantize(q, gamma, beta, K), np.float32(0))
    dw = G.run_conv_wgrad(s, K, o.pack_codes(q, K), st, dy, flags=B.ABL_MATH_BF16)
    assert rel(dw, o.conv_wgrad(a3t, dy, oshape(o, s))) < TOL_BF16
    assert rel(dw, o.conv_wgrad(to_bf16(a3t), to_bf16(dy), oshape(o, s))) < TOL


LAYER_CASES = [
    (synth.config1().shapes[0], "normal", "unit"),             # BASELINE config 1 as is
    (LayerShape(4, 32, 32, 16, 16), "normal", "random"),
    (LayerShape(4, 16, 16, 32, 32), "normal", "random"),
    (LayerShape(4, 32, 32, 16, 32, stride=2), "normal", "random"),
    (LayerShape(2, 14, 14, 256, 64, 1, 1, 1, 0), "relu_normal", "unit"),
    (LayerShape(2, 14, 14, 64, 64), "relu_normal", "unit"),
    (LayerShape(2, 14, 14, 64, 256, 1, 1, 1, 0), "relu_normal", "unit"),
    (LayerShape(2, 7, 7, 256, 256), "normal", "random"),
    (LayerShape(3, 7, 5, 6, 10), "normal", "random"),          # fallback path end to end
    (LayerShape(56, 5, 5, 256, 256), "normal", "random"),      # image-resident kernels: dgrad with the Eq. 6-7 sums
]


@pytest.mark.parametrize("case", LAYER_CASES, ids=lambda c: "x".join(map(str, c[0].as_tuple())))
@pytest.mark.parametrize("K", [4, 8])
def test_layer_forward_backward(G, oracle, case, K):
    o = oracle
    s, xd, aff = case
    print("case layer", s.as_tuple(), K, flush=True)
    x, w, gamma, beta, dy = synth.draw_layer(s, synth.DEFAULT_SEED, xd, aff)
    run = G.LayerRun(s, K)
    y = run.forward(x, w, gamma, beta)
    y_ref, saved = o.layer_forward(x, w, gamma, beta, K, oshape(o, s))
    sd = G.stats_to_dict(run.stats, s.Cin)
    np.testing.assert_array_equal(sd["mean"], saved.mean)
    np.testing.assert_array_equal(sd["var"], saved.var)
    np.testing.assert_array_equal(sd["rstd"], saved.rstd)
    assert run.packed.cpu().numpy().tobytes() == saved.store.tobytes()
    assert rel(y, y_ref) < TOL
    dx, dw, dg, db = run.backward(dy, w)
    dx_ref, dw_ref, dg_ref, db_ref = o.layer_backward(saved, dy, w)
    assert rel(dx, dx_ref) < TOL and rel(dw, dw_ref) < TOL
    assert rel(dg, dg_ref) < TOL and rel(db, db_ref) < TOL


@pytest.mark.parametrize("case", LAYER_CASES[:8], ids=lambda c: "x".join(map(str, c[0].as_tuple())))
def test_layer_bf16_variant(G, oracle, case):
    """Layer step with ABL_MATH_BF16: codes and statistics are untouched by the flag (bit-exact),
    outputs and gradients within 2e-2."""
    from paper_1901_07988_amd import binding as B
    o = oracle
    s, xd, aff = case
    print("case layer bf16", s.as_tuple(), flush=True)
    x, w, gamma, beta, dy = synth.draw_layer(s, synth.DEFAULT_SEED, xd, aff)
    run = G.LayerRun(s, 4, flags=B.ABL_MATH_BF16)
    y = run.forward(x, w, gamma, beta)
    y_ref, saved = o.layer_forward(x, w, gamma, beta, 4, oshape(o, s))
    assert run.packed.cpu().numpy().tobytes() == saved.store.tobytes()
    assert rel(y, y_ref) < TOL_BF16
    dx, dw, dg, db = run.backward(dy, w)
    dx_ref, dw_ref, dg_ref, db_ref = o.layer_backward(saved, dy, w)
    assert rel(dx, dx_ref) < TOL_BF16 and rel(dw, dw_ref) < TOL_BF16
    assert rel(dg, dg_ref) < TOL_BF16 and rel(db, db_ref) < TOL_BF16


def test_layer_forward_is_independent_of_K_and_repeatable(G):
    s = LayerShape(4, 32, 32, 16, 16)
    x, w, gamma, beta, dy = synth.draw_layer(s, 1, "normal", "random")
    outs = []
    for K in (4, 8, 4):
        run = G.LayerRun(s, K)
        y = run.forward(x, w, gamma, beta)
        outs.append((y, run.backward(dy, w), run.packed.cpu().numpy()))
    assert outs[0][0].tobytes() == outs[1][0].tobytes()             # y does not see the codes
    assert outs[0][1][3].tobytes() == outs[1][1][3].tobytes()       # dbeta is exact (Sec. 3.3)
    assert outs[0][0].tobytes() == outs[2][0].tobytes()             # run twice: identical bits
    assert outs[0][2].tobytes() == outs[2][2].tobytes()
    for a, b in zip(outs[0][1], outs[2][1]):
        assert a.tobytes() == b.tobytes()


def test_layer_skip_inplace_and_accumulate(G, oracle):
    o = oracle
    s = LayerShape(4, 16, 16, 32, 32)
    x, w, gamma, beta, dy = synth.draw_layer(s, 2, "normal", "random")
    rng = np.random.default_rng(5)
    skip = rng.standard_normal((s.N, s.Ho, s.Wo, s.Cout)).astype(np.float32)
    run = G.LayerRun(s, 4)
    y_ref, saved = o.layer_forward(x, w, gamma, beta, 4, oshape(o, s), skip=skip)
    assert rel(run.forward(x, w, gamma, beta, skip=skip), y_ref) < TOL
    y_plain, _ = o.layer_forward(x, w, gamma, beta, 4, oshape(o, s))
    assert rel(run.forward(x, w, gamma, beta, in_place=True), y_plain) < TOL
    base = rng.standard_normal(x.shape).astype(np.float32)
    dx, *_ = run.backward(dy, w, accum_into=base)
    dx_ref, *_ = o.layer_backward(saved, dy, w)
    assert rel(dx, base + dx_ref) < TOL


def _shrunk_stacks():
    c2 = synth.config2(N=8, layers=6)
    c3a, c3b = synth.config3(N=4, per_stage=4)
    c4 = synth.config4(N=2, HW=14)
    c5 = synth.config5(N=2, blocks=2, HW=7)
    odd = synth.Workload("chain of 5, skip/2 (trailing layer runs as a plain chain)",
                         [LayerShape(2, 8, 8, 16, 16)] * 5, 2, "normal", "random")
    return [c2, c3a, c3b, c4, c5, odd]


@pytest.mark.parametrize("wl", _shrunk_stacks(), ids=lambda w: w.name.split(":")[0])
@pytest.mark.parametrize("K", [4, 8])
def test_stack_forward_backward(G, oracle, wl, K):
    """The five workloads at reduced batch / depth / resolution, same structure."""
    o = oracle
    print("case stack", wl.name, K, flush=True)
    x, layers, dy = synth.draw_stack(wl, synth.DEFAULT_SEED)
    run = G.StackRun(layers, K, wl.skip_every)
    run.load(x)
    run.forward()
    y = run.output()
    olayers = [(oshape(o, s), w, g, b) for s, w, g, b in layers]
    y_ref, saved = o.stack_forward(x, olayers, K, np.float32, wl.skip_every)
    assert rel(y, y_ref) < TOL
    # the first layer's codes depend on x only: bit-exact; deeper layers quantize activations
    # that already differ by rounding between the two conv implementations
    assert run.descs[0]["packed"].cpu().numpy()[: saved[0].store.size].tobytes() == saved[0].store.tobytes()
    for d, sv in zip(run.descs, saved):
        got = d["packed"].cpu().numpy()[: sv.store.size]
        assert np.count_nonzero(got != sv.store) <= max(2, sv.store.size // 2000)
    # gradients (and every layer's codes): layer by layer on the GPU's own tensors
    teacher_forced(G, o, wl, K, verbose=False)


def test_error_codes(G):
    from paper_1901_07988_amd import binding as B
    import torch
    s = (2, 8, 8, 16, 16, 3, 3, 1, 1)
    t = torch.zeros(1 << 16, dtype=torch.float32, device="cuda")
    small = torch.zeros(16, dtype=torch.uint8, device="cuda")
    with pytest.raises(B.AblError) as e:
        B.abl_forward(s, 5, t, t, t, t, None, t, t, t, t)
    assert e.value.code == B.ABL_ERR_ARG
    with pytest.raises(B.AblError) as e:
        B.abl_forward((2, 8, 8, 0, 16, 3, 3, 1, 1), 4, t, t, t, t, None, t, t, t, t)
    assert e.value.code == B.ABL_ERR_SHAPE
    with pytest.raises(B.AblError) as e:
        B.abl_forward(s, 4, t, t, t, t, None, small, t, t, t)
    assert e.value.code == B.ABL_ERR_SCRATCH
    with pytest.raises(B.AblError) as e:
        B.abl_forward(s, 4, t.view(-1)[1:], t, t, t, None, t, t, t, t)     # 4-byte aligned only
    assert e.value.code == B.ABL_ERR_ARG
    assert B.abl_packed_bytes((2, 1, 1, 3, 16, 1, 1, 1, 0), 4) == 128
    assert B.abl_packed_bytes(s, 3) == 0


POSTACT_CASES = [
    LayerShape(4, 32, 32, 16, 16),
    LayerShape(4, 32, 32, 16, 32, stride=2),
    LayerShape(2, 14, 14, 64, 256, 1, 1, 1, 0),
    LayerShape(2, 14, 14, 256, 64, 1, 1, 1, 0),
    LayerShape(3, 7, 5, 6, 10),
]


@pytest.mark.parametrize("s", POSTACT_CASES, ids=lambda s: "x".join(map(str, s.as_tuple())))
@pytest.mark.parametrize("K", [4, 8])
def test_postact_layer(G, oracle, s, K):
    """conv -> BN -> ReLU grouping, exact fp32 conv input for the weight gradient.  Every stage is
    checked on the GPU's own intermediate tensors (codes bit for bit, gradients to 1e-4); against
    the oracle's own chain the codes quantize a conv output that differs by fp32 rounding, so a
    code at a bin edge may differ there: at most 1 byte in 2000."""
    o = oracle
    print("case postact", s.as_tuple(), K, flush=True)
    rng = np.random.default_rng(sum(s.as_tuple()) + K)
    x = rng.standard_normal((s.N, s.H, s.W, s.Cin)).astype(np.float32)
    w = synth.he_normal(rng, s)
    gamma, beta = rand_affine(rng, s.Cout)
    dy = rng.standard_normal((s.N, s.Ho, s.Wo, s.Cout)).astype(np.float32)
    run = G.PostactRun(s, K)
    y, dx, dw, _ = postact_teacher_forced(G, o, run, s, K, x, w, gamma, beta, dy)
    # end to end against the oracle's own chain: the output, and all but a few codes at bin edges
    y_ref, saved = o.postact_forward(x, w, gamma, beta, K, oshape(o, s))
    assert rel(y, y_ref) < TOL
    got = run.packed.cpu().numpy()
    assert got.size == saved.store.size
    assert np.count_nonzero(got != saved.store) <= max(1, got.size // 2000)
    # dx is optional
    _, dw2, _, _ = run.backward(dy, w, xin=x, want_dx=False)
    assert dw2.tobytes() == dw.tobytes()


@pytest.mark.parametrize("K", [4, 8])
def test_postact_chain_with_packed_inputs(G, oracle, K):
    """Two conv-first layers: the second one's weight gradient is taken from the first one's
    packed store (ABL_XIN_PACKED), never from a full-precision activation."""
    o = oracle
    rng = np.random.default_rng(31 + K)
    s0, s1 = LayerShape(4, 16, 16, 16, 32), LayerShape(4, 16, 16, 32, 48, 3, 3, 2, 1)
    x = rng.standard_normal((s0.N, s0.H, s0.W, s0.Cin)).astype(np.float32)
    w0, w1 = synth.he_normal(rng, s0), synth.he_normal(rng, s1)
    g0, b0 = rand_affine(rng, s0.Cout)
    g1, b1 = rand_affine(rng, s1.Cout)
    dy = rng.standard_normal((s1.N, s1.Ho, s1.Wo, s1.Cout)).astype(np.float32)
    import torch
    r0, r1 = G.PostactRun(s0, K), G.PostactRun(s1, K)
    # forward of both layers first (the second consumes the first one's GPU output), then the
    # backward from the top: each stage against the oracle on the GPU's own tensors
    y0 = r0.forward(x, w0, g0, b0)
    q0 = o.quantize(o.bn_relu(r0.scratch[: 4 * y0.size].view(torch.float32).cpu().numpy().reshape(y0.shape),
                              G.stats_to_dict(r0.stats, s0.Cout)["mean"], G.stats_to_dict(r0.stats, s0.Cout)["rstd"],
                              g0, b0)[0], g0, b0, K)
    y1, dx1, _, _ = postact_teacher_forced(G, o, r1, s1, K, y0, w1, g1, b1, dy, prev=(r0, q0, g0, b0))
    y0b, _, _, q0b = postact_teacher_forced(G, o, r0, s0, K, x, w0, g0, b0, dx1)
    assert y0b.tobytes() == y0.tobytes() and np.array_equal(q0, q0b)
    y0_ref, sv0 = o.postact_forward(x, w0, g0, b0, K, oshape(o, s0))
    y1_ref, sv1 = o.postact_forward(y0_ref, w1, g1, b1, K, oshape(o, s1))
    assert rel(y0, y0_ref) < TOL and rel(y1, y1_ref) < TOL
    # K-bit storage of the conv-first layer: K/32 of the fp32 tensor it replaces
    from paper_1901_07988_amd import binding as B
    assert B.abl_postact_packed_bytes(s1.as_tuple(), K) == (-(-s1.N * s1.Ho * s1.Wo * s1.Cout * K // 8) + 127) // 128 * 128


@pytest.mark.parametrize("s", [LayerShape(4, 32, 32, 16, 16), LayerShape(2, 16, 16, 32, 64),
                               LayerShape(2, 14, 14, 64, 64), LayerShape(1, 14, 14, 256, 256)],
                         ids=lambda s: "x".join(map(str, s.as_tuple())))
@pytest.mark.parametrize("K", [4, 8])
def test_fused_kernels_on_their_own(G, oracle, s, K):
    _fused_kernels_case(G, oracle, s, K, True)


@pytest.mark.parametrize("s", [LayerShape(3, 14, 14, 64, 32, 1, 1, 1, 0), LayerShape(2, 9, 7, 256, 64, 1, 1, 1, 0),
                               LayerShape(5, 8, 8, 48, 272, 1, 1, 1, 0), LayerShape(40, 14, 14, 32, 16, 1, 1, 1, 0)],
                         ids=lambda s: "x".join(map(str, s.as_tuple())))
@pytest.mark.parametrize("K", [4, 8])
def test_fused_forward_1x1(G, oracle, s, K):
    """abl_bn_conv_fwd on 1x1 convolutions (Eq. 1-3, 9 while the A tile is staged): ragged row
    tiles, several output-channel blocks, 16- and 32-channel chunks."""
    _fused_kernels_case(G, oracle, s, K, False)


@pytest.mark.parametrize("s", [LayerShape(2, 14, 14, 256, 64, 1, 1, 1, 0), LayerShape(3, 9, 7, 64, 256, 1, 1, 1, 0),
                               LayerShape(40, 14, 14, 32, 128, 1, 1, 1, 0), LayerShape(1, 5, 5, 1024, 256, 1, 1, 1, 0)],
                         ids=lambda s: "x".join(map(str, s.as_tuple())))
@pytest.mark.parametrize("K", [4, 8])
def test_fused_kernels_1x1_with_backward(G, oracle, s, K):
    """1x1 layers whose dgrad takes the Eq. 6-7 sums in its epilogue (the contraction runs over
    Cout: a multiple of 64, at most 256): ragged pixel tiles, one to four blocks of input channels."""
    _fused_kernels_case(G, oracle, s, K, True)


def test_dgrad_with_sums_rejects_long_contractions(G):
    import torch
    from paper_1901_07988_amd import binding as B
    t = torch.zeros(1 << 20, dtype=torch.float32, device="cuda")
    sc = G.zeros_bytes(B.abl_bn_scratch_bytes(50, 256))
    for shape in ((2, 5, 5, 256, 1024, 1, 1, 1, 0), (2, 5, 5, 256, 48, 1, 1, 1, 0)):
        with pytest.raises(B.AblError) as e:
            B.abl_conv_dgrad_bn_reduce(shape, 4, t, t, t, t, sc, t[1 << 19:])
        assert e.value.code == B.ABL_ERR_SHAPE


def _fused_kernels_case(G, oracle, s, K, backward):
    """abl_bn_conv_fwd (Eq. 1-3, 9, 4 in one kernel) and abl_conv_dgrad_bn_reduce (Eq. 5 with the
    Eq. 7 sums in the epilogue) against the oracle's separate steps."""
    import torch
    from paper_1901_07988_amd import binding as B
    o = oracle
    print("case fused", s.as_tuple(), K, flush=True)
    x, w, gamma, beta, dy = synth.draw_layer(s, 5, "normal", "random")
    st = G.run_bn_stats(x, gamma, beta, K)
    t = s.as_tuple()
    y = torch.empty(G.out_shape(s), dtype=torch.float32, device="cuda")
    packed = torch.full((B.abl_packed_bytes(t, K),), 0x77, dtype=torch.uint8, device="cuda")
    skip = np.random.default_rng(1).standard_normal(G.out_shape(s)).astype(np.float32)
    B.abl_bn_conv_fwd(t, K, G.dev(x), st, G.dev(w), G.dev(skip), y, packed)
    torch.cuda.synchronize()
    y_ref, saved = o.layer_forward(x, w, gamma, beta, K, oshape(o, s), skip=skip)
    assert packed.cpu().numpy().tobytes() == saved.store.tobytes()
    assert rel(y.cpu().numpy(), y_ref) < TOL
    if not backward:
        return
    # dgrad + reduce: da3 against the oracle, the partial rows against the oracle's Eq. 7 totals
    scratch = G.zeros_bytes(B.abl_bn_scratch_bytes(s.M, s.Cin))
    da3 = torch.empty((s.N, s.H, s.W, s.Cin), dtype=torch.float32, device="cuda")
    rows = B.abl_conv_dgrad_bn_reduce(t, K, G.dev(dy), G.dev(w), packed, st, scratch, da3)
    torch.cuda.synchronize()
    da3_ref = o.conv_dgrad(dy, w, oshape(o, s))
    assert rel(da3.cpu().numpy(), da3_ref) < TOL
    part = scratch[: rows * 2 * s.Cin * 8].cpu().numpy().view(np.float64).reshape(rows, 2, s.Cin).sum(0)
    _, dg_ref, db_ref = o.bn_relu_bwd(o.recover_a2(saved), da3_ref, saved.rstd, gamma, beta)
    scale = max(1.0, float(np.abs(da3_ref).sum((0, 1, 2)).max()))
    assert np.max(np.abs(part[0] - db_ref)) < TOL * scale and np.max(np.abs(part[1] - dg_ref)) < TOL * scale


def test_fused_kernels_reject_unsupported_shapes(G):
    import torch
    from paper_1901_07988_amd import binding as B
    t = torch.zeros(1 << 16, dtype=torch.float32, device="cuda")
    for shape in ((2, 8, 8, 16, 16, 1, 1, 2, 0), (2, 8, 8, 16, 16, 3, 3, 2, 1), (2, 8, 8, 12, 16, 3, 3, 1, 1)):
        with pytest.raises(B.AblError) as e:
            B.abl_bn_conv_fwd(shape, 4, t, t, t, None, t[4096:], t)
        assert e.value.code == B.ABL_ERR_SHAPE


@pytest.mark.parametrize("s", [LayerShape(4, 32, 32, 16, 16), LayerShape(3, 20, 28, 16, 16), LayerShape(10, 8, 8, 16, 16),
                               LayerShape(2, 5, 40, 16, 16)],
                         ids=lambda s: "x".join(map(str, s.as_tuple())))
@pytest.mark.parametrize("K", [4, 8])
def test_one_kernel_conv_backward(G, oracle, s, K):
    """abl_conv_bwd_bn_reduce (both contractions of Eq. 5 and the Eq. 7 sums in one kernel) against the
    oracle's separate steps; tiles that do not divide the image, several images per tile."""
    import torch
    from paper_1901_07988_amd import binding as B
    o = oracle
    print("case conv_bwd", s.as_tuple(), K, flush=True)
    x, w, gamma, beta, dy = synth.draw_layer(s, 9, "normal", "random")
    t = s.as_tuple()
    _, saved = o.layer_forward(x, w, gamma, beta, K, oshape(o, s))
    st = G.run_bn_stats(x, gamma, beta, K)
    packed = G.dev(saved.store)
    nred = (B.abl_bn_scratch_bytes(s.M, s.Cin) + 255) // 256 * 256
    scratch = G.zeros_bytes(nred + B.abl_wgrad_scratch_bytes(t))
    da3 = torch.empty((s.N, s.H, s.W, s.Cin), dtype=torch.float32, device="cuda")
    dw = torch.empty(w.shape, dtype=torch.float32, device="cuda")
    rows = B.abl_conv_bwd_bn_reduce(t, K, G.dev(dy), G.dev(w), packed, st, scratch, da3, dw)
    torch.cuda.synchronize()
    da3_ref = o.conv_dgrad(dy, w, oshape(o, s))
    a2t = o.recover_a2(saved)
    dw_ref = o.conv_wgrad(np.maximum(a2t, 0).astype(np.float32), dy, oshape(o, s))
    assert rel(da3.cpu().numpy(), da3_ref) < TOL
    assert rel(dw.cpu().numpy(), dw_ref) < TOL
    part = scratch[: rows * 2 * s.Cin * 8].cpu().numpy().view(np.float64).reshape(rows, 2, s.Cin).sum(0)
    _, dg_ref, db_ref = o.bn_relu_bwd(a2t, da3_ref, saved.rstd, gamma, beta)
    scale = max(1.0, float(np.abs(da3_ref).sum((0, 1, 2)).max()))
    assert np.max(np.abs(part[0] - db_ref)) < TOL * scale and np.max(np.abs(part[1] - dg_ref)) < TOL * scale


@pytest.mark.parametrize("case", LAYER_CASES[:10], ids=lambda c: "x".join(map(str, c[0].as_tuple())))
def test_layer_exact_storage(G, oracle, case):
    """K = 32 (Sec. 3.2 with alpha = 1: the fp32 A2 itself is stored): the store is bit-exact, the
    gradients are those of exact back-propagation."""
    o = oracle
    s, xd, aff = case
    print("case layer K=32", s.as_tuple(), flush=True)
    x, w, gamma, beta, dy = synth.draw_layer(s, synth.DEFAULT_SEED, xd, aff)
    run = G.LayerRun(s, 32)
    y = run.forward(x, w, gamma, beta)
    y_ref, saved = o.layer_forward(x, w, gamma, beta, 32, oshape(o, s))
    n = saved.store.size * saved.store.itemsize
    assert run.packed.cpu().numpy().tobytes()[:n] == saved.store.tobytes()
    assert rel(y, y_ref) < TOL
    dx, dw, dg, db = run.backward(dy, w)
    dx_ref, dw_ref, dg_ref, db_ref = o.layer_backward(saved, dy, w)
    assert rel(dx, dx_ref) < TOL and rel(dw, dw_ref) < TOL
    assert rel(dg, dg_ref) < TOL and rel(db, db_ref) < TOL


def test_exact_storage_stack_and_round_trip(G, oracle):
    """A residual stack with K = 32 against the oracle's exact mode, and pack -> unpack at K = 32
    returning the input bits."""
    from paper_1901_07988_amd import binding as B
    o = oracle
    wl = synth.config2(N=8, layers=6)
    x, layers, dy = synth.draw_stack(wl)
    run = G.StackRun(layers, 32, wl.skip_every)
    run.load(x)
    run.forward()
    ol = [(oshape(o, s), w, g, b) for s, w, g, b in layers]
    y_ref, saved = o.stack_forward(x, ol, 32, np.float32, wl.skip_every)
    assert rel(run.output(), y_ref) < TOL
    # exact back-propagation, layer by layer on the GPU's own tensors (the stored A2 bit for bit)
    teacher_forced(G, o, wl, 32, verbose=False)
    assert run.stored_bytes() >= sum(4 * s.E for s in wl.shapes)
    a2 = np.random.default_rng(3).standard_normal((50, 20)).astype(np.float32)
    st = G.run_bn_stats(a2, np.ones(20, np.float32), np.zeros(20, np.float32), 32)
    packed = G.run_pack(a2, st, 32)
    assert packed.tobytes()[: a2.size * 4] == a2.tobytes()
    assert G.run_unpack(packed, a2.shape, st, 32).tobytes() == a2.tobytes()


@pytest.mark.parametrize("s", [LayerShape(4, 16, 16, 16, 16), LayerShape(2, 14, 14, 64, 32, 1, 1, 1, 0),
                               LayerShape(3, 7, 5, 6, 10)], ids=lambda s: "x".join(map(str, s.as_tuple())))
@pytest.mark.parametrize("K", [4, 8])
def test_naive_forward_baseline(G, oracle, s, K):
    """ABL_NAIVE_FWD (the comparison baseline of Sec. 4): the convolution consumes the ReLU of the
    dequantized codes.  Codes bit-exact, outputs and gradients against the oracle's naive mode."""
    from paper_1901_07988_amd import binding as B
    o = oracle
    print("case naive", s.as_tuple(), K, flush=True)
    x, w, gamma, beta, dy = synth.draw_layer(s, 21, "normal", "random")
    run = G.LayerRun(s, K, flags=B.ABL_NAIVE_FWD)
    y = run.forward(x, w, gamma, beta)
    y_ref, saved = o.layer_forward(x, w, gamma, beta, K, oshape(o, s), naive=True)
    y_exact, _ = o.layer_forward(x, w, gamma, beta, K, oshape(o, s))
    assert run.packed.cpu().numpy().tobytes() == saved.store.tobytes()
    assert rel(y, y_ref) < TOL
    assert rel(y, y_exact) > 10 * TOL          # it really is another forward pass
    dx, dw, dg, db = run.backward(dy, w)
    dx_ref, dw_ref, dg_ref, db_ref = o.layer_backward(saved, dy, w)
    assert rel(dx, dx_ref) < TOL and rel(dw, dw_ref) < TOL
    assert rel(dg, dg_ref) < TOL and rel(db, db_ref) < TOL


def test_errors_do_not_compound_with_depth(G):
    """Sec. 3.2-3.3 on a 12-layer residual stack: with the proposed method the forward output is
    that of exact training and the weight-gradient error is of the same size at the top and at
    the bottom of the stack; with the naive baseline the output is wrong and the error of the
    bottom layers is several times that of the proposed method."""
    from paper_1901_07988_amd import error_study
    res = error_study.study(layers_n=12, batch=8, ks=(4,))
    p, n = res["proposed K=4"], res["naive K=4"]
    assert p["out"] < 1e-6                      # exact forward pass
    assert n["out"] > 1e-2                      # the baseline's forward pass has drifted
    assert max(p["dW"]) < 0.25 and max(p["dW"]) < 2 * min(p["dW"])   # proposed: no trend with depth
    assert all(a > 1.5 * b for a, b in zip(n["dW"], p["dW"]))        # the baseline is worse everywhere,
    assert n["dW"][0] > 1.2 * n["dW"][-1]                            # and worse the further the error travelled
    assert p["dx"] < 0.02 and n["dx"] > 10 * p["dx"]


@pytest.mark.parametrize("s", [LayerShape(128, 1, 1, 64, 10, 1, 1, 1, 0), LayerShape(37, 1, 1, 256, 48, 1, 1, 1, 0),
                               LayerShape(16, 1, 1, 100, 10, 1, 1, 1, 0)], ids=lambda s: "x".join(map(str, s.as_tuple())))
@pytest.mark.parametrize("K", [4, 8])
def test_fully_connected_layer(G, oracle, s, K):
    """A fully-connected layer is the same layer with 2-D activations (Sec. 3.1: [B, C] tensors,
    statistics over the batch): here a 1x1 convolution on 1x1 images.  Channel counts that are not
    multiples of 16 (a 10-way classifier) run on the element-wise kernels."""
    o = oracle
    print("case fc", s.as_tuple(), K, flush=True)
    x, w, gamma, beta, dy = synth.draw_layer(s, 33, "normal", "random")
    run = G.LayerRun(s, K)
    y = run.forward(x, w, gamma, beta)
    y_ref, saved = o.layer_forward(x, w, gamma, beta, K, oshape(o, s))
    assert run.packed.cpu().numpy().tobytes() == saved.store.tobytes()
    assert rel(y, y_ref) < TOL
    # the library routine this reduces to: batch norm over the batch, ReLU, matrix product
    a2 = (x.reshape(s.N, s.Cin).astype(np.float64) - saved.mean) * saved.rstd * gamma + beta
    assert rel(y.reshape(s.N, s.Cout), np.maximum(a2, 0) @ w.reshape(s.Cin, s.Cout).astype(np.float64)) < TOL
    dx, dw, dg, db = run.backward(dy, w)
    dx_ref, dw_ref, dg_ref, db_ref = o.layer_backward(saved, dy, w)
    assert rel(dx, dx_ref) < TOL and rel(dw, dw_ref) < TOL
    assert rel(dg, dg_ref) < TOL and rel(db, db_ref) < TOL


@pytest.mark.parametrize("L", [1, 2, 3, 4])
def test_plain_chain_alternates_buffers(G, oracle, L):
    """Stacks without shortcuts: the layers alternate between the two buffers (an odd chain runs
    its first layer in place) and the result still lands in the first buffer."""
    o = oracle
    wl = synth.Workload("plain chain of %d" % L, [LayerShape(4, 16, 16, 16, 16)] * L, 0, "normal", "random")
    x, layers, dy = synth.draw_stack(wl, 77)
    run = G.StackRun(layers, 4, 0)
    run.load(x)
    run.forward()
    ol = [(oshape(o, s), w, g, b) for s, w, g, b in layers]
    y_ref, saved = o.stack_forward(x, ol, 4, np.float32, 0)
    assert rel(run.output(), y_ref) < TOL
    teacher_forced(G, o, wl, 4, seed=77, verbose=False)


@pytest.mark.parametrize("K", [4, 8])
def test_quantizer_on_non_finite_and_huge_values(G, oracle, K):
    """Eq. 9 must be defined for any input: floor() is limited to +-2^24 before the integer
    conversion, a NaN takes the lowest code.  Same bytes on both sides."""
    o = oracle
    C = 16
    rng = np.random.default_rng(5)
    a2 = rng.standard_normal((64, C)).astype(np.float32)
    a2[0, :] = np.nan
    a2[1, :] = np.inf
    a2[2, :] = -np.inf
    a2[3, :] = 3e38
    a2[4, :] = -3e38
    a2[5, ::2] = 2.0 ** 25
    a2[5, 1::2] = -(2.0 ** 25)
    gamma = rng.uniform(0.5, 1.5, C).astype(np.float32)
    beta = (rng.standard_normal(C) * 0.1).astype(np.float32)
    st = G.run_bn_stats(rng.standard_normal((64, C)).astype(np.float32), gamma, beta, K)
    got = G.run_pack(a2, st, K)
    with np.errstate(all="ignore"):
        ref = o.pack_codes(o.quantize(a2, gamma, beta, K), K)
    assert got.tobytes()[: ref.size] == ref.tobytes()
    codes = o.unpack_codes(ref, a2.shape, K)
    assert np.all(codes[0] == 0) and np.all(codes[2] == 0) and np.all(codes[1] == 2 ** K - 1)


@pytest.mark.parametrize("n", [1, 3, 4, 5, 1023, 4099, 1 << 16])
def test_sgd_momentum_update(G, oracle, n):
    """The parameter update of Sec. 4's training setup: bit-exact against the fp32 oracle over
    several steps (every operation is rounded on its own on both sides), ragged tails included."""
    import torch
    from paper_1901_07988_amd import binding as B
    print("case sgd", n, flush=True)
    rng = np.random.default_rng(n)
    w = rng.standard_normal(n).astype(np.float32)
    v = np.zeros(n, np.float32)
    wt, vt = G.dev(w), G.dev(v)
    for step in range(4):
        g = rng.standard_normal(n).astype(np.float32)
        B.abl_sgd_momentum(wt, G.dev(g), vt, 0.1, 0.9, 2e-4)
        w, v = oracle.sgd_momentum(w, g, v, 0.1, 0.9, 2e-4, np.float32)
        assert wt.cpu().numpy().tobytes() == w.tobytes()
        assert vt.cpu().numpy().tobytes() == v.tobytes()
    with pytest.raises(B.AblError):
        B.abl_sgd_momentum(wt, None, vt, 0.1, 0.9, 0.0)
    B.abl_sgd_momentum(wt[:0], wt[:0], vt[:0], 0.1, 0.9, 0.0)   # n = 0: nothing to do


@pytest.mark.parametrize("s,pool", [(LayerShape(16, 8, 8, 64, 10, 8, 8, 1, 0), 8),      # global pool + classifier
                                    (LayerShape(8, 8, 8, 64, 32, 8, 8, 1, 0), 8),
                                    (LayerShape(4, 12, 12, 32, 32, 2, 2, 2, 0), 2)],    # 2x2 pool + 1x1 conv
                         ids=["global-pool+fc10", "global-pool+fc32", "pool2+conv1x1"])
def test_average_pool_folded_into_linear(G, oracle, s, pool):
    """Average pooling is folded into the linear transform that follows it (Sec. 3.4): BN -> ReLU
    -> pool x pool average -> 1x1 convolution V is the layer with the pool x pool, stride-pool
    kernel W[r, s] = V / pool^2.  Checked against the pooling written out on the oracle's A3, and
    the gradient of V, sum_rs dW[r, s] / pool^2, against pooling of the dequantized activation."""
    o = oracle
    K = 4
    print("case folded average pool", s.as_tuple(), flush=True)
    assert s.R == s.S == pool and s.stride in (1, pool) and s.pad == 0
    rng = np.random.default_rng(12)
    x = rng.standard_normal((s.N, s.H, s.W, s.Cin)).astype(np.float32)
    gamma, beta = rand_affine(rng, s.Cin)
    V = (rng.standard_normal((s.Cin, s.Cout)) * np.sqrt(2.0 / s.Cin)).astype(np.float32)
    w = np.ascontiguousarray(np.broadcast_to(V / np.float32(pool * pool), (pool, pool, s.Cin, s.Cout)))
    dy = rng.standard_normal((s.N, s.Ho, s.Wo, s.Cout)).astype(np.float32)
    run = G.LayerRun(s, K)
    y = run.forward(x, w, gamma, beta)
    y_ref, saved = o.layer_forward(x, w, gamma, beta, K, oshape(o, s))
    assert run.packed.cpu().numpy().tobytes() == saved.store.tobytes()
    assert rel(y, y_ref) < TOL

    def pooled(a):   # non-overlapping pool x pool average of an NHWC tensor, in fp64
        a = np.asarray(a, np.float64)
        return a.reshape(s.N, s.Ho, pool, s.Wo, pool, s.Cin).mean(axis=(2, 4))

    a2 = (x.astype(np.float64) - saved.mean) * saved.rstd * gamma + beta
    assert rel(y, pooled(np.maximum(a2, 0)) @ V.astype(np.float64)) < TOL
    dx, dw, dg, db = run.backward(dy, w)
    dx_ref, dw_ref, dg_ref, db_ref = o.layer_backward(saved, dy, w)
    assert rel(dx, dx_ref) < TOL and rel(dw, dw_ref) < TOL and rel(dg, dg_ref) < TOL and rel(db, db_ref) < TOL
    a3t = np.maximum(o.recover_a2(saved), 0)
    dV = np.einsum("nhwc,nhwk->ck", pooled(a3t), dy.astype(np.float64))
    assert rel(dw.astype(np.float64).sum(axis=(0, 1)) / (pool * pool), dV) < TOL


@pytest.mark.parametrize("N,H,W,Cin,Cout", [
    (1, 1, 1, 64, 16), (3, 5, 7, 128, 48), (2, 9, 9, 192, 96), (5, 6, 6, 256, 320), (1, 13, 11, 384, 64),
    (2, 8, 8, 512, 272), (7, 3, 3, 1024, 128), (1, 40, 40, 64, 64), (4, 17, 5, 640, 192), (2, 5, 5, 320, 64),
    (1, 67, 126, 512, 256), (1, 67, 126, 256, 512),
    (4, 77, 77, 512, 128), (3, 125, 125, 64, 512), (57, 14, 13, 512, 256), (2, 100, 60, 512, 512)],
    ids=lambda v: str(v))
def test_pointwise_convolutions(G, oracle, N, H, W, Cin, Cout):
    """1x1 stride-1 layers through the kernel that loads activations straight into MFMA layout:
    contractions held whole in LDS (up to 256 channels, four- and eight-wave blocks) and in 64- or
    128-channel chunks, one to four 16-channel tiles per wave, pixel counts that leave ragged
    tiles and idle blocks; the two largest cases have enough pixels (8442, not a multiple of 16)
    for the grid of whole rounds plus row groups split over the contraction, forward (512 -> 256)
    and data gradient (256 -> 512).  The last four have contractions of 512 channels and at least 224
    blocks of 208 rows (or whole images) x 64 output channels: the kernel that keeps the output tile
    in registers - forward only, data gradient only (with its Eq. 6-7 sums in the layer call),
    whole images per block, and both directions."""
    o = oracle
    s = LayerShape(N, H, W, Cin, Cout, 1, 1, 1, 0)
    print("case pointwise", s.as_tuple(), flush=True)
    x, w, gamma, beta, dy = synth.draw_layer(s, 17, "normal", "random")
    a3 = np.maximum(x, np.float32(0))
    skip = np.random.default_rng(3).standard_normal(G.out_shape(s)).astype(np.float32)
    y_ref = o.conv_fwd(a3, w, oshape(o, s))
    assert rel(G.run_conv_fwd(s, a3, w), y_ref) < TOL
    assert rel(G.run_conv_fwd(s, a3, w, skip=skip), y_ref + skip) < TOL
    assert rel(G.run_conv_dgrad(s, dy, w), o.conv_dgrad(dy, w, oshape(o, s))) < TOL
    # the whole layer (fused prologue where the output has at most 256 channels; sums epilogues)
    for K in (4, 8):
        run = G.LayerRun(s, K)
        y = run.forward(x, w, gamma, beta)
        yl_ref, saved = o.layer_forward(x, w, gamma, beta, K, oshape(o, s))
        assert run.packed.cpu().numpy().tobytes() == saved.store.tobytes()
        assert rel(y, yl_ref) < TOL
        dx, dw, dg, db = run.backward(dy, w)
        dx_ref, dw_ref, dg_ref, db_ref = o.layer_backward(saved, dy, w)
        assert rel(dx, dx_ref) < TOL and rel(dw, dw_ref) < TOL
        assert rel(dg, dg_ref) < TOL and rel(db, db_ref) < TOL
