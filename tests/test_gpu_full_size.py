"""The benchmark configurations at full size, in the launch configuration bench.py times: the whole
output of the fused kernels (kn2row, kn2col; fp32 and bf16 operands) against the oracle, element by
element, on every configuration; the staged variants whole on the small configurations and on sampled
outputs (which the oracle computes one by one) plus agreement with the fused kernel on the large ones."""
import functools

import numpy as np
import pytest

import oracle
from paper_1704_04428_amd import binding as B
from paper_1704_04428_amd import workloads as wl

from gpu_util import TOL_F32, announce, assert_within_bound, run_variant

pytestmark = pytest.mark.gpu

VARIANTS = [("kn2row", B.KN2ROW), ("kn2row_2pass", B.KN2ROW_2PASS), ("im2col", B.IM2COL), ("direct", B.DIRECT),
            ("kn2col", B.KN2COL), ("im2row", B.IM2ROW)]


@pytest.mark.parametrize("name,variant", VARIANTS)
@pytest.mark.parametrize("layer", ["cfg1_tiny", "cfg2_googlenet5x5", "cfg3_alexnet_conv2"])
def test_whole_output(layer, name, variant):
    L = wl.LAYERS[layer]
    announce("full", layer, name)
    I, K = wl.make_input(L), wl.make_kernel(L)
    ref, absref = oracle.mcmk(I, K, L.pad)
    got = run_variant(variant, I, K, L.pad)
    assert_within_bound(got, ref, absref, TOL_F32, f"{name} {layer}")


LARGE = ["cfg4_vgg_early", "cfg5a_vgg_deep56", "cfg5b_vgg_deep28", "cfg5c_vgg_deep14"]


@functools.lru_cache(maxsize=None)
def _whole_oracle(layer):
    """Inputs and the oracle's whole output of a large configuration (a few seconds on the host's cores), shared by
    the tests below."""
    L = wl.LAYERS[layer]
    I, K = wl.make_input(L), wl.make_kernel(L)
    ref, absref = oracle.mcmk(I, K, L.pad)
    return I, K, ref, absref


@pytest.mark.parametrize("dtype", [B.F32, B.BF16])
@pytest.mark.parametrize("name,variant", [("kn2row", B.KN2ROW), ("kn2col", B.KN2COL)])
@pytest.mark.parametrize("layer", LARGE)
def test_whole_output_of_the_fused_kernels_on_the_large_layers(layer, name, variant, dtype):
    """Every output element of the VGG-like layers, in the tile shape the selector picks for them (the one the
    benchmark times), within 1e-4 (fp32) / 1e-2 (bf16) of sum|K||I| of the oracle's value."""
    from gpu_util import TOL_BF16
    L = wl.LAYERS[layer]
    announce("whole", layer, name, "bf16" if dtype == B.BF16 else "f32")
    I, K, ref, absref = _whole_oracle(layer)
    got = run_variant(variant, I, K, L.pad, dtype=dtype)
    assert got.shape == (L.n, L.m, L.q, L.p)
    assert_within_bound(got, ref, absref, TOL_BF16 if dtype == B.BF16 else TOL_F32, f"{name} {layer} whole output")


@pytest.mark.parametrize("name,variant", VARIANTS)
@pytest.mark.parametrize("layer", LARGE)
def test_sampled_outputs(layer, name, variant):
    L = wl.LAYERS[layer]
    if variant == B.DIRECT and L.flops > 1e10:
        pytest.skip("the plain-ALU direct kernel is a comparison point for the small layers only")
    announce("sampled", layer, name)
    I, K = wl.make_input(L), wl.make_kernel(L)
    pts = wl.sample_points(L, 3000)
    ref, absref = oracle.mcmk_at(I, K, L.pad, pts)
    got = run_variant(variant, I, K, L.pad)
    assert np.all(np.isfinite(got))
    sampled = got[pts[:, 0], pts[:, 1], pts[:, 2], pts[:, 3]]
    assert_within_bound(sampled, ref, absref, TOL_F32, f"{name} {layer}")
    # every variant must agree with the fused kernel everywhere (any-size property)
    if variant != B.KN2ROW:
        fused = run_variant(B.KN2ROW, I, K, L.pad)
        scale = np.abs(fused).max()
        assert np.abs(got - fused).max() <= 2e-4 * max(scale, 1.0) * 4


@pytest.mark.parametrize("dtype", [B.F32, B.BF16])
@pytest.mark.parametrize("name,variant", [("kn2row", B.KN2ROW), ("kn2col", B.KN2COL), ("im2col", B.IM2COL)])
@pytest.mark.parametrize("layer", list(wl.GENERALISED_LAYERS))
def test_generalised_layers_sampled(layer, name, variant, dtype):
    """The deep VGG-like shape with stride 2, with an even kernel side and as a 1 x 1 layer, at the
    size bench.py times them: sampled outputs against the oracle."""
    from gpu_util import TOL_BF16
    L = wl.GENERALISED_LAYERS[layer]
    if B.conv_mcmk_check(B.desc(L.n, L.c, L.h, L.w, L.m, L.k, L.pad, L.stride, dtype), variant) == B.ERR_UNSUPPORTED:
        pytest.skip("channels-last variants need C to be a multiple of 4 (fp32) or 8 (bf16)")
    announce("generalised", layer, name, dtype)
    I, K = wl.make_input(L), wl.make_kernel(L)
    pts = wl.sample_points(L, 2000)
    ref, absref = oracle.mcmk_at(I, K, L.pad, pts, L.stride)
    got = run_variant(variant, I, K, L.pad, dtype=dtype, stride=L.stride)
    assert got.shape == (L.n, L.m, L.q, L.p)
    sampled = got[pts[:, 0], pts[:, 1], pts[:, 2], pts[:, 3]]
    assert_within_bound(sampled, ref, absref, TOL_BF16 if dtype == B.BF16 else TOL_F32, f"{name} {layer}")
    if layer == "gen_vgg56_1x1" and variant == B.KN2ROW:
        one = run_variant(B.KN2ROW, I, K, L.pad, dtype=dtype, one_by_one=True)
        sampled = one[pts[:, 0], pts[:, 1], pts[:, 2], pts[:, 3]]
        assert_within_bound(sampled, ref, absref, TOL_BF16 if dtype == B.BF16 else TOL_F32, f"1x1 entry {layer}")
