"""GPU parity for what the library adds beyond the paper's unit-stride, odd-k, bare convolution:
strides, the bias / rectifier epilogue of the fused kernels, and the 1 x 1 entry point.  Same
bounds as the main parity tests; the oracle's strided sum is pinned against the subsampled
unit-stride result and a hand-worked example."""
import numpy as np
import pytest

import oracle
from paper_1704_04428_amd import binding as B
from paper_1704_04428_amd import workloads as wl

from gpu_util import TOL_BF16, TOL_F32, announce, assert_within_bound, run_variant

pytestmark = pytest.mark.gpu

ALL = [("kn2row", B.KN2ROW), ("kn2row_2pass", B.KN2ROW_2PASS), ("im2col", B.IM2COL), ("direct", B.DIRECT),
       ("kn2col", B.KN2COL), ("im2row", B.IM2ROW)]

# (n, c, h, w, m, k, pad, stride): channel counts the channels-last variants take; odd and even
# extents, so the last output row / column sits on and off the last input row / column
STRIDED = [
    (1, 16, 32, 32, 16, 3, 1, 2),
    (2, 20, 17, 19, 35, 3, 1, 2),
    (1, 8, 30, 61, 7, 5, 2, 2),
    (1, 36, 15, 16, 18, 1, 0, 2),
    (1, 8, 41, 40, 9, 7, 3, 2),
    (2, 12, 29, 43, 70, 2, 0, 2),
    (1, 4, 9, 9, 5, 3, 0, 2),
    (1, 4, 6, 7, 5, 3, 2, 2),
    (1, 24, 57, 59, 40, 4, 1, 2),
    (1, 8, 33, 35, 24, 6, 2, 2),
    (1, 4, 2, 2, 3, 1, 0, 2),            # one output
]


def _inputs(case, seed):
    n, c, h, w, m, k = case[:6]
    I = wl.uniform(seed, n * c * h * w, -1, 1).reshape(n, c, h, w)
    K = wl.normal(seed + 1, m * c * k * k, 0.5).reshape(m, c, k, k)
    return I, K


@pytest.mark.parametrize("name,variant", ALL)
@pytest.mark.parametrize("case", STRIDED)
def test_stride_two_matches_oracle(name, variant, case):
    announce("stride2", name, case)
    I, K = _inputs(case, 3000 + sum(case))
    pad, stride = case[6], case[7]
    ref, absref = oracle.mcmk(I, K, pad, stride)
    got = run_variant(variant, I, K, pad, stride=stride)
    assert got.shape == ref.shape
    assert_within_bound(got, ref, absref, TOL_F32, f"{name} {case}")


@pytest.mark.parametrize("name,variant", [("kn2row", B.KN2ROW), ("kn2col", B.KN2COL), ("im2col", B.IM2COL), ("im2row", B.IM2ROW),
                                          ("kn2row_2pass", B.KN2ROW_2PASS)])
@pytest.mark.parametrize("case", [(2, 40, 30, 33, 35, 3, 1, 2), (1, 64, 31, 29, 20, 5, 2, 2), (1, 32, 35, 30, 17, 7, 3, 2)])
def test_stride_two_bf16(name, variant, case):
    announce("stride2-bf16", name, case)
    I, K = _inputs(case, 3100 + sum(case))
    pad, stride = case[6], case[7]
    ref, absref = oracle.mcmk(I, K, pad, stride)
    got = run_variant(variant, I, K, pad, dtype=B.BF16, stride=stride)
    assert_within_bound(got, ref, absref, TOL_BF16, f"{name} bf16 {case}")


@pytest.mark.parametrize("name,variant", [a for a in ALL if a[1] not in (B.KN2ROW, B.KN2COL)])
@pytest.mark.parametrize("case", [(1, 8, 20, 23, 6, 3, 1, 3), (2, 4, 25, 19, 9, 5, 0, 4), (1, 12, 11, 11, 5, 2, 1, 5)])
def test_larger_strides_on_the_staged_variants(name, variant, case):
    announce("stride>2", name, case)
    I, K = _inputs(case, 3200 + sum(case))
    pad, stride = case[6], case[7]
    ref, absref = oracle.mcmk(I, K, pad, stride)
    got = run_variant(variant, I, K, pad, stride=stride)
    assert got.shape == ref.shape
    assert_within_bound(got, ref, absref, TOL_F32, f"{name} {case}")


@pytest.mark.parametrize("name,variant", ALL)
def test_strided_integer_data_is_bit_exact(name, variant):
    n, c, h, w, m, k, pad, stride = 2, 20, 31, 33, 35, 3, 1, 2
    announce("stride2 exact-int", name)
    I = wl.small_integers(41, n * c * h * w, 0, 8).reshape(n, c, h, w)
    K = wl.small_integers(42, m * c * k * k, -4, 4).reshape(m, c, k, k)
    ref, _ = oracle.mcmk(I, K, pad, stride)
    got = run_variant(variant, I, K, pad, stride=stride)
    np.testing.assert_array_equal(got.astype(np.float64), ref)


@pytest.mark.parametrize("dtype", [B.F32, B.BF16])
@pytest.mark.parametrize("k,pad", [(1, 0), (2, 0), (3, 1), (4, 2), (5, 2), (6, 2), (7, 3)])
def test_every_strided_tile_shape(k, pad, dtype, monkeypatch):
    """Force each menu entry; the strided kernels exist for the first three shapes (x channel split
    1 and 2), any other index falls back to the selector's own choice."""
    case = (2, 72, 37, 30, 80, k, pad, 2)
    n, c, h, w, m = case[:5]
    I, K = _inputs(case, 3300 + k)
    ref, absref = oracle.mcmk(I, K, pad, 2)
    tol = TOL_BF16 if dtype == B.BF16 else TOL_F32
    for index in (0, 1, 2, 3, 6, 7, 8, 9):
        for variant in (B.KN2ROW, B.KN2COL):
            announce("strided menu", "k", k, "dtype", dtype, "tile", index, "variant", variant)
            B.conv_mcmk_force_tile(index)
            got = run_variant(variant, I, K, pad, dtype=dtype, stride=2)
            assert_within_bound(got, ref, absref, tol, f"strided tile {index} k={k} dtype={dtype} variant={variant}")
    B.conv_mcmk_force_tile(-1)


# ------------------------------------------------------------------ bias / rectifier epilogue

@pytest.mark.parametrize("variant", [B.KN2ROW, B.KN2COL])
@pytest.mark.parametrize("dtype", [B.F32, B.BF16])
@pytest.mark.parametrize("case", [(2, 24, 17, 19, 35, 3, 1, 1), (1, 16, 30, 31, 20, 5, 2, 2), (1, 40, 14, 14, 33, 1, 0, 1),
                                  (2, 512, 14, 14, 64, 3, 1, 1),           # a shape whose plain call splits the channels
                                  (2, 3, 30, 31, 20, 3, 1, 1), (1, 4, 40, 33, 24, 7, 3, 2)])   # few channels: one channel quad
def test_bias_and_rectifier_epilogue(variant, dtype, case):
    if B.conv_mcmk_check(B.desc(*case[:7], case[7], dtype), variant) == B.ERR_UNSUPPORTED:
        pytest.skip("channels-last variants need C to be a multiple of 4 (fp32) or 8 (bf16)")
    announce("epilogue", variant, dtype, case)
    I, K = _inputs(case, 3400 + sum(case))
    m, pad, stride = case[4], case[6], case[7]
    bias = wl.uniform(3499, m, -0.5, 0.5)
    ref, absref = oracle.mcmk(I, K, pad, stride)
    tol = TOL_BF16 if dtype == B.BF16 else TOL_F32
    for b, relu in ((bias, True), (bias, False), (None, True), (None, False)):
        want = oracle.bias_relu(ref, b, relu)
        # the rectifier never widens an error; the bias adds one rounding of a value of size |sum| + |bias|
        bound = absref + (np.abs(b).reshape(1, -1, 1, 1) if b is not None else 0.0)
        got = run_variant(variant, I, K, pad, dtype=dtype, stride=stride, epilogue=(b, relu))
        assert_within_bound(got, want, bound, tol, f"epilogue bias={b is not None} relu={relu} {case}")
        if relu:
            assert got.min() >= 0.0 and (got == 0.0).any() and (got > 0.0).any()


def test_epilogue_on_integer_data_is_bit_exact(monkeypatch):
    n, c, h, w, m, k, pad = 2, 20, 17, 19, 35, 3, 1
    I = wl.small_integers(51, n * c * h * w, 0, 8).reshape(n, c, h, w)
    K = wl.small_integers(52, m * c * k * k, -4, 4).reshape(m, c, k, k)
    bias = wl.small_integers(53, m, -100, 100)
    ref, _ = oracle.mcmk(I, K, pad)
    want = oracle.bias_relu(ref, bias, True)
    for index in (None, 0, 2, 5, 6, 7, 13):          # 7 and 13 ask for a channel split, which the epilogue must refuse to use
        announce("epilogue exact-int", "tile", index)
        if index is None:
            B.conv_mcmk_force_tile(-1)
        else:
            B.conv_mcmk_force_tile(index)
        for variant in (B.KN2ROW, B.KN2COL):
            got = run_variant(variant, I, K, pad, epilogue=(bias, True))
            np.testing.assert_array_equal(got.astype(np.float64), want)
    B.conv_mcmk_force_tile(-1)


# ------------------------------------------------------------------ the 1 x 1 entry point (section III-A's building block)

@pytest.mark.parametrize("dtype", [B.F32, B.BF16])
@pytest.mark.parametrize("case", [(1, 33, 15, 15, 18, 1, 0, 1), (3, 64, 28, 28, 70, 1, 0, 1), (1, 8, 3, 500, 16, 1, 0, 1),
                                  (2, 20, 9, 11, 5, 1, 1, 1), (2, 20, 9, 11, 5, 1, 0, 2), (1, 1, 1, 1, 1, 1, 0, 1)])
def test_one_by_one_entry_point(dtype, case):
    announce("1x1", dtype, case)
    if dtype == B.BF16 and case[2] * case[3] < 2:
        assert B.conv_mcmk_check(B.desc(*case[:7], case[7], dtype), B.KN2ROW) == B.ERR_UNSUPPORTED
        pytest.skip("[C][H][W] bf16 input needs at least two elements per plane")
    I, K = _inputs(case, 3500 + sum(case))
    pad, stride = case[6], case[7]
    ref, absref = oracle.mcmk(I, K, pad, stride)
    got = run_variant(B.KN2ROW, I, K, pad, dtype=dtype, stride=stride, one_by_one=True)
    assert_within_bound(got, ref, absref, TOL_BF16 if dtype == B.BF16 else TOL_F32, f"1x1 {case}")
    if pad == 0 and stride == 1:
        # Without padding the result is the matrix product itself (section III-A)
        n, c, h, w, m = case[:5]
        if dtype == B.F32:
            prod = np.einsum("mc,ncp->nmp", K.reshape(m, c).astype(np.float64), I.reshape(n, c, h * w).astype(np.float64))
            assert_within_bound(got.reshape(n, m, h * w), prod, absref.reshape(n, m, h * w), TOL_F32, "1x1 as a product")


@pytest.mark.parametrize("variant", [B.KN2ROW, B.KN2COL], ids=["kn2row", "kn2col"])
@pytest.mark.parametrize("dtype,case", [(B.F32, (8, 48, 40, 40, 256, 1, 0, 1)), (B.F32, (8, 128, 50, 30, 500, 1, 0, 1)), (B.F32, (8, 128, 51, 29, 500, 1, 0, 1)),
                                        (B.BF16, (8, 256, 40, 40, 512, 1, 0, 1))])
def test_one_by_one_layers_run_as_a_plain_product(dtype, case, variant):
    """Large 1 x 1 layers without padding or stride, [C][H][W] input: the fused call runs on the flat tile shape over
    the flattened plane, and the plan text says so (channels last: the 2-D tiles, same checks).  Plain, with the
    epilogue, and on exact integer data."""
    announce("1x1 as a product", dtype, case, variant)
    n, c, h, w, m = case[:5]
    plan = B.conv_mcmk_describe_plan(B.desc(*case[:7], case[7], dtype), variant)
    assert ("flattened plane" in plan) == (variant == B.KN2ROW), plan
    I, K = _inputs(case, 3600 + sum(case))
    ref, absref = oracle.mcmk(I, K, 0)
    tol = TOL_BF16 if dtype == B.BF16 else TOL_F32
    assert_within_bound(run_variant(variant, I, K, 0, dtype=dtype), ref, absref, tol, f"1x1 product {case}")
    if variant == B.KN2ROW:
        assert_within_bound(run_variant(variant, I, K, 0, dtype=dtype, one_by_one=True), ref, absref, tol, f"1x1 entry {case}")
    bias = wl.uniform(3699, m, -0.5, 0.5)
    got = run_variant(variant, I, K, 0, dtype=dtype, epilogue=(bias, True))
    assert_within_bound(got, oracle.bias_relu(ref, bias, True), absref + np.abs(bias).reshape(1, -1, 1, 1), tol, f"1x1 product + epilogue {case}")
    assert got.min() >= 0.0 and (got == 0.0).any() and (got > 0.0).any()
    Ii = wl.small_integers(3601, n * c * h * w, 0, 8).reshape(n, c, h, w)
    Ki = wl.small_integers(3602, m * c, -4, 4).reshape(m, c, 1, 1)
    np.testing.assert_array_equal(run_variant(variant, Ii, Ki, 0, dtype=dtype).astype(np.float64), oracle.mcmk(Ii, Ki, 0)[0])


def test_one_by_one_entry_point_refuses_larger_kernels():
    import torch
    d = B.desc(1, 4, 8, 8, 4, 3, 1)
    buf = torch.zeros(4096, device="cuda")
    with pytest.raises(B.ConvMcmkError) as e:
        B.conv_mcmk_1x1(d, buf, buf, buf)
    assert e.value.code == B.ERR_UNSUPPORTED


# ------------------------------------------------------------------ per-layer choice among the algorithms

@pytest.mark.parametrize("case", [
    (1, 3, 227, 227, 96, 11, 0, 4),      # first-layer-like: outside the fused kernels
    (1, 64, 30, 30, 64, 9, 4, 1),
    (1, 32, 28, 28, 96, 5, 2, 1),
    (2, 128, 28, 28, 128, 3, 1, 1),
    (1, 16, 32, 32, 16, 3, 1, 1),
    (1, 8, 64, 64, 8, 8, 4, 3),
    (2, 3, 224, 224, 64, 7, 3, 2),       # an RGB first layer, 7 x 7 with stride 2: the one-channel-quad kernels
    (2, 3, 112, 112, 32, 3, 1, 1),
])
def test_selected_variant_is_correct(case):
    """conv_mcmk_select + Plan.auto: the chosen variant runs and gives the oracle's result.  (How close the choice
    is to the fastest variant is a timing question: the `selector` entry of bench.py's output reports it.)"""
    import torch
    announce("select", case)
    n, c, h, w, m, k, pad, stride = case
    I, K = _inputs(case, 3600 + sum(case))
    ref, absref = oracle.mcmk(I, K, pad, stride)
    d = B.desc(n, c, h, w, m, k, pad, stride)
    I_dev, K_dev = torch.from_numpy(I).cuda(), torch.from_numpy(K).cuda()
    chosen, est = B.conv_mcmk_select(d)
    assert est > 0
    plan = B.Plan.auto(d, K_dev)
    assert plan.variant == chosen
    got = plan.run(I_dev).cpu().numpy()
    assert_within_bound(got, ref, absref, TOL_F32, f"selected variant {chosen} {case}")
    # every other variant that takes the layer agrees with the oracle too, so the choice is a matter of time only
    for variant in (B.KN2ROW, B.KN2ROW_2PASS, B.IM2COL, B.DIRECT):
        if variant != chosen and B.conv_mcmk_check(d, variant) == B.OK:
            got = B.Plan(d, variant, K_dev).run(I_dev).cpu().numpy()
            assert_within_bound(got, ref, absref, TOL_F32, f"variant {variant} {case}")


# ------------------------------------------------------------------ the one-call form of the binding

def test_one_call_form():
    import torch
    case = (2, 24, 19, 21, 20, 3, 1, 1)
    I, K = _inputs(case, 3700)
    bias = wl.uniform(3701, case[4], -0.5, 0.5)
    ref, absref = oracle.mcmk(I, K, 1)
    ref2, absref2 = oracle.mcmk(I, K, 1, 2)
    I_dev, K_dev = torch.from_numpy(I).cuda(), torch.from_numpy(K).cuda()
    announce("one-call")
    got = B.conv_mcmk(I_dev, K_dev, pad=1).cpu().numpy()
    assert_within_bound(got, ref, absref, TOL_F32, "auto")
    for name, variant in ALL:
        cl = variant in B.CHANNELS_LAST
        x = I_dev.permute(0, 2, 3, 1).contiguous() if cl else I_dev
        got = B.conv_mcmk(x, K_dev, pad=1, stride=2, variant=variant, channels_last=cl)
        got = (got.permute(0, 3, 1, 2) if cl else got).cpu().numpy()
        assert_within_bound(got, ref2, absref2, TOL_F32, f"one-call {name} stride 2")
    got = B.conv_mcmk(I_dev, K_dev, pad=1, bias=torch.from_numpy(bias).cuda(), relu=True).cpu().numpy()
    assert_within_bound(got, oracle.bias_relu(ref, bias, True), absref + np.abs(bias).reshape(1, -1, 1, 1), TOL_F32, "epilogue")
    got = B.conv_mcmk(I_dev, K_dev, pad=1, bf16=True).cpu().numpy()
    assert_within_bound(got, ref, absref, TOL_BF16, "bf16")
    with pytest.raises(ValueError):
        B.conv_mcmk(I_dev, K_dev, pad=1, variant=B.KN2COL)                      # layout and variant disagree
    with pytest.raises(ValueError):
        B.conv_mcmk(I_dev, K_dev, pad=1, variant=B.IM2COL, relu=True)
