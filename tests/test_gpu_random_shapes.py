"""A seeded sweep of random small shapes through every variant and both operand types: shapes no
one thought of (single rows, kernels larger than the image with padding, one channel, M not a
multiple of anything), checked against the oracle under the stated bounds."""
import numpy as np
import pytest

import oracle
from paper_1704_04428_amd import binding as B
from paper_1704_04428_amd import workloads as wl

from gpu_util import TOL_BF16, TOL_F32, announce, assert_within_bound, run_variant

pytestmark = pytest.mark.gpu

VARIANTS = [("kn2row", B.KN2ROW), ("kn2row_2pass", B.KN2ROW_2PASS), ("im2col", B.IM2COL), ("direct", B.DIRECT),
            ("kn2col", B.KN2COL), ("im2row", B.IM2ROW)]


def _random_cases(count, seed):
    r = wl.splitmix64(seed, np.arange(count * 8)).reshape(count, 8)
    cases = []
    for row in r:
        v = [int(x % 1000003) for x in row]
        k = (1, 3, 5, 7, 2, 4)[v[0] % 6]
        pad = v[1] % k
        n = 1 + v[2] % 3
        c = 1 + v[3] % 70
        if v[7] % 2:
            c = 4 * (1 + c // 4)            # every other case is eligible for the channels-last variants
        h = max(1, k - 2 * pad) + v[4] % 36
        w = max(1, k - 2 * pad) + v[5] % 36
        m = 1 + v[6] % 90
        cases.append((n, c, h, w, m, k, pad))
    return cases


CASES = _random_cases(48, 20240611)


@pytest.mark.parametrize("case", CASES)
def test_random_shape(case):
    n, c, h, w, m, k, pad = case
    I = wl.uniform(sum(case), n * c * h * w, -1, 1).reshape(n, c, h, w)
    K = wl.normal(sum(case) + 1, m * c * k * k, 0.5).reshape(m, c, k, k)
    ref, absref = oracle.mcmk(I, K, pad)
    ran = 0
    for dtype, tol in ((B.F32, TOL_F32), (B.BF16, TOL_BF16)):
        for name, variant in VARIANTS:
            d = B.desc(n, c, h, w, m, k, pad, 1, dtype)
            rc = B.conv_mcmk_check(d, variant)
            if rc == B.ERR_UNSUPPORTED:
                continue                      # even k in the fused kernels, channel vectors, bf16 direct
            assert rc == B.OK, (case, name, dtype, rc)
            announce("random", case, name, "bf16" if dtype else "f32")
            got = run_variant(variant, I, K, pad, dtype=dtype)
            assert got.shape == ref.shape
            assert_within_bound(got, ref, absref, tol, f"{name} dtype={dtype} {case}")
            ran += 1
    assert ran >= 3          # the two staged variants and direct take every shape


def _random_strided_cases(count, seed):
    r = wl.splitmix64(seed, np.arange(count * 10)).reshape(count, 10)
    cases = []
    for row in r:
        v = [int(x % 1000003) for x in row]
        k = 1 + v[0] % 7
        pad = v[1] % k
        stride = 2 + v[8] % 2                 # 2 or 3 (the fused kernels refuse 3)
        n = 1 + v[2] % 2
        c = 1 + v[3] % 48
        if v[7] % 2:
            c = 8 * (1 + c // 8)              # eligible for the channels-last variants, bf16 included
        h = max(1, k - 2 * pad) + v[4] % 45
        w = max(1, k - 2 * pad) + v[5] % 45
        m = 1 + v[6] % 70
        cases.append((n, c, h, w, m, k, pad, stride, v[9] % 2 == 0))
    return cases


@pytest.mark.parametrize("case", _random_strided_cases(32, 20250314))
def test_random_strided_shape_with_epilogue(case):
    """Random shapes with a stride, every variant and operand type that takes them, and -- for the fused
    variants -- the same call through the bias / rectifier entry point."""
    n, c, h, w, m, k, pad, stride, relu = case
    I = wl.uniform(sum(case[:8]), n * c * h * w, -1, 1).reshape(n, c, h, w)
    K = wl.normal(sum(case[:8]) + 1, m * c * k * k, 0.5).reshape(m, c, k, k)
    bias = wl.uniform(sum(case[:8]) + 2, m, -1, 1)
    ref, absref = oracle.mcmk(I, K, pad, stride)
    want = oracle.bias_relu(ref, bias, relu)
    ran = 0
    for dtype, tol in ((B.F32, TOL_F32), (B.BF16, TOL_BF16)):
        for name, variant in VARIANTS:
            d = B.desc(n, c, h, w, m, k, pad, stride, dtype)
            rc = B.conv_mcmk_check(d, variant)
            if rc == B.ERR_UNSUPPORTED:
                continue
            assert rc == B.OK, (case, name, dtype, rc)
            announce("random strided", case, name, "bf16" if dtype else "f32")
            got = run_variant(variant, I, K, pad, dtype=dtype, stride=stride)
            assert got.shape == ref.shape
            assert_within_bound(got, ref, absref, tol, f"{name} dtype={dtype} {case}")
            ran += 1
            if variant in (B.KN2ROW, B.KN2COL):
                got = run_variant(variant, I, K, pad, dtype=dtype, stride=stride, epilogue=(bias, relu))
                assert_within_bound(got, want, absref + np.abs(bias).reshape(1, -1, 1, 1), tol, f"{name} epilogue dtype={dtype} {case}")
    assert ran >= 3


def test_large_tensors_sampled():
    """Indices beyond 2^31 bytes: a 1 GiB output and a 0.5 GiB two-pass workspace; sampled outputs."""
    L = wl.Layer("big", 1, 4, 2048, 2048, 64, 3, 1, "u11", "u11", 4711)
    announce("large", L)
    I, K = wl.make_input(L), wl.make_kernel(L)
    pts = wl.sample_points(L, 4000)
    pts[:8] = [(0, 63, 2047, 2047), (0, 63, 2047, 0), (0, 32, 1024, 1024), (0, 0, 0, 2047),
               (0, 63, 0, 0), (0, 1, 2046, 2046), (0, 62, 1, 1), (0, 31, 2047, 1023)]
    ref, absref = oracle.mcmk_at(I, K, L.pad, pts)
    for name, variant in (("kn2row", B.KN2ROW), ("kn2col", B.KN2COL), ("im2col", B.IM2COL)):
        got = run_variant(variant, I, K, L.pad)
        assert_within_bound(got[pts[:, 0], pts[:, 1], pts[:, 2], pts[:, 3]], ref, absref, TOL_F32, f"{name} large")
        del got
