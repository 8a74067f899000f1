"""GPU parity for bfloat16 operands (fp32 accumulation), through the C ABI.

Two bounds per case: against the oracle on the un-rounded fp32 inputs, |err| <= 1e-2 * sum|K||I|
(each product carries at most 2 * 2^-9 relative rounding error from the two bf16 roundings); and
against the oracle fed the inputs rounded to bf16 by the oracle's own rounding routine, the fp32
bound 1e-4 * sum|K||I|, because products of two bf16 values are exact in fp32 and only the
accumulation order differs.
"""
import numpy as np
import pytest

import oracle
from oracle import steps
from paper_1704_04428_amd import binding as B
from paper_1704_04428_amd import workloads as wl

from gpu_util import TOL_BF16, TOL_F32, announce, assert_within_bound, run_variant

pytestmark = pytest.mark.gpu

MFMA = [("kn2row", B.KN2ROW), ("kn2row_2pass", B.KN2ROW_2PASS), ("im2col", B.IM2COL)]
KN2COL_CASES = [           # channels-last bf16 needs C % 8 == 0
    (1, 16, 32, 32, 16, 3, 1), (2, 24, 17, 19, 35, 3, 1), (1, 40, 30, 9, 7, 5, 2), (1, 8, 15, 15, 18, 1, 0),
    (1, 72, 20, 21, 9, 7, 3), (2, 64, 28, 28, 48, 5, 2),
]

CASES = [
    (1, 16, 32, 32, 16, 3, 1),
    (2, 20, 17, 19, 35, 3, 1),     # channels not a multiple of 32, rows not of 16, ragged tiles
    (1, 40, 30, 9, 7, 5, 2),
    (1, 33, 15, 15, 18, 1, 0),
    (1, 7, 20, 21, 9, 7, 3),
    (3, 70, 29, 43, 70, 3, 1),
    (1, 4, 9, 9, 5, 3, 0),
    (1, 4, 6, 7, 5, 3, 2),
    (1, 1, 1, 2, 1, 1, 0),         # the smallest plane the [C][H][W] bf16 path takes: two elements
    (1, 3, 2, 1, 2, 1, 0),         # one column: every pair of columns has a single valid element
    (1, 5, 1, 7, 3, 3, 1),         # one row, odd width
    (2, 9, 5, 3, 4, 2, 1),         # even kernel side: odd tile width, the last pair has one column
    (2, 64, 28, 28, 48, 5, 2),
]


def _inputs(case, seed):
    n, c, h, w, m, k, pad = case
    I = wl.uniform(seed, n * c * h * w, -1, 1).reshape(n, c, h, w)
    K = wl.normal(seed + 1, m * c * k * k, 0.5).reshape(m, c, k, k)
    return I, K


@pytest.mark.parametrize("name,variant", MFMA)
@pytest.mark.parametrize("case", CASES)
def test_bf16_matches_oracle(name, variant, case):
    announce("bf16", name, case)
    I, K = _inputs(case, 3000 + sum(case))
    pad = case[-1]
    got = run_variant(variant, I, K, pad, dtype=B.BF16)
    ref, absref = oracle.mcmk(I, K, pad)
    assert_within_bound(got, ref, absref, TOL_BF16, f"bf16 {name} {case} vs fp32 inputs")
    Ir, Kr = steps.round_to_bf16(I), steps.round_to_bf16(K)
    ref_r, abs_r = oracle.mcmk(Ir, Kr, pad)
    assert_within_bound(got, ref_r, abs_r, TOL_F32, f"bf16 {name} {case} vs rounded inputs")


def test_bf16_single_element_plane_is_refused():
    """[C][H][W] bf16 input is staged two positions at a time; H*W = 1 is left to fp32 or channels last."""
    with pytest.raises(B.ConvMcmkError) as e:
        run_variant(B.KN2ROW, np.ones((1, 8, 1, 1), np.float32), np.ones((4, 8, 1, 1), np.float32), 0, dtype=B.BF16)
    assert e.value.code == B.ERR_UNSUPPORTED
    got = run_variant(B.KN2COL, np.ones((1, 8, 1, 1), np.float32), np.ones((4, 8, 1, 1), np.float32), 0, dtype=B.BF16)
    np.testing.assert_array_equal(got, np.full((1, 4, 1, 1), 8.0, np.float32))


@pytest.mark.parametrize("variant", [B.KN2COL, B.IM2ROW])
@pytest.mark.parametrize("case", KN2COL_CASES)
def test_bf16_channels_last_matches_oracle(case, variant):
    announce("bf16 channels-last", variant, case)
    I, K = _inputs(case, 3500 + sum(case))
    pad = case[-1]
    got = run_variant(variant, I, K, pad, dtype=B.BF16)
    ref, absref = oracle.mcmk(I, K, pad)
    assert_within_bound(got, ref, absref, TOL_BF16, f"bf16 kn2col {case} vs fp32 inputs")
    ref_r, abs_r = oracle.mcmk(steps.round_to_bf16(I), steps.round_to_bf16(K), pad)
    assert_within_bound(got, ref_r, abs_r, TOL_F32, f"bf16 kn2col {case} vs rounded inputs")


@pytest.mark.parametrize("name,variant", MFMA + [("kn2col", B.KN2COL), ("im2row", B.IM2ROW)])
def test_bf16_integer_data_is_bit_exact(name, variant):
    case = (2, 40, 17, 19, 35, 3, 1)
    announce("bf16 exact-int", name, case)
    n, c, h, w, m, k, pad = case
    I = wl.small_integers(41, n * c * h * w, 0, 8).reshape(n, c, h, w)
    K = wl.small_integers(42, m * c * k * k, -4, 4).reshape(m, c, k, k)
    ref, _ = oracle.mcmk(I, K, pad)
    got = run_variant(variant, I, K, pad, dtype=B.BF16)
    np.testing.assert_array_equal(got.astype(np.float64), ref)


def _expected_packing_bf16(K, im2col):
    """The bf16 packed-kernel layout documented in conv_mcmk.h, written out with plain loops."""
    m, c, k, _ = K.shape
    mb = (m + 15) // 16
    if im2col:
        A = K.reshape(1, m, c * k * k)
    else:
        A = np.stack([K[:, :, i, j] for i in range(k) for j in range(k)])
    taps, _, kc = A.shape
    cg = (kc + 31) // 32
    bits = steps.round_to_bf16_bits(A).reshape(A.shape)
    out = np.zeros((taps, mb, cg, 64, 8), dtype=np.uint16)
    for t in range(taps):
        for row in range(m):
            for col in range(kc):
                lane = ((col % 32) // 8) * 16 + row % 16
                out[t, row // 16, col // 32, lane, col % 8] = bits[t, row, col]
    return out


@pytest.mark.parametrize("variant", [B.KN2ROW, B.IM2COL])
def test_bf16_prepack_layout(variant):
    import torch
    m, c, k = 35, 45, 3
    announce("bf16 prepack", variant)
    K = wl.normal(9, m * c * k * k, 1.0).reshape(m, c, k, k)
    d = B.desc(1, c, 8, 8, m, k, 1, 1, B.BF16)
    nbytes = B.conv_mcmk_packed_kernel_bytes(d, variant)
    Kp = torch.full((nbytes,), 0xFF, dtype=torch.uint8, device="cuda")
    B.conv_mcmk_prepack(d, variant, torch.from_numpy(K).cuda(), Kp)
    torch.cuda.synchronize()
    got = Kp.cpu().numpy().view(np.uint16)
    want = _expected_packing_bf16(K, variant == B.IM2COL).reshape(-1)
    assert got.size == want.size
    np.testing.assert_array_equal(got, want)


def test_bf16_im2col_workspace_holds_the_rounded_patch_matrix():
    case = (2, 6, 9, 13, 10, 3, 1)
    announce("bf16 im2col-workspace", case)
    n, c, h, w, m, k, pad = case
    I, K = _inputs(case, 4343)
    _, ws = run_variant(B.IM2COL, I, K, pad, dtype=B.BF16, return_ws=True)
    cols = ws.view(np.uint16).reshape(n, c * k * k, h * w)
    for i in range(n):
        want = steps.round_to_bf16_bits(steps.input_patch_matrix(I[i], k, pad).astype(np.float32))
        np.testing.assert_array_equal(cols[i], want.reshape(cols[i].shape))


@pytest.mark.parametrize("name,variant", MFMA + [("kn2col", B.KN2COL), ("im2row", B.IM2ROW)])
@pytest.mark.parametrize("layer", ["cfg5a_vgg_deep56", "cfg5b_vgg_deep28", "cfg5c_vgg_deep14"])
def test_bf16_full_size_sampled(layer, name, variant):
    L = wl.LAYERS[layer]
    announce("bf16 sampled", layer, name)
    I, K = wl.make_input(L), wl.make_kernel(L)
    pts = wl.sample_points(L, 2000)
    got = run_variant(variant, I, K, L.pad, dtype=B.BF16)
    assert np.all(np.isfinite(got))
    sampled = got[pts[:, 0], pts[:, 1], pts[:, 2], pts[:, 3]]
    ref, absref = oracle.mcmk_at(I, K, L.pad, pts)
    assert_within_bound(sampled, ref, absref, TOL_BF16, f"bf16 {name} {layer} vs fp32 inputs")
    ref_r, abs_r = oracle.mcmk_at(steps.round_to_bf16(I), steps.round_to_bf16(K), L.pad, pts)
    assert_within_bound(sampled, ref_r, abs_r, TOL_F32, f"bf16 {name} {layer} vs rounded inputs")
