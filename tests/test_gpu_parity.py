"""GPU parity: every variant of the library, called through the C ABI, against the CPU oracle.

Bounds: fp32 operands |gpu - oracle| <= 1e-4 * sum|K||I| per output element (the oracle's second
output is that sum); data made of small integers must match bit for bit in any summation order.
"""
import numpy as np
import pytest

import oracle
from oracle import steps
from paper_1704_04428_amd import binding as B
from paper_1704_04428_amd import workloads as wl

from gpu_util import TOL_BF16, TOL_F32, Guarded, announce, assert_within_bound, run_variant

pytestmark = pytest.mark.gpu

ALL = [("kn2row", B.KN2ROW), ("kn2row_2pass", B.KN2ROW_2PASS), ("im2col", B.IM2COL), ("direct", B.DIRECT),
       ("kn2col", B.KN2COL), ("im2row", B.IM2ROW)]

# (n, c, h, w, m, k, pad): several tiles, ragged tails in every dimension, degenerate sizes
SMALL = [
    (1, 16, 32, 32, 16, 3, 1),     # the tiny benchmark shape
    (2, 20, 17, 19, 35, 3, 1),     # nothing a multiple of a tile
    (1, 5, 30, 9, 7, 5, 2),
    (1, 33, 15, 15, 18, 1, 0),     # 1x1: the plain GEMM of section III
    (1, 7, 20, 21, 9, 7, 3),
    (1, 3, 14, 14, 64, 3, 1),      # exactly one spatial tile, few channels (first-layer-like)
    (3, 17, 29, 43, 70, 3, 1),     # several row tiles
    (1, 4, 9, 9, 5, 3, 0),         # no padding: output smaller than input
    (1, 4, 6, 7, 5, 3, 2),         # padding k-1: output larger than input
    (1, 1, 1, 1, 1, 1, 0),         # a single product
    (1, 2, 3, 3, 2, 3, 1),
    (2, 40, 28, 28, 48, 5, 2),
]
EVEN_K = [(1, 6, 12, 13, 10, 2, 1), (2, 5, 11, 10, 20, 4, 1), (1, 3, 10, 10, 4, 6, 0)]


def _skip_unless_supported(variant, case, dtype=B.F32):
    """kn2col reads whole channel vectors (4 floats / 8 bf16); other channel counts are refused."""
    n, c, h, w, m, k, pad = case
    if B.conv_mcmk_check(B.desc(n, c, h, w, m, k, pad, 1, dtype), variant) == B.ERR_UNSUPPORTED:
        assert variant in B.CHANNELS_LAST and c % 4 != 0
        pytest.skip("the channels-last variants need a channel count that is a multiple of 4")


# channel counts kn2col accepts, otherwise as ragged as SMALL
KN2COL_CASES = [
    (2, 20, 17, 19, 35, 3, 1), (1, 4, 30, 9, 7, 5, 2), (1, 36, 15, 15, 18, 1, 0), (1, 8, 20, 21, 9, 7, 3),
    (3, 12, 29, 43, 70, 3, 1), (1, 4, 9, 9, 5, 3, 0), (1, 4, 6, 7, 5, 3, 2), (1, 4, 1, 1, 1, 1, 0), (2, 40, 28, 28, 49, 5, 2),
]


def _inputs(case, seed):
    n, c, h, w, m, k, pad = case
    I = wl.uniform(seed, n * c * h * w, -1, 1).reshape(n, c, h, w)
    K = wl.normal(seed + 1, m * c * k * k, 0.5).reshape(m, c, k, k)
    return I, K


@pytest.mark.parametrize("name,variant", ALL)
@pytest.mark.parametrize("case", SMALL)
def test_small_shapes_match_oracle(name, variant, case):
    _skip_unless_supported(variant, case)
    announce("small", name, case)
    I, K = _inputs(case, 1000 + sum(case))
    ref, absref = oracle.mcmk(I, K, case[-1])
    got = run_variant(variant, I, K, case[-1])
    assert got.shape == ref.shape
    assert_within_bound(got, ref, absref, TOL_F32, f"{name} {case}")


@pytest.mark.parametrize("name,variant", [("kn2col", B.KN2COL), ("im2row", B.IM2ROW)])
@pytest.mark.parametrize("case", KN2COL_CASES)
def test_channels_last_shapes_match_oracle(name, variant, case):
    announce(name, case)
    I, K = _inputs(case, 1500 + sum(case))
    ref, absref = oracle.mcmk(I, K, case[-1])
    got = run_variant(variant, I, K, case[-1])
    assert_within_bound(got, ref, absref, TOL_F32, f"{name} {case}")


@pytest.mark.parametrize("name,variant", ALL)
@pytest.mark.parametrize("case", EVEN_K + [(1, 8, 12, 13, 10, 2, 1), (2, 4, 11, 10, 20, 4, 1), (2, 24, 31, 33, 40, 6, 3)])
def test_even_kernel_sizes(name, variant, case):
    _skip_unless_supported(variant, case)
    announce("even-k", name, case)
    I, K = _inputs(case, 2000 + sum(case))
    ref, absref = oracle.mcmk(I, K, case[-1])
    got = run_variant(variant, I, K, case[-1])
    assert_within_bound(got, ref, absref, TOL_F32, f"{name} {case}")


@pytest.mark.parametrize("name,variant", ALL)
@pytest.mark.parametrize("case", [(2, 20, 17, 19, 35, 3, 1), (1, 24, 31, 16, 40, 5, 2), (1, 9, 15, 16, 33, 1, 0)])
def test_integer_data_is_bit_exact(name, variant, case):
    """Integer-valued inputs keep every partial sum below 2^24, so any summation order is exact."""
    _skip_unless_supported(variant, case)
    announce("exact-int", name, case)
    n, c, h, w, m, k, pad = case
    I = wl.small_integers(31, n * c * h * w, 0, 8).reshape(n, c, h, w)
    K = wl.small_integers(32, m * c * k * k, -4, 4).reshape(m, c, k, k)
    ref, _ = oracle.mcmk(I, K, pad)
    got = run_variant(variant, I, K, pad)
    np.testing.assert_array_equal(got.astype(np.float64), ref)


@pytest.mark.parametrize("name,variant", ALL)
def test_delta_kernels_shift_without_row_wrap(name, variant):
    """A single tap copies the input displaced by the tap's offset; values leaving a row are dropped
    (section III-A), including at tile borders."""
    c, h, w, k, pad = 4, 30, 17, 3, 1
    I = wl.uniform(77, c * h * w, -1, 1).reshape(1, c, h, w)
    K = np.zeros((k * k, c, k, k), dtype=np.float32)
    for i in range(k):
        for j in range(k):
            K[i * k + j, 1, i, j] = 1.0          # kernel t is the delta at tap t on channel 1
    announce("delta", name)
    got = run_variant(variant, I, K, pad)
    for i in range(k):
        for j in range(k):
            want = np.zeros((h, w), dtype=np.float32)
            di, dj = i - pad, j - pad
            q0, q1 = max(0, -di), min(h, h - di)
            p0, p1 = max(0, -dj), min(w, w - dj)
            want[q0:q1, p0:p1] = I[0, 1, q0 + di:q1 + di, p0 + dj:p1 + dj]
            np.testing.assert_array_equal(got[0, i * k + j], want)


def test_zero_terms_give_exact_zero():
    """Where sum|K||I| is 0 the result must be exactly 0."""
    announce("zeros")
    I = np.zeros((1, 4, 16, 16), dtype=np.float32)
    K = wl.normal(5, 8 * 4 * 9, 1.0).reshape(8, 4, 3, 3)
    for _, variant in ALL:
        assert not run_variant(variant, I, K, 1).any()


# ------------------------------------------------------------------ stage outputs

def _expected_packing(K, im2col):
    """The packed-kernel layout documented in conv_mcmk.h, written out with plain loops."""
    m, c, k, _ = K.shape
    mb = (m + 15) // 16
    if im2col:
        A = K.reshape(1, m, c * k * k)
    else:
        A = np.stack([K[:, :, i, j] for i in range(k) for j in range(k)])      # [t][m][c]
    taps, _, kc = A.shape
    cg = (kc + 15) // 16
    out = np.zeros((taps, mb, cg, 64, 4), dtype=np.float32)
    for t in range(taps):
        for row in range(m):
            for col in range(kc):
                lane = (col % 4) * 16 + row % 16
                out[t, row // 16, col // 16, lane, (col % 16) // 4] = A[t, row, col]
    return out


@pytest.mark.parametrize("variant", [B.KN2ROW, B.KN2ROW_2PASS, B.IM2COL, B.KN2COL, B.IM2ROW])
def test_prepack_layout(variant):
    import torch
    m, c, k = 35, 20, 3
    announce("prepack", variant)
    K = wl.normal(9, m * c * k * k, 1.0).reshape(m, c, k, k)
    d = B.desc(1, c, 8, 8, m, k, 1)
    nbytes = B.conv_mcmk_packed_kernel_bytes(d, variant)
    Kp = torch.full((nbytes,), 0xFF, dtype=torch.uint8, device="cuda")
    B.conv_mcmk_prepack(d, variant, torch.from_numpy(K).cuda(), Kp)
    torch.cuda.synchronize()
    got = Kp.view(torch.float32).cpu().numpy()
    if variant == B.IM2ROW:          # one row per kernel, contraction index ordered (i, j, c)
        want = _expected_packing(np.ascontiguousarray(K.transpose(0, 2, 3, 1)).reshape(m, k * k * c, 1, 1), True).reshape(-1)
    else:
        want = _expected_packing(K, variant == B.IM2COL).reshape(-1)
    assert got.size == want.size
    np.testing.assert_array_equal(got, want)


def test_two_pass_workspace_holds_the_gemm_result():
    """After the two-pass call the workspace is the [k*k*M] x [H*W] product of section III-A."""
    case = (2, 12, 13, 11, 21, 3, 1)
    announce("2pass-workspace", case)
    n, c, h, w, m, k, pad = case
    I, K = _inputs(case, 4242)
    O, ws = run_variant(B.KN2ROW_2PASS, I, K, pad, return_ws=True)
    T = ws.view(np.float32).reshape(n, k * k * m, h * w)
    for i in range(n):
        ref = steps.kn2row_gemm(I[i], K)
        absref = steps.kn2row_gemm(np.abs(I[i]), np.abs(K))
        assert_within_bound(T[i], ref, absref, TOL_F32, "kn2row GEMM result")
        # and the post pass applied to the library's own product gives the library's output
        again = steps.shift_add(T[i], m, h, w, k, pad)
        assert np.all(np.abs(again - O[i]) <= 1e-6 * steps.shift_add(np.abs(T[i]), m, h, w, k, pad) + 1e-30)


def test_im2col_workspace_holds_the_patch_matrix():
    case = (2, 6, 9, 13, 10, 3, 1)
    announce("im2col-workspace", case)
    n, c, h, w, m, k, pad = case
    I, K = _inputs(case, 4343)
    _, ws = run_variant(B.IM2COL, I, K, pad, return_ws=True)
    cols = ws.view(np.float32).reshape(n, c * k * k, h * w)
    for i in range(n):
        np.testing.assert_array_equal(cols[i], steps.input_patch_matrix(I[i], k, pad).astype(np.float32))


def test_im2row_workspace_holds_the_patch_rows():
    case = (2, 8, 9, 13, 10, 3, 1)
    announce("im2row-workspace", case)
    n, c, h, w, m, k, pad = case
    I, K = _inputs(case, 4444)
    _, ws = run_variant(B.IM2ROW, I, K, pad, return_ws=True)
    rows = ws.view(np.float32).reshape(n, h * w, k * k * c)
    for i in range(n):
        want = steps.input_patch_matrix_rows(np.ascontiguousarray(I[i].transpose(1, 2, 0)), k, pad)
        np.testing.assert_array_equal(rows[i], want.astype(np.float32))


def test_cvt_f32_bf16_bit_exact():
    import torch
    announce("cvt")
    x = np.concatenate([wl.normal(1, 100000, 1.0), wl.uniform(2, 1000, -1e-30, 1e-30),
                        np.array([0.0, -0.0, np.inf, -np.inf, np.nan, 1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8,
                                  3.3e38, 3.4e38, 1e-45], dtype=np.float32)]).astype(np.float32)
    src = torch.from_numpy(x).cuda()
    dst = torch.zeros(x.size, dtype=torch.int16, device="cuda")
    B.conv_mcmk_cvt_f32_bf16(src, dst)
    torch.cuda.synchronize()
    got = dst.cpu().numpy().view(np.uint16)
    np.testing.assert_array_equal(got, steps.round_to_bf16_bits(x))


def test_repeat_calls_are_bitwise_identical():
    """No atomics, no races: the same call twice gives the same bits."""
    case = (2, 40, 28, 28, 48, 3, 1)
    announce("repeat", case)
    I, K = _inputs(case, 555)
    a = run_variant(B.KN2ROW, I, K, 1)
    b = run_variant(B.KN2ROW, I, K, 1)
    np.testing.assert_array_equal(a, b)


def test_runtime_errors_through_binding():
    import torch
    announce("errors")
    d = B.desc(1, 4, 8, 8, 4, 3, 1)
    I = torch.zeros(4 * 64, device="cuda")
    K = torch.zeros(4 * 4 * 9, device="cuda")
    O = torch.zeros(4 * 64, device="cuda")
    with pytest.raises(B.ConvMcmkError) as e:
        B.conv_mcmk_im2col(d, I, K, O, None)
    assert e.value.code == B.ERR_WORKSPACE
    with pytest.raises(B.ConvMcmkError) as e:
        B.conv_mcmk_kn2row(B.desc(1, 4, 8, 8, 4, 3, 1, stride=3), I, K, O)
    assert e.value.code == B.ERR_UNSUPPORTED
    with pytest.raises(B.ConvMcmkError) as e:
        B.conv_mcmk_kn2row(d, I[1:], K, O)
    assert e.value.code == B.ERR_ALIGN


@pytest.mark.parametrize("dtype", [B.F32, B.BF16])
@pytest.mark.parametrize("k,pad", [(1, 0), (2, 1), (3, 1), (4, 1), (5, 2), (6, 3), (7, 3)])
def test_every_tile_shape_of_the_menu(k, pad, dtype, monkeypatch):
    """The selector only ever launches the shape it prefers; force each of the 34 menu entries (7 common tile / wave
    shapes; then 4 bf16-only shapes with two row blocks per wave, the quarter tiles, the two fp32-only pairs of tiles
    under sixteen waves and the fp32-only quarter tiles with two channel groups; then the two bf16-only four-wave
    shapes; each with channel split 1 and 2; entries the operand type or kernel side does not have fall back to the
    selector) so every instantiation is checked."""
    from gpu_util import TOL_BF16
    case = (2, 72, 33, 30, 80, k, pad)        # 5 (fp32) / 3 (bf16) channel chunks: an uneven split
    n, c, h, w, m, _, _ = case
    I = wl.uniform(600 + k, n * c * h * w, -1, 1).reshape(n, c, h, w)
    K = wl.normal(601 + k, m * c * k * k, 0.5).reshape(m, c, k, k)
    ref, absref = oracle.mcmk(I, K, pad)
    tol = TOL_BF16 if dtype == B.BF16 else TOL_F32
    for index in range(34):
        for variant in (B.KN2ROW, B.KN2COL):
            announce("menu", "k", k, "dtype", dtype, "tile", index, "variant", variant)
            B.conv_mcmk_force_tile(index)
            got = run_variant(variant, I, K, pad, dtype=dtype)
            assert_within_bound(got, ref, absref, tol, f"tile {index} k={k} dtype={dtype} variant={variant}")
    B.conv_mcmk_force_tile(-1)


@pytest.mark.parametrize("dtype", [B.F32, B.BF16])
@pytest.mark.parametrize("case", [(2, 24, 19, 22, 40, 3, 1, 1), (1, 40, 30, 17, 24, 2, 1, 1), (2, 16, 21, 21, 20, 3, 1, 2)])
def test_every_tile_shape_of_the_staged_variants_matrix_product(case, dtype):
    """The matrix product of im2col, im2row and the two-pass variant (sections II-B, III-A) runs on the same tile
    kernels as a 1 x 1 convolution over the patch matrix / the input, with the tile shape picked from the fused
    kernel's menu (34 entries) plus the flat shapes (8 entries, from index 100); force every entry, so that each instantiation is checked with
    rows that are (tap, kernel) pairs, with the channel split and with channel groups."""
    from gpu_util import TOL_BF16
    n, c, h, w, m, k, pad, stride = case
    I = wl.uniform(700 + k, n * c * h * w, -1, 1).reshape(n, c, h, w)
    K = wl.normal(701 + k, m * c * k * k, 0.5).reshape(m, c, k, k)
    ref, absref = oracle.mcmk(I, K, pad, stride)
    tol = TOL_BF16 if dtype == B.BF16 else TOL_F32
    for index in list(range(34)) + list(range(100, 110)) + [-1]:
        for variant in (B.IM2COL, B.KN2ROW_2PASS, B.IM2ROW):
            announce("gemm menu", case, "dtype", dtype, "tile", index, "variant", variant)
            B.conv_mcmk_force_gemm_tile(index)
            got = run_variant(variant, I, K, pad, dtype=dtype, stride=stride)
            assert_within_bound(got, ref, absref, tol, f"gemm tile {index} {case} dtype={dtype} variant={variant}")
    B.conv_mcmk_force_gemm_tile(-1)


@pytest.mark.parametrize("c", [128, 144, 176, 272])
def test_layers_deep_enough_for_a_barrier_every_second_chunk(c, monkeypatch):
    """From eight 16-channel chunks on, the fp32 shapes that have four LDS buffers stage two chunks ahead and meet
    at a barrier after every second chunk: even and odd chunk counts (8, 9, 11, 17), with and without the two-way
    channel split (which hands each half 8 and 9 chunks of the 17), every such shape; integer data, exact."""
    n, h, w, m, k, pad = 1, 30, 33, 40, 3, 1
    I = wl.small_integers(950 + c, n * c * h * w, 0, 4).reshape(n, c, h, w)
    K = wl.small_integers(951 + c, m * c * k * k, -3, 3).reshape(m, c, k, k)
    ref, _ = oracle.mcmk(I, K, pad)
    for index in (None, 0, 1, 18, 19, 21, 7, 8, 26, 6, 13, 20, 28, 29):        # the last five: channel groups, alone and under the split
        for variant in (B.KN2ROW, B.KN2COL):
            announce("deep", c, "tile", index, "variant", variant)
            if index is None:
                B.conv_mcmk_force_tile(-1)
            else:
                B.conv_mcmk_force_tile(index)
            got = run_variant(variant, I, K, pad)
            np.testing.assert_array_equal(got.astype(np.float64), ref)
    B.conv_mcmk_force_tile(-1)


@pytest.mark.parametrize("k,pad", [(3, 1), (5, 2), (7, 3), (3, 0), (7, 6)])
@pytest.mark.parametrize("c", [1, 2, 3, 4, 5])
def test_few_channel_layers(c, k, pad, monkeypatch):
    """Layers of up to four channels run an instantiation of three tile shapes that stages and multiplies one
    channel quad instead of four (five channels: the general kernels); every such shape against the oracle,
    integer data so that the comparison is exact."""
    n, h, w, m = 2, 37, 45, 40
    I = wl.small_integers(900 + c, n * c * h * w, 0, 8).reshape(n, c, h, w)
    K = wl.small_integers(901 + k, m * c * k * k, -4, 4).reshape(m, c, k, k)
    ref, _ = oracle.mcmk(I, K, pad)
    for index in (None, 0, 3, 4, 1):
        announce("few channels", c, k, pad, "tile", index)
        if index is None:
            B.conv_mcmk_force_tile(-1)
        else:
            B.conv_mcmk_force_tile(index)
        got = run_variant(B.KN2ROW, I, K, pad)
        np.testing.assert_array_equal(got.astype(np.float64), ref)
    ref2, _ = oracle.mcmk(I, K, pad, 2)
    for index in (None, 0, 1, 2):                 # stride 2: shapes 0 and 1 have the lean form, 2 has not
        announce("few channels, stride 2", c, k, pad, "tile", index)
        if index is None:
            B.conv_mcmk_force_tile(-1)
        else:
            B.conv_mcmk_force_tile(index)
        got = run_variant(B.KN2ROW, I, K, pad, stride=2)
        np.testing.assert_array_equal(got.astype(np.float64), ref2)
    B.conv_mcmk_force_tile(-1)


@pytest.mark.parametrize("case", [
    (1, 3, 600, 500, 8, 7, 3),        # large image, first-layer-like channel count
    (1, 8, 9, 2000, 16, 3, 1),        # very wide, few rows
    (1, 8, 2000, 9, 16, 3, 1),        # very tall
    (4, 130, 20, 20, 300, 3, 1),      # many kernels, channels just past a chunk boundary
    (1, 1, 40, 40, 1, 5, 2),          # one channel, one kernel
])
def test_stretched_shapes(case):
    announce("stretched", case)
    n, c, h, w, m, k, pad = case
    I = wl.uniform(700 + c, n * c * h * w, -1, 1).reshape(n, c, h, w)
    K = wl.normal(701 + c, m * c * k * k, 0.5).reshape(m, c, k, k)
    ref, absref = oracle.mcmk(I, K, pad)
    for name, variant in ALL:
        if variant in B.CHANNELS_LAST and c % 4:
            continue
        got = run_variant(variant, I, K, pad)
        assert_within_bound(got, ref, absref, TOL_F32, f"{name} {case}")


@pytest.mark.parametrize("case", [(2, 40, 28, 28, 48, 3, 1),        # single launch
                                  (8, 128, 14, 14, 128, 3, 1),      # quarter tiles with channel groups
                                  (1, 512, 14, 14, 512, 3, 1)])     # ... under the channel split: zero-fill kernel + atomics
def test_calls_can_be_captured_into_a_graph(case):
    """The library launches only kernels on the caller's stream (no allocation, no synchronisation,
    no memset node), so a call can be captured once and replayed; every replay must reproduce the
    eager result bit for bit, also after the input changes."""
    import torch
    n, c, h, w, m, k, pad = case
    announce("graph", case, B.conv_mcmk_describe_plan(B.desc(n, c, h, w, m, k, pad), B.KN2ROW))
    d = B.desc(n, c, h, w, m, k, pad)
    dev = torch.device("cuda:0")
    I1, K = _inputs(case, 8100)
    I2, _ = _inputs(case, 8200)
    K_dev = torch.from_numpy(K).to(dev)
    plan = B.Plan(d, B.KN2ROW, K_dev)
    I_static = torch.from_numpy(I1).to(dev)
    eager1 = plan.run(I_static).clone()
    I_static.copy_(torch.from_numpy(I2).to(dev))
    eager2 = plan.run(I_static).clone()
    torch.cuda.synchronize()
    I_static.copy_(torch.from_numpy(I1).to(dev))
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        plan.run(I_static)                      # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        plan.run(I_static)
    for rep in range(3):
        for src, want in ((I1, eager1), (I2, eager2)):
            I_static.copy_(torch.from_numpy(src).to(dev))
            plan.out.fill_(float("nan"))
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            assert torch.equal(plan.out, want), f"replay {rep} differs from the eager result"
    ref, absref = oracle.mcmk(I2, K, pad)
    assert_within_bound(plan.out.cpu().numpy(), ref, absref, TOL_F32, f"graph replay {case}")


def test_machine_rate_probes():
    """The benchmark's two probe kernels: the copy moves exactly the bytes it is told to (and nothing beyond them),
    the register-only matrix-core loop writes one finite value per lane; bad arguments are return codes."""
    import torch
    announce("probes")
    nbytes = 3 * 4096 + 16 * 5                                   # not a multiple of the workgroup's 4 KiB
    src = Guarded(nbytes)
    dst = Guarded(nbytes)
    src.payload.copy_(torch.arange(nbytes, device="cuda", dtype=torch.int64).to(torch.uint8))
    B.conv_mcmk_probe_copy(src.payload, dst.payload, nbytes)
    torch.cuda.synchronize()
    assert torch.equal(src.payload, dst.payload) and dst.intact() and src.intact()
    for dtype in (B.F32, B.BF16):
        sink = Guarded(8 * 256 * 4)
        B.conv_mcmk_probe_mfma(dtype, 8, 10, sink.payload)
        torch.cuda.synchronize()
        vals = sink.payload.view(torch.float32)
        assert sink.intact() and bool(torch.isfinite(vals).all()) and float(vals.abs().max()) > 0.0
    with pytest.raises(B.ConvMcmkError) as e:
        B.conv_mcmk_probe_copy(src.payload, dst.payload, 24)     # not a multiple of 16
    assert e.value.code == B.ERR_SHAPE
    with pytest.raises(B.ConvMcmkError) as e:
        B.conv_mcmk_probe_mfma(7, 8, 10, dst.payload)
    assert e.value.code == B.ERR_UNSUPPORTED
    with pytest.raises(B.ConvMcmkError) as e:
        B.conv_mcmk_probe_mfma(B.F32, 0, 10, dst.payload)
    assert e.value.code == B.ERR_SHAPE
    with pytest.raises(B.ConvMcmkError) as e:
        B.conv_mcmk_probe_copy(None, dst.payload, 16)
    assert e.value.code == B.ERR_NULL


@pytest.mark.parametrize("k", [3, 5])
@pytest.mark.parametrize("w", [16, 12, 10, 9, 1])          # output widths that are multiples of 8, 4, 2, odd, and a single column
def test_streaming_forms_of_the_builds_and_the_post_pass(k, w):
    """Unit stride with kernel side 3 or 5 takes the streaming forms of the patch-matrix builds (section II-B) and of
    the shift-add post pass (section III-A): vector widths 8 / 4 / 2 / 1 by output width, every padding from none to
    k - 1 (vectors that hang over either end of a row, rows outside the image, the first and the last element of the
    whole product), fp32 and bf16.  The workspaces must BE the paper's matrices, bit for bit, and on integer data the
    two-pass output must equal the oracle exactly."""
    n, c, h, m = 2, 8, 7, 5
    for pad in range(0, k):
        if h + 2 * pad < k or w + 2 * pad < k:
            continue
        win = w - 2 * pad + k - 1                           # input width that gives output width w
        if win < 1:
            continue
        announce("streaming forms", "k", k, "out width", w, "pad", pad)
        I = wl.small_integers(7000 + 10 * k + pad, n * c * h * win, 0, 8).reshape(n, c, h, win)
        K = wl.small_integers(7001 + 10 * k + pad, m * c * k * k, -4, 4).reshape(m, c, k, k)
        ref, _ = oracle.mcmk(I, K, pad)
        q, p = ref.shape[2], ref.shape[3]
        assert p == w
        got, ws = run_variant(B.KN2ROW_2PASS, I, K, pad, return_ws=True)
        np.testing.assert_array_equal(got.astype(np.float64), ref)
        T = ws.view(np.float32).reshape(n, k * k * m, h * win)
        for i in range(n):
            np.testing.assert_array_equal(T[i].astype(np.float64), steps.kn2row_gemm(I[i], K))
        for dtype in (B.F32, B.BF16):
            got, ws = run_variant(B.IM2COL, I, K, pad, dtype=dtype, return_ws=True)
            np.testing.assert_array_equal(got.astype(np.float64), ref)          # small integers are exact in bf16 too
            cols = ws.view(np.uint16 if dtype == B.BF16 else np.float32).reshape(n, c * k * k, q * p)
            for i in range(n):
                want = steps.input_patch_matrix(I[i], k, pad).astype(np.float32)
                np.testing.assert_array_equal(cols[i], steps.round_to_bf16_bits(want).reshape(want.shape) if dtype == B.BF16 else want)
            got, ws = run_variant(B.IM2ROW, I, K, pad, dtype=dtype, return_ws=True)
            np.testing.assert_array_equal(got.astype(np.float64), ref)
            rows = ws.view(np.uint16 if dtype == B.BF16 else np.float32).reshape(n, q * p, k * k * c)
            for i in range(n):
                want = steps.input_patch_matrix_rows(np.ascontiguousarray(I[i].transpose(1, 2, 0)), k, pad).astype(np.float32)
                np.testing.assert_array_equal(rows[i], steps.round_to_bf16_bits(want).reshape(want.shape) if dtype == B.BF16 else want)


@pytest.mark.parametrize("variant", [B.IM2COL, B.IM2ROW], ids=["im2col", "im2row"])
@pytest.mark.parametrize("dtype", [B.F32, B.BF16], ids=["f32", "bf16"])
@pytest.mark.parametrize("case", [(2, 64, 7, 7, 48, 3, 1), (1, 96, 13, 13, 40, 5, 2), (3, 128, 6, 10, 35, 3, 0)])
def test_split_products_meet_in_copies_or_in_atomics(case, dtype, variant):
    """A deep contraction with a small result is split into parts.  With the workspace the library asks for, each part
    stores a copy of the result and a last pass adds the copies in a fixed order (the same bits on every call);
    with room for the patch matrix alone the parts add into the zeroed output with atomics.  Small integers make
    every sum exact, so both ways must equal the oracle bit for bit."""
    announce("split-product", case, dtype, variant)
    n, c, h, w, m, k, pad = case
    d = B.desc(n, c, h, w, m, k, pad, 1, dtype)
    plan = B.conv_mcmk_describe_plan(d, variant)
    parts = int(plan.split("channel split ")[1].split(",")[0])
    assert parts > 1 or dtype == B.BF16, plan    # the cases are here to cover the split (fp32 splits all of them)
    matrix = n * c * k * k * ((h + 2 * pad - k) + 1) * ((w + 2 * pad - k) + 1) * (2 if dtype == B.BF16 else 4)
    copies = (n * m * ((h + 2 * pad - k) + 1) * ((w + 2 * pad - k) + 1) + 3) // 4 * 16
    assert B.conv_mcmk_workspace_bytes(d, variant) == (matrix if parts == 1 else (matrix + 255) // 256 * 256 + parts * copies)
    I = wl.small_integers(9100 + c, n * c * h * w, 0, 8).reshape(n, c, h, w)
    K = wl.small_integers(9101 + c, m * c * k * k, -4, 4).reshape(m, c, k, k)
    ref, _ = oracle.mcmk(I, K, pad)
    np.testing.assert_array_equal(run_variant(variant, I, K, pad, dtype=dtype).astype(np.float64), ref)
    np.testing.assert_array_equal(run_variant(variant, I, K, pad, dtype=dtype, matrix_only=True).astype(np.float64), ref)
    # inexact sums: the copies are added in a fixed order, so two calls agree in every bit; both ways stay in the bound
    If, Kf = _inputs(case, 9200 + c)
    ref, absref = oracle.mcmk(If, Kf, pad)
    tol = TOL_BF16 if dtype == B.BF16 else TOL_F32
    first = run_variant(variant, If, Kf, pad, dtype=dtype)
    second = run_variant(variant, If, Kf, pad, dtype=dtype)
    np.testing.assert_array_equal(first.view(np.uint32), second.view(np.uint32))
    assert_within_bound(first, ref, absref, tol, "copies")
    assert_within_bound(run_variant(variant, If, Kf, pad, dtype=dtype, matrix_only=True), ref, absref, tol, "atomics")
