"""Pins for the CPU oracle: checks against things other than the oracle itself.

Hand-worked values (tests/golden), closed forms, invariants, two independent
reformulations (im2col and kn2row, section II-B and III-A) and a library
convolution in float64.  Each pin is chosen so that a plausible slip in the
oracle (kernel flip, row/column swap, wrong padding offset, dropped channel,
row wrap-around) fails at least one of them.
"""
import glob
import json
import os

import numpy as np
import pytest

import oracle
from oracle import steps
from paper_1704_04428_amd import workloads as wl


def _rand_int_case(seed, n, c, h, w, m, k):
    I = wl.small_integers(seed, n * c * h * w, 0, 8).reshape(n, c, h, w)
    K = wl.small_integers(seed + 1, m * c * k * k, -4, 4).reshape(m, c, k, k)
    return I, K


# ------------------------------------------------------------------ hand-worked values

def test_golden_hand_worked(golden_dir):
    files = sorted(glob.glob(os.path.join(golden_dir, "*.json")))
    assert len(files) >= 4
    for path in files:
        with open(path) as f:
            g = json.load(f)
        I = np.array(g["I"], dtype=np.float32)
        K = np.array(g["K"], dtype=np.float32)
        O, _ = oracle.mcmk(I, K, g["pad"], g.get("stride", 1))
        np.testing.assert_array_equal(O, np.array(g["O"], dtype=np.float64), err_msg=path)


def test_abs_sum_hand_worked(golden_dir):
    with open(os.path.join(golden_dir, "eq123_two_channel_two_kernel_2x3.json")) as f:
        g = json.load(f)
    I = np.array(g["I"], dtype=np.float32)
    K = np.array(g["K"], dtype=np.float32)
    _, A = oracle.mcmk(I, K, g["pad"])
    # kernel 1: |I0[q][p+1]| + 2 |I1[q][p]|, by hand
    np.testing.assert_array_equal(A[1], np.array([[4, 3, 4], [11, 8, 4]], dtype=np.float64))
    # kernel 0 at (0,0): 3*|I0[1][1]| + |I1[1][0]| = 15 + 3
    assert A[0, 0, 0] == 18.0


# ------------------------------------------------------------------ delta kernels (section III-A offsets)

@pytest.mark.parametrize("k,pad", [(3, 1), (5, 2), (3, 0), (3, 2), (2, 1), (4, 0)])
def test_delta_kernel_is_a_shifted_copy(k, pad):
    c, h, w = 3, 6, 7
    I = wl.uniform(11, c * h * w, -1.0, 1.0).reshape(c, h, w)
    q_out, p_out = h + 2 * pad - k + 1, w + 2 * pad - k + 1
    for ch in range(c):
        for i0 in range(k):
            for j0 in range(k):
                K = np.zeros((1, c, k, k), dtype=np.float32)
                K[0, ch, i0, j0] = 1.0
                O, _ = oracle.mcmk(I, K, pad)
                want = np.zeros((q_out, p_out))
                for q in range(q_out):
                    for p in range(p_out):
                        y, x = q - pad + i0, p - pad + j0
                        if 0 <= y < h and 0 <= x < w:      # never wraps into the next row
                            want[q, p] = I[ch, y, x]
                np.testing.assert_array_equal(O[0], want)


def test_centre_tap_aligned_and_corner_tap_offset():
    """Section III-A: the centre tap's plane is aligned with the output; the upper-left tap of a
    3 x 3 kernel pairs output (q, p) with the input one row up and one column left."""
    I = np.arange(20, dtype=np.float32).reshape(1, 4, 5)
    K = np.zeros((1, 1, 3, 3), dtype=np.float32)
    K[0, 0, 1, 1] = 1
    np.testing.assert_array_equal(oracle.mcmk(I, K, 1)[0][0], I[0])
    K[:] = 0
    K[0, 0, 0, 0] = 1
    O = oracle.mcmk(I, K, 1)[0][0]
    assert O[0].tolist() == [0] * 5 and O[:, 0].tolist() == [0] * 4
    np.testing.assert_array_equal(O[1:, 1:], I[0, :-1, :-1])


# ------------------------------------------------------------------ invariants and closed forms

def test_linearity_in_input_and_kernel():
    n, c, h, w, m, k, pad = 2, 3, 5, 6, 4, 3, 1
    I1, K1 = _rand_int_case(21, n, c, h, w, m, k)
    I2, K2 = _rand_int_case(23, n, c, h, w, m, k)
    a, b = 3.0, -2.0
    lhs = oracle.mcmk(a * I1 + b * I2, K1, pad)[0]
    rhs = a * oracle.mcmk(I1, K1, pad)[0] + b * oracle.mcmk(I2, K1, pad)[0]
    np.testing.assert_array_equal(lhs, rhs)          # integers: exact
    lhs = oracle.mcmk(I1, a * K1 + b * K2, pad)[0]
    rhs = a * oracle.mcmk(I1, K1, pad)[0] + b * oracle.mcmk(I1, K2, pad)[0]
    np.testing.assert_array_equal(lhs, rhs)


@pytest.mark.parametrize("c,h,w,k,pad", [(4, 5, 7, 3, 1), (2, 6, 6, 5, 2), (3, 4, 5, 3, 0), (2, 5, 4, 3, 2)])
def test_constant_input_constant_kernel_closed_form(c, h, w, k, pad):
    a, b = 2.0, 3.0
    I = np.full((c, h, w), a, dtype=np.float32)
    K = np.full((2, c, k, k), b, dtype=np.float32)
    O, A = oracle.mcmk(I, K, pad)
    q_out, p_out = h + 2 * pad - k + 1, w + 2 * pad - k + 1

    def taps(o, size):       # how many of the k taps land inside the image
        return min(k - 1, size - 1 - o + pad) - max(0, pad - o) + 1

    want = np.array([[a * b * c * taps(q, h) * taps(p, w) for p in range(p_out)] for q in range(q_out)])
    np.testing.assert_array_equal(O[0], want)
    np.testing.assert_array_equal(O[1], want)
    np.testing.assert_array_equal(A[0], want)
    if k == 3 and pad == 1:
        assert O[0, 0, 0] == 4 * c * a * b and O[0, 0, 1] == 6 * c * a * b and O[0, 1, 1] == 9 * c * a * b


def test_constant_input_general_kernel():
    c, h, w, m, k, pad = 3, 6, 5, 2, 3, 1
    K = wl.small_integers(31, m * c * k * k, -4, 4).reshape(m, c, k, k)
    I = np.full((c, h, w), 2.0, dtype=np.float32)
    O, _ = oracle.mcmk(I, K, pad)
    # interior: every tap inside; top-left corner: taps i>=1, j>=1 only
    assert O[0, 2, 2] == 2.0 * K[0].sum()
    assert O[1, 0, 0] == 2.0 * K[1][:, 1:, 1:].sum()
    assert O[1, h - 1, 2] == 2.0 * K[1][:, :2, :].sum()
    assert O[0, 3, w - 1] == 2.0 * K[0][:, :, :2].sum()


def test_images_and_kernels_are_independent():
    """Eq. 3 concatenates per-kernel planes; batch images never mix."""
    n, c, h, w, m, k, pad = 3, 2, 5, 5, 3, 3, 1
    I, K = _rand_int_case(41, n, c, h, w, m, k)
    O, _ = oracle.mcmk(I, K, pad)
    for i in range(n):
        for j in range(m):
            np.testing.assert_array_equal(O[i, j], oracle.mcmk(I[i], K[j:j + 1], pad)[0][0])


# ------------------------------------------------------------------ reformulations

CASES = [
    # n, c, h, w, m, k, pad
    (1, 1, 3, 3, 1, 3, 1),
    (1, 2, 3, 4, 2, 3, 1),
    (2, 5, 9, 7, 4, 3, 1),
    (1, 3, 8, 11, 5, 5, 2),
    (1, 4, 6, 6, 3, 1, 0),
    (1, 2, 7, 5, 2, 3, 0),
    (1, 2, 4, 6, 2, 3, 2),
    (1, 3, 6, 5, 2, 2, 1),
    (1, 2, 9, 8, 3, 4, 1),
    (1, 2, 9, 9, 2, 7, 3),
]


@pytest.mark.parametrize("case", CASES)
def test_im2col_reformulation_matches(case):
    n, c, h, w, m, k, pad = case
    I = wl.uniform(51, n * c * h * w, -1, 1).reshape(n, c, h, w)
    K = wl.normal(52, m * c * k * k, 0.5).reshape(m, c, k, k)
    O, A = oracle.mcmk(I, K, pad)
    for i in range(n):
        got = steps.im2col_mcmk(I[i], K, pad)
        assert np.all(np.abs(got - O[i]) <= 1e-13 * A[i] + 1e-300)


@pytest.mark.parametrize("case", CASES)
def test_im2row_reformulation_matches(case):
    n, c, h, w, m, k, pad = case
    I = wl.uniform(55, n * c * h * w, -1, 1).reshape(n, c, h, w)
    K = wl.normal(56, m * c * k * k, 0.5).reshape(m, c, k, k)
    O, A = oracle.mcmk(I, K, pad)
    for i in range(n):
        got = steps.im2row_mcmk(np.ascontiguousarray(I[i].transpose(1, 2, 0)), K, pad)      # [Q][P][M]
        assert np.all(np.abs(got.transpose(2, 0, 1) - O[i]) <= 1e-13 * A[i] + 1e-300)
    rows = steps.input_patch_matrix_rows(np.ascontiguousarray(I[0].transpose(1, 2, 0)), k, pad)
    cols = steps.input_patch_matrix(I[0], k, pad)
    # same patches, transposed and with (i, j, c) instead of (c, i, j) ordering
    np.testing.assert_array_equal(rows.reshape(-1, k * k, c).transpose(2, 1, 0).reshape(c * k * k, -1), cols)


@pytest.mark.parametrize("case", CASES)
def test_kn2row_reformulation_matches(case):
    n, c, h, w, m, k, pad = case
    I = wl.uniform(61, n * c * h * w, -1, 1).reshape(n, c, h, w)
    K = wl.normal(62, m * c * k * k, 0.5).reshape(m, c, k, k)
    O, A = oracle.mcmk(I, K, pad)
    for i in range(n):
        got = steps.kn2row_mcmk(I[i], K, pad)
        assert np.all(np.abs(got - O[i]) <= 1e-13 * A[i] + 1e-300)


@pytest.mark.parametrize("case", CASES)
def test_kn2col_reformulation_matches(case):
    """kn2col is kn2row with the channel innermost: same numbers, transposed layouts."""
    n, c, h, w, m, k, pad = case
    I = wl.uniform(65, n * c * h * w, -1, 1).reshape(n, c, h, w)
    K = wl.normal(66, m * c * k * k, 0.5).reshape(m, c, k, k)
    O, A = oracle.mcmk(I, K, pad)
    for i in range(n):
        got = steps.kn2col_mcmk(np.ascontiguousarray(I[i].transpose(1, 2, 0)), K, pad)      # [Q][P][M]
        assert got.shape == (O.shape[2], O.shape[3], m)
        assert np.all(np.abs(got.transpose(2, 0, 1) - O[i]) <= 1e-13 * A[i] + 1e-300)
    T = steps.kn2col_gemm(np.ascontiguousarray(I[0].transpose(1, 2, 0)), K)
    assert T.shape == (h * w, k * k * m)
    np.testing.assert_allclose(T, steps.kn2row_gemm(I[0], K).T, rtol=0, atol=1e-13)


def test_one_by_one_is_a_matrix_product():
    """Section III: for k = 1 the layer is [M x C] times [C x HW]."""
    c, h, w, m = 7, 5, 6, 4
    I = wl.uniform(71, c * h * w, -1, 1).reshape(c, h, w)
    K = wl.uniform(72, m * c, -1, 1).reshape(m, c, 1, 1)
    want = np.zeros((m, h * w))
    for a in range(m):
        for b in range(h * w):
            for cc in range(c):
                want[a, b] += float(K[a, cc, 0, 0]) * float(I.reshape(c, -1)[cc, b])
    O, _ = oracle.mcmk(I, K, 0)
    np.testing.assert_allclose(O.reshape(m, -1), want, rtol=0, atol=1e-14)


def test_matches_library_convolution_float64():
    torch = pytest.importorskip("torch")
    for (n, c, h, w, m, k, pad) in CASES:
        I = wl.uniform(81, n * c * h * w, -1, 1).reshape(n, c, h, w)
        K = wl.normal(82, m * c * k * k, 0.5).reshape(m, c, k, k)
        O, A = oracle.mcmk(I, K, pad)
        ref = torch.nn.functional.conv2d(torch.from_numpy(I).double(), torch.from_numpy(K).double(),
                                         padding=pad).numpy()
        assert ref.shape == O.shape
        assert np.all(np.abs(ref - O) <= 1e-13 * A + 1e-300)


def test_sampled_outputs_equal_full_output():
    L = wl.LAYERS["cfg1_tiny"]
    I, K = wl.make_input(L), wl.make_kernel(L)
    O, A = oracle.mcmk(I, K, L.pad)
    pts = wl.sample_points(L, 200)
    o, a = oracle.mcmk_at(I, K, L.pad, pts)
    np.testing.assert_array_equal(o, O[pts[:, 0], pts[:, 1], pts[:, 2], pts[:, 3]])
    np.testing.assert_array_equal(a, A[pts[:, 0], pts[:, 1], pts[:, 2], pts[:, 3]])


def test_rejects_bad_shapes():
    I = np.zeros((1, 2, 2), dtype=np.float32)
    with pytest.raises(ValueError):
        oracle.mcmk(I, np.zeros((1, 1, 5, 5), dtype=np.float32), 0)     # empty output
    with pytest.raises(ValueError):
        oracle.mcmk(I, np.zeros((1, 2, 3, 3), dtype=np.float32), 1)     # channel mismatch


# ------------------------------------------------------------------ the staged matrices themselves

def test_patch_matrix_shapes_and_replication():
    """The column matrix is k^2 times the input (section I); the kn2row product is k^2 times the
    output and the input is used as is (section III)."""
    c, h, w, m, k, pad = 3, 6, 5, 4, 3, 1
    I = wl.uniform(91, c * h * w, 0, 1).reshape(c, h, w)
    K = wl.uniform(92, m * c * k * k, -1, 1).reshape(m, c, k, k)
    cols = steps.input_patch_matrix(I, k, pad)
    assert cols.shape == (c * k * k, h * w)
    T = steps.kn2row_gemm(I, K)
    assert T.shape == (k * k * m, h * w)
    A = steps.kn2row_kernel_matrix(K)
    assert A.shape == (k * k * m, c)
    # slice t = i*k + j of the re-ordered kernel is K[:, :, i, j]
    for i in range(k):
        for j in range(k):
            np.testing.assert_array_equal(A[(i * k + j) * m:(i * k + j + 1) * m], K[:, :, i, j])
    # the centre rows of the patch matrix are the image itself
    for ch in range(c):
        np.testing.assert_array_equal(cols[(ch * k + 1) * k + 1], I[ch].reshape(-1))


# ------------------------------------------------------------------ bf16 rounding

def test_bf16_rounding_known_values():
    x = np.array([1.0, 1.0 + 2.0 ** -8, 1.0 + 2.0 ** -7, 1.0 + 3 * 2.0 ** -8, -2.5, 0.0, 3.0e38,
                  1.0 + 2.0 ** -8 + 2.0 ** -20], dtype=np.float32)
    bits = steps.round_to_bf16_bits(x)
    #        1.0     tie->even  exact    tie->even(up)  exact   zero    rounds to a finite bf16   above tie -> up
    assert bits.tolist() == [0x3F80, 0x3F80, 0x3F81, 0x3F82, 0xC020, 0x0000, 0x7F62, 0x3F81]
    assert np.isnan(steps.round_to_bf16(np.array([np.nan], dtype=np.float32)))[0]
    assert np.isinf(steps.round_to_bf16(np.array([3.4e38], dtype=np.float32)))[0]


def test_bf16_rounding_matches_library_cast():
    torch = pytest.importorskip("torch")
    x = np.concatenate([wl.normal(101, 20000, 1.0), wl.uniform(102, 20000, -1e-3, 1e-3),
                        wl.normal(103, 1000, 1e20)]).astype(np.float32)
    want = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    np.testing.assert_array_equal(steps.round_to_bf16_bits(x), want)


# ------------------------------------------------------------------ the input generator

def test_generator_is_reproducible_and_distributed_as_stated():
    L = wl.LAYERS["cfg2_googlenet5x5"]
    I, K = wl.make_input(L), wl.make_kernel(L)
    assert I.shape == (1, 32, 28, 28) and K.shape == (96, 32, 5, 5)
    np.testing.assert_array_equal(I, wl.make_input(L))
    assert 0.0 <= I.min() and I.max() < 1.0 and abs(I.mean() - 0.5) < 0.01
    sigma = np.sqrt(2.0 / (32 * 25))
    assert abs(K.std() - sigma) < 0.02 * sigma and abs(K.mean()) < 0.02 * sigma
    # splitmix64 reference values: the first outputs of the generator seeded with 0 and with 1234567
    z = wl.splitmix64(0, np.arange(2))
    assert [int(v) for v in z] == [0xE220A8397B1DCDAF, 0x6E789E6AA1B965F4]
    z = wl.splitmix64(1234567, np.arange(2))
    assert [int(v) for v in z] == [6457827717110365317, 3203168211198807973]


# ------------------------------------------------------------------ strides (generalisation; section II-A treats unit stride only)

STRIDED = [
    # n, c, h, w, m, k, pad, stride
    (1, 2, 7, 9, 2, 3, 1, 2),
    (2, 3, 8, 11, 3, 3, 0, 2),
    (1, 2, 9, 8, 2, 5, 2, 3),
    (1, 3, 6, 7, 2, 1, 0, 2),
    (1, 2, 10, 6, 2, 2, 1, 2),
    (1, 1, 5, 5, 1, 3, 1, 4),
    (1, 2, 12, 13, 2, 7, 3, 2),
]


@pytest.mark.parametrize("case", STRIDED)
def test_strided_output_is_the_unit_stride_output_subsampled(case):
    """The definition of a stride: the same sums, kept at every s-th row and column only.  The
    unit-stride oracle is pinned above; integer data makes the comparison exact."""
    n, c, h, w, m, k, pad, s = case
    I, K = _rand_int_case(300 + s, n, c, h, w, m, k)
    full, full_abs = oracle.mcmk(I, K, pad)
    O, A = oracle.mcmk(I, K, pad, s)
    assert O.shape == (n, m, (h + 2 * pad - k) // s + 1, (w + 2 * pad - k) // s + 1)
    np.testing.assert_array_equal(O, full[:, :, ::s, ::s])
    np.testing.assert_array_equal(A, full_abs[:, :, ::s, ::s])


def test_strided_delta_kernel_picks_every_second_pixel():
    c, h, w, k, pad, s = 2, 7, 8, 3, 1, 2
    I = wl.uniform(311, c * h * w, -1.0, 1.0).reshape(c, h, w)
    for i0 in range(k):
        for j0 in range(k):
            K = np.zeros((1, c, k, k), dtype=np.float32)
            K[0, 1, i0, j0] = 1.0
            O, _ = oracle.mcmk(I, K, pad, s)
            for q in range(O.shape[1]):
                for p in range(O.shape[2]):
                    y, x = s * q - pad + i0, s * p - pad + j0
                    want = float(I[1, y, x]) if 0 <= y < h and 0 <= x < w else 0.0
                    assert O[0, q, p] == want


@pytest.mark.parametrize("case", STRIDED)
def test_strided_reformulations_match(case):
    """im2col / im2row keep only the patches a stride uses; kn2row / kn2col keep the GEMM and
    subsample in the post pass.  All four must reproduce the strided sum."""
    n, c, h, w, m, k, pad, s = case
    I = wl.uniform(321, n * c * h * w, -1, 1).reshape(n, c, h, w)
    K = wl.normal(322, m * c * k * k, 0.5).reshape(m, c, k, k)
    O, A = oracle.mcmk(I, K, pad, s)
    for i in range(n):
        hwc = np.ascontiguousarray(I[i].transpose(1, 2, 0))
        for got in (steps.im2col_mcmk(I[i], K, pad, s), steps.kn2row_mcmk(I[i], K, pad, s),
                    steps.im2row_mcmk(hwc, K, pad, s).transpose(2, 0, 1), steps.kn2col_mcmk(hwc, K, pad, s).transpose(2, 0, 1)):
            assert got.shape == O[i].shape
            assert np.all(np.abs(got - O[i]) <= 1e-13 * A[i] + 1e-300)


def test_strided_sampled_outputs_equal_full_output():
    n, c, h, w, m, k, pad, s = 2, 3, 9, 10, 4, 3, 1, 2
    I = wl.uniform(331, n * c * h * w, -1, 1).reshape(n, c, h, w)
    K = wl.normal(332, m * c * k * k, 0.5).reshape(m, c, k, k)
    O, A = oracle.mcmk(I, K, pad, s)
    pts = [(a, b, q, p) for a in range(n) for b in range(m) for q in range(O.shape[2]) for p in range(O.shape[3])][::7]
    Os, As = oracle.mcmk_at(I, K, pad, pts, s)
    np.testing.assert_array_equal(Os, np.array([O[t] for t in pts]))
    np.testing.assert_array_equal(As, np.array([A[t] for t in pts]))
    with pytest.raises(ValueError):
        oracle.mcmk_at(I, K, pad, [(0, 0, O.shape[2], 0)], s)          # a row the strided output does not have


# ------------------------------------------------------------------ bias and rectifier (layer epilogue; not in the paper)

def test_bias_relu_closed_forms():
    O = np.array([[[-2.0, 0.5], [1.5, -0.25]], [[3.0, -3.0], [0.0, 1.0]]])       # [M=2][2][2]
    bias = np.array([1.0, -2.0])
    np.testing.assert_array_equal(oracle.bias_relu(O), O)
    np.testing.assert_array_equal(oracle.bias_relu(O, bias), [[[-1.0, 1.5], [2.5, 0.75]], [[1.0, -5.0], [-2.0, -1.0]]])
    np.testing.assert_array_equal(oracle.bias_relu(O, bias, True), [[[0.0, 1.5], [2.5, 0.75]], [[1.0, 0.0], [0.0, 0.0]]])
    np.testing.assert_array_equal(oracle.bias_relu(O, None, True), [[[0.0, 0.5], [1.5, 0.0]], [[3.0, 0.0], [0.0, 1.0]]])
    # a batch axis in front is carried along; the bias still goes with the kernel axis
    np.testing.assert_array_equal(oracle.bias_relu(np.stack([O, -O]), bias, True)[1],
                                  np.maximum(-O + bias.reshape(2, 1, 1), 0.0))
