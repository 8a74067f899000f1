"""The paper's GEMM-based algorithms written out step by step in numpy float64.

TEST INFRASTRUCTURE ONLY (see conv_oracle.c).  Two uses: they pin the direct
oracle (both must reproduce the defining sum), and they give the intermediate
matrices of the two staged GPU variants something to be compared with.

Each function handles one image I[C][H][W] and kernels K[M][C][k][k]; taps are
numbered t = i*k + j with i the row tap and j the column tap.  `np.matmul` in
float64 serves as the GEMM step; nothing is blocked, fused or reordered.

`stride` (default 1) is the generalisation the paper leaves out (section II-A): output (q, p) is the
unit-stride output (s q, s p).  The patch matrices then hold only the patches that are used; the
kn2row GEMM is unchanged (it has no notion of an output position) and the post pass reads every
s-th value of the shifted planes.
"""
from __future__ import annotations

import numpy as np


def _f64(a):
    return np.asarray(a, dtype=np.float64)


def _out(size, k, pad, stride):
    return (size + 2 * pad - k) // stride + 1


# ---------------------------------------------------------------- im2col (section II-B)

def kernel_patch_matrix(K):
    """K-hat: each of the M kernels unrolled into one row, [M] x [C*k*k], columns ordered (c, i, j)."""
    K = _f64(K)
    m = K.shape[0]
    return K.reshape(m, -1)


def input_patch_matrix(I, k, pad, stride=1):
    """I-hat: one column per output position holding the k x k x C patch under the kernel there,
    [C*k*k] x [Q*P]; rows ordered (c, i, j) to match K-hat, columns ordered (q, p).
    Patch elements outside the image are zero (the padding of section II-A)."""
    I = _f64(I)
    c, h, w = I.shape
    q_out, p_out = _out(h, k, pad, stride), _out(w, k, pad, stride)
    cols = np.zeros((c * k * k, q_out * p_out), dtype=np.float64)
    for ch in range(c):
        for i in range(k):
            for j in range(k):
                row = (ch * k + i) * k + j
                for q in range(q_out):
                    y = q * stride - pad + i
                    if y < 0 or y >= h:
                        continue
                    for p in range(p_out):
                        x = p * stride - pad + j
                        if 0 <= x < w:
                            cols[row, q * p_out + p] = I[ch, y, x]
    return cols


def im2col_mcmk(I, K, pad, stride=1):
    """O-hat = K-hat x I-hat, read back as M planes of Q x P."""
    K = _f64(K)
    m, _, k, _ = K.shape
    c, h, w = np.shape(I)
    q_out, p_out = _out(h, k, pad, stride), _out(w, k, pad, stride)
    out = np.matmul(kernel_patch_matrix(K), input_patch_matrix(I, k, pad, stride))
    return out.reshape(m, q_out, p_out)


def input_patch_matrix_rows(I_hwc, k, pad, stride=1):
    """im2row: the patches unrolled into ROWS, [Q*P] x [k*k*C], from a channel-innermost input
    I[H][W][C]; columns ordered (i, j, c) so that consecutive patch elements are consecutive in memory."""
    I_hwc = _f64(I_hwc)
    h, w, c = I_hwc.shape
    q_out, p_out = _out(h, k, pad, stride), _out(w, k, pad, stride)
    rows = np.zeros((q_out * p_out, k * k * c), dtype=np.float64)
    for q in range(q_out):
        for p in range(p_out):
            for i in range(k):
                for j in range(k):
                    y, x = q * stride - pad + i, p * stride - pad + j
                    if 0 <= y < h and 0 <= x < w:
                        rows[q * p_out + p, (i * k + j) * c:(i * k + j + 1) * c] = I_hwc[y, x, :]
    return rows


def kernel_patch_matrix_cols(K):
    """im2row: each kernel unrolled into one COLUMN, [k*k*C] x [M], rows ordered (i, j, c)."""
    K = _f64(K)
    m = K.shape[0]
    return np.ascontiguousarray(K.transpose(2, 3, 1, 0)).reshape(-1, m)


def im2row_mcmk(I_hwc, K, pad, stride=1):
    """O = I-hat x K-hat, read back as O[Q][P][M]."""
    K = _f64(K)
    m, _, k, _ = K.shape
    h, w, _ = np.shape(I_hwc)
    q_out, p_out = _out(h, k, pad, stride), _out(w, k, pad, stride)
    return np.matmul(input_patch_matrix_rows(I_hwc, k, pad, stride), kernel_patch_matrix_cols(K)).reshape(q_out, p_out, m)


# ---------------------------------------------------------------- kn2row (section III-A)

def kn2row_kernel_matrix(K):
    """The re-ordered kernel: k*k slices of [M] x [C] stacked into [k*k*M] x [C], row t*M + m,
    channel index innermost (contiguous)."""
    K = _f64(K)
    m, c, k, _ = K.shape
    return np.ascontiguousarray(K.transpose(2, 3, 0, 1)).reshape(k * k * m, c)


def kn2row_gemm(I, K):
    """The single GEMM: [k*k*M] x [C] times [C] x [H*W] gives [k*k*M] x [H*W]: the k*k results of the
    1 x 1 convolutions, each M planes of H x W in the multi-channel representation."""
    I = _f64(I)
    c, h, w = I.shape
    return np.matmul(kn2row_kernel_matrix(K), I.reshape(c, h * w))


def shift_add(T, m, h, w, k, pad, stride=1):
    """The post pass: add the k*k sub-matrices of T ([k*k*M] x [H*W]) into O[M][Q][P], each offset
    by its tap's row and column distance from the output position.  Offsets act on the 2-D planes
    (a value that leaves a row is dropped, never carried into the next row); values that fall
    outside the output are discarded."""
    T = _f64(T).reshape(k * k, m, h, w)
    q_out, p_out = _out(h, k, pad, stride), _out(w, k, pad, stride)
    O = np.zeros((m, q_out, p_out), dtype=np.float64)
    for i in range(k):
        for j in range(k):
            di, dj = i - pad, j - pad
            # output (q, p) takes plane value (s q + di, s p + dj) when that lies inside the plane
            qs = [q for q in range(q_out) if 0 <= q * stride + di < h]
            ps = [p for p in range(p_out) if 0 <= p * stride + dj < w]
            if not qs or not ps:
                continue
            q0, q1, p0, p1 = qs[0], qs[-1] + 1, ps[0], ps[-1] + 1
            O[:, q0:q1, p0:p1] += T[i * k + j, :, q0 * stride + di:(q1 - 1) * stride + di + 1:stride,
                                    p0 * stride + dj:(p1 - 1) * stride + dj + 1:stride]
    return O


def kn2row_mcmk(I, K, pad, stride=1):
    K = _f64(K)
    m, _, k, _ = K.shape
    c, h, w = np.shape(I)
    return shift_add(kn2row_gemm(I, K), m, h, w, k, pad, stride)


# ---------------------------------------------------------------- kn2col (section III-A, last paragraph)

def kn2col_kernel_matrix(K):
    """The kernel matrix with the dimensions swapped: [C] x [k*k*M], column t*M + m."""
    return np.ascontiguousarray(kn2row_kernel_matrix(K).T)


def kn2col_gemm(I_hwc, K):
    """[H*W] x [C] (channel innermost input, I[H][W][C]) times [C] x [k*k*M] gives [H*W] x [k*k*M]."""
    I_hwc = _f64(I_hwc)
    h, w, c = I_hwc.shape
    return np.matmul(I_hwc.reshape(h * w, c), kn2col_kernel_matrix(K))


def shift_add_channels_last(T, m, h, w, k, pad, stride=1):
    """The same post pass on the channel-innermost product T ([H*W] x [k*k*M]): O[Q][P][M]."""
    T = _f64(T).reshape(h, w, k * k, m)
    q_out, p_out = _out(h, k, pad, stride), _out(w, k, pad, stride)
    O = np.zeros((q_out, p_out, m), dtype=np.float64)
    for i in range(k):
        for j in range(k):
            di, dj = i - pad, j - pad
            qs = [q for q in range(q_out) if 0 <= q * stride + di < h]
            ps = [p for p in range(p_out) if 0 <= p * stride + dj < w]
            if not qs or not ps:
                continue
            q0, q1, p0, p1 = qs[0], qs[-1] + 1, ps[0], ps[-1] + 1
            O[q0:q1, p0:p1, :] += T[q0 * stride + di:(q1 - 1) * stride + di + 1:stride,
                                    p0 * stride + dj:(p1 - 1) * stride + dj + 1:stride, i * k + j, :]
    return O


def kn2col_mcmk(I_hwc, K, pad, stride=1):
    """kn2col: input I[H][W][C], kernels K[M][C][k][k], output O[Q][P][M]."""
    K = _f64(K)
    m, _, k, _ = K.shape
    h, w, _ = np.shape(I_hwc)
    return shift_add_channels_last(kn2col_gemm(I_hwc, K), m, h, w, k, pad, stride)


# ---------------------------------------------------------------- bf16 rounding

def round_to_bf16_bits(x):
    """float32 -> bfloat16 bit patterns (uint16), round to nearest, ties to even.
    bfloat16 is the upper half of the float32 encoding; NaNs stay NaNs (quiet bit set)."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    bits = x.view(np.uint32).astype(np.uint64)
    lower = bits & 0xFFFF
    upper = bits >> 16
    round_up = (lower > 0x8000) | ((lower == 0x8000) & ((upper & 1) == 1))
    out = (upper + round_up.astype(np.uint64)) & 0xFFFF
    nan = np.isnan(x)
    out = np.where(nan, (upper | 0x40) & 0xFFFF, out)
    return out.astype(np.uint16)


def bf16_bits_to_f32(bits):
    bits = np.ascontiguousarray(bits, dtype=np.uint16)
    return (bits.astype(np.uint32) << 16).view(np.float32)


def round_to_bf16(x):
    """float32 values rounded to the nearest bfloat16 and widened back to float32."""
    return bf16_bits_to_f32(round_to_bf16_bits(x)).reshape(np.shape(x))
