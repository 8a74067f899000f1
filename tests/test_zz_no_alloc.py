"""conv_mcmk_kn2row_2pass_static: the two-pass kn2row whose k*k*M x H*W product lives in a buffer inside the
library's device image, for callers that cannot allocate.  Called through the C ABI and checked against
conv_mcmk_kn2row_2pass (same kernels, caller-provided workspace) and against the oracle, on two calls in a row,
the second with a smaller input (the buffer then still holds the first call's product)."""
import numpy as np
import pytest

import oracle
from paper_1704_04428_amd import binding as B
from paper_1704_04428_amd import workloads as wl

from gpu_util import TOL_F32, Guarded, announce, assert_within_bound, run_variant

pytestmark = pytest.mark.gpu


def _static_two_pass(I, K, pad, dtype=B.F32):
    import torch
    n, c, h, w = I.shape
    m, _, k, _ = K.shape
    d = B.desc(n, c, h, w, m, k, pad, 1, dtype)
    dev = torch.device("cuda:0")
    I_dev = torch.from_numpy(np.ascontiguousarray(I)).to(dev)
    K_dev = torch.from_numpy(np.ascontiguousarray(K)).to(dev)
    if dtype == B.BF16:
        I_bf = torch.empty(I_dev.shape, dtype=torch.bfloat16, device=dev)
        B.conv_mcmk_cvt_f32_bf16(I_dev, I_bf)
        I_dev = I_bf
    kp = Guarded(B.conv_mcmk_packed_kernel_bytes(d, B.KN2ROW_2PASS))
    B.conv_mcmk_prepack(d, B.KN2ROW_2PASS, K_dev, kp.payload)
    q, p = B.conv_mcmk_output_dims(d)
    out = Guarded(n * m * q * p * 4)
    B.conv_mcmk_kn2row_2pass_static(d, I_dev, kp.payload, out.payload)
    torch.cuda.synchronize()
    assert out.intact() and kp.intact(), "guard band overwritten"
    return out.payload.view(torch.float32).reshape(n, m, q, p).cpu().numpy()


def test_static_scratch_two_pass_matches_the_workspace_form_twice_in_a_row():
    cases = [(2, 40, 45, 52, 48, 3, 1),       # 2 * 9 * 48 * 45 * 52 floats = 8.1 MB of product: several tiles, ragged edges
             (1, 24, 19, 21, 20, 3, 1),       # smaller: 0.3 MB, the rest of the buffer keeps the first call's values
             (1, 8, 17, 17, 12, 5, 2)]        # another kernel side, smaller still
    for dtype in (B.F32, B.BF16):
        for case in cases:
            n, c, h, w, m, k, pad = case
            announce("static scratch", case, "dtype", dtype)
            I = wl.uniform(5100 + h, n * c * h * w, -1, 1).reshape(n, c, h, w)
            K = wl.normal(5101 + h, m * c * k * k, 0.5).reshape(m, c, k, k)
            assert B.conv_mcmk_workspace_bytes(B.desc(n, c, h, w, m, k, pad), B.KN2ROW_2PASS) <= B.STATIC_SCRATCH_BYTES
            got = _static_two_pass(I, K, pad, dtype)
            want = run_variant(B.KN2ROW_2PASS, I, K, pad, dtype=dtype)
            ref, absref = oracle.mcmk(I, K, pad)
            # the same kernels on the same inputs: within the fp32 bound of each other (in fact equal), and of the oracle
            assert_within_bound(got, want.astype(np.float64), absref, TOL_F32, f"static vs workspace form {case}")
            np.testing.assert_array_equal(got, want)
            assert_within_bound(got, ref, absref, 1e-2 if dtype == B.BF16 else TOL_F32, f"static vs oracle {case}")


def test_static_scratch_rejects_what_does_not_fit():
    import torch
    L = wl.LAYERS["cfg4_vgg_early"]                       # 115.6 MB of product
    d = B.desc(L.n, L.c, L.h, L.w, L.m, L.k, L.pad)
    assert B.conv_mcmk_workspace_bytes(d, B.KN2ROW_2PASS) > B.STATIC_SCRATCH_BYTES
    buf = torch.zeros(1 << 20, device="cuda")
    with pytest.raises(B.ConvMcmkError) as e:
        B.conv_mcmk_kn2row_2pass_static(d, buf, buf, buf)
    assert e.value.code == B.ERR_WORKSPACE
    with pytest.raises(B.ConvMcmkError) as e:
        B.conv_mcmk_kn2row_2pass_static(B.desc(1, 4, 8, 8, 4, 3, 1), None, buf, buf)
    assert e.value.code == B.ERR_NULL
