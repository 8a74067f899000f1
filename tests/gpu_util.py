"""Helpers for the GPU parity tests: run one variant through the C ABI with guard bands around the
output and the workspace, and compare with the oracle under the stated error bound."""
import sys

import numpy as np

from paper_1704_04428_amd import binding as B

GUARD = 4096          # bytes of canary on each side
CANARY = 0x5A
TOL_F32 = 1e-4        # |gpu - oracle| <= TOL * sum|K||I| per output element (fp32 operands)
TOL_BF16 = 1e-2       # same norm, bf16 operands, oracle on the un-rounded inputs


def announce(*what):
    print("[gpu-case]", *what, flush=True)
    sys.stdout.flush()


class Guarded:
    """A device byte buffer with canaries before and after the payload."""

    def __init__(self, nbytes, device="cuda"):
        import torch
        self.nbytes = nbytes
        self.raw = torch.full((nbytes + 2 * GUARD,), CANARY, dtype=torch.uint8, device=device)
        self.payload = self.raw[GUARD:GUARD + nbytes]

    def intact(self):
        head = self.raw[:GUARD]
        tail = self.raw[GUARD + self.nbytes:]
        return bool((head == CANARY).all().item()) and bool((tail == CANARY).all().item())


def run_variant(variant, I, K, pad, dtype=B.F32, return_ws=False, stride=1, epilogue=None, one_by_one=False, matrix_only=False):
    """I [N][C][H][W] float32 numpy, K [M][C][k][k] float32 numpy -> O float32 numpy via the C ABI.
    epilogue = (bias [M] float32 numpy or None, relu) routes the call through the *_bias_relu entry
    point of the variant (kn2row / kn2col); one_by_one = True through conv_mcmk_1x1."""
    import torch
    n, c, h, w = I.shape
    m, _, k, _ = K.shape
    d = B.desc(n, c, h, w, m, k, pad, stride, dtype)
    rc = B.conv_mcmk_check(d, variant)
    if rc != B.OK:
        raise B.ConvMcmkError(rc, B.strerror(rc))
    q, p = (h + 2 * pad - k) // stride + 1, (w + 2 * pad - k) // stride + 1
    dev = torch.device("cuda:0")
    channels_last = variant in B.CHANNELS_LAST
    if channels_last:
        I = I.transpose(0, 2, 3, 1)                      # the library sees I[N][H][W][C]
    I_dev = torch.from_numpy(np.ascontiguousarray(I)).to(dev)
    K_dev = torch.from_numpy(np.ascontiguousarray(K)).to(dev)
    if dtype == B.BF16:
        I_bf = torch.empty(I_dev.shape, dtype=torch.bfloat16, device=dev)
        B.conv_mcmk_cvt_f32_bf16(I_dev, I_bf)
        I_dev = I_bf
    if variant == B.DIRECT:
        kern = K_dev
    else:
        kp = Guarded(B.conv_mcmk_packed_kernel_bytes(d, variant))
        B.conv_mcmk_prepack(d, variant, K_dev, kp.payload)
        kern = kp.payload
    out = Guarded(n * m * q * p * 4)
    ws_bytes = B.conv_mcmk_workspace_bytes(d, variant)
    # the matrix a staged variant keeps in its workspace; im2col / im2row may ask for room behind it (copies of the
    # result for the parts of a split contraction) and must also run, on atomics, when given the matrix alone
    matrix_bytes = {B.KN2ROW_2PASS: n * k * k * m * h * w * 4, B.IM2COL: n * c * k * k * q * p * (2 if dtype == B.BF16 else 4),
                    B.IM2ROW: n * c * k * k * q * p * (2 if dtype == B.BF16 else 4)}.get(variant, 0)
    assert ws_bytes >= matrix_bytes
    if matrix_only:
        ws_bytes = matrix_bytes
    ws = Guarded(ws_bytes) if ws_bytes else None
    if epilogue is not None:
        bias, relu = epilogue
        bias_dev = torch.from_numpy(np.ascontiguousarray(bias, dtype=np.float32)).to(dev) if bias is not None else None
        fn = {B.KN2ROW: B.conv_mcmk_kn2row_bias_relu, B.KN2COL: B.conv_mcmk_kn2col_bias_relu}[variant]
        fn(d, I_dev, kern, bias_dev, relu, out.payload)
    elif one_by_one:
        assert variant == B.KN2ROW
        B.conv_mcmk_1x1(d, I_dev, kern, out.payload)
    else:
        B.RUNNERS[variant](d, I_dev, kern, out.payload, ws.payload if ws else None)
    torch.cuda.synchronize()
    assert out.intact(), "output guard band overwritten"
    if ws is not None:
        assert ws.intact(), "workspace guard band overwritten"
    if variant != B.DIRECT:
        assert kp.intact(), "packed-kernel guard band overwritten"
    if channels_last:                                    # O[N][Q][P][M] back to the oracle's [N][M][Q][P]
        O = np.ascontiguousarray(out.payload.view(torch.float32).reshape(n, q, p, m).cpu().numpy().transpose(0, 3, 1, 2))
    else:
        O = out.payload.view(torch.float32).reshape(n, m, q, p).cpu().numpy()
    if return_ws:
        return O, (ws.payload[:matrix_bytes].cpu().numpy() if ws is not None else None)
    return O


def assert_within_bound(got, ref, absref, tol, what=""):
    got = np.asarray(got, dtype=np.float64)
    err = np.abs(got - ref)
    bound = tol * absref
    bad = err > bound
    if bad.any():
        idx = np.unravel_index(np.argmax(err - bound), err.shape)
        raise AssertionError(
            f"{what}: {int(bad.sum())} of {bad.size} outputs outside {tol:g} * sum|K||I|; worst at {idx}: "
            f"got {got[idx]!r}, oracle {ref[idx]!r}, bound {bound[idx]!r}")
    assert np.all(np.isfinite(got)), f"{what}: non-finite output"
