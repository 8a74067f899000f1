"""Thin ctypes binding over libconv_mcmk.so: argument marshalling only.

Every function here has the name and the meaning of the C entry point in
include/conv_mcmk.h; torch tensors are used for device memory and streams and
nothing else.  There is no CPU fallback: if the HIP library has not been built
the first call raises.
"""
from __future__ import annotations

import ctypes
import os

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libconv_mcmk.so")

F32, BF16 = 0, 1
KN2ROW, KN2ROW_2PASS, IM2COL, DIRECT, KN2COL, IM2ROW = 0, 1, 2, 3, 4, 5
CHANNELS_LAST = (KN2COL, IM2ROW)       # variants that take I[N][H][W][C] and give O[N][Q][P][M]
VARIANTS = {"kn2row": KN2ROW, "kn2row_2pass": KN2ROW_2PASS, "im2col": IM2COL, "direct": DIRECT, "kn2col": KN2COL,
            "im2row": IM2ROW}

OK, ERR_NULL, ERR_SHAPE, ERR_UNSUPPORTED, ERR_WORKSPACE, ERR_DEVICE, ERR_ALIGN = range(7)
STATIC_SCRATCH_BYTES = 32 << 20        # CONV_MCMK_STATIC_SCRATCH_BYTES

EXPORTS = (
    "conv_mcmk_strerror", "conv_mcmk_check", "conv_mcmk_describe_plan", "conv_mcmk_workspace_bytes", "conv_mcmk_packed_kernel_bytes",
    "conv_mcmk_prepack", "conv_mcmk_kn2row", "conv_mcmk_kn2row_2pass", "conv_mcmk_im2col",
    "conv_mcmk_direct", "conv_mcmk_kn2col", "conv_mcmk_im2row", "conv_mcmk_cvt_f32_bf16",
    "conv_mcmk_kn2row_bias_relu", "conv_mcmk_kn2col_bias_relu", "conv_mcmk_1x1", "conv_mcmk_select", "conv_mcmk_run",
    "conv_mcmk_kn2row_2pass_static", "conv_mcmk_output_dims", "conv_mcmk_force_tile", "conv_mcmk_force_gemm_tile", "conv_mcmk_probe_mfma", "conv_mcmk_probe_copy",
)


class Desc(ctypes.Structure):
    _fields_ = [(name, ctypes.c_int32) for name in ("n", "c", "h", "w", "m", "k", "pad", "stride", "dtype")]


class ConvMcmkError(RuntimeError):
    def __init__(self, code: int, text: str):
        super().__init__(f"conv_mcmk error {code}: {text}")
        self.code = code


_lib = None


def lib():
    """Load libconv_mcmk.so (built in-tree by paper_1704_04428_amd.build); raises when it is missing."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                f"{LIB_PATH} is missing: build it with `python -m paper_1704_04428_amd.build` "
                "(there is no CPU fallback)")
        # torch first: it brings its own copy of the HIP runtime, and the device pointers and streams
        # handed to the library belong to that copy.  Loading the library before torch would bind its
        # kernels to whichever libamdhip64 the system resolves instead, and every launch would fail.
        import torch  # noqa: F401
        L = ctypes.CDLL(LIB_PATH)
        dp = ctypes.POINTER(Desc)
        vp, sz, i = ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int
        L.conv_mcmk_strerror.argtypes = [i]
        L.conv_mcmk_strerror.restype = ctypes.c_char_p
        L.conv_mcmk_check.argtypes = [dp, i]
        L.conv_mcmk_check.restype = i
        L.conv_mcmk_describe_plan.argtypes = [dp, i, ctypes.c_char_p, sz]
        L.conv_mcmk_describe_plan.restype = i
        L.conv_mcmk_workspace_bytes.argtypes = [dp, i]
        L.conv_mcmk_workspace_bytes.restype = sz
        L.conv_mcmk_packed_kernel_bytes.argtypes = [dp, i]
        L.conv_mcmk_packed_kernel_bytes.restype = sz
        L.conv_mcmk_prepack.argtypes = [dp, i, vp, vp, vp]
        L.conv_mcmk_prepack.restype = i
        for name in ("conv_mcmk_kn2row", "conv_mcmk_kn2row_2pass", "conv_mcmk_im2col", "conv_mcmk_direct",
                     "conv_mcmk_kn2col", "conv_mcmk_im2row"):
            fn = getattr(L, name)
            fn.argtypes = [dp, vp, vp, vp, vp, sz, vp]
            fn.restype = i
        for name in ("conv_mcmk_kn2row_bias_relu", "conv_mcmk_kn2col_bias_relu"):
            fn = getattr(L, name)
            fn.argtypes = [dp, vp, vp, vp, i, vp, vp]
            fn.restype = i
        L.conv_mcmk_select.argtypes = [dp, i, sz, ctypes.POINTER(ctypes.c_int), ctypes.POINTER(ctypes.c_double)]
        L.conv_mcmk_select.restype = i
        L.conv_mcmk_run.argtypes = [dp, i, vp, vp, vp, vp, sz, vp]
        L.conv_mcmk_run.restype = i
        L.conv_mcmk_1x1.argtypes = [dp, vp, vp, vp, vp]
        L.conv_mcmk_1x1.restype = i
        L.conv_mcmk_cvt_f32_bf16.argtypes = [vp, vp, sz, vp]
        L.conv_mcmk_cvt_f32_bf16.restype = i
        L.conv_mcmk_kn2row_2pass_static.argtypes = [dp, vp, vp, vp, vp]
        L.conv_mcmk_kn2row_2pass_static.restype = i
        L.conv_mcmk_output_dims.argtypes = [dp, ctypes.POINTER(ctypes.c_int), ctypes.POINTER(ctypes.c_int)]
        L.conv_mcmk_output_dims.restype = i
        L.conv_mcmk_force_tile.argtypes = [i]
        L.conv_mcmk_force_tile.restype = None
        L.conv_mcmk_force_gemm_tile.argtypes = [i]
        L.conv_mcmk_force_gemm_tile.restype = None
        L.conv_mcmk_probe_mfma.argtypes = [i, i, i, vp, vp]
        L.conv_mcmk_probe_mfma.restype = i
        L.conv_mcmk_probe_copy.argtypes = [vp, vp, sz, vp]
        L.conv_mcmk_probe_copy.restype = i
        _lib = L
    return _lib


def desc(n, c, h, w, m, k, pad, stride=1, dtype=F32) -> Desc:
    return Desc(n, c, h, w, m, k, pad, stride, dtype)


def strerror(code: int) -> str:
    return lib().conv_mcmk_strerror(code).decode()


def _raise(code: int):
    if code != OK:
        raise ConvMcmkError(code, strerror(code))


def _ptr(t):
    return ctypes.c_void_p(t.data_ptr()) if t is not None else ctypes.c_void_p(0)


def _stream(stream):
    import torch
    s = stream if stream is not None else torch.cuda.current_stream()
    return ctypes.c_void_p(s.cuda_stream)


def conv_mcmk_check(d: Desc, variant: int) -> int:
    return lib().conv_mcmk_check(ctypes.byref(d), variant)


def conv_mcmk_output_dims(d: Desc):
    """(Q, P): rows and columns of one output plane."""
    q, p = ctypes.c_int(0), ctypes.c_int(0)
    _raise(lib().conv_mcmk_output_dims(ctypes.byref(d), ctypes.byref(q), ctypes.byref(p)))
    return q.value, p.value


def conv_mcmk_force_tile(index: int) -> None:
    lib().conv_mcmk_force_tile(int(index))


def conv_mcmk_force_gemm_tile(index: int) -> None:
    lib().conv_mcmk_force_gemm_tile(int(index))


def conv_mcmk_probe_mfma(dtype: int, blocks: int, iters: int, sink, stream=None) -> None:
    _raise(lib().conv_mcmk_probe_mfma(dtype, blocks, iters, _ptr(sink), _stream(stream)))


def conv_mcmk_probe_copy(src, dst, nbytes: int, stream=None) -> None:
    _raise(lib().conv_mcmk_probe_copy(_ptr(src), _ptr(dst), nbytes, _stream(stream)))


def conv_mcmk_describe_plan(d: Desc, variant: int) -> str:
    buf = ctypes.create_string_buffer(512)
    _raise(lib().conv_mcmk_describe_plan(ctypes.byref(d), variant, buf, len(buf)))
    return buf.value.decode()


def conv_mcmk_workspace_bytes(d: Desc, variant: int) -> int:
    return lib().conv_mcmk_workspace_bytes(ctypes.byref(d), variant)


def conv_mcmk_packed_kernel_bytes(d: Desc, variant: int) -> int:
    return lib().conv_mcmk_packed_kernel_bytes(ctypes.byref(d), variant)


def conv_mcmk_prepack(d: Desc, variant: int, K, Kp, stream=None) -> None:
    _raise(lib().conv_mcmk_prepack(ctypes.byref(d), variant, _ptr(K), _ptr(Kp), _stream(stream)))


def _run(name, d, I, Kp, O, ws, stream):
    ws_bytes = ws.numel() * ws.element_size() if ws is not None else 0
    fn = getattr(lib(), name)
    _raise(fn(ctypes.byref(d), _ptr(I), _ptr(Kp), _ptr(O), _ptr(ws), ws_bytes, _stream(stream)))


def conv_mcmk_kn2row(d, I, Kp, O, ws=None, stream=None):
    _run("conv_mcmk_kn2row", d, I, Kp, O, ws, stream)


def conv_mcmk_kn2row_2pass(d, I, Kp, O, ws=None, stream=None):
    _run("conv_mcmk_kn2row_2pass", d, I, Kp, O, ws, stream)


def conv_mcmk_kn2row_2pass_static(d, I, Kp, O, stream=None):
    _raise(lib().conv_mcmk_kn2row_2pass_static(ctypes.byref(d), _ptr(I), _ptr(Kp), _ptr(O), _stream(stream)))


def conv_mcmk_im2col(d, I, Kp, O, ws=None, stream=None):
    _run("conv_mcmk_im2col", d, I, Kp, O, ws, stream)


def conv_mcmk_direct(d, I, K, O, ws=None, stream=None):
    _run("conv_mcmk_direct", d, I, K, O, ws, stream)


def conv_mcmk_kn2col(d, I, Kp, O, ws=None, stream=None):
    _run("conv_mcmk_kn2col", d, I, Kp, O, ws, stream)


def conv_mcmk_im2row(d, I, Kp, O, ws=None, stream=None):
    _run("conv_mcmk_im2row", d, I, Kp, O, ws, stream)


def conv_mcmk_kn2row_bias_relu(d, I, Kp, bias, relu, O, stream=None):
    _raise(lib().conv_mcmk_kn2row_bias_relu(ctypes.byref(d), _ptr(I), _ptr(Kp), _ptr(bias), int(relu), _ptr(O), _stream(stream)))


def conv_mcmk_kn2col_bias_relu(d, I, Kp, bias, relu, O, stream=None):
    _raise(lib().conv_mcmk_kn2col_bias_relu(ctypes.byref(d), _ptr(I), _ptr(Kp), _ptr(bias), int(relu), _ptr(O), _stream(stream)))


def conv_mcmk_1x1(d, I, Kp, O, stream=None):
    _raise(lib().conv_mcmk_1x1(ctypes.byref(d), _ptr(I), _ptr(Kp), _ptr(O), _stream(stream)))


def conv_mcmk_select(d, channels_last=False, ws_limit_bytes=2 ** 62):
    """(variant, estimated microseconds) of the cheapest variant for this layer."""
    variant, est = ctypes.c_int(-1), ctypes.c_double(0.0)
    _raise(lib().conv_mcmk_select(ctypes.byref(d), int(channels_last), ws_limit_bytes, ctypes.byref(variant), ctypes.byref(est)))
    return variant.value, est.value


def conv_mcmk_run(d, variant, I, K, O, ws=None, stream=None):
    ws_bytes = ws.numel() * ws.element_size() if ws is not None else 0
    _raise(lib().conv_mcmk_run(ctypes.byref(d), variant, _ptr(I), _ptr(K), _ptr(O), _ptr(ws), ws_bytes, _stream(stream)))


def conv_mcmk_cvt_f32_bf16(src, dst, count=None, stream=None):
    n = src.numel() if count is None else count
    _raise(lib().conv_mcmk_cvt_f32_bf16(_ptr(src), _ptr(dst), n, _stream(stream)))


RUNNERS = {KN2ROW: conv_mcmk_kn2row, KN2ROW_2PASS: conv_mcmk_kn2row_2pass, IM2COL: conv_mcmk_im2col,
           DIRECT: conv_mcmk_direct, KN2COL: conv_mcmk_kn2col, IM2ROW: conv_mcmk_im2row}


class Plan:
    """Device buffers for one layer and one variant: packed kernel, workspace and output, allocated
    once with torch; run() is a single library call on the current stream."""

    def __init__(self, d: Desc, variant: int, K_dev):
        import torch
        _raise(conv_mcmk_check(d, variant))
        self.d, self.variant = d, variant
        dev = K_dev.device
        if variant == DIRECT:
            self.kernel = K_dev
        else:
            nbytes = conv_mcmk_packed_kernel_bytes(d, variant)
            self.kernel = torch.empty(nbytes, dtype=torch.uint8, device=dev)
            conv_mcmk_prepack(d, variant, K_dev, self.kernel)
        ws_bytes = conv_mcmk_workspace_bytes(d, variant)
        self.ws = torch.empty(ws_bytes, dtype=torch.uint8, device=dev) if ws_bytes else None
        q, p = conv_mcmk_output_dims(d)
        shape = (d.n, q, p, d.m) if variant in CHANNELS_LAST else (d.n, d.m, q, p)
        self.out = torch.empty(shape, dtype=torch.float32, device=dev)

    @classmethod
    def auto(cls, d: Desc, K_dev, channels_last=False, ws_limit_bytes=2 ** 62):
        """The plan for the variant conv_mcmk_select prefers."""
        variant, _ = conv_mcmk_select(d, channels_last, ws_limit_bytes)
        return cls(d, variant, K_dev)

    def run(self, I_dev, stream=None):
        conv_mcmk_run(self.d, self.variant, I_dev, self.kernel, self.out, self.ws, stream)
        return self.out


def conv_mcmk(I, K, pad=0, stride=1, variant=None, bias=None, relu=False, channels_last=False, bf16=False):
    """One-call form for device tensors: I float32 [N][C][H][W] (or [N][H][W][C] with channels_last),
    K float32 [M][C][k][k]; returns O float32 [N][M][Q][P] (or [N][Q][P][M]).  Picks the variant with
    conv_mcmk_select unless one is named, re-orders the kernel (in a real network: once per layer, keep
    the Plan instead), converts the input to bfloat16 when bf16 is set, and applies the bias / rectifier
    epilogue of the fused variants when asked.  Every step runs in the library's kernels."""
    import torch
    if I.dim() != 4 or K.dim() != 4 or K.shape[2] != K.shape[3]:
        raise ValueError("I must be 4-D and K [M][C][k][k]")
    n = I.shape[0]
    c, h, w = (I.shape[3], I.shape[1], I.shape[2]) if channels_last else (I.shape[1], I.shape[2], I.shape[3])
    m, kc, k, _ = K.shape
    if kc != c:
        raise ValueError("input and kernel disagree on the number of channels")
    d = desc(n, c, h, w, m, k, pad, stride, BF16 if bf16 else F32)
    epilogue = bias is not None or relu
    if variant is None:
        variant = (KN2COL if channels_last else KN2ROW) if epilogue else conv_mcmk_select(d, channels_last)[0]
    if (variant in CHANNELS_LAST) != bool(channels_last):
        raise ValueError("the variant does not take this layout")
    if epilogue and variant not in (KN2ROW, KN2COL):
        raise ValueError("the bias / rectifier epilogue belongs to the fused variants")
    I = I.contiguous()
    plan = Plan(d, variant, K.contiguous())
    if bf16:
        I_bf = torch.empty(I.shape, dtype=torch.bfloat16, device=I.device)
        conv_mcmk_cvt_f32_bf16(I, I_bf)
        I = I_bf
    if epilogue:
        fn = conv_mcmk_kn2col_bias_relu if variant == KN2COL else conv_mcmk_kn2row_bias_relu
        fn(d, I, plan.kernel, bias.contiguous() if bias is not None else None, relu, plan.out)
        return plan.out
    return plan.run(I)
