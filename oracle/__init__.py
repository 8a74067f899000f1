"""CPU oracle for MCMK convolution: TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's cpu_baseline leg may import this
package.  It imports nothing from the GPU package and the GPU package imports
nothing from here.

  mcmk(I, K, pad, stride=1)              whole output in float64 (+ sum |K||I| per element)
  mcmk_at(I, K, pad, points, stride=1)   selected outputs
  bias_relu(O, bias, relu)               the per-kernel offset and the rectifier applied to an output
  oracle.steps                 the im2col and kn2row algorithms step by step (numpy, float64)
"""
from __future__ import annotations

import ctypes
import os

import numpy as np

from . import build as _build

_lib = None


class OracleDesc(ctypes.Structure):
    """conv_oracle_desc of oracle/conv_oracle.h."""
    _fields_ = [(name, ctypes.c_int) for name in ("n", "c", "h", "w", "m", "k", "pad", "stride")]


def _load():
    global _lib
    if _lib is None:
        path = _build.build(force=False)
        lib = ctypes.CDLL(path)
        i = ctypes.c_int
        fp = ctypes.POINTER(ctypes.c_float)
        dp = ctypes.POINTER(ctypes.c_double)
        ip = ctypes.POINTER(ctypes.c_int)
        desc = ctypes.POINTER(OracleDesc)
        lib.conv_mcmk_oracle_f64.argtypes = [desc, fp, fp, dp, dp]
        lib.conv_mcmk_oracle_f64.restype = i
        lib.conv_mcmk_oracle_f64_at.argtypes = [desc, fp, fp, i, ip, dp, dp]
        lib.conv_mcmk_oracle_f64_at.restype = i
        _lib = lib
    return _lib


def _as4d(I):
    I = np.ascontiguousarray(I, dtype=np.float32)
    if I.ndim == 3:
        I = I[None]
    if I.ndim != 4:
        raise ValueError("input must be [C][H][W] or [N][C][H][W]")
    return I


def _check(I, K):
    K = np.ascontiguousarray(K, dtype=np.float32)
    if K.ndim != 4 or K.shape[2] != K.shape[3]:
        raise ValueError("kernel must be [M][C][k][k]")
    if K.shape[1] != I.shape[1]:
        raise ValueError("input and kernel disagree on the number of channels")
    return K


def _f(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_float))


def _d(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def mcmk(I, K, pad, stride=1):
    """Eq. 1-3 evaluated directly.  Returns (O, absO), both float64 [N][M][Q][P]
    (batch axis dropped when I is 3-D); absO = sum of |K||I| over the same terms."""
    squeeze = np.ndim(I) == 3
    I = _as4d(I)
    K = _check(I, K)
    n, c, h, w = I.shape
    m, _, k, _ = K.shape
    if h + 2 * pad - k + 1 < 1 or w + 2 * pad - k + 1 < 1 or stride < 1:
        raise ValueError("empty output")
    q, p = (h + 2 * pad - k) // stride + 1, (w + 2 * pad - k) // stride + 1
    O = np.empty((n, m, q, p), dtype=np.float64)
    A = np.empty_like(O)
    d = OracleDesc(n, c, h, w, m, k, pad, stride)
    rc = _load().conv_mcmk_oracle_f64(ctypes.byref(d), _f(I), _f(K), _d(O), _d(A))
    if rc:
        raise ValueError(f"oracle rejected the shape (code {rc})")
    return (O[0], A[0]) if squeeze else (O, A)


def mcmk_at(I, K, pad, points, stride=1):
    """Selected outputs: points is [npts][4] of (n, m, q, p).  Returns (O, absO), float64 [npts]."""
    I = _as4d(I)
    K = _check(I, K)
    n, c, h, w = I.shape
    m, _, k, _ = K.shape
    pts = np.ascontiguousarray(points, dtype=np.int32).reshape(-1, 4)
    O = np.empty(len(pts), dtype=np.float64)
    A = np.empty_like(O)
    d = OracleDesc(n, c, h, w, m, k, pad, stride)
    rc = _load().conv_mcmk_oracle_f64_at(ctypes.byref(d), _f(I), _f(K), len(pts),
                                         pts.ctypes.data_as(ctypes.POINTER(ctypes.c_int)), _d(O), _d(A))
    if rc:
        raise ValueError(f"oracle rejected the request (code {rc})")
    return O, A


def bias_relu(O, bias=None, relu=False):
    """What commonly follows the convolution in a network layer (not part of the paper's method, which
    stops at Eq. 3): add bias[m] to every element of plane m of O[...][M][Q][P], then clamp negative
    values to zero.  float64 in, float64 out."""
    O = np.asarray(O, dtype=np.float64)
    if bias is not None:
        O = O + np.asarray(bias, dtype=np.float64).reshape((-1, 1, 1))
    if relu:
        O = np.maximum(O, 0.0)
    return O
