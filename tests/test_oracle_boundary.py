"""The oracle's own C boundary (oracle/conv_oracle.h): the descriptor-taking entry points called directly
through ctypes, and the pinned cases run through a host program built with AddressSanitizer and
UndefinedBehaviorSanitizer.  No GPU; nothing here touches the HIP library."""
import ctypes
import glob
import json
import os
import re
import subprocess

import numpy as np
import pytest

import oracle
from oracle import build as oracle_build
from paper_1704_04428_amd import workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _goldens(golden_dir):
    for path in sorted(glob.glob(os.path.join(golden_dir, "*.json"))):
        with open(path) as f:
            g = json.load(f)
        I = np.array(g["I"], dtype=np.float32)
        K = np.array(g["K"], dtype=np.float32)
        if I.ndim == 3:
            I = I[None]
        O = np.array(g["O"], dtype=np.float64)
        yield path, I, K, g["pad"], g.get("stride", 1), O.reshape((I.shape[0], K.shape[0]) + O.shape[-2:])


def test_header_declares_what_the_library_exports():
    with open(os.path.join(ROOT, "oracle", "conv_oracle.h")) as f:
        text = re.sub(r"/\*.*?\*/", "", f.read(), flags=re.S)
    names = sorted(set(re.findall(r"\b(conv_mcmk_oracle_[a-z0-9_]+)\s*\(", text)))
    assert names == ["conv_mcmk_oracle_f64", "conv_mcmk_oracle_f64_at"]
    lib = ctypes.CDLL(oracle_build.build(force=False))
    for name in names:
        assert getattr(lib, name) is not None
    assert "hip" not in text.lower()


def test_descriptor_entry_point_gives_the_hand_worked_values(golden_dir):
    """conv_mcmk_oracle_f64(desc, I, K, O, absO) called as a C program would, on the hand-worked examples."""
    lib = ctypes.CDLL(oracle_build.build(force=False))
    fp, dp = ctypes.POINTER(ctypes.c_float), ctypes.POINTER(ctypes.c_double)
    lib.conv_mcmk_oracle_f64.argtypes = [ctypes.POINTER(oracle.OracleDesc), fp, fp, dp, dp]
    lib.conv_mcmk_oracle_f64.restype = ctypes.c_int
    seen = 0
    for path, I, K, pad, stride, want in _goldens(golden_dir):
        n, c, h, w = I.shape
        m, _, k, _ = K.shape
        d = oracle.OracleDesc(n, c, h, w, m, k, pad, stride)
        O = np.full(want.shape, np.nan)
        I, K = np.ascontiguousarray(I), np.ascontiguousarray(K)
        rc = lib.conv_mcmk_oracle_f64(ctypes.byref(d), I.ctypes.data_as(fp), K.ctypes.data_as(fp), O.ctypes.data_as(dp), None)
        assert rc == 0, path
        np.testing.assert_array_equal(O, want, err_msg=path)
        seen += 1
    assert seen >= 4
    # errors are codes and nothing is written
    d = oracle.OracleDesc(1, 1, 2, 2, 1, 5, 0, 1)                      # empty output
    O = np.full(4, 7.0)
    z = np.zeros(25, dtype=np.float32)
    assert lib.conv_mcmk_oracle_f64(ctypes.byref(d), z.ctypes.data_as(fp), z.ctypes.data_as(fp), O.ctypes.data_as(dp), None) == 1
    assert (O == 7.0).all()
    assert lib.conv_mcmk_oracle_f64(None, z.ctypes.data_as(fp), z.ctypes.data_as(fp), O.ctypes.data_as(dp), None) == 1
    d = oracle.OracleDesc(1, 1, 3, 3, 1, 3, 1, 1)
    assert lib.conv_mcmk_oracle_f64(ctypes.byref(d), None, z.ctypes.data_as(fp), O.ctypes.data_as(dp), None) == 1


def _case_text(I, K, pad, stride, pts):
    n, c, h, w = I.shape
    m, _, k, _ = K.shape
    head = f"{n} {c} {h} {w} {m} {k} {pad} {stride} {len(pts)}"
    body = " ".join(repr(float(v)) for v in I.ravel()) + "\n" + " ".join(repr(float(v)) for v in K.ravel())
    return head + "\n" + body + "\n" + " ".join(str(int(v)) for v in np.asarray(pts, dtype=np.int64).ravel()) + "\n"


def _parse(out):
    tokens = out.split()
    pos, results = 0, []
    while pos < len(tokens):
        assert tokens[pos] == "rc"
        rc, count = int(tokens[pos + 1]), int(tokens[pos + 2])
        pos += 3
        vals = np.array(tokens[pos:pos + 2 * count], dtype=np.float64)
        pos += 2 * count
        assert tokens[pos] == "at"
        rc_at, npts = int(tokens[pos + 1]), int(tokens[pos + 2])
        pos += 3
        at = np.array(tokens[pos:pos + 2 * npts], dtype=np.float64)
        pos += 2 * npts
        results.append((rc, vals[:count], vals[count:], rc_at, at[:npts], at[npts:]))
    return results


def test_pins_hold_under_address_and_undefined_behaviour_sanitizers(golden_dir):
    """The hand-worked examples, a delta kernel in a corner tap with pad k-1 (every index reaches the image
    border from outside), a strided constant-input case and two rejected shapes, through the oracle built
    with -fsanitize=address,undefined: the values must be the pinned ones and the sanitizers must stay silent."""
    try:
        exe = oracle_build.build_sanitized()
    except (subprocess.CalledProcessError, FileNotFoundError) as e:      # no sanitizer runtime in this image
        pytest.skip(f"cannot build with sanitizers: {e}")
    text, want = "", []
    for path, I, K, pad, stride, O in _goldens(golden_dir):
        pts = [(0, 0, 0, 0), (I.shape[0] - 1, K.shape[0] - 1, O.shape[2] - 1, O.shape[3] - 1)]
        text += _case_text(I, K, pad, stride, pts)
        want.append(("golden " + os.path.basename(path), 0, O, 0, np.array([O[p] for p in pts])))
    # delta kernel at tap (0, 2) of a 3 x 3 kernel, pad 2: O[q][p] = I[q - 2][p] (zero outside)
    I = wl.uniform(91, 2 * 4 * 5, -1.0, 1.0).reshape(1, 2, 4, 5)
    K = np.zeros((1, 2, 3, 3), dtype=np.float32)
    K[0, 1, 0, 2] = 1.0
    O = np.zeros((1, 1, 6, 7))
    O[0, 0, 2:6, 0:5] = I[0, 1].astype(np.float64)
    text += _case_text(I, K, 2, 1, [(0, 0, 5, 6)])
    want.append(("delta", 0, O, 0, np.array([O[0, 0, 5, 6]])))
    # constant input a, constant kernel b, stride 2, k 3, pad 1 on 5 x 5: a b C |R(q)| |R'(p)| at the kept positions
    a, b, c = 0.5, 0.25, 3
    I = np.full((1, c, 5, 5), a, dtype=np.float32)
    K = np.full((2, c, 3, 3), b, dtype=np.float32)
    cnt = np.array([2, 3, 2], dtype=np.float64)                            # rows 0, 2, 4 of a 5-row image
    O = np.broadcast_to(a * b * c * cnt[:, None] * cnt[None, :], (1, 2, 3, 3)).copy()
    text += _case_text(I, K, 1, 2, [(0, 1, 2, 2)])
    want.append(("constant stride 2", 0, O, 0, np.array([O[0, 1, 2, 2]])))
    # rejected: empty output; a point outside the output (whole output fine, selection refused)
    text += _case_text(np.zeros((1, 1, 2, 2), np.float32), np.zeros((1, 1, 5, 5), np.float32), 0, 1, [])
    want.append(("empty output", 1, None, 1, None))
    text += _case_text(np.ones((1, 1, 2, 2), np.float32), np.ones((1, 1, 1, 1), np.float32), 0, 1, [(0, 0, 2, 0)])
    want.append(("point outside", 0, np.ones((1, 1, 2, 2)), 2, None))
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:verify_asan_link_order=0", UBSAN_OPTIONS="print_stacktrace=1")
    env.pop("LD_PRELOAD", None)                                             # the sanitizer runtime must come first
    done = subprocess.run([exe], input=text, capture_output=True, text=True, timeout=120, env=env)
    assert done.returncode == 0, done.stderr[-2000:]
    assert "Sanitizer" not in done.stderr and "runtime error" not in done.stderr, done.stderr[-2000:]
    got = _parse(done.stdout)
    assert len(got) == len(want)
    for (what, rc, O, rc_at, at), (g_rc, g_O, g_A, g_rc_at, g_at, _) in zip(want, got):
        assert (g_rc, g_rc_at) == (rc, rc_at), what
        if O is not None:
            np.testing.assert_allclose(g_O, O.ravel(), rtol=0, atol=1e-15, err_msg=what)
            assert (g_A >= np.abs(g_O) - 1e-15).all(), what
        if at is not None:
            np.testing.assert_allclose(g_at, at, rtol=0, atol=1e-15, err_msg=what)
