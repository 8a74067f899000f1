"""Host-side checks of bench.py and the workload module: no GPU needed."""
import os
import subprocess
import sys

import numpy as np

from paper_1704_04428_amd import workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_bench_refuses_more_than_one_gpu():
    """One process, one MI355X: --gpus 2 exits with a message before anything touches a device."""
    p = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert p.returncode != 0
    assert "one GPU" in p.stderr and p.stdout.strip() == ""


def test_benchmark_layers_match_the_stated_configurations():
    """Shapes, flop counts and workspace sizes of the benchmark layers (2 M C k^2 P Q N flop per call)."""
    want = {
        "cfg1_tiny": (1, 16, 32, 32, 16, 3, 1, 4_718_592),
        "cfg2_googlenet5x5": (1, 32, 28, 28, 96, 5, 2, 120_422_400),
        "cfg3_alexnet_conv2": (1, 96, 27, 27, 256, 5, 2, 895_795_200),
        "cfg4_vgg_early": (1, 64, 224, 224, 64, 3, 1, 3_699_376_128),
        "cfg5a_vgg_deep56": (8, 256, 56, 56, 256, 3, 1, 29_595_009_024),
        "cfg5b_vgg_deep28": (8, 512, 28, 28, 512, 3, 1, 29_595_009_024),
        "cfg5c_vgg_deep14": (8, 512, 14, 14, 512, 3, 1, 7_398_752_256),
    }
    assert set(wl.LAYERS) == set(want)
    for name, (n, c, h, w, m, k, pad, flops) in want.items():
        L = wl.LAYERS[name]
        assert (L.n, L.c, L.h, L.w, L.m, L.k, L.pad, L.stride) == (n, c, h, w, m, k, pad, 1), name
        assert (L.q, L.p) == (h, w) and L.flops == flops, name
    s2 = wl.GENERALISED_LAYERS["gen_vgg56_stride2"]
    assert (s2.q, s2.p, s2.stride) == (28, 28, 2) and s2.flops == 29_595_009_024 // 4
    rgb = wl.GENERALISED_LAYERS["gen_rgb224_k7_stride2"]
    assert (rgb.c, rgb.q, rgb.p, rgb.stride) == (3, 112, 112, 2) and rgb.flops == 2 * 8 * 64 * 3 * 49 * 112 * 112
    assert wl.GENERALISED_LAYERS["gen_rgb224_k3"].flops == 2 * 8 * 64 * 3 * 9 * 224 * 224


def test_inputs_follow_the_stated_distributions():
    L = wl.LAYERS["cfg3_alexnet_conv2"]
    I, K = wl.make_input(L), wl.make_kernel(L)
    assert I.dtype == np.float32 and K.dtype == np.float32
    assert I.shape == (1, 96, 27, 27) and K.shape == (256, 96, 5, 5)
    assert 0.0 <= I.min() and I.max() < 1.0 and abs(float(I.mean()) - 0.5) < 0.01       # uniform [0, 1)
    sigma = np.sqrt(2.0 / (96 * 25))
    assert abs(float(K.std()) / sigma - 1.0) < 0.01 and abs(float(K.mean())) < 0.01 * sigma * 10
    np.testing.assert_array_equal(I, wl.make_input(L))                                  # seeded: reproducible
    t = wl.LAYERS["cfg1_tiny"]
    It = wl.make_input(t)
    assert -1.0 <= It.min() < -0.9 and 0.9 < It.max() < 1.0                             # uniform [-1, 1)
    pts = wl.sample_points(L, 100)
    assert pts.shape == (100, 4) and (pts[:, 1] < L.m).all() and (pts[:, 2] < L.q).all() and (pts[0] == 0).all()
