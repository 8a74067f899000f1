"""Times every tile shape of the fused kernels' menu on a set of layers (needs the GPU) and writes the table the
selector's constants are fitted to and checked against.

    python -m paper_1704_04428_amd.tuning.sweep_tiles --set heldout --out tests/fixtures/selector_heldout.json
    python -m paper_1704_04428_amd.tuning.sweep_tiles --set fit     --out paper_1704_04428_amd/tuning/selector_fit.json

Layer sets: "fit", "fit2", "fit3" and "heldout" are seeded draws from the same distribution of layer shapes (batch 1-16, 3-768
channels, 7-224 pixels a side, 16-512 kernels, kernel side 1-7, unit stride, 20 MFLOP to 30 GFLOP); "network" is the
layer list of the networks the paper takes its layers from, single image and batch 8.  For every layer, operand type
(f32, bf16) and layout (kn2row: [C][H][W], kn2col: channels last) each menu entry is forced in turn
(conv_mcmk_force_tile), entries the layer cannot use are skipped, and the average time per call is recorded under the
plan text the library reports for it, so that a later run of the selector can be scored against the table without a
GPU: tests/test_selector_fixture.py.
"""
from __future__ import annotations

import argparse
import json
import os
import re
import sys

import numpy as np

MENU_INDICES = list(range(34))
# An index that names no menu entry leaves the choice to the estimate, among the menu's entries alone: a 1 x 1 layer
# is then not run as a plain matrix product on the flat shape, which these tables do not time.
MENU_ONLY = 1 << 20


def plan_key(text: str) -> str:
    """'14x14/4x2/rb1/kg1/cs1' (tile, waves, row blocks per wave, channel groups, channel split) from a plan line."""
    m = re.search(r"tile (\d+x\d+), waves (\d+x\d+), row blocks (\d+), channel groups (\d+), channel split (\d+)", text)
    if not m:
        raise ValueError(f"no tile in plan text {text!r}")
    return "%s/%s/rb%s/kg%s/cs%s" % m.groups()


def random_layers(seed: int, count: int):
    rng = np.random.default_rng(seed)
    layers = []
    while len(layers) < count:
        n = int(rng.choice([1, 1, 2, 4, 8, 16]))
        c = int(rng.choice([3, 16, 24, 32, 48, 64, 96, 128, 160, 192, 256, 320, 384, 512, 768]))
        h = int(rng.choice([7, 13, 14, 17, 27, 28, 35, 56, 73, 112, 224]))
        m = int(rng.choice([16, 32, 64, 96, 128, 192, 256, 384, 512]))
        k = int(rng.choice([1, 3, 3, 5, 7]))
        flop = 2.0 * n * c * k * k * m * h * h
        if flop > 3e10 or flop < 2e7 or n * max(c, m) * h * h * 4 > 4e8:
            continue
        layers.append((n, c, h, m, k))
    return layers


NETWORK_LAYERS = [  # (C, H, M, k): AlexNet 13 x 13, GoogLeNet inception and reductions, VGG-16
    (256, 13, 384, 3), (384, 13, 384, 3), (384, 13, 256, 3), (96, 28, 128, 3), (128, 28, 192, 3), (16, 28, 32, 5),
    (96, 14, 208, 3), (112, 14, 224, 3), (160, 7, 320, 3), (192, 56, 64, 1), (64, 56, 192, 3), (480, 14, 192, 1),
    (832, 7, 384, 1), (3, 224, 64, 3), (64, 224, 64, 3), (64, 112, 128, 3), (128, 112, 128, 3), (128, 56, 256, 3),
    (256, 56, 256, 3), (256, 28, 512, 3), (512, 28, 512, 3), (512, 14, 512, 3),
]


def layer_set(name: str):
    if name == "fit":
        return random_layers(20260, 60)
    if name == "fit2":
        return random_layers(20262, 60)
    if name == "fit3":
        return random_layers(20263, 60)
    if name == "heldout":
        return random_layers(20261, 60)
    if name == "network":
        return [(n, c, h, m, k) for n in (1, 8) for (c, h, m, k) in NETWORK_LAYERS]
    raise ValueError(name)


def timed(fn, warm_ms=12.0, timed_ms=25.0):
    import torch
    for _ in range(3):
        fn()
    torch.cuda.synchronize()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record(); fn(); fn(); b.record(); torch.cuda.synchronize()
    ms = max(a.elapsed_time(b) / 2, 1e-3)
    warm, steps = max(5, int(warm_ms / ms)), max(10, int(timed_ms / ms))
    for _ in range(warm):
        fn()
    a.record()
    for _ in range(steps):
        fn()
    b.record(); torch.cuda.synchronize()
    return a.elapsed_time(b) / steps


def sweep(layers, log=sys.stderr):
    import torch
    from paper_1704_04428_amd import binding as B
    out = []
    for li, (n, c, h, m, k) in enumerate(layers):
        I = torch.rand(n, c, h, h, device="cuda")
        K = torch.randn(m, c, k, k, device="cuda") * 0.05
        for dtype_name, dtype in (("f32", B.F32), ("bf16", B.BF16)):
            for variant_name, variant in (("kn2row", B.KN2ROW), ("kn2col", B.KN2COL)):
                d = B.desc(n, c, h, h, m, k, k // 2, 1, dtype)
                if B.conv_mcmk_check(d, variant) != B.OK:
                    continue
                x = I.to(torch.bfloat16) if dtype == B.BF16 else I
                if variant == B.KN2COL:
                    x = x.permute(0, 2, 3, 1).contiguous()
                plan = B.Plan(d, variant, K)
                B.conv_mcmk_force_tile(-1)
                times = {}
                print(f"[sweep] layer {li} {(n, c, h, m, k)} {dtype_name} {variant_name}", file=log, flush=True)
                for index in MENU_INDICES:
                    B.conv_mcmk_force_tile(index)
                    key = plan_key(B.conv_mcmk_describe_plan(d, variant))
                    if key in times:
                        continue                       # an entry this layer cannot use: the estimate's own choice again
                    times[key] = round(timed(lambda: plan.run(x)) * 1e3, 3)
                B.conv_mcmk_force_tile(-1)
                out.append({"layer": [n, c, h, m, k], "dtype": dtype_name, "variant": variant_name, "us": times})
                del plan
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--set", default="heldout", choices=["fit", "fit2", "fit3", "heldout", "network"])
    ap.add_argument("--out", required=True)
    args = ap.parse_args()
    rows = sweep(layer_set(args.set))
    os.makedirs(os.path.dirname(os.path.abspath(args.out)) or ".", exist_ok=True)
    with open(args.out, "w") as f:
        json.dump({"set": args.set, "unit": "microseconds per call, average of back-to-back launches after warm-up",
                   "rows": rows}, f, indent=0, separators=(",", ":"))
    print(f"{len(rows)} rows -> {args.out}")


if __name__ == "__main__":
    main()
