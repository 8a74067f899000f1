"""Fits the constants of the tile-cost estimate to the timing tables written by sweep_tiles (no GPU needed) and
rewrites csrc/selector_constants.h.

    python -m paper_1704_04428_amd.tuning.fit [--iterations 4000] [--seed 1] [--write]

One set of constants per operand type and layout, each fitted on its own rows of selector_fit*.json and
selector_network.json (random layers and the layers of the networks the paper draws from, every menu entry timed).
What is minimised is what the selector is for: the time lost by picking the entry with the lowest estimate instead of
the fastest one (squared, so that a few large losses count for more than many small ones), plus the squared log error
of the estimates of the entries near the best one, which keeps the constants meaningful where picks are already right.
Random multiplicative steps on one to three constants at a time, kept when the objective falls.  The held-out table
(tests/fixtures/selector_heldout.json) is only scored, never fitted to.
"""
from __future__ import annotations

import argparse
import json
import math
import os
import random

from paper_1704_04428_amd.tuning import cost_model as cm

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(os.path.dirname(HERE))
FIT_TABLES = [os.path.join(HERE, name) for name in ("selector_fit.json", "selector_fit2.json", "selector_fit3.json", "selector_network.json")]
HELDOUT = os.path.join(ROOT, "tests", "fixtures", "selector_heldout.json")

# constants that are not fitted: the data holds no strided layer, and the caps are structural
FROZEN = {"stride2", "reuse_a_cap", "type_scale"}
FP32_UNUSED = {"reuse_a0", "reuse_a1", "reuse_b", "extra_wg_alone", "extra_wg_16", "partial_out", "out_write_rb2"}
BF16_UNUSED = {"stage_partial"}
UPPER = {"pipe_multi": 1.0, "pipe_single": 1.0}


def load(paths):
    rows = []
    for path in paths:
        if os.path.exists(path):
            rows += json.load(open(path))["rows"]
    return rows


def regime_of(row):
    return (2 if row["dtype"] == "bf16" else 0) + (1 if row["variant"] == "kn2col" else 0)


# the benchmark configurations that occur in the tables (VGG-like layers) count ten-fold: whatever else the constants
# trade off, the headline layers keep the entry that measured fastest
BENCHMARK_LAYERS = {(1, 64, 224, 64, 3), (8, 256, 56, 256, 3), (8, 512, 28, 512, 3), (8, 512, 14, 512, 3)}


def prepared(rows, regime):
    out = []
    for row in rows:
        if regime_of(row) != regime:
            continue
        layer = tuple(row["layer"])
        cands = [(key, cm.parse_key(key), us) for key, us in row["us"].items()]
        best = min(us for _, _, us in cands)
        out.append((layer, cands, best, 10.0 if layer in BENCHMARK_LAYERS else 1.0))
    return out


def objective(data, P, bf16, channels_last):
    total = 0.0
    for layer, cands, best, row_weight in data:
        pick_us, pick_cost, pick_wgs, err, weight = None, None, None, 0.0, 0.0
        n, c, h, m, k = layer
        for key, cand, us in cands:
            est = cm.tile_cost(layer, cand, bf16, channels_last, P)
            w = math.exp(-(us / best - 1.0) / 0.25)
            err += w * math.log(est / us) ** 2
            weight += w
            if not cm.allowed(layer, cand, bf16):
                continue
            th, tw, wm, wp, rb, kg, cs = cand
            wgs = n * cm.cd(h, tw) * cm.cd(h, th) * cm.cd(cm.cd(m, 16), wm * rb) * cs
            if pick_cost is None or est < pick_cost - 1e-6 or (abs(est - pick_cost) <= 1e-6 and wgs > pick_wgs):
                pick_us, pick_cost, pick_wgs = us, est, wgs
        loss = pick_us / best - 1.0
        total += row_weight * (25.0 * loss * loss + err / weight)
    return total / max(1, len(data))


def losses(data, P, bf16, channels_last):
    out = []
    for layer, cands, best, _ in data:
        key = cm.pick(layer, [k for k, _, _ in cands], bf16, channels_last, P)
        out.append(dict((k, us) for k, _, us in cands)[key] / best - 1.0)
    return out


def summary(tag, ls):
    ls = sorted(ls)
    return (f"{tag}: {len(ls)} layers, mean loss {100 * sum(ls) / len(ls):.1f} %, over 5 %: {sum(l > 0.05 for l in ls)}, "
            f"over 15 %: {sum(l > 0.15 for l in ls)}, worst {100 * ls[-1]:.0f} %")


def fit_regime(regime, names, start, data, iterations, rng):
    bf16, channels_last = regime >= 2, regime % 2 == 1
    unused = BF16_UNUSED if bf16 else FP32_UNUSED
    free = [i for i, name in enumerate(names) if name not in FROZEN and name not in unused and start[i] != 0.0]
    cur = list(start)
    best_obj = objective(data, dict(zip(names, cur)), bf16, channels_last)
    for it in range(iterations):
        sigma = 0.3 * (0.1 ** (it / max(1, iterations - 1)))            # 0.3 -> 0.03
        trial = list(cur)
        for i in rng.sample(free, rng.choice((1, 1, 2, 3))):
            trial[i] = cur[i] * math.exp(rng.gauss(0.0, sigma))
            if names[i] in UPPER:
                trial[i] = min(trial[i], UPPER[names[i]])
        obj = objective(data, dict(zip(names, trial)), bf16, channels_last)
        if obj < best_obj:
            cur, best_obj = trial, obj
    return cur, best_obj


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--iterations", type=int, default=4000)
    ap.add_argument("--seed", type=int, default=1)
    ap.add_argument("--write", action="store_true", help="rewrite csrc/selector_constants.h with the fitted constants")
    args = ap.parse_args()
    names, values = cm.read_header()
    fit_rows, held_rows = load(FIT_TABLES), load([HELDOUT])
    rng = random.Random(args.seed)
    fitted = []
    for regime in range(4):
        bf16, channels_last = regime >= 2, regime % 2 == 1
        data, held = prepared(fit_rows, regime), prepared(held_rows, regime)
        before = dict(zip(names, values[regime]))
        print(summary(f"{cm.REGIMES[regime]} fit set, before", losses(data, before, bf16, channels_last)))
        print(summary(f"{cm.REGIMES[regime]} held out, before", losses(held, before, bf16, channels_last)))
        new, obj = fit_regime(regime, names, values[regime], data, args.iterations, rng)
        after = dict(zip(names, new))
        print(summary(f"{cm.REGIMES[regime]} fit set, after ", losses(data, after, bf16, channels_last)), f"(objective {obj:.4f})")
        print(summary(f"{cm.REGIMES[regime]} held out, after ", losses(held, after, bf16, channels_last)), flush=True)
        fitted.append(new)
    if args.write:
        cm.write_header(names, fitted)
        print("wrote", cm.HEADER)


if __name__ == "__main__":
    main()
