"""Scores the selector against a table written by sweep_tiles (no GPU needed): for every row the tile the library
would pick now, its measured time and the best measured time.

    python -m paper_1704_04428_amd.tuning.score tests/fixtures/selector_heldout.json [--worst 15] [--estimates]
"""
from __future__ import annotations

import argparse
import json

from paper_1704_04428_amd import binding as B
from paper_1704_04428_amd.tuning.sweep_tiles import MENU_INDICES, MENU_ONLY, plan_key

VARIANTS = {"kn2row": B.KN2ROW, "kn2col": B.KN2COL}
DTYPES = {"f32": B.F32, "bf16": B.BF16}


def pick(row):
    n, c, h, m, k = row["layer"]
    d = B.desc(n, c, h, h, m, k, k // 2, 1, DTYPES[row["dtype"]])
    B.conv_mcmk_force_tile(MENU_ONLY)
    try:
        return plan_key(B.conv_mcmk_describe_plan(d, VARIANTS[row["variant"]]))
    finally:
        B.conv_mcmk_force_tile(-1)


def estimates(row):
    """{tile key: the library's estimate in microseconds} for every menu entry the layer can use."""
    n, c, h, m, k = row["layer"]
    d = B.desc(n, c, h, h, m, k, k // 2, 1, DTYPES[row["dtype"]])
    out = {}
    for index in MENU_INDICES:
        B.conv_mcmk_force_tile(index)
        text = B.conv_mcmk_describe_plan(d, VARIANTS[row["variant"]])
        key = plan_key(text)
        if key not in out:
            out[key] = float(text.rsplit("est ", 1)[1].split(" us")[0])
    B.conv_mcmk_force_tile(-1)
    return out


def score(rows):
    """[(loss, row, picked key, best key)], loss = time of the pick / best time - 1; a pick that was not timed counts
    as infinitely bad."""
    out = []
    for row in rows:
        p = pick(row)
        best = min(row["us"], key=row["us"].get)
        loss = row["us"][p] / row["us"][best] - 1.0 if p in row["us"] else float("inf")
        out.append((loss, row, p, best))
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("table")
    ap.add_argument("--worst", type=int, default=12)
    ap.add_argument("--estimates", action="store_true", help="for the worst rows, list estimate and measurement of every entry")
    args = ap.parse_args()
    rows = json.load(open(args.table))["rows"]
    scored = score(rows)
    for dtype in DTYPES:
        for variant in VARIANTS:
            sel = [s for s in scored if s[1]["dtype"] == dtype and s[1]["variant"] == variant]
            if not sel:
                continue
            losses = sorted(s[0] for s in sel)
            print(f"{dtype} {variant}: {len(sel)} layers, mean loss {100 * sum(losses) / len(losses):.1f} %, "
                  f"over 5 %: {sum(l > 0.05 for l in losses)}, over 15 %: {sum(l > 0.15 for l in losses)}, worst {100 * losses[-1]:.0f} %")
    for loss, row, p, best in sorted(scored, key=lambda s: -s[0])[:args.worst]:
        print(f"  {100 * loss:5.0f} %  {row['layer']} {row['dtype']} {row['variant']}: picked {p} ({row['us'].get(p)} us), best {best} ({row['us'][best]} us)")
        if args.estimates:
            est = estimates(row)
            for key, us in sorted(row["us"].items(), key=lambda kv: kv[1]):
                print(f"            {key:28s} measured {us:8.1f}  estimate {est.get(key, float('nan')):8.1f}")


if __name__ == "__main__":
    main()
