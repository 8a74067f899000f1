"""Python replica of the library's tile-cost estimate (csrc/conv_mcmk.hip, tile_cost) for fitting its constants
without a GPU.  The constants are read from csrc/selector_constants.h, the same file the library is compiled from;
tests/test_selector_fixture.py checks that this replica and the library give the same estimates."""
from __future__ import annotations

import os
import re

HERE = os.path.dirname(os.path.abspath(__file__))
HEADER = os.path.join(os.path.dirname(HERE), "csrc", "selector_constants.h")
NUM_CU = 256
REGIMES = ("f32 kn2row", "f32 kn2col", "bf16 kn2row", "bf16 kn2col")     # the order of kCost[] in the header


def read_header(path=HEADER):
    """(field names, [four lists of values]) from the header."""
    text = open(path).read()
    struct = text[text.index("struct CostParams {"):text.index("};", text.index("struct CostParams {"))]
    names = re.findall(r"^\s*double (\w+);", struct, flags=re.M)
    table = text[text.index("kCost[4] = {"):]
    rows = re.findall(r"^\s*\{([^{}]*)\},\s*$", table, flags=re.M)
    values = [[float(v) for v in row.split(",")] for row in rows]
    assert len(values) == 4 and all(len(v) == len(names) for v in values), "selector_constants.h: unexpected layout"
    return names, values


def write_header(names, values, path=HEADER):
    text = open(path).read()
    head = text[:text.index("constexpr CostParams kCost[4] = {")]
    rows = "".join("    {" + ", ".join(("%.6g" % v) for v in row) + "},\n" for row in values)
    open(path, "w").write(head + "constexpr CostParams kCost[4] = {\n" + rows + "};\n\n}  // namespace mcmk\n")


def params(regime_index, names=None, values=None):
    if names is None:
        names, values = read_header()
    return dict(zip(names, values[regime_index]))


def cd(a, b):
    return -(-a // b)


def parse_key(key):
    """'14x14/4x2/rb1/kg1/cs1' -> (th, tw, wm, wp, rb, kg, cs)."""
    tile, waves, rb, kg, cs = key.split("/")
    th, tw = map(int, tile.split("x"))
    wm, wp = map(int, waves.split("x"))
    return th, tw, wm, wp, int(rb[2:]), int(kg[2:]), int(cs[2:])


def lean_applies(layer, cand, bf16, channels_last):
    n, c, h, m, k = layer
    th, tw, wm, wp, rb, kg, cs = cand
    shape_ok = (th, tw, wm, wp) in ((14, 14, 4, 2), (16, 16, 4, 2), (16, 16, 2, 4)) and rb == 1 and kg == 1
    return (not bf16) and c <= 4 and not channels_last and cs == 1 and k in (3, 5, 7) and shape_ok


def tile_cost(layer, cand, bf16, channels_last, P):
    """Estimated microseconds of candidate `cand` on `layer` = (n, c, h, m, k), square image, pad k // 2, unit stride."""
    n, c, h, m, k = layer
    th, tw, wm, wp, rb, kg, cs = cand
    q = p = h + 2 * (k // 2) - k + 1
    mb = cd(m, 16)
    wgs = n * cd(p, tw) * cd(q, th) * cd(mb, wm * rb) * cs
    npb = cd(th * tw, 16)
    group_waves = wm * wp
    waves = group_waves * kg
    simd = [0, 0, 0, 0]
    rem, pbw = npb % wp, cd(npb, wp)
    for w in range(waves):
        g = w // group_waves
        wpi = ((w % group_waves + g * wm) % group_waves) // wm
        simd[w % 4] += rb * (pbw if (rem == 0 or wpi < rem) else pbw - 1)
    simd_load, simd_sum = max(simd), sum(simd)
    chunks = cd(cd(cd(c, 32 if bf16 else 16), cs), kg)
    lean = lean_applies(layer, cand, bf16, channels_last)
    steps = chunks * k * k * (0.5 if bf16 else 1.0 if lean else 4.0)
    per_cu = cd(wgs, NUM_CU)
    can_hold = max(1, (8 if bf16 else 16) // waves)
    if bf16 and rb == 2 and wp == 1 and th * tw > 128:
        can_hold = 1
    halo = (th - 1 + k) * (tw - 1 + k)
    if not bf16:
        fit = 163840 // (2 * kg * 16 * (((halo + 15) // 32) * 32 + 16) * 4)
        can_hold = max(1, min(can_hold, fit))
    held = min(per_cu, can_hold)
    pipe_use = (P["pipe_multi"] if held * waves / 4.0 >= 2.0 else P["pipe_single"]) * P["type_scale"]
    if bf16:
        reuse_a = min(P["reuse_a_cap"], P["reuse_a0"] + P["reuse_a1"] * cd(npb, wp))
        rows = 16.0 * wm * rb
        reuse_b = min(1.0, rows / (rows + 16.0) / P["reuse_b"])
        pipe_use *= reuse_a * reuse_b
    if k > 3:
        pipe_use *= 1.0 + P["taps_gain"] * (1.0 - 9.0 / (k * k))
    pipe_use = min(pipe_use, 1.0)
    blocks = 0.5 * simd_load + 0.125 * simd_sum if (not bf16 and held >= 2) else float(simd_load)
    us = per_cu * blocks * steps * 0.0139 / pipe_use
    floor_us = cd(per_cu, can_hold) * chunks * P["floor_chunk"] * (P["floor_small"] if th == 7 else 1.0)
    us = max(us, floor_us)
    if k == 1:
        us *= P["k1_tile256"] if th * tw == 256 else P["k1_other"]
    if bf16:
        us += per_cu * chunks * halo * kg / waves * (P["stage"] / 64.0)
    us += P["fixed"]
    if not bf16:
        us += P["stage"] * wgs * halo * (c / cs) * 4.0e-6 * (1.0 if (tw % 16 == 0 or tw >= 28) else P["stage_partial"])
        if per_cu > 1:
            us += (per_cu - 1) * P["extra_wg"] / can_hold
    elif per_cu > 1:
        us += (per_cu - 1) * (P["extra_wg_16"] if waves == 16 else P["extra_wg_alone"] if can_hold == 1 else P["extra_wg"])
    out_mb = n * m * q * p * 4.0e-6
    partial_lines = (not channels_last) and tw % 16 != 0 and tw < 28
    if bf16 and partial_lines:
        us += P["partial_out"] * out_mb
    us += (P["out_write"] + (P["out_write_rb2"] if rb == 2 else 0.0)) * out_mb
    if lean:
        us += 0.5 * 4.0 * n * m * q * p / (5.0e6 if tw % 16 == 0 else 3.3e6)
    if cs > 1:
        us += P["split_fixed"] + (P["split_mb_partial"] if partial_lines else P["split_mb"]) * out_mb * (cs / 2.0)
    if kg > 1:
        us += P["kg4"] if kg == 4 else P["kg2_16"] if waves == 16 else P["kg2"]
    return us


def allowed(layer, cand, bf16):
    """The selector's own exclusions among the entries a layer can run (search_fused): channel groups are not
    offered to 1 x 1 kernels, except fp32 layers of 256 channels or more."""
    n, c, h, m, k = layer
    kg = cand[5]
    return not (kg > 1 and k == 1 and (c < 256 or bf16))


def pick(layer, keys, bf16, channels_last, P):
    """The entry of `keys` the estimate prefers (ties: more workgroups)."""
    best, best_cost, best_wgs = None, None, None
    n, c, h, m, k = layer
    for key in keys:
        cand = parse_key(key)
        if not allowed(layer, cand, bf16):
            continue
        cost = tile_cost(layer, cand, bf16, channels_last, P)
        th, tw, wm, wp, rb, kg, cs = cand
        wgs = n * cd(h, tw) * cd(h, th) * cd(cd(m, 16), wm * rb) * cs
        if best is None or cost < best_cost - 1e-6 or (abs(cost - best_cost) <= 1e-6 and wgs > best_wgs):
            best, best_cost, best_wgs = key, cost, wgs
    return best
