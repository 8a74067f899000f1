"""The per-layer tile selector (the paper's conclusion: choose per layer) against a table of measured times: no GPU
needed.  tests/fixtures/selector_heldout.json holds, for 60 random layers per operand type and layout that the
constants were NOT fitted to, the time of every menu entry measured on an MI355X
(python -m paper_1704_04428_amd.tuning.sweep_tiles --set heldout).  The tests score the entry the library picks now
against the fastest one, and check that the Python replica of the estimate that the constants are fitted with
(paper_1704_04428_amd/tuning/cost_model.py) is the library's estimate."""
import json
import os

import pytest

from paper_1704_04428_amd import binding as B
from paper_1704_04428_amd.tuning import cost_model as cm
from paper_1704_04428_amd.tuning import score

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HELDOUT = os.path.join(ROOT, "tests", "fixtures", "selector_heldout.json")
MAX_LOSS = 0.15          # a pick may be this much slower than the fastest entry of its layer
# ... except on held-out layers named here with a bound of their own, where the estimate is known to miss (none at
# present: the 1 x 1 layer on 27 x 27 images that was listed -- 16 x 16 tiles estimated ahead of quarter tiles 20 %
# faster -- is picked right by the present constants)
KNOWN_MISSES = {}


@pytest.fixture(scope="module")
def heldout():
    if not os.path.exists(B.LIB_PATH):
        from paper_1704_04428_amd import build
        build.build()
    B.lib()
    with open(HELDOUT) as f:
        return json.load(f)["rows"]


def test_table_covers_sixty_layers_per_type_and_layout(heldout):
    for dtype in ("f32", "bf16"):
        assert sum(r["dtype"] == dtype and r["variant"] == "kn2row" for r in heldout) >= 60
        assert sum(r["dtype"] == dtype and r["variant"] == "kn2col" for r in heldout) >= 55     # C = 3 has no channels-last form
    assert all(len(r["us"]) >= 4 and min(r["us"].values()) > 0 for r in heldout)


def test_replica_of_the_estimate_is_the_librarys(heldout):
    names, values = cm.read_header()
    checked = 0
    for row in heldout[::7]:
        bf16, channels_last = row["dtype"] == "bf16", row["variant"] == "kn2col"
        P = cm.params((2 if bf16 else 0) + (1 if channels_last else 0), names, values)
        for key, est in score.estimates(row).items():
            mine = cm.tile_cost(tuple(row["layer"]), cm.parse_key(key), bf16, channels_last, P)
            assert abs(mine - est) <= 0.06, (row["layer"], row["dtype"], row["variant"], key, est, mine)     # printed to 0.1 us
            checked += 1
        assert score.pick(row) == cm.pick(tuple(row["layer"]), list(row["us"]), bf16, channels_last, P)
    assert checked > 500


def test_picks_on_held_out_layers_lose_at_most_fifteen_per_cent(heldout):
    scored = score.score(heldout)
    bad = [(round(100 * loss), row["layer"], row["dtype"], row["variant"], picked, best)
           for loss, row, picked, best in scored
           if loss > KNOWN_MISSES.get((row["dtype"], row["variant"], tuple(row["layer"])), MAX_LOSS)]
    assert len(KNOWN_MISSES) <= len(scored) // 100
    assert not bad, f"{len(bad)} of {len(scored)} picks lose more than {100 * MAX_LOSS:.0f} %: {sorted(bad, reverse=True)[:10]}"
    mean = sum(s[0] for s in scored) / len(scored)
    assert mean <= 0.03, mean
