"""Hand-worked pins of oracle/prune.py's per-tile TW branch (fp64 and exact integer scores) and
of the 2:4 step over condensed rows.  The examples live in tests/golden/ with every step of
Algorithm 3 written out; nothing here comes from a second implementation."""
import os

import numpy as np
import pytest

from oracle import prune as op

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _examples(name):
    out, cur = [], None
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            tok = line.split()
            if not tok or tok[0].startswith("#"):
                continue
            if tok[0] == "example":
                cur = {"w": [], "m": []}
                i = 2
                while i < len(tok):                    # key followed by one or more integers
                    key, vals = tok[i], []
                    i += 1
                    while i < len(tok) and tok[i].lstrip("-").isdigit():
                        vals.append(int(tok[i]))
                        i += 1
                    cur[key] = vals[0] if len(vals) == 1 and key != "kept_rows" else vals
                out.append(cur)
            else:
                cur[tok[0]].append([int(x) for x in tok[1:]])
    for e in out:
        e["w"] = np.array(e["w"], dtype=np.float16)
        e["m"] = np.array(e["m"], dtype=np.uint8)
        assert e["w"].shape == e["m"].shape == (e["K"], e["N"])
    return out


TW_EXAMPLES = _examples("tw_per_tile_worked_example.txt")


@pytest.mark.parametrize("exact", [False, True])
@pytest.mark.parametrize("ex", TW_EXAMPLES, ids=lambda e: f"K{e['K']}N{e['N']}")
def test_tw_per_tile_worked_by_hand(ex, exact):
    got = op.tw(ex["w"], ex["G"], n_cols_pruned=ex["cols_pruned"], rows_kept_per_tile=ex["rows_kept"], exact=exact)
    assert got.tolist() == ex["m"].tolist()


def test_worked_examples_tell_the_directions_apart():
    """The first example is built so that the plausible mistakes give another mask: keeping the
    lowest rows, pruning the highest column, cutting tiles on the original columns."""
    ex = TW_EXAMPLES[0]
    w, G, want = ex["w"].astype(np.float64), ex["G"], ex["m"]
    sq = w ** 2
    col_low = int(np.argmin(sq.sum(0)))
    kept = [n for n in range(ex["N"]) if n != col_low]

    def build(tiles, keep_highest):
        m = np.zeros_like(want)
        for cols in tiles:
            order = np.argsort(sq[:, cols].sum(1))
            rows = order[-ex["rows_kept"]:] if keep_highest else order[:ex["rows_kept"]]
            m[np.ix_(rows, cols)] = 1
        return m
    right = build([kept[i:i + G] for i in range(0, len(kept), G)], True)
    assert right.tolist() == want.tolist()
    lowest_rows = build([kept[i:i + G] for i in range(0, len(kept), G)], False)
    original_tiles = build([[n for n in range(i, min(i + G, ex["N"])) if n != col_low]
                            for i in range(0, ex["N"], G)], True)
    kept_hi = [n for n in range(ex["N"]) if n != int(np.argmax(sq.sum(0)))]
    highest_col = build([kept_hi[i:i + G] for i in range(0, len(kept_hi), G)], True)
    for wrong in (lowest_rows, original_tiles, highest_col):
        assert wrong.tolist() != want.tolist()


def test_vw24_over_condensed_rows_worked_by_hand():
    (ex,) = _examples("vw24_condensed_worked_example.txt")
    tile_mask = np.zeros((ex["K"], ex["N"]), dtype=np.uint8)
    tile_mask[ex["kept_rows"], :] = 1
    got = op.vw24_condensed(ex["w"], tile_mask, ex["G"])
    assert got.tolist() == ex["m"].tolist()
