"""One-shot TW / VW(2:4) / TVW / TEW pruning masks, following Algorithms 2 and 3.

TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).

The paper prunes in many prune+fine-tune stages (Algorithm 1) with a
first-order Taylor importance score (Section IV, "Importance Score"); neither
is reproducible without its datasets.  What is kept here is a single call of
the pattern functions with the magnitude score the same section calls the most
intuitive one: an element scores w^2, a vector scores the sum of its elements'
scores.

Readings where the algorithms are silent:
  * `Percentile(scores, s)` followed by the strict `score < threshold` test is
    made deterministic as: order the units by (score, index) ascending and
    prune the first floor(s * n_units).
  * 2:4 (Algorithm 3's `VW(w, 0.5, 4)` inside TVW) runs along K over the
    *condensed* kept rows of each tile, 4 consecutive kept rows at a time; of
    equal magnitudes the lower position is kept.
  * a last tile narrower than G scores its rows by the mean, not the sum, when
    one threshold is shared by all tiles.
  * TEW's remedy step (Section III-A; Algorithm 3, TEW, where the scores of kept
    elements are zeroed and the threshold sits at the (1 - delta) percentile over
    all K*N scores) puts back a delta share of the weight's elements, the
    highest-scored ones.  Made deterministic as: of the elements the TW step
    pruned, restore the floor(delta * K * N) highest by (score descending, flat
    index ascending); fewer if fewer were pruned.
"""
from __future__ import annotations

import math

import numpy as np


def tw_split_sparsity(s_t: float) -> float:
    """Algorithm 3, TW: the target is divided equally between the column and
    the row step: (1-s)^2 = 1-s_t."""
    return 1.0 - math.sqrt(1.0 - s_t)


def tvw_tw_sparsity(s_t: float) -> float:
    """Algorithm 3, TVW: the TW part carries s with (1-s)/2 = 1-s_t."""
    return 1.0 - 2.0 * (1.0 - s_t)


def n_tiles(n_cols: int, G: int) -> int:
    """Section III-A: a width-N matrix is cut into ceil(N/G) B tiles."""
    return -(-n_cols // G)


def _prune_lowest(scores, count):
    """Set of unit ids pruned: the `count` lowest by (score, id)."""
    ranked = sorted(range(len(scores)), key=lambda i: (scores[i], i))
    return set(ranked[:count])


def exact_square_scores(w16: np.ndarray):
    """Element scores w^2 as exact Python integers in units of 2^-48.  An fp16
    value is an integer multiple of 2^-24 (below 2^40 in those units), so its
    square and any sum of squares are exact integers: ranking by them does not
    depend on the order of summation."""
    bits = w16.astype(np.float16).view(np.uint16).reshape(-1).tolist()
    out = []
    for h in bits:
        e, m = (h >> 10) & 31, h & 1023
        if e == 31:
            raise ValueError("non-finite weight")
        mag = m if e == 0 else (m | 1024) << (e - 1)
        out.append(mag * mag)
    return out


def ew(w: np.ndarray, s_t: float) -> np.ndarray:
    """Algorithm 2, EW: element scores, one global threshold."""
    sc = (w.astype(np.float64) ** 2).reshape(-1).tolist()
    pruned = _prune_lowest(sc, int(math.floor(s_t * len(sc))))
    m = np.ones(w.size, dtype=np.uint8)
    for i in pruned:
        m[i] = 0
    return m.reshape(w.shape)


def tw(w: np.ndarray, G: int, *, s_cols: float | None = None, n_cols_pruned: int | None = None,
       s_rows: float | None = None, rows_kept_per_tile: int | None = None,
       exact: bool = False) -> np.ndarray:
    """Algorithm 3, TW, with the two steps parameterised separately.

    TW-C: columns (K,1) scored and pruned, either a fraction s_cols or a count.
    Condense, then TW-R: the kept columns are cut into tiles of G and every
    (1,G) row piece is a unit; either one global threshold prunes a fraction
    s_rows of all units, or every tile keeps its `rows_kept_per_tile` best.
    `exact` scores with integers (exact_square_scores) instead of fp64 sums; only
    with rows_kept_per_tile (a shared threshold over tiles of different width
    needs the mean).  Returns the 0/1 mask (K x N).
    """
    K, N = w.shape
    if exact:
        if rows_kept_per_tile is None:
            raise ValueError("exact scores are defined for the per-tile row count only")
        sq = np.array(exact_square_scores(w), dtype=object).reshape(K, N)
        col_scores = [sum(sq[:, n].tolist()) for n in range(N)]
    else:
        sq = w.astype(np.float64) ** 2
        col_scores = [float(sq[:, n].sum()) for n in range(N)]
    if n_cols_pruned is None:
        n_cols_pruned = int(math.floor((s_cols or 0.0) * N))
    pruned_cols = _prune_lowest(col_scores, n_cols_pruned)
    kept_cols = [n for n in range(N) if n not in pruned_cols]          # Condense
    tiles = [kept_cols[i:i + G] for i in range(0, len(kept_cols), G)]  # split by (1,G)
    mask = np.zeros((K, N), dtype=np.uint8)
    if rows_kept_per_tile is not None:
        for cols in tiles:
            sc = [sum(sq[k, cols].tolist()) if exact else float(sq[k, cols].sum()) for k in range(K)]
            gone = _prune_lowest(sc, K - rows_kept_per_tile)
            for k in range(K):
                if k not in gone:
                    mask[k, cols] = 1
        return mask
    units = []            # (tile, row) in tile-major order
    scores = []
    for t, cols in enumerate(tiles):
        for k in range(K):
            units.append((t, k))
            scores.append(float(sq[k, cols].mean()))
    gone = _prune_lowest(scores, int(math.floor((s_rows or 0.0) * len(units))))
    for u, (t, k) in enumerate(units):
        if u not in gone:
            mask[k, tiles[t]] = 1
    return mask


def tw_paper(w: np.ndarray, s_t: float, G: int) -> np.ndarray:
    """Algorithm 3, TW exactly as listed: equal split, global row threshold."""
    s = tw_split_sparsity(s_t)
    return tw(w, G, s_cols=s, s_rows=s)


def vw24_condensed(w: np.ndarray, tile_mask: np.ndarray, G: int) -> np.ndarray:
    """Algorithm 2's VW with vectors of 4 along K and s_t = 0.5, applied the
    way TVW needs it: inside every tile, over the kept rows in ascending
    order, 4 at a time; in each (vector, column) the 2 smallest |w| go."""
    K, N = w.shape
    mag = np.abs(w.astype(np.float64))
    kept_cols = [n for n in range(N) if tile_mask[:, n].any()]
    out = np.zeros((K, N), dtype=np.uint8)
    for i in range(0, len(kept_cols), G):
        cols = kept_cols[i:i + G]
        rows = [k for k in range(K) if tile_mask[k, cols].any()]
        for g in range(0, len(rows), 4):
            vec = rows[g:g + 4]
            for n in cols:
                ranked = sorted(range(len(vec)), key=lambda p: (-mag[vec[p], n], p))
                for p in ranked[:2]:
                    out[vec[p], n] = 1
    return out


def tvw_paper(w: np.ndarray, s_t: float, G: int):
    """Algorithm 3, TVW: TW at 1-2(1-s_t), then 2:4.  Returns (mask, tile_mask)."""
    tile_mask = tw_paper(w, tvw_tw_sparsity(s_t), G)
    return vw24_condensed(w, tile_mask, G), tile_mask


def tew(w: np.ndarray, G: int, s_t: float, delta: float, tw_fn=None):
    """Algorithm 3, TEW: TW at sparsity s_t + delta, then the remedy step puts
    back the delta * K * N pruned elements with the highest scores.
    `tw_fn(w, s, G)` is the TW step (default: Algorithm 3's TW as listed).
    Returns (mask, tile_mask): the element mask and the TW-level mask inside it."""
    K, N = w.shape
    tile_mask = (tw_fn or tw_paper)(w, s_t + delta, G)
    scores = (w.astype(np.float64) ** 2).reshape(-1).tolist()
    flat_tm = tile_mask.reshape(-1)
    pruned = [i for i in range(K * N) if not flat_tm[i]]
    pruned.sort(key=lambda i: (-scores[i], i))
    mask = tile_mask.copy().reshape(-1)
    for i in pruned[:int(math.floor(delta * K * N))]:
        mask[i] = 1
    return mask.reshape(K, N), tile_mask


def rows_per_tile(K: int, N: int, n_kept: int, density: float, multiple: int = 1) -> int:
    """Kept rows per tile so that the whole matrix keeps `density` of its
    elements when only n_kept of N columns survive: round(density*N/n_kept*K),
    to a multiple of `multiple`, halves rounded up."""
    x = min(1.0, density * N / n_kept) * K / multiple
    r = int(math.floor(x + 0.5)) * multiple
    return max(0, min(K - K % multiple, r))
