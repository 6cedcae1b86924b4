"""Canonical logical packed form of a TW / TVW / TEW pruned weight, on the CPU.

TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).

Section V keeps B condensed per tile ("remove the pruned rows and columns in
the weight matrix tile B_tile ... offline") and replaces the per-tile mask
vectors by the indices of the unpruned rows/columns, then by offsets
(index minus position: the compressed tile offset, CTO).  Written out:

  col_idx      ascending original indices of the kept columns       (CTO_n)
  tiles        condensed column j belongs to tile j // G (Algorithm 3:
               Condense, then split by (1,G)); the last tile may be narrower
  row_idx[t]   ascending original K indices kept in tile t            (CTO_k)
  cto_k, cto_n row_idx[t][j] - j  and  col_idx[j] - j
  TW values    V[t][j][w] = B[row_idx[t][j], col_idx[t*G + w]]   (fp16 bits)
  TVW          per tile, runs of 4 consecutive entries of row_idx[t] form a
               group; per (group g, column w) exactly two positions p0 < p1 of
               {0,1,2,3} are stored: the mask-set ones, topped up with the
               lowest unset positions when fewer than two are set (their
               values are +0 and their `valid` bit is 0).
               meta[t][g][w] = p0 | p1 << 2, valid[t][g][w] = v0 | v1 << 1,
               values V2[t][g][i][w], i in {0,1}.

  TEW          the TW form of the TW-level `tile_mask`, plus the restored
               elements (mask set, tile_mask clear) in compressed sparse column
               form over the ORIGINAL columns (Section III-A, "TEW": the EW
               part is kept in CSC; here one CSC for the matrix, which also
               covers restored elements in columns the TW step dropped):
               ew_col_ptr[N+1], ew_row[nnz] ascending inside a column,
               ew_val[nnz] fp16 bits.

A mask is TW-conformant when mask[k,n] == (n kept) and (k in row_idx[tile(n)]).
For TVW the kept rows/columns come from the TW-level `tile_mask` when given,
else from the element mask itself; the element mask must lie inside it with at
most two set positions per (group, column).
"""
from __future__ import annotations

import numpy as np

PATTERN_TW = 0
PATTERN_TVW = 1
PATTERN_TEW = 2


class MaskError(ValueError):
    """The mask does not have the TW / TVW structure."""


def _structure(m: np.ndarray, G: int):
    K, N = m.shape
    col_idx = [n for n in range(N) if m[:, n].any()]
    tiles = [col_idx[i:i + G] for i in range(0, len(col_idx), G)]
    row_idx = [[k for k in range(K) if m[k, cols].any()] for cols in tiles]
    return col_idx, tiles, row_idx


def _check_tw(m: np.ndarray, col_idx, tiles, row_idx):
    want = np.zeros_like(m, dtype=bool)
    for cols, rows in zip(tiles, row_idx):
        want[np.ix_(rows, cols)] = True
    if not np.array_equal(want, m != 0):
        raise MaskError("mask is not tile-wise: a kept row of a tile has a hole, "
                        "or a kept column misses one of its tile's rows")


def cto(indices):
    """Index -> offset: the value to add to position j to reach index j."""
    return [int(v) - j for j, v in enumerate(indices)]


def ref_pack(B16: np.ndarray, mask: np.ndarray, G: int, pattern: int,
             tile_mask: np.ndarray | None = None) -> dict:
    if B16.dtype != np.float16 or B16.shape != mask.shape:
        raise ValueError("B must be fp16 and mask must match its shape")
    K, N = B16.shape
    bits = B16.view(np.uint16)
    m = mask != 0
    if pattern == PATTERN_TW:
        col_idx, tiles, row_idx = _structure(m, G)
        _check_tw(m, col_idx, tiles, row_idx)
    elif pattern == PATTERN_TVW:
        tm = m if tile_mask is None else (tile_mask != 0)
        col_idx, tiles, row_idx = _structure(tm, G)
        if tile_mask is not None:
            _check_tw(tm, col_idx, tiles, row_idx)
            if (m & ~tm).any():
                raise MaskError("element mask has bits outside the tile mask")
    elif pattern == PATTERN_TEW:
        if tile_mask is None:
            raise ValueError("TEW needs the TW-level tile_mask")
        tm = tile_mask != 0
        col_idx, tiles, row_idx = _structure(tm, G)
        _check_tw(tm, col_idx, tiles, row_idx)
        if (tm & ~m).any():
            raise MaskError("tile mask has bits outside the element mask")
    else:
        raise ValueError("pattern")
    out = dict(K=K, N=N, G=G, pattern=pattern, col_idx=np.array(col_idx, np.int32),
               n_kept=len(col_idx), n_tiles=len(tiles),
               row_idx=[np.array(r, np.int32) for r in row_idx],
               cto_n=np.array(cto(col_idx), np.int32),
               cto_k=[np.array(cto(r), np.int32) for r in row_idx])
    if pattern in (PATTERN_TW, PATTERN_TEW):
        out["values"] = [bits[np.ix_(rows, cols)].copy() if rows else
                         np.zeros((0, len(cols)), np.uint16)
                         for cols, rows in zip(tiles, row_idx)]
        if pattern == PATTERN_TEW:
            ptr, rows_e, vals_e = [0], [], []
            for n in range(N):
                for k in range(K):
                    if m[k, n] and not tm[k, n]:
                        rows_e.append(k)
                        vals_e.append(int(bits[k, n]))
                ptr.append(len(rows_e))
            out.update(ew_col_ptr=np.array(ptr, np.int32), ew_row=np.array(rows_e, np.int32),
                       ew_val=np.array(vals_e, np.uint16))
        return out
    vals, metas, valids = [], [], []
    for cols, rows in zip(tiles, row_idx):
        ng = -(-len(rows) // 4)
        v = np.zeros((ng, 2, len(cols)), np.uint16)
        me = np.zeros((ng, len(cols)), np.uint8)
        va = np.zeros((ng, len(cols)), np.uint8)
        for g in range(ng):
            grp = rows[4 * g:4 * g + 4]
            for w, n in enumerate(cols):
                setpos = [p for p, k in enumerate(grp) if m[k, n]]
                if len(setpos) > 2:
                    raise MaskError("more than 2 of 4 kept in a group")
                pos = list(setpos)
                p = 0
                while len(pos) < 2:
                    if p not in pos:
                        pos.append(p)
                    p += 1
                pos.sort()
                me[g, w] = pos[0] | (pos[1] << 2)
                for i, p in enumerate(pos):
                    if p in setpos:
                        va[g, w] |= 1 << i
                        v[g, i, w] = bits[grp[p], n]
        vals.append(v); metas.append(me); valids.append(va)
    out.update(values=vals, meta=metas, valid=valids)
    return out


def ref_unpack(p: dict):
    """Packed form -> (B (.) mask as fp16 bits, mask); inverse of ref_pack."""
    K, N, G = p["K"], p["N"], p["G"]
    Bm = np.zeros((K, N), np.uint16)
    mask = np.zeros((K, N), np.uint8)
    col_idx = p["col_idx"]
    for t in range(p["n_tiles"]):
        cols = col_idx[t * G:(t + 1) * G]
        rows = p["row_idx"][t]
        if p["pattern"] in (PATTERN_TW, PATTERN_TEW):
            if len(rows):
                Bm[np.ix_(rows, cols)] = p["values"][t]
                mask[np.ix_(rows, cols)] = 1
            continue
        v, me, va = p["values"][t], p["meta"][t], p["valid"][t]
        for g in range(me.shape[0]):
            for w, n in enumerate(cols):
                for i in range(2):
                    if (va[g, w] >> i) & 1:
                        k = rows[4 * g + ((me[g, w] >> (2 * i)) & 3)]
                        Bm[k, n] = v[g, i, w]
                        mask[k, n] = 1
    if p["pattern"] == PATTERN_TEW:
        ptr = p["ew_col_ptr"]
        for n in range(N):
            for e in range(ptr[n], ptr[n + 1]):
                Bm[p["ew_row"][e], n] = p["ew_val"][e]
                mask[p["ew_row"][e], n] = 1
    return Bm, mask
