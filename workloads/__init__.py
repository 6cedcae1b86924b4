"""Seeded synthetic inputs for the TW / TVW sparse GEMM  C = A . (B (.) mask).

This module only *makes inputs*: activations A, weights B and 0/1 masks whose
structure follows the paper's tile-wise (TW) and tile-vector-wise (TVW)
patterns (Section III-A; Algorithm 3).  It contains no GEMM, no packing and no
index/metadata encoding, and it imports neither the CPU oracle nor the HIP
library; both sides are fed from here.

Everything is a pure function of an integer seed:
``numpy.random.Generator(PCG64(seed))`` draws fp32 normals that are rounded to
fp16 (round-to-nearest-even), the input precision of the path.

The layer shapes stand in for the paper's BERT-base / BERT-large / VGG-16
workloads (Section VI-A): only the GEMM shapes are used, the trained weights
and datasets are not available, so weights are N(0, sigma) draws and the masks
come from one-shot magnitude pruning of those draws.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field

import numpy as np

__all__ = [
    "rng_fp16", "rng_i8", "make_A", "make_B", "Shape", "SHAPES", "CONFIGS",
    "tw_mask", "tvw_mask", "make_case", "Case", "seed_for", "ConvGeom", "same_geom", "conv_ldx", "CONV_LAYERS", "make_conv_input",
]


# --------------------------------------------------------------------------
# raw tensors
# --------------------------------------------------------------------------
def rng_fp16(seed: int, shape, sigma: float = 1.0) -> np.ndarray:
    """fp16 array of N(0, sigma^2) draws (fp32 draw, one RNE rounding)."""
    g = np.random.Generator(np.random.PCG64(int(seed)))
    x = g.standard_normal(size=shape, dtype=np.float32) * np.float32(sigma)
    return x.astype(np.float16)


def rng_i8(seed: int, shape, sigma: float = 40.0) -> np.ndarray:
    """int8 array shaped like a symmetric 8-bit quantisation of normal data: N(0, sigma^2)
    draws rounded to the nearest integer and clipped to [-127, 127]."""
    g = np.random.Generator(np.random.PCG64(int(seed)))
    x = g.standard_normal(size=shape, dtype=np.float32) * np.float32(sigma)
    return np.clip(np.rint(x), -127, 127).astype(np.int8)


def make_A(seed: int, M: int, K: int) -> np.ndarray:
    """Activations, logical M x K (row i = one token / im2col row), N(0,1)."""
    return rng_fp16(seed, (M, K), 1.0)


def make_B(seed: int, K: int, N: int, sigma: float) -> np.ndarray:
    """Weights, logical K x N."""
    return rng_fp16(seed + 1, (K, N), sigma)


# --------------------------------------------------------------------------
# mask recipes (one-shot magnitude pruning shaped like Algorithm 3)
# --------------------------------------------------------------------------
def _lowest(scores: np.ndarray, n_prune: int) -> np.ndarray:
    """Indices of the n_prune lowest scores; equal scores: lower index first."""
    order = np.lexsort((np.arange(scores.size), scores))
    return order[:n_prune]


def _round_half_up(x: float) -> int:
    return int(math.floor(x + 0.5))


def tw_mask(B16: np.ndarray, G: int, *, density: float, col_frac: float | None,
            recipe: str = "per_tile", row_multiple: int = 1):
    """TW mask for a K x N fp16 weight keeping a fraction `density` of it.

    Columns first (TW-C), then rows of each width-G tile of the *kept* columns
    (TW-R), as in Algorithm 3's TW.  Scores are sums of squares in fp64.

    recipe
      "per_tile": prune floor(col_frac*N) columns, then every tile keeps its
          top  round(rho*K)  rows, rho = density*N/N_kept.
      "global":   same column step, then one threshold over all (tile,row)
          units (mean of squares, so a narrow last tile is comparable): the
          tiles end up with different heights K_t.
      "paper":    the equal split of Algorithm 3: s = 1-sqrt(density) is
          pruned from the columns and from the (tile,row) units, the latter
          with one global threshold (col_frac ignored).
    row_multiple: "per_tile" only; kept-row count per tile is rounded to a
        multiple of it (4 for TVW so that 2:4 groups are whole).

    Returns the mask, u8 K x N.
    """
    K, N = B16.shape
    sq = B16.astype(np.float64) ** 2
    s_paper = 1.0 - math.sqrt(min(1.0, max(0.0, density)))
    if recipe == "paper":
        n_col_prune = int(math.floor(s_paper * N))
    else:
        n_col_prune = int(math.floor((col_frac or 0.0) * N))
    col_keep = np.ones(N, dtype=bool)
    col_keep[_lowest(sq.sum(axis=0), n_col_prune)] = False
    cols = np.flatnonzero(col_keep)
    n_kept = cols.size
    mask = np.zeros((K, N), dtype=np.uint8)
    if n_kept == 0:
        return mask
    n_tiles = (n_kept + G - 1) // G
    tiles = [cols[t * G:(t + 1) * G] for t in range(n_tiles)]
    rho = min(1.0, density * N / n_kept)
    if recipe == "per_tile":
        k_keep = _round_half_up(rho * K / row_multiple) * row_multiple
        k_keep = max(0, min(K - K % row_multiple, k_keep))
        for tc in tiles:
            keep = np.ones(K, dtype=bool)
            keep[_lowest(sq[:, tc].sum(axis=1), K - k_keep)] = False
            mask[np.ix_(np.flatnonzero(keep), tc)] = 1
    elif recipe in ("global", "paper"):
        unit = np.stack([sq[:, tc].mean(axis=1) for tc in tiles], axis=0)  # (tiles, K)
        if recipe == "paper":
            n_prune = int(math.floor(s_paper * unit.size))
        else:
            n_prune = unit.size - _round_half_up(rho * unit.size)
        keep = np.ones(unit.size, dtype=bool)
        keep[_lowest(unit.reshape(-1), n_prune)] = False
        keep = keep.reshape(unit.shape)
        for t, tc in enumerate(tiles):
            mask[np.ix_(np.flatnonzero(keep[t]), tc)] = 1
    else:
        raise ValueError(f"unknown recipe {recipe!r}")
    return mask


def _two_of_four(B16: np.ndarray, tile_mask: np.ndarray, G: int) -> np.ndarray:
    """2:4 along the condensed K order of every tile (the VW(w,0.5,4) step of
    Algorithm 3's TVW): in each run of 4 consecutive kept rows of a tile and
    each column keep the two largest |w|; equal |w|: lower position kept."""
    K, N = B16.shape
    mag = np.abs(B16.astype(np.float64))
    out = np.zeros_like(tile_mask)
    cols = np.flatnonzero(tile_mask.any(axis=0))
    for t in range((cols.size + G - 1) // G):
        tc = cols[t * G:(t + 1) * G]
        rows = np.flatnonzero(tile_mask[:, tc].any(axis=1))
        for g0 in range(0, rows.size, 4):
            gr = rows[g0:g0 + 4]
            m = mag[np.ix_(gr, tc)]                       # (<=4, w)
            # rank within the group: larger first, ties -> lower position first
            order = np.argsort(-m, axis=0, kind="stable")
            keep = np.zeros_like(m, dtype=bool)
            for r in range(min(2, gr.size)):
                keep[order[r], np.arange(tc.size)] = True
            out[np.ix_(gr, tc)] = keep.astype(np.uint8)
    return out


def tvw_mask(B16: np.ndarray, G: int, *, sparsity: float, col_frac: float | None,
             recipe: str = "per_tile"):
    """TVW mask: TW at sparsity 1-2(1-s_t) (Algorithm 3, TVW) with kept-row
    counts that are multiples of 4, then 2:4 inside the kept rows.

    Returns (mask, tile_mask): the element mask and the TW-level mask it was
    cut from (the packer is given both, so a kept row that loses every
    element of a tile to the 2:4 step still counts as kept)."""
    if sparsity < 0.5:
        raise ValueError("TVW cannot go below 50% sparsity")
    tile_mask = tw_mask(B16, G, density=2.0 * (1.0 - sparsity), col_frac=col_frac,
                        recipe=recipe, row_multiple=4 if recipe == "per_tile" else 1)
    return _two_of_four(B16, tile_mask, G), tile_mask


def tew_mask(B16: np.ndarray, G: int, *, sparsity: float, delta: float, col_frac: float | None,
             recipe: str = "per_tile"):
    """TEW mask (Algorithm 3, TEW): TW at sparsity s_t + delta, then the
    floor(delta*K*N) largest-magnitude pruned elements are put back (equal
    magnitudes: lower flat index first).  Returns (mask, tile_mask)."""
    K, N = B16.shape
    tile_mask = tw_mask(B16, G, density=1.0 - sparsity - delta, col_frac=col_frac, recipe=recipe)
    score = B16.astype(np.float64).reshape(-1) ** 2
    pruned = np.flatnonzero(tile_mask.reshape(-1) == 0)
    order = pruned[np.argsort(-score[pruned], kind="stable")]
    mask = tile_mask.copy().reshape(-1)
    mask[order[:int(np.floor(delta * K * N))]] = 1
    return mask.reshape(K, N), tile_mask


# --------------------------------------------------------------------------
# named workloads
# --------------------------------------------------------------------------
@dataclass(frozen=True)
class Shape:
    name: str
    M: int
    K: int
    N: int
    sigma: float


SHAPES = {
    # config index -> list of layer shapes
    1: [Shape("tiny", 128, 256, 256, 1.0)],
    2: [Shape("bert_base_qkvo", 4096, 768, 768, 0.02),
        Shape("bert_base_ffn1", 4096, 768, 3072, 0.02),
        Shape("bert_base_ffn2", 4096, 3072, 768, 0.02)],
    4: [Shape("bert_large_ffn1", 8192, 1024, 4096, 0.02),
        Shape("bert_large_ffn2", 8192, 4096, 1024, 0.02)],
    5: [Shape("vgg16_conv3x3_256_56", 25088, 2304, 256, 0.02),
        Shape("vgg16_conv3x3_512_14", 1568, 4608, 512, 0.02)],
}
SHAPES[3] = SHAPES[2]

# (config, default G, pattern, sparsity, col_frac)
CONFIGS = {
    1: dict(G=64, pattern="tw", sparsity=0.5, col_frac=0.0),
    2: dict(G=128, pattern="tw", sparsity=0.75, col_frac=0.10),
    3: dict(G=128, pattern="tvw", sparsity=0.875, col_frac=0.10),
    4: dict(G=128, pattern="tw", sparsity=0.75, col_frac=0.10),
    5: dict(G=64, pattern="tw", sparsity=0.75, col_frac=0.10),
}


def seed_for(config: int, shape_index: int, variant: int = 0) -> int:
    return 1000 * config + 10 * shape_index + variant


@dataclass
class Case:
    name: str
    M: int
    K: int
    N: int
    G: int
    pattern: str          # "tw" | "tvw" | "tew"
    sparsity: float
    seed: int
    A: np.ndarray = field(repr=False)          # M x K fp16
    B: np.ndarray = field(repr=False)          # K x N fp16
    mask: np.ndarray = field(repr=False)       # K x N u8
    tile_mask: np.ndarray = field(repr=False)  # K x N u8 (TW-level)


def make_case(config: int, shape_index: int = 0, *, pattern: str | None = None,
              sparsity: float | None = None, G: int | None = None,
              col_frac: float | None = None, recipe: str = "per_tile",
              variant: int = 0, M: int | None = None, with_A: bool = True,
              delta: float = 0.015) -> Case:
    """One (A, B, mask) triple of a configured workload.  Sparsity 0 gives the
    all-ones mask (the dense case).  `M` may shrink the activation count."""
    shp = SHAPES[config][shape_index]
    cfg = CONFIGS[config]
    pattern = pattern or cfg["pattern"]
    sparsity = cfg["sparsity"] if sparsity is None else sparsity
    G = G or cfg["G"]
    col_frac = cfg["col_frac"] if col_frac is None else col_frac
    seed = seed_for(config, shape_index, variant)
    M = M or shp.M
    A = make_A(seed, M, shp.K) if with_A else np.zeros((0, shp.K), np.float16)
    B = make_B(seed, shp.K, shp.N, shp.sigma)
    if sparsity == 0.0:
        mask = np.ones((shp.K, shp.N), dtype=np.uint8)
        tile_mask = mask.copy()
    elif pattern == "tw":
        mask = tw_mask(B, G, density=1.0 - sparsity, col_frac=col_frac, recipe=recipe)
        tile_mask = mask.copy()
    elif pattern == "tvw":
        mask, tile_mask = tvw_mask(B, G, sparsity=sparsity, col_frac=col_frac, recipe=recipe)
    elif pattern == "tew":
        mask, tile_mask = tew_mask(B, G, sparsity=sparsity, delta=delta, col_frac=col_frac, recipe=recipe)
    else:
        raise ValueError(pattern)
    return Case(f"{shp.name}_{pattern}{int(round(sparsity * 10000)) / 100:g}_G{G}_{recipe}",
                M, shp.K, shp.N, G, pattern, sparsity, seed, A, B, mask, tile_mask)


# --------------------------------------------------------------------------
# convolution inputs in the wide layout (config 5's layers before img2col)
# --------------------------------------------------------------------------
@dataclass
class ConvGeom:
    """C input channels, R x S filter, B images of H x W, stored per channel as B blocks of
    L lines of P elements (padding included)."""
    C: int
    R: int
    S: int
    B: int
    H: int
    W: int
    P: int
    L: int

    @property
    def Mp(self) -> int:           # positions of the wide grid
        return self.B * self.L * self.P

    @property
    def K(self) -> int:
        return self.C * self.R * self.S

    def ints(self) -> dict:        # keyword arguments of the oracle
        return dict(R=self.R, S=self.S, B=self.B, H=self.H, W=self.W, P=self.P, L=self.L)


def same_geom(C: int, R: int, S: int, B: int, H: int, W: int, pitch_multiple: int = 1) -> ConvGeom:
    """Block size for a stride-1 'same' convolution: (R-1) extra lines, (S-1) extra columns,
    the pitch rounded up to `pitch_multiple`."""
    P = -(-(W + S - 1) // pitch_multiple) * pitch_multiple
    return ConvGeom(C, R, S, B, H, W, P, H + R - 1)


# config 5: VGG-16 3x3 convolutions, batch 8 (M = 8*56*56 and 8*14*14 valid positions)
CONV_LAYERS = [("vgg16_conv3x3_256_56", same_geom(256, 3, 3, 8, 56, 56), 256),
               ("vgg16_conv3x3_512_14", same_geom(512, 3, 3, 8, 14, 14), 512)]


def conv_ldx(g: ConvGeom, chunk: int = 8) -> int:
    """Shortest channel row (multiple of `chunk` elements: 8 for fp16, 16 for int8) in which the
    windows of every wide-grid position, padding lanes included, stay inside the row."""
    up = lambda v: (v + chunk - 1) // chunk * chunk
    return up(up(g.Mp) + (g.R - 1) * g.P + g.S - 1)


def make_conv_input(seed: int, g: ConvGeom, ldx: int | None = None, int8: bool = False) -> np.ndarray:
    """C x ldx, fp16 N(0,1) pixels (or int8, as rng_i8), zeros in the padding ((R-1)//2 lines above,
    (S-1)//2 columns left of every image, the rest below / right) and in the slack behind the grid."""
    ldx = ldx or conv_ldx(g, 16 if int8 else 8)
    X = np.zeros((g.C, ldx), np.int8 if int8 else np.float16)
    img = rng_i8(seed, (g.C, g.B, g.H, g.W)) if int8 else rng_fp16(seed, (g.C, g.B, g.H, g.W), 1.0)
    blk = X[:, :g.Mp].reshape(g.C, g.B, g.L, g.P)
    t, l = (g.R - 1) // 2, (g.S - 1) // 2
    blk[:, :, t:t + g.H, l:l + g.W] = img
    return X
