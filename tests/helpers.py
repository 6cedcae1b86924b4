"""Shared test helpers: acceptance bars and small mask builders."""
import numpy as np

REL_FRO = 1e-3      # ||C - C_ref||_F / ||C_ref||_F
ELEM = 4e-3         # |C - C_ref|_ij <= ELEM * (|A| . |B (.) mask|)_ij


def assert_C_close(C, C_ref, S):
    """The two bars of the benchmark spec.  Derivation of why they hold for a
    correct kernel: fp32 accumulation of n terms errs by at most about
    n * 2^-24 * S (2e-4 * S at n = 3072), the final rounding to fp16 adds
    2^-11 * |C| <= 4.9e-4 * S; both sit well inside 4e-3 * S.  Below fp16's
    normal range (|C| < 2^-14) the output format itself is coarser than that:
    its values are 2^-24 apart, so the correctly rounded result may be 2^-25
    away (a single product 6.9e-6 rounds to 7.0e-6: 4.3e-3 relative), and that
    half spacing is allowed on top.  Where S is 0 (pruned columns) the result
    must be exactly 0."""
    C = np.asarray(C, dtype=np.float64)
    assert C.shape == C_ref.shape
    assert np.isfinite(C).all()
    err = np.abs(C - C_ref)
    allowed = ELEM * S + np.where(S > 0, 2.0 ** -25, 0.0)
    bad = err > allowed
    assert not bad.any(), (f"{bad.sum()} elements outside {ELEM}*S; worst ratio "
                           f"{(err / np.maximum(S, 1e-300)).max():.3e} at "
                           f"{np.unravel_index(np.argmax(err - allowed), err.shape)}")
    den = np.linalg.norm(C_ref)
    if den > 0:
        # (the same half spacing per kept element, as a norm, for matrices of tiny values)
        slack = 2.0 ** -25 * np.sqrt(np.count_nonzero(S > 0))
        rel = max(np.linalg.norm(C - C_ref) - slack, 0.0) / den
        assert rel <= REL_FRO, f"relative Frobenius error {rel:.3e} > {REL_FRO}"
    else:
        assert not C.any()


def random_tw_mask(rng, K, N, G, col_keep=0.8, row_keep=0.5):
    """A random TW-conformant mask (random, not magnitude-based)."""
    cols = np.flatnonzero(rng.random(N) < col_keep)
    mask = np.zeros((K, N), np.uint8)
    for i in range(0, cols.size, G):
        tc = cols[i:i + G]
        rows = np.flatnonzero(rng.random(K) < row_keep)
        mask[np.ix_(rows, tc)] = 1
    return mask


def random_tvw_mask(rng, K, N, G, col_keep=0.8, row_keep=0.5, full=True):
    """Random TVW mask + its tile mask.  full=False leaves some groups with
    fewer than two kept elements."""
    tm = random_tw_mask(rng, K, N, G, col_keep, row_keep)
    mask = np.zeros_like(tm)
    cols = np.flatnonzero(tm.any(axis=0))
    for i in range(0, cols.size, G):
        tc = cols[i:i + G]
        rows = np.flatnonzero(tm[:, tc].any(axis=1))
        for g in range(0, rows.size, 4):
            grp = rows[g:g + 4]
            for n in tc:
                k = 2 if full else int(rng.integers(0, 3))
                pick = rng.permutation(grp.size)[:k]
                mask[grp[pick], n] = 1
    return mask, tm
