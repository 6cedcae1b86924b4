"""Pins of the convolution oracle (CPU): the img2col GEMM of Section VI-A against a library
cross-correlation, against seven plain loops, and against special cases."""
import numpy as np
import pytest
from scipy.signal import correlate2d

from oracle import conv as oc
from oracle import gemm as og
from tests.helpers import random_tw_mask
import workloads as wl


def _weights(seed, g, N):
    return wl.rng_fp16(seed, (g.K, N), 0.5)


def _images(X, g):
    """The pixels back out of the wide layout: C x B x H x W."""
    t, l = (g.R - 1) // 2, (g.S - 1) // 2
    return X[:, :g.Mp].reshape(g.C, g.B, g.L, g.P)[:, :, t:t + g.H, l:l + g.W]


@pytest.mark.parametrize("R,S,pitch", [(3, 3, 1), (3, 3, 8), (5, 3, 1), (1, 1, 1), (1, 3, 4)])
def test_equals_same_mode_cross_correlation(R, S, pitch):
    """Odd filters, zero padding: position (y, x) of the result is scipy's 'same' cross-correlation
    of the image with the filter, summed over input channels."""
    g = wl.same_geom(3, R, S, 2, 6, 7, pitch)
    N = 4
    X, Bw = wl.make_conv_input(1, g), _weights(2, g, N)
    mask = np.ones((g.K, N), np.uint8)
    Cw = oc.conv_wide_oracle(X, Bw, mask, **g.ints())
    img = _images(X, g).astype(np.float64)
    valid = oc.valid_positions(B=g.B, H=g.H, W=g.W, P=g.P, L=g.L)
    assert valid.sum() == g.B * g.H * g.W
    got = Cw[valid].reshape(g.B, g.H, g.W, N)
    for b in range(g.B):
        for n in range(N):
            want = sum(correlate2d(img[c, b], Bw[c * R * S:(c + 1) * R * S, n].astype(np.float64).reshape(R, S),
                                   mode="same") for c in range(g.C))
            assert np.allclose(got[b, :, :, n], want, rtol=1e-12, atol=1e-12)
    assert not Cw[~valid].any()


def test_equals_seven_plain_loops_with_a_tw_mask():
    g = wl.same_geom(4, 3, 3, 2, 3, 4)
    N = 6
    rng = np.random.default_rng(3)
    mask = random_tw_mask(rng, g.K, N, 4, col_keep=0.8, row_keep=0.5)
    X, Bw = wl.make_conv_input(4, g), _weights(5, g, N)
    a = oc.conv_wide_oracle(X, Bw, mask, **g.ints())
    b = oc.conv_bruteforce(X, Bw, mask, **g.ints())
    assert np.allclose(a, b, rtol=1e-13, atol=1e-13)
    assert np.abs(a).max() > 0.1


def test_pointwise_filter_is_the_plain_product():
    """R = S = 1 with no padding: the img2col matrix is X transposed."""
    g = wl.ConvGeom(5, 1, 1, 2, 3, 4, 4, 3)
    X, Bw = wl.make_conv_input(6, g), _weights(7, g, 3)
    mask = (np.arange(15).reshape(5, 3) % 2).astype(np.uint8)
    A = oc.im2col_wide(X, **g.ints())
    assert np.array_equal(A, X[:, :g.Mp].T)
    assert np.array_equal(oc.conv_wide_oracle(X, Bw, mask, **g.ints()), og.gemm_oracle(X[:, :g.Mp].T, Bw, mask))


def test_one_hot_input_and_weight_pick_one_window_element():
    """A single 1 in the input and a single 1 in the weight: the output is 1 exactly where the
    window of the position covers the pixel at the filter tap (pins the order k = (c, r, s) and the
    direction of the shifts)."""
    g = wl.ConvGeom(2, 2, 3, 1, 4, 5, 7, 5)
    X = np.zeros((g.C, g.Mp + 8), np.float16)
    c0, yy, xx = 1, 3, 4
    X[c0, yy * g.P + xx] = 1
    for r in range(g.R):
        for s in range(g.S):
            Bw = np.zeros((g.K, 1), np.float16)
            Bw[(c0 * g.R + r) * g.S + s, 0] = 1
            Cw = oc.conv_wide_oracle(X, Bw, np.ones((g.K, 1), np.uint8), **g.ints())
            want = np.zeros(g.Mp)
            y, x = yy - r, xx - s
            if 0 <= y < g.H and 0 <= x < g.W:
                want[y * g.P + x] = 1
            assert np.array_equal(Cw[:, 0], want), (r, s)


def test_planted_mistakes_are_caught():
    g = wl.same_geom(3, 3, 3, 1, 5, 5)
    N = 2
    X, Bw = wl.make_conv_input(8, g), _weights(9, g, N)
    mask = np.ones((g.K, N), np.uint8)
    ref = oc.conv_bruteforce(X, Bw, mask, **g.ints())
    A = oc.im2col_wide(X, **g.ints())
    # filter rows and columns exchanged; filter-major instead of channel-major rows of B
    rs_swapped = A.reshape(-1, g.C, g.R, g.S).transpose(0, 1, 3, 2).reshape(A.shape)
    k_order = A.reshape(-1, g.C, g.R * g.S).transpose(0, 2, 1).reshape(A.shape)
    for wrong in (rs_swapped, k_order):
        assert not np.allclose(og.gemm_oracle(wrong, Bw, mask), ref, atol=1e-3)
    assert np.allclose(og.gemm_oracle(A, Bw, mask), ref, rtol=1e-13, atol=1e-13)


def test_configured_layers_have_the_configured_sizes():
    (n1, g1, N1), (n2, g2, N2) = wl.CONV_LAYERS
    assert (g1.K, N1, g1.B * g1.H * g1.W) == (2304, 256, 25088)
    assert (g2.K, N2, g2.B * g2.H * g2.W) == (4608, 512, 1568)


def test_row_subset_is_a_slice_of_the_matrix():
    g = wl.same_geom(3, 3, 2, 2, 5, 4)
    X = wl.make_conv_input(9, g)
    full = oc.im2col_wide(X, **g.ints())
    rows = np.array([0, g.Mp - 1, 7, 7, 3, g.P - 1, g.L * g.P + 2])      # valid and padding positions, a repeat
    assert np.array_equal(oc.im2col_wide(X, rows=rows, **g.ints()), full[rows])
