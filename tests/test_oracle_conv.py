"""Pins of the convolution oracle against things other than itself: a pure-Python evaluation
of the paper's sum, scipy's correlation routine, closed forms and invariants.  Each would fail
for a plausible mistake (flipped filter, swapped x/y, dropped weighing factor, wrong halo)."""
import numpy as np
import pytest
from scipy import signal

from oracle import conv_oracle as co
from oracle import conv_space_oracle as cs
from paper_1703_06503_amd import synth


def test_matches_plain_python_loops_on_a_tiny_asymmetric_case():
    A, F = synth.make_conv_inputs(7, 5, 3, 5, seed=1)      # Xf != Yf, X != Y
    got = co.conv2d(A, F, 0.37, 7, 5)
    want = np.array(co.conv2d_python(A.tolist(), F.tolist(), 0.37, 7, 5))
    assert np.allclose(got, want, rtol=1e-13, atol=1e-13)


def test_is_scipys_valid_correlation_not_its_convolution():
    A, F = synth.make_conv_inputs(40, 23, 7, 3, seed=2)
    got = co.conv2d(A, F, -1.5, 40, 23)
    corr = -1.5 * signal.correlate2d(A.astype(np.float64), F.astype(np.float64), mode="valid")
    conv = -1.5 * signal.convolve2d(A.astype(np.float64), F.astype(np.float64), mode="valid")
    assert np.allclose(got, corr, rtol=1e-12, atol=1e-12)
    assert not np.allclose(got, conv, rtol=1e-3, atol=1e-3)   # the filter is not flipped


def test_single_tap_filter_shifts_the_image():
    """F = unit impulse at (j0, i0): B[y, x] = w * A[y + j0, x + i0] exactly."""
    A, _ = synth.make_conv_inputs(31, 17, 5, 7, seed=3)
    for j0, i0 in [(0, 0), (6, 4), (2, 3), (5, 0)]:
        F = np.zeros((7, 5), dtype=np.float32)
        F[j0, i0] = 1.0
        got = co.conv2d(A, F, 2.0, 31, 17)
        assert np.array_equal(got, 2.0 * A[j0:j0 + 17, i0:i0 + 31].astype(np.float64))


def test_box_filter_on_a_ramp_has_a_closed_form():
    """A[r, c] = 3 r + 5 c, F = ones: the sum over a Yf x Xf window is
    Xf*Yf*(3 y + 5 x) + 3 Xf * Yf(Yf-1)/2 + 5 Yf * Xf(Xf-1)/2."""
    X, Y, Xf, Yf = 19, 11, 5, 3
    r, c = np.meshgrid(np.arange(Y + Yf - 1), np.arange(X + Xf - 1), indexing="ij")
    A = (3.0 * r + 5.0 * c).astype(np.float32)
    got = co.conv2d(A, np.ones((Yf, Xf), np.float32), 0.5, X, Y)
    y, x = np.meshgrid(np.arange(Y), np.arange(X), indexing="ij")
    want = 0.5 * (Xf * Yf * (3.0 * y + 5.0 * x) + 3.0 * Xf * Yf * (Yf - 1) / 2 + 5.0 * Yf * Xf * (Xf - 1) / 2)
    assert np.array_equal(got, want)


def test_linear_in_filter_and_image_and_only_the_used_part_of_a_wide_row_matters():
    A, F = synth.make_conv_inputs(25, 14, 3, 3, seed=4, lda=40)
    A2, F2 = synth.make_conv_inputs(25, 14, 3, 3, seed=5, lda=40)
    base = co.conv2d(A, F, 1.0, 25, 14)
    assert np.allclose(co.conv2d(A, F.astype(np.float64) + F2, 1.0, 25, 14), base + co.conv2d(A, F2, 1.0, 25, 14), atol=1e-12)
    assert np.allclose(co.conv2d(A.astype(np.float64) + A2, F, 1.0, 25, 14), base + co.conv2d(A2, F, 1.0, 25, 14), atol=1e-12)
    A3 = A.copy()
    A3[:, 27:] = 99.0                                       # beyond X + Xf - 1 = 27 columns
    assert np.array_equal(co.conv2d(A3, F, 1.0, 25, 14), base)
    with pytest.raises(ValueError):
        co.conv2d(A[:, :26], F, 1.0, 25, 14)                # halo missing


def test_separable_filter_equals_a_row_pass_followed_by_a_column_pass():
    """F = v u^T (outer product): the 2-D sum factors into a 1-D pass along x with u and a 1-D
    pass along y with v.  Each pass is itself the oracle with a one-row or one-column filter, and
    is checked against numpy's 1-D correlation on one line."""
    X, Y, Xf, Yf = 37, 21, 5, 3
    A, _ = synth.make_conv_inputs(X, Y, Xf, Yf, seed=7)
    rng = np.random.default_rng(8)
    u, v = rng.uniform(-1, 1, Xf), rng.uniform(-1, 1, Yf)
    rows = co.conv2d(A, u[None, :], 1.0, X, Y + Yf - 1)            # along x, all stored rows
    assert np.allclose(rows[4], np.correlate(A[4].astype(np.float64), u, mode="valid"), atol=1e-13)
    both = co.conv2d(rows, v[:, None], 0.75, X, Y)                  # then along y
    assert np.allclose(both, co.conv2d(A, np.outer(v, u), 0.75, X, Y), rtol=1e-12, atol=1e-12)


def test_translation_of_the_image_translates_the_result():
    A, F = synth.make_conv_inputs(30, 20, 3, 5, seed=9)
    full = co.conv2d(A, F, 1.0, 30, 20)
    assert np.array_equal(co.conv2d(A[3:, 4:], F, 1.0, 26, 17), full[3:, 4:])


def test_sampled_values_equal_the_full_result():
    A, F = synth.make_conv_inputs(64, 48, 7, 7, seed=6)
    full = co.conv2d(A, F, 1.0 / 49, 64, 48)
    ys, xs = [0, 47, 13, 30], [0, 63, 50, 7]
    assert np.allclose(co.conv2d_sample(A, F, 1.0 / 49, ys, xs), full[ys, xs], rtol=1e-13)


# ---- the space -----------------------------------------------------------------------------
def test_space_counts_follow_from_counting():
    """Pairs (Xwpt, VW) with VW | Xwpt: 1+2+3+4 = 10.  With L$ = 0 (PAD = 0) only the thread limit
    prunes: (Xwg, Ywg) pairs with Xwg*Ywg <= 1024 are all 16 but (32,64), (64,32), (64,64) = 13;
    so 13 * 10 * 4 (Ywpt) * 2 (UNR) = 1040 configurations, whatever the filter."""
    for Xf, Yf in [(3, 3), (7, 7), (11, 11)]:
        space = cs.enumerate_space(Xf, Yf)
        assert sum(1 for c in space if c[4] == 0) == 1040
        assert len(set(space)) == len(space) and space == sorted(space)
        for c in space:
            assert c[2] % c[5] == 0 and cs.threads(c, Xf, Yf) <= 1024
            assert cs.lds_bytes(c, Xf, Yf) <= 160 * 1024
    # a 1x1 filter needs no halo: L$ = 2 has no helper threads and caches exactly the tile
    one = cs.enumerate_space(1, 1)
    assert sum(1 for c in one if c[4] == 1) == sum(1 for c in one if c[4] == 2)
    # larger filters can only remove configurations
    assert len(cs.enumerate_space(3, 3)) >= len(cs.enumerate_space(7, 7)) >= len(cs.enumerate_space(11, 11))


def test_the_papers_best_found_configurations_lie_in_the_space():
    """Table "Best-found parameters for 2D convolution": both devices, three filter sizes."""
    rows = {3: [(32, 8, 1, 8, 0, 1, 0, 1), (64, 8, 1, 4, 0, 1, 0, 1)],
            7: [(32, 16, 2, 4, 2, 2, 1, 1), (32, 8, 2, 8, 2, 2, 0, 1)],
            11: [(32, 8, 2, 8, 2, 2, 1, 1), (32, 8, 2, 4, 1, 2, 0, 1)]}
    for f, cfgs in rows.items():
        space = set(cs.enumerate_space(f, f))
        for c in cfgs:
            assert c in space
