"""Pins for the separable-filter oracle (no GPU)."""
import numpy as np
import pytest
from scipy import ndimage

import oracle
from oracle import merit_literal as lit


def _gauss(k, sigma):
    a = np.arange(k) - k // 2
    g = np.exp(-0.5 * (a / sigma) ** 2)
    return (g / g.sum()).astype(np.float32)


def test_single_tap_and_constant_image():
    rng = np.random.default_rng(3)
    x = rng.standard_normal((2, 9, 11)).astype(np.float32)
    one = np.ones(1, np.float32)
    assert np.array_equal(oracle.sepfilter(x, one, one), x)
    assert np.array_equal(oracle.sepfilter(x, 2 * one, 3 * one), 6 * x)
    c = np.full((1, 7, 8), 1.5, np.float32)
    kx = np.array([1, 2, 3, 4], np.float32)
    ky = np.array([0.5, -1, 2, 0.25], np.float32)
    # clamped borders keep a constant image constant: the product of the two tap sums
    assert np.allclose(oracle.sepfilter(c, kx, ky), 1.5 * kx.sum() * ky.sum(), rtol=1e-6)


@pytest.mark.parametrize("k", [3, 4, 5])
def test_impulse_shows_the_unflipped_window_indexing(k):
    """y[p] = sum_a w[a] x[p + a - k//2]: an impulse at c puts w[a] at c - a + k//2 (axis by axis),
    kx along the width, ky along the height.  A flipped kernel, swapped axes or a window centred
    at (k-1)//2 fails for asymmetric taps."""
    H, W, cy, cx = 12, 13, 6, 5
    x = np.zeros((1, H, W), np.float32)
    x[0, cy, cx] = 1.0
    kx = (np.arange(k) + 1).astype(np.float32)              # 1, 2, 3 ...
    ky = (10 * (np.arange(k) + 1)).astype(np.float32)       # 10, 20, 30 ...
    y = oracle.sepfilter(x, kx, ky)[0]
    want = np.zeros((H, W), np.float32)
    for a1 in range(k):
        for a2 in range(k):
            want[cy - a1 + k // 2, cx - a2 + k // 2] = ky[a1] * kx[a2]
    assert np.array_equal(y, want)


@pytest.mark.parametrize("k", [1, 3, 6, 9])
def test_matches_library_correlation_with_nearest_border(k):
    rng = np.random.default_rng(10 + k)
    x = rng.standard_normal((2, 14, 17)).astype(np.float32)
    kx = rng.standard_normal(k).astype(np.float32)
    ky = rng.standard_normal(k).astype(np.float32)
    got = oracle.sepfilter(x, kx, ky).astype(np.float64)
    t = ndimage.correlate1d(x.astype(np.float64), kx.astype(np.float64), axis=2, mode="nearest")
    ref = ndimage.correlate1d(t, ky.astype(np.float64), axis=1, mode="nearest")
    scale = np.abs(kx).sum() * np.abs(ky).sum() * np.abs(x).max()
    assert np.all(np.abs(got - ref) <= 1e-6 * scale)


def test_equals_the_full_2d_window_with_outer_product_taps_on_the_interior():
    """Away from the border the two passes are one k x k correlation with taps ky[a1] kx[a2]."""
    rng = np.random.default_rng(5)
    k = 5
    x = rng.standard_normal((1, 16, 18)).astype(np.float32)
    kx, ky = _gauss(k, 1.0), _gauss(k, 2.0)
    got = oracle.sepfilter(x, kx, ky)[0].astype(np.float64)
    w2 = np.outer(ky, kx).astype(np.float64)
    for (p1, p2) in [(2, 2), (7, 9), (13, 15)]:
        win = x[0, p1 - 2:p1 + 3, p2 - 2:p2 + 3].astype(np.float64)
        assert abs(got[p1, p2] - (win * w2).sum()) <= 1e-6


@pytest.mark.parametrize("k", [2, 3, 7])
def test_matches_literal_transform_evaluator(k):
    rng = np.random.default_rng(20 + k)
    x = rng.standard_normal((2, 6, 9)).astype(np.float32)
    kx = rng.standard_normal(k).astype(np.float32)
    ky = rng.standard_normal(k).astype(np.float32)
    a = oracle.sepfilter(x, kx, ky).astype(np.float64)
    b = lit.sepfilter(x, kx, ky).astype(np.float64)
    assert np.all(np.abs(a - b) <= 1e-6 * np.abs(kx).sum() * np.abs(ky).sum() * np.abs(x).max())


def test_bad_shapes_are_rejected():
    x = np.zeros((1, 4, 4), np.float32)
    with pytest.raises(ValueError):
        oracle.sepfilter(x, np.ones(3, np.float32), np.ones(2, np.float32))
    with pytest.raises(ValueError):
        oracle.sepfilter(x[0], np.ones(3, np.float32), np.ones(3, np.float32))
