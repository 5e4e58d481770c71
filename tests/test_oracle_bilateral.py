"""Pins for the bilateral-filter oracle (no GPU)."""
import numpy as np
import pytest

import oracle


def _gauss(k, sigma):
    a = np.arange(k) - k // 2
    return np.exp(-0.5 * (a / sigma) ** 2).astype(np.float32)


def test_without_a_range_term_it_is_the_normalised_separable_filter():
    """norm = 0: every range weight is 1, so wxsum / wsum is the separable filter with taps
    gy[a1] gx[a2] divided by the sum of all taps (clamped pixels count like any other) —
    checked against the separately pinned separable oracle.  A window offset, an axis swap or
    a missing normalisation fails here."""
    rng = np.random.default_rng(1)
    for k in (3, 4, 7):
        x = rng.uniform(0, 255, (2, 11, 13)).astype(np.float32)
        gx, gy = _gauss(k, 1.0), (np.arange(k) + 1).astype(np.float32)      # gy asymmetric
        got = oracle.bilateral(x, gx, gy, 0.0).astype(np.float64)
        ref = oracle.sepfilter(x, gx, gy).astype(np.float64) / (gx.astype(np.float64).sum() * gy.astype(np.float64).sum())
        assert np.allclose(got, ref, rtol=2e-6, atol=1e-4)


def test_constant_image_single_tap_and_a_strong_range_term_give_the_input_back():
    c = np.full((1, 6, 7), 42.5, np.float32)
    g = _gauss(5, 1.5)
    assert np.array_equal(oracle.bilateral(c, g, g, -0.01), c)
    rng = np.random.default_rng(2)
    x = rng.uniform(0, 255, (1, 8, 9)).astype(np.float32)
    one = np.array([0.7], np.float32)
    assert np.array_equal(oracle.bilateral(x, one, one, -0.3), x)           # k = 1: w v / w
    # distinct integers and a range term that kills every other pixel: only the centre counts
    xi = rng.permutation(72).reshape(1, 8, 9).astype(np.float32)
    assert np.array_equal(oracle.bilateral(xi, g, g, -200.0), xi)


def test_edge_is_preserved_and_noise_is_smoothed():
    """A step of 100 with small noise: with sigma_r = 10 the far side's weight is exp(-50), so
    each side is averaged on its own (the mean of its own pixels in the window), unlike the
    plain Gaussian, which blurs the step."""
    rng = np.random.default_rng(3)
    H, W, k = 12, 16, 5
    base = np.zeros((1, H, W), np.float32)
    base[:, :, W // 2:] = 100.0
    x = base + rng.uniform(-1, 1, base.shape).astype(np.float32)
    g = _gauss(k, 2.0)
    y = oracle.bilateral(x, g, g, -1.0 / (2 * 10.0 ** 2))
    assert np.all(np.abs(y - base) < 1.0)                                   # no blur across the step
    assert np.abs(y - base).mean() < 0.6 * np.abs(x - base).mean()          # noise reduced
    blurred = oracle.sepfilter(x, g, g) / (g.sum() ** 2)
    assert np.abs(blurred - base).max() > 20.0


@pytest.mark.parametrize("k,norm", [(3, -0.02), (4, -0.005), (5, 0.001)])
def test_one_pixel_by_hand(k, norm):
    """The three strategy functions written out for a few pixels, borders included
    (positive norm too: the constant is used as given)."""
    rng = np.random.default_rng(k)
    x = rng.uniform(0, 50, (1, 7, 8)).astype(np.float32)
    gx = rng.uniform(0.2, 1.0, k).astype(np.float32)
    gy = rng.uniform(0.2, 1.0, k).astype(np.float32)
    y = oracle.bilateral(x, gx, gy, norm)
    for (p1, p2) in [(0, 0), (3, 4), (6, 7), (0, 5)]:
        wsum = wxsum = 0.0
        center = float(x[0, p1, p2])
        for a1 in range(k):
            for a2 in range(k):
                v = float(x[0, min(max(p1 + a1 - k // 2, 0), 6), min(max(p2 + a2 - k // 2, 0), 7)])
                w = np.exp((center - v) ** 2 * norm) * float(gy[a1]) * float(gx[a2])
                wsum += w
                wxsum += w * v
        assert abs(float(y[0, p1, p2]) - wxsum / wsum) <= 1e-6 * abs(wxsum / wsum) + 1e-6


def test_range_factor_closed_form_half_weight():
    """Section VI-A, Listing 2: a neighbour's range factor is exp(norm * (difference)^2).  A row
    `b a b` with (a - b)^2 * norm = -ln 2 gives both neighbours exactly half their spatial
    weight, so the centre output is (g1 a + (g0 + g2) b / 2) / (g1 + (g0 + g2) / 2); the table
    along the other window index multiplies numerator and denominator alike and cancels (all
    three window rows clamp to the one image row).  Numbers worked by hand: a = 10, b = 4,
    g = (1, 2, 3) -> (20 + 8) / (2 + 2) = 7.  A factor of 2 in the exponent would give
    (20 + 4) / (2 + 1) = 8, a missing square (a - b = 6 instead of 36) a weight of 2^(-1/6)."""
    norm = -np.log(2.0) / 36.0
    g = np.array([1, 2, 3], np.float32)
    other = np.array([0.3, 1.7, 0.9], np.float32)
    row = np.array([[[4, 10, 4]]], np.float32)                  # [N=1, H=1, W=3]
    y = oracle.bilateral(row, g, other, norm)
    assert abs(float(y[0, 0, 1]) - 7.0) < 1e-6
    # the same column-wise: now the table along the height carries the weights
    col = row.reshape(1, 3, 1).copy()
    y = oracle.bilateral(col, other, g, norm)
    assert abs(float(y[0, 1, 0]) - 7.0) < 1e-6
    # the border pixels: window `b b a` (left edge clamps): neighbours b (full weight, d = 0)
    # and a (half weight): (1*4 + 2*4 + 3*10/2) / (1 + 2 + 3/2) = 27 / 4.5 = 6
    y = oracle.bilateral(row, g, other, norm)
    assert abs(float(y[0, 0, 0]) - 6.0) < 1e-6
    # a quarter weight: (a - b)^2 * norm = -2 ln 2 with a - b = 6 -> norm = -2 ln 2 / 36
    y = oracle.bilateral(row, g, other, 2 * norm)
    assert abs(float(y[0, 0, 1]) - 8.0) < 1e-6


def test_output_stays_within_the_window_range():
    rng = np.random.default_rng(7)
    x = rng.uniform(0, 255, (1, 20, 20)).astype(np.float32)
    g = _gauss(7, 2.0)
    y = oracle.bilateral(x, g, g, -1.0 / (2 * 30.0 ** 2))
    assert y.min() >= x.min() and y.max() <= x.max()


def test_bad_shapes_are_rejected():
    x = np.zeros((1, 4, 4), np.float32)
    with pytest.raises(ValueError):
        oracle.bilateral(x, np.ones(3, np.float32), np.ones(2, np.float32), -1.0)
