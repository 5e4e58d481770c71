"""Pins for the pool2d oracle (no GPU)."""
import numpy as np
import pytest
import torch

import oracle
from oracle import merit_literal as lit

GEOMS = [
    # H  W  kh kw sh sw ph pw
    (7, 9, 3, 3, 2, 2, 1, 1),
    (8, 8, 2, 2, 2, 2, 0, 0),
    (9, 6, 3, 2, 1, 2, 1, 0),
    (12, 10, 5, 5, 3, 3, 2, 2),
    (6, 7, 3, 3, 1, 1, 1, 1),
]


def test_max_of_constant_is_that_constant():
    for c in (1.0, -2.5, 0.0, 3.25e-3):
        x = np.full((2, 3, 10, 12), c, np.float32)
        y = oracle.pool2d(x, (3, 3), (2, 2), (1, 1), "max")
        assert y.shape == (2, 3, 5, 6)
        assert np.all(y == np.float32(c))


def test_avg_of_constant_excludes_padding():
    """An implementation that counted padding would give 4c/9 at the corner."""
    for c in (1.0, -2.5):
        x = np.full((1, 2, 8, 8), c, np.float32)
        y = oracle.pool2d(x, (3, 3), (2, 2), (1, 1), "avg")
        assert np.all(y == np.float32(c))


def test_avg_counts_4_6_9():
    """Ramp input: closed form of the mean over the in-range part of each window."""
    H = W = 8
    x = np.arange(H * W, dtype=np.float32).reshape(1, 1, H, W)
    y = oracle.pool2d(x, (3, 3), (2, 2), (1, 1), "avg")[0, 0]
    for oy in range(4):
        for ox in range(4):
            rows = [r for r in range(2 * oy - 1, 2 * oy + 2) if 0 <= r < H]
            cols = [c for c in range(2 * ox - 1, 2 * ox + 2) if 0 <= c < W]
            # mean of an affine function over a rectangle = value at its centre
            want = W * (sum(rows) / len(rows)) + sum(cols) / len(cols)
            assert y[oy, ox] == np.float32(want)
            assert len(rows) * len(cols) == (4 if (oy == 0 and ox == 0) else 6 if (oy == 0 or ox == 0) else 9)


def test_avg_sum_identity_non_overlapping():
    rng = np.random.default_rng(5)
    x = rng.integers(-8, 9, size=(1, 1, 8, 12)).astype(np.float32)
    y = oracle.pool2d(x, (2, 2), (2, 2), (0, 0), "avg")
    assert float(y.sum()) * 4 == float(x.sum())


def test_max_is_attained_and_dominates_window():
    rng = np.random.default_rng(6)
    x = rng.standard_normal((1, 1, 9, 11)).astype(np.float32)
    y = oracle.pool2d(x, (3, 3), (2, 2), (1, 1), "max")[0, 0]
    for oy in range(y.shape[0]):
        for ox in range(y.shape[1]):
            win = [x[0, 0, r, c] for r in range(2 * oy - 1, 2 * oy + 2)
                   for c in range(2 * ox - 1, 2 * ox + 2) if 0 <= r < 9 and 0 <= c < 11]
            assert y[oy, ox] in win and all(y[oy, ox] >= v for v in win)


def test_max_monotone_under_shift():
    rng = np.random.default_rng(8)
    x = rng.integers(-100, 100, size=(1, 2, 7, 7)).astype(np.float32)
    a = oracle.pool2d(x, (3, 3), (2, 2), (1, 1), "max")
    b = oracle.pool2d(x + 16.0, (3, 3), (2, 2), (1, 1), "max")
    assert np.array_equal(b, a + 16.0)


def test_negative_inputs_do_not_see_zero_padding():
    x = np.full((1, 1, 6, 6), -3.0, np.float32)
    assert np.all(oracle.pool2d(x, (3, 3), (2, 2), (1, 1), "max") == -3.0)


@pytest.mark.parametrize("g", GEOMS)
@pytest.mark.parametrize("mode", ["max", "avg"])
def test_matches_literal_transform_evaluator(g, mode):
    H, W, kh, kw, sh, sw, ph, pw = g
    rng = np.random.default_rng(H * 100 + W)
    x = rng.standard_normal((2, 2, H, W)).astype(np.float32)
    a = oracle.pool2d(x, (kh, kw), (sh, sw), (ph, pw), mode)
    b = lit.pool2d(x, (kh, kw), (sh, sw), (ph, pw), mode)
    assert a.shape == b.shape
    if mode == "max":
        assert np.array_equal(a, b)
    else:
        assert np.all(np.abs(a.astype(np.float64) - b) <= np.spacing(np.abs(b))), "more than 1 ulp"


@pytest.mark.parametrize("g", GEOMS)
def test_matches_torch(g):
    H, W, kh, kw, sh, sw, ph, pw = g
    rng = np.random.default_rng(99)
    x = rng.standard_normal((2, 3, H, W)).astype(np.float32)
    t = torch.from_numpy(x).double()
    mx = torch.nn.functional.max_pool2d(t, (kh, kw), (sh, sw), (ph, pw)).numpy()
    av = torch.nn.functional.avg_pool2d(t, (kh, kw), (sh, sw), (ph, pw),
                                        count_include_pad=False).numpy()
    assert np.array_equal(oracle.pool2d(x, (kh, kw), (sh, sw), (ph, pw), "max"), mx.astype(np.float32))
    got = oracle.pool2d(x, (kh, kw), (sh, sw), (ph, pw), "avg")
    assert np.array_equal(got, av.astype(np.float32)) or \
        np.all(np.abs(got - av) <= np.spacing(np.abs(av).astype(np.float32)))
