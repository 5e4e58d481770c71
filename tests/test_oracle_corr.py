"""Pins for the correlation-layer oracle (Section III-C, Eq. 8); no GPU."""
import numpy as np
import pytest
import torch

import oracle
from oracle import merit_literal as lit


def _rand_half(rng, shape, scale=1.0):
    return (rng.standard_normal(shape) * scale).astype(np.float16)


def test_delta_images_answer_only_at_their_displacement():
    """One-hot tensors: the only non-zero output is at pixel (y0,x0), displacement
    ((y1-y0)/sd, (x1-x0)/sd); a swapped operand or a wrong sign moves or loses it."""
    H, W, R, sd = 9, 11, 2, 2
    x1 = np.zeros((1, 1, H, W), np.float16)
    x2 = np.zeros((1, 1, H, W), np.float16)
    x1[0, 0, 3, 4] = 2.0
    x2[0, 0, 7, 2] = 3.0                                   # displacement (+4, -2) = (+2, -1) * sd
    y = oracle.correlation(x1, x2, R, sd).astype(np.float64)
    want = np.zeros_like(y)
    want[0, 3, 4, R + 2, R - 1] = 6.0
    assert np.array_equal(y, want)


def test_zero_range_is_the_per_pixel_dot_product():
    rng = np.random.default_rng(51)
    a, b = _rand_half(rng, (2, 5, 6, 7)), _rand_half(rng, (2, 5, 6, 7))
    y = oracle.correlation(a, b, 0, 1)
    want = np.einsum("nchw,nchw->nhw", a.astype(np.float64), b.astype(np.float64)).astype(np.float16)
    assert y.shape == (2, 6, 7, 1, 1)
    assert np.array_equal(y[..., 0, 0].view(np.uint16), want.view(np.uint16))


def test_outside_the_image_contributes_zero():
    a = np.ones((1, 3, 4, 5), np.float16)
    y = oracle.correlation(a, a, 1, 1).astype(np.float64)
    assert y[0, 0, 0, 0, 0] == 0 and y[0, 0, 0, 1, 1] == 3 and y[0, 3, 4, 2, 2] == 0 and y[0, 1, 1, 0, 0] == 3


def test_swapping_the_operands_mirrors_the_displacement():
    """corr(a,b)[p, d] = corr(b,a)[p + d, -d] wherever p + d is inside the image."""
    rng = np.random.default_rng(52)
    a, b = _rand_half(rng, (1, 4, 8, 9)), _rand_half(rng, (1, 4, 8, 9))
    R, sd = 2, 1
    y, z = oracle.correlation(a, b, R, sd), oracle.correlation(b, a, R, sd)
    for p1, p2, d1, d2 in [(3, 4, 1, -2), (0, 0, 2, 2), (7, 8, -1, 0), (4, 1, -2, 1)]:
        assert y[0, p1, p2, R + d1, R + d2] == z[0, p1 + d1, p2 + d2, R - d1, R - d2]


@pytest.mark.parametrize("R,sd", [(1, 1), (2, 2), (3, 1)])
def test_matches_literal_evaluator_and_torch(R, sd):
    rng = np.random.default_rng(53)
    a, b = _rand_half(rng, (2, 6, 7, 9)), _rand_half(rng, (2, 6, 7, 9))
    got = oracle.correlation(a, b, R, sd)
    assert np.array_equal(got.view(np.uint16), lit.correlation(a, b, R, sd).view(np.uint16))
    # third opinion: unfold the padded second tensor with a dilated (2R+1)^2 window
    n = 2 * R + 1
    tb = torch.nn.functional.unfold(torch.from_numpy(b.astype(np.float64)), kernel_size=n, dilation=sd, padding=R * sd)
    tb = tb.reshape(2, 6, n, n, 7, 9)
    ref = torch.einsum("nchw,ncijhw->nhwij", torch.from_numpy(a.astype(np.float64)), tb).numpy()
    assert np.allclose(got.astype(np.float64), ref, rtol=2e-3, atol=1e-3)
