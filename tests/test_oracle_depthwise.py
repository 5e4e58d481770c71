"""Pins for the depthwise-convolution oracle; no GPU."""
import numpy as np
import pytest
import torch

import oracle
from oracle import merit_literal as lit


def _rand_half(rng, shape, scale=1.0):
    return (rng.standard_normal(shape) * scale).astype(np.float16)


@pytest.mark.parametrize("k,stride,pad", [(3, (1, 1), (1, 1)), (3, (2, 2), (1, 1)), (5, (1, 2), (2, 0))])
def test_equals_full_convolution_with_block_diagonal_weights(k, stride, pad):
    """Pinned to the (already pinned) full convolution: weights that are zero off the
    channel diagonal give the same sums, bit for bit."""
    rng = np.random.default_rng(61)
    C = 5
    x = _rand_half(rng, (2, C, 9, 11))
    w = _rand_half(rng, (C, k, k), 0.4)
    full = np.zeros((C, C, k, k), np.float16)
    for c in range(C):
        full[c, c] = w[c]
    got = oracle.conv2d_depthwise(x, w, stride, pad)
    want = oracle.conv2d(x, full, stride, pad)
    assert got.shape == want.shape
    assert np.array_equal(got.view(np.uint16), want.view(np.uint16))


def test_channels_do_not_mix():
    rng = np.random.default_rng(62)
    x = _rand_half(rng, (1, 3, 6, 8))
    w = _rand_half(rng, (3, 3, 3))
    y = oracle.conv2d_depthwise(x, w, (1, 1), (1, 1))
    x2 = x.copy()
    x2[:, 1] = 0                                             # channel 1 changes, 0 and 2 must not
    y2 = oracle.conv2d_depthwise(x2, w, (1, 1), (1, 1))
    assert np.array_equal(y[:, 0], y2[:, 0]) and np.array_equal(y[:, 2], y2[:, 2])
    assert not np.any(y2[:, 1]) and np.any(y[:, 1])


def test_one_hot_tap_shifts_each_channel_by_its_own_tap():
    rng = np.random.default_rng(63)
    x = _rand_half(rng, (1, 2, 7, 9))
    w = np.zeros((2, 3, 3), np.float16)
    w[0, 0, 2] = 1.0                                         # channel 0: up 1, right 1 (pad 1)
    w[1, 1, 1] = 1.0                                         # channel 1: identity
    y = oracle.conv2d_depthwise(x, w, (1, 1), (1, 1))
    assert np.array_equal(y[0, 1].view(np.uint16), x[0, 1].view(np.uint16))
    want = np.zeros((7, 9), np.float16)
    want[1:, :-1] = x[0, 0, :-1, 1:]
    assert np.array_equal(y[0, 0].view(np.uint16), want.view(np.uint16))


def test_matches_literal_evaluator_and_torch():
    rng = np.random.default_rng(64)
    x = _rand_half(rng, (2, 4, 8, 10))
    w = _rand_half(rng, (4, 3, 3), 0.4)
    got = oracle.conv2d_depthwise(x, w, (2, 1), (1, 1))
    assert np.array_equal(got.view(np.uint16), lit.conv2d_depthwise(x, w, (2, 1), (1, 1)).view(np.uint16))
    ref = torch.nn.functional.conv2d(torch.from_numpy(x.astype(np.float64)),
                                     torch.from_numpy(w.astype(np.float64))[:, None], stride=(2, 1), padding=(1, 1),
                                     groups=4).numpy()
    assert np.allclose(got.astype(np.float64), ref, rtol=2e-3, atol=1e-3)
