"""Pins for the conv2d oracle (no GPU): closed forms, invariants, the literal
Eq.-5 evaluator on tiny inputs, and CPU library routines as a third opinion."""
import numpy as np
import pytest
import torch

import oracle
from oracle import merit_literal as lit


# ---------------------------------------------------------------- fp16 codec
def test_half_to_double_all_patterns_match_numpy():
    bits = np.arange(65536, dtype=np.uint16)
    want = bits.view(np.float16).astype(np.float64)
    got = np.array([oracle.half_to_double(int(b)) for b in bits])
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan], want[~nan])
    assert np.array_equal(np.signbit(got[~nan]), np.signbit(want[~nan]))


def test_double_to_half_matches_numpy_rounding():
    rng = np.random.default_rng(7)
    vals = np.concatenate([
        rng.standard_normal(20000),
        rng.standard_normal(5000) * 1e-6,            # subnormal range
        rng.standard_normal(5000) * 3e4,             # near overflow
        np.array([0.0, -0.0, 65504.0, 65519.999, 65520.0, 1e9, -1e9, 2.0 ** -24,
                  2.0 ** -25, 2.0 ** -25 * 1.0000001, 2.0 ** -14, np.inf, -np.inf]),
    ])
    # exact ties between neighbouring halves (must go to even)
    h = rng.integers(0, 0x7bff, size=5000).astype(np.uint16)
    lo = h.view(np.float16).astype(np.float64)
    hi = (h + 1).astype(np.uint16).view(np.float16).astype(np.float64)
    vals = np.concatenate([vals, 0.5 * (lo + hi), -0.5 * (lo + hi)])
    with np.errstate(over="ignore"):
        want = vals.astype(np.float16).view(np.uint16)
    got = np.array([oracle.double_to_half(float(v)) for v in vals], dtype=np.uint16)
    assert np.array_equal(got, want)


# ---------------------------------------------------------------- invariants
def _rand_half(rng, shape, scale=1.0):
    return (rng.standard_normal(shape) * scale).astype(np.float16)


def test_identity_kernel_returns_input_bit_exact():
    rng = np.random.default_rng(1)
    C = 5
    x = _rand_half(rng, (2, C, 9, 11))
    w = np.zeros((C, C, 3, 3), np.float16)
    for c in range(C):
        w[c, c, 1, 1] = 1.0
    y = oracle.conv2d(x, w, (1, 1), (1, 1))
    assert np.array_equal(y.view(np.uint16), x.view(np.uint16))


def test_all_ones_counts_valid_taps():
    Cin = 3
    x = np.ones((1, Cin, 6, 7), np.float16)
    w = np.ones((2, Cin, 3, 3), np.float16)
    y = oracle.conv2d(x, w, (1, 1), (1, 1)).astype(np.float64)
    want = np.full((6, 7), 9.0 * Cin)
    want[0, :] = want[-1, :] = 6.0 * Cin
    want[:, 0] = want[:, -1] = 6.0 * Cin
    for cy, cx in [(0, 0), (0, -1), (-1, 0), (-1, -1)]:
        want[cy, cx] = 4.0 * Cin
    assert np.array_equal(y[0, 0], want) and np.array_equal(y[0, 1], want)


def test_shifted_delta_kernel_is_a_shift_without_flip():
    """w = delta at (ky,kx) => y[oy,ox] = x[oy+ky-p, ox+kx-p]: the window index is
    ADDED (correlation, no kernel flip), and zeros enter from the border."""
    rng = np.random.default_rng(2)
    x = _rand_half(rng, (1, 1, 7, 8))
    for ky in range(3):
        for kx in range(3):
            w = np.zeros((1, 1, 3, 3), np.float16)
            w[0, 0, ky, kx] = 1.0
            y = oracle.conv2d(x, w, (1, 1), (1, 1))[0, 0]
            want = np.zeros((7, 8), np.float16)
            for oy in range(7):
                for ox in range(8):
                    iy, ix = oy + ky - 1, ox + kx - 1
                    if 0 <= iy < 7 and 0 <= ix < 8:
                        want[oy, ox] = x[0, 0, iy, ix]
            assert np.array_equal(y.view(np.uint16), want.view(np.uint16)), (ky, kx)


def test_power_of_two_scaling_is_exact():
    rng = np.random.default_rng(3)
    x = _rand_half(rng, (1, 4, 8, 8))
    w = _rand_half(rng, (3, 4, 3, 3), 0.1)
    y1 = oracle.conv2d(x, w, (1, 1), (1, 1)).astype(np.float64)
    y4 = oracle.conv2d(x, (w.astype(np.float32) * 4).astype(np.float16), (1, 1), (1, 1)).astype(np.float64)
    # no value here is near the subnormal or overflow range, so scaling commutes with rounding
    assert np.array_equal(y4, 4.0 * y1)


def test_channel_and_output_channel_indexing():
    """Distinct weights per (co, ci) catch a transposed OIHW operand."""
    x = np.zeros((1, 2, 3, 3), np.float16)
    x[0, 0, 1, 1] = 1.0
    x[0, 1, 1, 1] = 2.0
    w = np.zeros((3, 2, 1, 1), np.float16)
    w[:, 0, 0, 0] = [1, 10, 100]
    w[:, 1, 0, 0] = [3, 5, 7]
    y = oracle.conv2d(x, w, (1, 1), (0, 0)).astype(np.float64)
    assert y[0, :, 1, 1].tolist() == [1 + 6, 10 + 10, 100 + 14]
    assert np.count_nonzero(y) == 3


# -------------------------------------------------- brute force / libraries
CASES = [
    # N Cin H  W Cout kh kw sh sw ph pw
    (1, 2, 5, 6, 3, 3, 3, 1, 1, 1, 1),
    (2, 3, 9, 7, 2, 3, 3, 2, 2, 1, 1),
    (1, 3, 11, 12, 4, 7, 7, 2, 2, 3, 3),
    (1, 1, 6, 6, 1, 2, 3, 1, 2, 0, 1),
    (1, 2, 8, 5, 2, 5, 1, 3, 1, 2, 0),
]


@pytest.mark.parametrize("case", CASES)
def test_matches_literal_transform_evaluator(case):
    N, Cin, H, W, Cout, kh, kw, sh, sw, ph, pw = case
    rng = np.random.default_rng(hash(case) % 2 ** 31)
    x = _rand_half(rng, (N, Cin, H, W))
    w = _rand_half(rng, (Cout, Cin, kh, kw), 0.2)
    a = oracle.conv2d(x, w, (sh, sw), (ph, pw))
    b = lit.conv2d(x, w, (sh, sw), (ph, pw))
    assert a.shape == b.shape
    # both accumulate in double but in different orders: allow one fp16 ulp
    da = a.astype(np.float64)
    db = b.astype(np.float64)
    ulp = np.spacing(np.abs(db).astype(np.float16)).astype(np.float64)
    assert np.all(np.abs(da - db) <= ulp)
    assert np.mean(a.view(np.uint16) == b.view(np.uint16)) > 0.99


@pytest.mark.parametrize("case", CASES)
def test_matches_torch_fp64_conv(case):
    N, Cin, H, W, Cout, kh, kw, sh, sw, ph, pw = case
    rng = np.random.default_rng(11)
    x = _rand_half(rng, (N, Cin, H, W))
    w = _rand_half(rng, (Cout, Cin, kh, kw), 0.2)
    got = oracle.conv2d(x, w, (sh, sw), (ph, pw)).astype(np.float64)
    ref = torch.nn.functional.conv2d(torch.from_numpy(x.astype(np.float64)),
                                     torch.from_numpy(w.astype(np.float64)),
                                     stride=(sh, sw), padding=(ph, pw)).numpy()
    assert got.shape == ref.shape
    ulp = np.spacing(np.abs(ref).astype(np.float16)).astype(np.float64)
    assert np.all(np.abs(got - ref) <= 0.5 * ulp + 1e-12)


def test_output_extent_rule():
    # floor((I + 2p - k)/s) + 1 at the three workload shapes
    assert oracle.out_extent(112, 3, 2, 1) == 56
    assert oracle.out_extent(56, 3, 1, 1) == 56
    assert oracle.out_extent(224, 7, 2, 3) == 112


# ------------------------------------------- product function max(v1.v2, 0) (Section III-B)
def test_relu_identity_kernel_clips_the_input_at_zero():
    """Identity weights: the fused-ReLU product returns max(x, 0), with +0 for every
    non-positive input (a dropped clip or a clip of the wrong sign fails here)."""
    rng = np.random.default_rng(21)
    C = 4
    x = _rand_half(rng, (2, C, 7, 9))
    x[0, 0, 0, :3] = [-0.0, 0.0, -6.1e-5]                    # signed zero, negative subnormal
    w = np.zeros((C, C, 3, 3), np.float16)
    for c in range(C):
        w[c, c, 1, 1] = 1.0
    y = oracle.conv2d(x, w, (1, 1), (1, 1), relu=True)
    want = np.where(x > 0, x, np.float16(0.0))
    assert np.array_equal(y.view(np.uint16), want.view(np.uint16))
    assert not np.signbit(y).any()


def test_relu_closed_forms_on_constant_tensors():
    """Ones times +1 weights: the valid-tap count; times -1 weights: zero everywhere."""
    Cin = 3
    x = np.ones((1, Cin, 6, 7), np.float16)
    for sign, scale in ((1.0, 1.0), (-1.0, 0.0)):
        w = np.full((2, Cin, 3, 3), sign, np.float16)
        y = oracle.conv2d(x, w, (1, 1), (1, 1), relu=True).astype(np.float64)
        assert y[0, 0, 0, 0] == scale * Cin * 4 and y[0, 1, 0, 3] == scale * Cin * 6
        assert y[0, 0, 2, 3] == scale * Cin * 9


def test_relu_clips_before_the_single_rounding():
    """A sum just below zero must give +0, not the rounded negative; a sum in the binary16
    subnormal range must survive (clip first, round once)."""
    x = np.array([[[[1.0, 1.0]]]], np.float16).reshape(1, 2, 1, 1)
    w = np.array([[2.0 ** -14, -(2.0 ** -14) - 2.0 ** -24]], np.float16).reshape(1, 2, 1, 1)
    y = oracle.conv2d(x, w, relu=True)
    assert y.view(np.uint16)[0, 0, 0, 0] == 0                 # -2^-24 -> +0
    y = oracle.conv2d(x, -w, relu=True)
    assert float(y[0, 0, 0, 0]) == 2.0 ** -24


@pytest.mark.parametrize("stride,pad", [((1, 1), (1, 1)), ((2, 2), (3, 3)), ((2, 1), (0, 2))])
def test_relu_matches_literal_evaluator_and_torch(stride, pad):
    rng = np.random.default_rng(33)
    k = 7 if pad == (3, 3) else 3
    x = _rand_half(rng, (2, 3, 9, 10))
    w = _rand_half(rng, (4, 3, k, k), 0.3)
    got = oracle.conv2d(x, w, stride, pad, relu=True)
    assert np.array_equal(got.view(np.uint16), lit.conv2d(x, w, stride, pad, relu=True).view(np.uint16))
    ref = torch.relu(torch.nn.functional.conv2d(torch.from_numpy(x.astype(np.float64)),
                                                torch.from_numpy(w.astype(np.float64)),
                                                stride=stride, padding=pad)).numpy()
    assert np.allclose(got.astype(np.float64), ref, rtol=2e-3, atol=1e-3)
    plain = oracle.conv2d(x, w, stride, pad).astype(np.float64)
    assert np.array_equal(got.astype(np.float64), np.maximum(plain, 0.0))
    assert (plain < 0).any() and (plain > 0).any()


# ------------------------------------------- residual layer (Section III-B, remark after Listing 1)
def test_residual_special_cases_reduce_to_known_results():
    rng = np.random.default_rng(41)
    x = _rand_half(rng, (2, 3, 8, 9))
    w = _rand_half(rng, (5, 3, 3, 3), 0.3)
    plain = oracle.conv2d(x, w, (1, 1), (1, 1))
    zero = np.zeros(plain.shape, np.float16)
    # r = 0: the convolution itself, bit for bit, with and without the clip
    assert np.array_equal(oracle.conv2d_residual(x, w, zero, (1, 1), (1, 1)).view(np.uint16), plain.view(np.uint16))
    assert np.array_equal(oracle.conv2d_residual(x, w, zero, (1, 1), (1, 1), relu=True),
                          oracle.conv2d(x, w, (1, 1), (1, 1), relu=True))
    # w = 0: the added tensor itself (clipped when asked)
    r = _rand_half(rng, plain.shape)
    assert np.array_equal(oracle.conv2d_residual(x, np.zeros_like(w), r, (1, 1), (1, 1)), r)
    assert np.array_equal(oracle.conv2d_residual(x, np.zeros_like(w), r, (1, 1), (1, 1), relu=True),
                          np.maximum(r, np.float16(0)))
    # identity kernel: fp16(x + r), one rounding of the exact sum; a subtraction or a dropped term fails
    C = 3
    wi = np.zeros((C, C, 3, 3), np.float16)
    for c in range(C):
        wi[c, c, 1, 1] = 1.0
    r = _rand_half(rng, x.shape)
    want = (x.astype(np.float64) + r.astype(np.float64)).astype(np.float16)
    assert np.array_equal(oracle.conv2d_residual(x, wi, r, (1, 1), (1, 1)).view(np.uint16), want.view(np.uint16))


def test_residual_is_added_before_the_clip_and_the_single_rounding():
    # sum = 2049 (a binary16 tie: alone it rounds to 2048), r = 1: the exact 2050 is representable.
    # Rounding the sum first and adding then gives 2048.
    x = np.array([2048.0, 1.0], np.float16).reshape(1, 2, 1, 1)
    w = np.ones((1, 2, 1, 1), np.float16)
    r = np.ones((1, 1, 1, 1), np.float16)
    assert float(oracle.conv2d(x, w)[0, 0, 0, 0]) == 2048.0
    assert float(oracle.conv2d_residual(x, w, r)[0, 0, 0, 0]) == 2050.0
    # sum = -3, r = +2: clip after the addition gives 0; clipping the sum first would give 2
    x = np.array([-3.0], np.float16).reshape(1, 1, 1, 1)
    w = np.ones((1, 1, 1, 1), np.float16)
    r = np.full((1, 1, 1, 1), 2.0, np.float16)
    assert float(oracle.conv2d_residual(x, w, r, relu=True)[0, 0, 0, 0]) == 0.0
    assert float(oracle.conv2d_residual(x, w, r)[0, 0, 0, 0]) == -1.0
    # sum = +3, r = -5 -> -2 -> clipped; sum = 3, r = -1 -> 2
    assert float(oracle.conv2d_residual(-x, w, np.full((1, 1, 1, 1), -5.0, np.float16), relu=True)[0, 0, 0, 0]) == 0.0
    assert float(oracle.conv2d_residual(-x, w, np.full((1, 1, 1, 1), -1.0, np.float16), relu=True)[0, 0, 0, 0]) == 2.0


@pytest.mark.parametrize("stride,pad,relu", [((1, 1), (1, 1), True), ((2, 2), (3, 3), False), ((2, 1), (0, 2), True)])
def test_residual_matches_literal_evaluator_and_torch(stride, pad, relu):
    rng = np.random.default_rng(43)
    k = 7 if pad == (3, 3) else 3
    x = _rand_half(rng, (2, 3, 9, 10))
    w = _rand_half(rng, (4, 3, k, k), 0.3)
    shape = oracle.conv2d(x, w, stride, pad).shape
    r = _rand_half(rng, shape)
    got = oracle.conv2d_residual(x, w, r, stride, pad, relu=relu)
    want = lit.conv2d(x, w, stride, pad, relu=relu, residual=r)
    assert np.array_equal(got.view(np.uint16), want.view(np.uint16))
    ref = torch.nn.functional.conv2d(torch.from_numpy(x.astype(np.float64)), torch.from_numpy(w.astype(np.float64)),
                                     stride=stride, padding=pad) + torch.from_numpy(r.astype(np.float64))
    ref = (torch.relu(ref) if relu else ref).numpy()
    assert np.allclose(got.astype(np.float64), ref, rtol=2e-3, atol=1e-3)
    with pytest.raises(ValueError):
        oracle.conv2d_residual(x, w, r[:, :1], stride, pad)


# ------------------------------------------- dilated window (Section III-C, after Eq. 6)
def _stuff(w, dh, dw):
    """The dilated kernel written out: zeros between the taps."""
    Cout, Cin, kh, kw = w.shape
    ws = np.zeros((Cout, Cin, (kh - 1) * dh + 1, (kw - 1) * dw + 1), w.dtype)
    ws[:, :, ::dh, ::dw] = w
    return ws


@pytest.mark.parametrize("dil,stride,pad", [((2, 2), (1, 1), (2, 2)), ((3, 1), (2, 1), (1, 0)), ((1, 4), (1, 2), (0, 5))])
def test_dilated_equals_plain_conv_with_zero_stuffed_kernel(dil, stride, pad):
    """Dilation pinned to the already pinned plain convolution: same products, extra zeros."""
    rng = np.random.default_rng(41)
    x = _rand_half(rng, (2, 3, 13, 15))
    w = _rand_half(rng, (4, 3, 3, 3), 0.3)
    for relu in (False, True):
        got = oracle.conv2d(x, w, stride, pad, relu=relu, dilation=dil)
        want = oracle.conv2d(x, _stuff(w, *dil), stride, pad, relu=relu)
        assert got.shape == want.shape
        assert np.array_equal(got.view(np.uint16), want.view(np.uint16))


def test_dilated_index_expression_of_the_paper():
    """x = p + 2a with no padding: a one-hot kernel at tap (a2, a3) returns the input shifted
    by (2 a2, 2 a3), bit-exactly."""
    rng = np.random.default_rng(42)
    x = _rand_half(rng, (1, 1, 12, 14))
    for a2, a3 in ((0, 0), (1, 2), (2, 1)):
        w = np.zeros((1, 1, 3, 3), np.float16)
        w[0, 0, a2, a3] = 1.0
        y = oracle.conv2d(x, w, dilation=(2, 2))
        assert y.shape == (1, 1, 8, 10)
        assert np.array_equal(y.view(np.uint16), x[:, :, 2 * a2:2 * a2 + 8, 2 * a3:2 * a3 + 10].view(np.uint16))


def test_dilated_matches_literal_evaluator_and_torch():
    rng = np.random.default_rng(43)
    x = _rand_half(rng, (1, 4, 11, 12))
    w = _rand_half(rng, (3, 4, 3, 2), 0.3)
    got = oracle.conv2d(x, w, (2, 1), (2, 3), dilation=(2, 3))
    assert np.array_equal(got.view(np.uint16), lit.conv2d(x, w, (2, 1), (2, 3), dilation=(2, 3)).view(np.uint16))
    ref = torch.nn.functional.conv2d(torch.from_numpy(x.astype(np.float64)), torch.from_numpy(w.astype(np.float64)),
                                     stride=(2, 1), padding=(2, 3), dilation=(2, 3)).numpy()
    assert np.allclose(got.astype(np.float64), ref, rtol=2e-3, atol=1e-3)


# ------------------------------------------- convolution followed by 3x3 / s2 / p1 max pooling
def test_conv_pool_closed_form_and_library():
    """Ones * ones: conv gives the valid-tap count, whose 3x3 maximum is the full count
    Cin*9 everywhere for a 3x3 / s1 / p1 conv on >= 3x3 interiors; random data against the
    CPU library's relu -> max_pool2d."""
    x = np.ones((1, 2, 8, 8), np.float16)
    w = np.ones((3, 2, 3, 3), np.float16)
    y = oracle.conv2d_pool(x, w, (1, 1), (1, 1), relu=True).astype(np.float64)
    assert y.shape == (1, 3, 4, 4)
    assert y[0, 0, 0, 0] == 2 * 9 and np.all(y[0, :, 1:, 1:] == 18) and y[0, 2, 0, 3] == 18
    rng = np.random.default_rng(71)
    x = _rand_half(rng, (2, 3, 16, 16))
    w = _rand_half(rng, (4, 3, 7, 7), 0.1)
    got = oracle.conv2d_pool(x, w, (2, 2), (3, 3), relu=True).astype(np.float64)
    t = torch.nn.functional.conv2d(torch.from_numpy(x.astype(np.float64)), torch.from_numpy(w.astype(np.float64)),
                                   stride=2, padding=3)
    ref = torch.nn.functional.max_pool2d(torch.relu(t), 3, 2, 1).numpy()
    assert got.shape == ref.shape == (2, 4, 4, 4)
    assert np.allclose(got, ref, rtol=2e-3, atol=1e-3)
    plain = oracle.conv2d_pool(x, w, (2, 2), (3, 3), relu=False).astype(np.float64)
    assert np.array_equal(np.maximum(plain, 0.0), got)        # ReLU and max commute
