"""Parity of the wave-specialised many-channel convolution kernel (merit_conv2d_chws) against
the CPU oracle, through the C ABI: the caller's weights and the packed copy.  Needs a real MI355X.

Bar: 2e-2*|r| + 1e-3 (fp16 products, fp32 accumulate, one rounding, against a double sum); the
packed-weights entry point must give the same bits as merit_conv2d.
"""
import numpy as np
import pytest

import oracle
from paper_1911_03458_amd import workloads as wl

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def mb():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_1911_03458_amd import binding
    binding.lib()
    return binding


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0")


def guarded(shape, fill=777.0):
    n = int(np.prod(shape))
    pad = 64
    buf = torch.full((n + 2 * pad,), fill, dtype=torch.float16, device="cuda:0")
    return buf, buf[pad:pad + n].view(shape), pad


def canary_ok(buf, pad, fill=777.0):
    host = buf.cpu()
    return bool((host[:pad] == fill).all()) and bool((host[-pad:] == fill).all())


CHWS_CASES = [
    # N Cin H   W  Cout kh kw sh sw ph pw dh dw relu tile
    ((1, 256, 12, 56, 64, 3, 3, 1, 1, 1, 1), (1, 1), 0, None),       # 64-channel tile, 8-pixel input units
    ((2, 128, 30, 56, 160, 3, 3, 1, 1, 1, 1), (1, 1), 1, None),      # 128-channel tile, ragged last channel block
    ((1, 200, 14, 14, 70, 3, 3, 1, 1, 1, 1), (1, 1), 0, None),       # one-pixel input units, last pass half empty
    ((1, 128, 24, 24, 64, 3, 3, 2, 2, 1, 1), (1, 1), 0, (0, 0, 8, 64)),   # stride 2
    ((3, 136, 16, 24, 200, 3, 3, 1, 1, 1, 1), (1, 1), 0, (0, 0, 8, 128)),   # Cin = 8 mod 16, ragged blocks
    ((1, 512, 16, 64, 64, 1, 1, 1, 1, 0, 0), (1, 1), 0, (0, 0, 8, 64)),     # 1x1 (on request only)
    ((1, 520, 12, 64, 96, 1, 1, 1, 1, 0, 0), (1, 1), 1, (0, 0, 8, 64)),     # 1x1, ragged channels both ways
    ((2, 128, 30, 56, 160, 3, 3, 1, 1, 1, 1), (1, 1), 0, (0, 0, 8, 128)),   # 128-channel tile on 4 multiplying wavefronts
    ((2, 96, 20, 33, 256, 3, 3, 1, 1, 1, 1), (1, 1), 0, (0, 0, 12, 64)),    # 8 multiplying wavefronts, one-pixel input units
    ((1, 64, 36, 224, 128, 3, 3, 1, 1, 1, 1), (1, 1), 1, (0, 0, 12, 64)),   # 8 multiplying wavefronts, wide rows
    ((1, 64, 36, 224, 64, 3, 3, 1, 1, 1, 1), (1, 1), 0, (0, 0, 8, 64)),   # wide rows: two input units per moving thread
    ((2, 144, 20, 40, 128, 3, 3, 1, 1, 2, 2), (2, 2), 0, (0, 0, 8, 128)),   # dilated window
    ((40, 64, 48, 48, 128, 3, 3, 1, 1, 1, 1), (1, 1), 0, (0, 0, 8, 128)),   # 360 work items on 256 workgroups
    ((300, 32, 16, 16, 64, 3, 3, 1, 1, 1, 1), (1, 1), 0, (0, 0, 8, 64)),    # two passes per item, two items per workgroup
    ((2, 16, 40, 40, 64, 3, 3, 1, 1, 1, 1), (1, 1), 0, (0, 0, 8, 64)),      # a single pass per item
    ((2, 48, 27, 27, 256, 3, 3, 1, 1, 0, 0), (1, 1), 1, (0, 0, 8, 128)),    # no padding, odd width, three passes
    ((1, 64, 9, 10, 64, 1, 1, 2, 2, 0, 0), (1, 1), 0, (0, 0, 8, 64)),       # 1x1 stride 2, tiny image
    ((2, 128, 15, 28, 96, 1, 1, 2, 2, 0, 0), (1, 1), 1, None),              # 1x1 stride 2: only every second row is staged; 64 channels per pass
    ((1, 256, 30, 56, 128, 1, 1, 3, 3, 0, 0), (1, 1), 0, None),             # 1x1 stride 3
    # tiles of whole rows (wide images: two rows of 112, one of 224 in a 256-pixel tile)
    ((1, 32, 21, 112, 70, 3, 3, 1, 1, 1, 1), (1, 1), 0, (0, 0, 8, 64)),     # odd row count: the last tile is one row; ragged channels
    ((1, 64, 9, 112, 64, 1, 1, 1, 1, 0, 0), (1, 1), 1, (0, 0, 8, 64)),      # 1x1
    ((1, 32, 24, 224, 64, 3, 3, 2, 2, 1, 1), (1, 1), 0, (0, 0, 8, 64)),     # stride 2 from 224 columns to 112
    ((2, 48, 10, 112, 160, 3, 3, 1, 1, 1, 1), (1, 1), 1, (0, 0, 12, 64)),   # 128-channel tiles on 12 wavefronts
    # 5x5 windows (256 x 64 tiles; a pass's weights are 25 x 2 x 64 fragments)
    ((2, 96, 27, 27, 256, 5, 5, 1, 1, 2, 2), (1, 1), 1, None),              # the 5x5 layer of the per-layer table: one-pixel units, 6 passes
    ((1, 32, 24, 56, 64, 5, 5, 1, 1, 2, 2), (1, 1), 0, None),               # 8-pixel input units, two passes
    ((1, 40, 24, 32, 70, 5, 5, 2, 2, 2, 2), (1, 1), 0, (0, 0, 8, 64)),      # stride 2, last pass half empty, ragged channels
    ((1, 32, 30, 40, 64, 5, 5, 1, 1, 4, 4), (2, 2), 1, (0, 0, 8, 64)),      # dilated 5x5 window
    ((1, 64, 12, 16, 96, 5, 5, 1, 1, 0, 0), (1, 1), 0, (0, 0, 8, 64)),      # no padding
    # 128-pixel tiles, 32 channels per pass (the 3x3 workload's shape class)
    ((2, 64, 28, 56, 64, 3, 3, 1, 1, 1, 1), (1, 1), 0, (0, 0, 8, 32)),      # two passes
    ((3, 80, 17, 24, 40, 3, 3, 1, 1, 1, 1), (1, 1), 1, (0, 0, 8, 32)),      # last pass half empty, ragged channel block
    ((1, 40, 13, 11, 64, 3, 3, 2, 2, 1, 1), (1, 1), 0, (0, 0, 8, 32)),      # one-pixel input units, stride 2, one group of padding
    ((300, 32, 12, 16, 64, 3, 3, 1, 1, 1, 1), (1, 1), 0, (0, 0, 8, 32)),    # a single pass per item, several items per workgroup
    ((1, 96, 20, 40, 64, 1, 1, 1, 1, 0, 0), (1, 1), 0, (0, 0, 8, 32)),      # 1x1
    # two-pixel input units (W % 4 == 2: rows start on 4-byte boundaries)
    ((2, 128, 14, 14, 40, 3, 3, 1, 1, 1, 1), (1, 1), 0, None),              # the 14x14 layers' shape class, ragged channel block
    ((1, 200, 13, 14, 64, 3, 3, 1, 1, 1, 1), (1, 1), 1, None),              # last pass half empty, odd height
    ((3, 64, 14, 14, 96, 1, 1, 1, 1, 0, 0), (1, 1), 0, None),               # 1x1
    ((2, 96, 30, 30, 64, 3, 3, 2, 2, 1, 1), (1, 1), 0, None),               # stride 2 from 30 to 15 columns
    ((2, 64, 20, 42, 128, 3, 3, 1, 1, 2, 2), (2, 2), 1, (0, 0, 8, 64)),     # 256-pixel tiles, dilated
    ((1, 48, 12, 22, 256, 3, 3, 1, 1, 1, 1), (1, 1), 0, (0, 0, 12, 64)),    # 8 multiplying wavefronts: four units per moving thread
    ((1, 128, 14, 14, 256, 1, 1, 2, 2, 0, 0), (1, 1), 0, None),             # 1x1 stride 2: every second row staged
]


@pytest.mark.parametrize("case,dil,relu,tile", CHWS_CASES)
def test_chws_against_the_oracle_raw_and_packed(mb, case, dil, relu, tile):
    N, Cin, H, W, Cout, kh, kw, sh, sw, ph, pw = case
    rng = np.random.default_rng(abs(hash(case)) % 2 ** 31)
    x = rng.standard_normal((N, Cin, H, W)).astype(np.float16)
    w = (rng.standard_normal((Cout, Cin, kh, kw)) / np.sqrt(Cin * kh * kw)).astype(np.float16)
    if dil != (1, 1):
        plan = mb.merit_plan_conv2d_dilated(N, Cin, H, W, Cout, kh, kw, sh, sw, ph, pw, *dil, relu)
    elif relu:
        plan = mb.merit_plan_conv2d_relu(N, Cin, H, W, Cout, kh, kw, sh, sw, ph, pw)
    else:
        plan = mb.merit_plan_conv2d(N, Cin, H, W, Cout, kh, kw, sh, sw, ph, pw)
    if tile is not None:
        plan.set_tile(tile)
    li = plan.launch_info()
    print("chws", case, dil, relu, li, flush=True)
    assert li["kernel"] == "merit_conv2d_chws" and li["block"][0] in (512, 768) and li["lds_bytes"] <= 160 * 1024
    dx, dw_ = dev(x), dev(w)
    buf, y, pad = guarded(plan.out_shape())
    mb.merit_conv2d(plan, dx, dw_, y)
    torch.cuda.synchronize()
    assert canary_ok(buf, pad), "write outside the output"
    got = y.cpu().numpy()
    ref = oracle.conv2d(x, w, (sh, sw), (ph, pw), relu=bool(relu), dilation=dil).astype(np.float64)
    err = np.abs(got.astype(np.float64) - ref)
    tol = 2e-2 * np.abs(ref) + 1e-3
    assert np.all(err <= tol), f"max excess {np.max(err - tol)} at {np.unravel_index(np.argmax(err - tol), err.shape)}"
    if relu:
        assert not np.signbit(got).any()
    # the packed copy: same bits
    packed = mb.merit_conv2d_pack_weights(plan, dw_)
    buf2, y2, pad2 = guarded(plan.out_shape(), 555.0)
    mb.merit_conv2d_packed(plan, dx, packed, y2)
    torch.cuda.synchronize()
    assert canary_ok(buf2, pad2, 555.0), "write outside the output (packed)"
    assert np.array_equal(y2.cpu().numpy().view(np.uint16), got.view(np.uint16))


def test_chws_identity_kernel_is_exact(mb):
    rng = np.random.default_rng(11)
    C = 64
    x = rng.standard_normal((2, C, 24, 32)).astype(np.float16)
    w = np.zeros((C, C, 3, 3), np.float16)
    for c in range(C):
        w[c, c, 1, 1] = 1.0
    plan = mb.merit_plan_conv2d(2, C, 24, 32, C, 3, 3, 1, 1, 1, 1)
    plan.set_tile((0, 0, 8, 64))
    assert plan.launch_info()["kernel"] == "merit_conv2d_chws"
    y = mb.merit_conv2d(plan, dev(x), dev(w)).cpu().numpy()
    assert np.array_equal(y, x)


def test_chws_one_hot_tap_and_channel_pick_the_right_input(mb):
    """w[co, ci, ky, kx] = 1 for one (ci, ky, kx) per output channel: the output is a shifted input
    channel, so a swapped tap, a transposed window or a wrong channel group shows up exactly."""
    rng = np.random.default_rng(12)
    Cin, Cout, H, W = 48, 128, 20, 24
    x = rng.standard_normal((1, Cin, H, W)).astype(np.float16)
    w = np.zeros((Cout, Cin, 3, 3), np.float16)
    pick = [(int(rng.integers(Cin)), int(rng.integers(3)), int(rng.integers(3))) for _ in range(Cout)]
    for co, (ci, ky, kx) in enumerate(pick):
        w[co, ci, ky, kx] = 1.0
    plan = mb.merit_plan_conv2d(1, Cin, H, W, Cout, 3, 3, 1, 1, 1, 1)
    plan.set_tile((0, 0, 8, 128))
    assert plan.launch_info()["kernel"] == "merit_conv2d_chws"
    y = mb.merit_conv2d(plan, dev(x), dev(w)).cpu().numpy()
    xp = np.zeros((Cin, H + 2, W + 2), np.float16)
    xp[:, 1:-1, 1:-1] = x[0]
    for co, (ci, ky, kx) in enumerate(pick):
        assert np.array_equal(y[0, co], xp[ci, ky:ky + H, kx:kx + W]), (co, ci, ky, kx)


def test_chws_many_channel_workload_four_images(mb):
    """The 256 -> 256 3x3 layer at full size, in the launch configuration bench.py times; the
    oracle checks the first, the last and two middle images, every output of each."""
    c = wl.CFG_CONV256
    x, w = wl.make_conv_inputs(c)
    plan = mb.merit_plan_conv2d(c.N, c.Cin, c.H, c.W, c.Cout, c.kh, c.kw, c.sh, c.sw, c.ph, c.pw)
    assert plan.launch_info()["kernel"] == "merit_conv2d_chws"
    dx, dw_ = dev(x), dev(w)
    y = mb.merit_conv2d(plan, dx, dw_)
    yp = mb.merit_conv2d_packed(plan, dx, mb.merit_conv2d_pack_weights(plan, dw_))
    torch.cuda.synchronize()
    assert torch.equal(y, yp)
    y = y.cpu().numpy().astype(np.float64)
    for n in (0, 3, 4, c.N - 1):
        print("oracle image", n, flush=True)
        ref = oracle.conv2d(x[n:n + 1], w, (c.sh, c.sw), (c.ph, c.pw)).astype(np.float64)
        assert np.all(np.abs(y[n:n + 1] - ref) <= 2e-2 * np.abs(ref) + 1e-3)


def test_chws_512_channel_layer_on_28x28(mb):
    """512 -> 512 at 28x28, batch 8 (a width that is not a multiple of 8: one-pixel staging units, 32
    passes): the planner's own choice at full size; the oracle checks every output of two images."""
    N, C, H, W = 8, 512, 28, 28
    rng = np.random.default_rng(512)
    x = rng.standard_normal((N, C, H, W)).astype(np.float16)
    w = (rng.standard_normal((C, C, 3, 3)) / np.sqrt(C * 9)).astype(np.float16)
    plan = mb.merit_plan_conv2d(N, C, H, W, C, 3, 3, 1, 1, 1, 1)
    assert plan.launch_info()["kernel"] == "merit_conv2d_chws"
    y = mb.merit_conv2d(plan, dev(x), dev(w)).cpu().numpy().astype(np.float64)
    for n in (0, 5):
        ref = oracle.conv2d(x[n:n + 1], w, (1, 1), (1, 1)).astype(np.float64)
        assert np.all(np.abs(y[n:n + 1] - ref) <= 2e-2 * np.abs(ref) + 1e-3)


def test_chws_many_channel_workload_on_a_batch_of_64(mb):
    """The 256 -> 256 layer on 64 images (the bench's larger launch: three rounds of tiles per CU);
    the oracle checks every output of the first, a middle and the last image."""
    from paper_1911_03458_amd import workloads as wl
    c = wl.CFG_CONV256_B64
    x, w = wl.make_conv_inputs(c)
    plan = mb.merit_plan_conv2d(c.N, c.Cin, c.H, c.W, c.Cout, c.kh, c.kw, c.sh, c.sw, c.ph, c.pw)
    assert plan.launch_info()["kernel"] == "merit_conv2d_chws"
    y = mb.merit_conv2d(plan, dev(x), dev(w))
    for n in (0, 37, 63):
        ref = oracle.conv2d(x[n:n + 1], w, (1, 1), (1, 1)).astype(np.float64)
        got = y[n:n + 1].cpu().numpy().astype(np.float64)
        assert np.all(np.abs(got - ref) <= 2e-2 * np.abs(ref) + 1e-3), n


def test_chws_whole_row_tiles_with_an_added_tensor(mb):
    """Tiles of two whole rows of 112 (224 of the 256 pixels used) on the residual instance: the
    added tensor is read per tile, the pixels past a tile's end are never stored."""
    N, Cin, H, W, Cout = 1, 32, 11, 112, 64
    rng = np.random.default_rng(112)
    x = rng.standard_normal((N, Cin, H, W)).astype(np.float16)
    w = (rng.standard_normal((Cout, Cin, 3, 3)) / np.sqrt(Cin * 9)).astype(np.float16)
    r = rng.standard_normal((N, Cout, H, W)).astype(np.float16)
    plan = mb.merit_plan_conv2d_residual(N, Cin, H, W, Cout, 3, 3, 1, 1, 1, 1, 1)
    plan.set_tile((0, 0, 8, 64))
    li = plan.launch_info()
    assert li["kernel"] == "merit_conv2d_chws" and li["tile"][2] == 2 and li["grid"][0] == 6
    buf, y, pad = guarded(plan.out_shape())
    mb.merit_conv2d_residual(plan, dev(x), dev(w), dev(r), y)
    torch.cuda.synchronize()
    assert canary_ok(buf, pad)
    ref = oracle.conv2d_residual(x, w, r, (1, 1), (1, 1), True).astype(np.float64)
    got = y.cpu().numpy().astype(np.float64)
    assert np.all(np.abs(got - ref) <= 2e-2 * np.abs(ref) + 1e-3)


@pytest.mark.parametrize("shape", [(2, 128, 28, 28, 512), (1, 256, 14, 14, 1000), (3, 136, 9, 20, 70)])
def test_chws_1x1_layer_with_an_added_tensor(mb, shape):
    """1x1 windows with an added tensor and clipping (the closing layer of a bottleneck block) on the
    residual instance: the planner's own choice from 128 input channels on."""
    N, Cin, H, W, Cout = shape
    rng = np.random.default_rng(Cin + Cout)
    x = rng.standard_normal((N, Cin, H, W)).astype(np.float16)
    w = (rng.standard_normal((Cout, Cin, 1, 1)) / np.sqrt(Cin)).astype(np.float16)
    r = rng.standard_normal((N, Cout, H, W)).astype(np.float16)
    plan = mb.merit_plan_conv2d_residual(N, Cin, H, W, Cout, 1, 1, 1, 1, 0, 0, 1)
    assert plan.launch_info()["kernel"] == "merit_conv2d_chws", plan.launch_info()
    buf, y, pad = guarded(plan.out_shape())
    mb.merit_conv2d_residual(plan, dev(x), dev(w), dev(r), y)
    torch.cuda.synchronize()
    assert canary_ok(buf, pad)
    ref = oracle.conv2d_residual(x, w, r, (1, 1), (0, 0), True).astype(np.float64)
    got = y.cpu().numpy().astype(np.float64)
    assert np.all(np.abs(got - ref) <= 2e-2 * np.abs(ref) + 1e-3)


def test_packed_entry_points_refuse_other_plans(mb):
    plan = mb.merit_plan_conv2d(1, 3, 32, 32, 16, 7, 7, 2, 2, 3, 3)
    with pytest.raises(mb.MeritError) as e:
        mb.merit_plan_packed_weights_bytes(plan)
    assert e.value.status == mb.MERIT_ERR_UNSUPPORTED
