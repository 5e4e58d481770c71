"""Parity of the HIP library against the CPU oracle, element by element, through
the C ABI.  Needs a real MI355X.

Bars: SAD values and vectors bit-exact; max-pool exact; avg-pool within
1e-5*|r| + 1e-6 (fp32 sum of at most kh*kw terms against a double sum);
conv within 2e-2*|r| + 1e-3 (fp16 products, fp32 accumulate, against double).
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


def guarded_empty(shape, dtype, fill):
    """Output tensor inside a larger buffer whose margins hold a canary."""
    n = int(np.prod(shape))
    pad = 64
    buf = torch.full((n + 2 * pad,), fill, dtype=dtype, device="cuda:0")
    return buf, buf[pad:pad + n].view(shape), pad


def check_canary(buf, pad, fill):
    host = buf.cpu()
    assert bool((host[:pad] == fill).all()) and bool((host[-pad:] == fill).all()), "write outside the output"


# ------------------------------------------------------------------ pooling
POOL_CASES = [
    # N  C  H    W    kh kw sh sw ph pw   (rows variants: W%4==0 and OW%4==0)
    (2, 3, 32, 32, 3, 3, 2, 2, 1, 1),
    (1, 2, 70, 40, 3, 3, 2, 2, 1, 1),      # several strips and a ragged last strip
    (1, 5, 16, 24, 2, 2, 2, 2, 0, 0),
    (1, 2, 20, 12, 3, 3, 1, 1, 1, 1),
    (1, 3, 37, 29, 3, 3, 2, 2, 1, 1),      # generic kernel: odd sizes
    (2, 2, 33, 50, 5, 4, 3, 2, 2, 1),      # generic kernel: asymmetric window
    (1, 1, 130, 200, 3, 3, 2, 2, 1, 1),    # wide plane, several tiles
    (1, 1, 9, 9, 9, 9, 1, 1, 4, 4),        # window as large as the image
    (1, 2, 4, 4, 2, 2, 2, 2, 1, 1),        # corner windows hold a single element
    # 3x3 / stride 2 on widths the 16-byte kernels do not take: a lane per output column
    (2, 5, 55, 55, 3, 3, 2, 2, 0, 0),      # 27 outputs per row: two items per wavefront
    (1, 3, 13, 13, 3, 3, 2, 2, 0, 0),      # 6 outputs per row: four items per wavefront
    (1, 2, 9, 150, 3, 3, 2, 2, 1, 1),      # 75 outputs per row: two column chunks
    (1, 4, 6, 5, 3, 3, 2, 2, 0, 1),        # mixed padding, tiny plane
    (3, 7, 27, 27, 3, 3, 2, 2, 0, 0),      # items not a multiple of the wavefront's share
    # ... two output columns per lane (W >= 8): the lane's columns picked out of a 16-byte load moved inside the row
    (2, 3, 30, 301, 3, 3, 2, 2, 1, 1),     # 151 outputs per row: two chunks of 128, left padding, the last pair half outside
    (1, 3, 21, 147, 3, 3, 2, 2, 0, 0),     # 73 outputs per row on 64 lanes
    (2, 2, 17, 71, 3, 3, 2, 2, 0, 1),      # 36 outputs per row: the last lane's second column is outside
    (3, 1, 10, 35, 3, 3, 2, 2, 1, 1),      # 18 outputs per row: the narrowest rows the kernel takes, 9 of 16 lanes
    (1, 2, 11, 38, 3, 3, 2, 2, 1, 0),      # mixed padding
    (1, 2, 12, 42, 3, 3, 2, 2, 0, 0),      # even width the 16-byte kernels do not take (OW % 4 != 0)
    (3, 1, 10, 9, 3, 3, 2, 2, 1, 1),       # 9 columns on groups of 4 lanes: every lane's load is moved
    (1, 2, 11, 8, 3, 3, 2, 2, 1, 0),       # the narrowest plane the kernel takes
    # ... and 2x2 / stride 2 where the output rows are not whole 16-byte vectors
    # ... and 3x3 at stride 1 (8 output rows per group; any width of 4 and more)
    (2, 5, 35, 35, 3, 3, 1, 1, 1, 1),      # 35 outputs per row on 32 lanes, five strips with a ragged last one
    (3, 7, 17, 17, 3, 3, 1, 1, 1, 1),      # 17 outputs on 16 lanes
    (2, 9, 7, 7, 3, 3, 1, 1, 1, 1),        # 7 outputs on 4 lanes: sixteen items per wavefront
    (1, 3, 9, 5, 3, 3, 1, 1, 0, 1),        # mixed padding, 5 columns
    (1, 2, 21, 150, 3, 3, 1, 1, 1, 1),     # two chunks of 128 outputs
    (2, 3, 10, 4, 3, 3, 1, 1, 1, 1),       # the narrowest plane the kernel takes
    (1, 2, 12, 13, 3, 3, 1, 1, 0, 0),      # no padding: 11 outputs from 13 columns
    # (launches of 512 workgroups and more)
    (8, 600, 28, 28, 2, 2, 2, 2, 0, 0),    # 14 outputs per row on 8 lanes
    (40, 500, 14, 14, 2, 2, 2, 2, 0, 0),   # 7 outputs: the last lane's second column is outside the output
    (66, 300, 15, 15, 2, 2, 2, 2, 0, 0),   # odd extents: the last row and column are not used
    (9, 130, 9, 262, 2, 2, 2, 2, 0, 0),    # 131 outputs: two chunks
    (64, 257, 10, 9, 2, 2, 2, 2, 0, 0),    # 9 columns: the second lane's load is moved
    # one output per plane: the wavefront-per-plane kernel
    (3, 37, 7, 7, 7, 7, 1, 1, 0, 0),       # global pooling of 7x7 planes, planes not a multiple of 4
    (1, 5, 9, 13, 9, 13, 2, 3, 0, 0),      # 117 elements: two rounds of lanes
    (2, 6, 5, 6, 7, 8, 1, 1, 1, 1),        # window larger than the plane: padding on every side
    (1, 4, 1, 1, 1, 1, 1, 1, 0, 0),        # a single element per plane
    # padding as large as the window: the first output rows see no input element (mean of nothing = 0)
    (1, 2, 16, 32, 3, 3, 2, 2, 3, 1),      # row-strip kernel
    (1, 2, 16, 32, 3, 3, 2, 2, 4, 1),
    (1, 2, 9, 11, 3, 3, 2, 2, 3, 3),       # generic kernel, rows and columns
    # rows so wide that a strip needs more than 64 KB of LDS
    (1, 1, 16, 8192, 3, 3, 2, 2, 1, 1),
]


@pytest.mark.parametrize("case", POOL_CASES)
@pytest.mark.parametrize("mode", ["max", "avg"])
def test_pool_small(mb, case, mode):
    N, C, H, W, kh, kw, sh, sw, ph, pw = case
    rng = np.random.default_rng(abs(hash(case)) % 2 ** 31)
    x = rng.standard_normal((N, C, H, W)).astype(np.float32)
    plan = mb.merit_plan_pool2d(N, C, H, W, kh, kw, sh, sw, ph, pw, mode == "avg")
    buf, y, pad = guarded_empty(plan.out_shape(), torch.float32, 1234.5)
    print("pool", case, mode, plan.launch_info(), flush=True)
    mb.merit_pool2d(plan, dev(x), y)
    torch.cuda.synchronize()
    check_canary(buf, pad, 1234.5)
    got = y.cpu().numpy()
    ref = oracle.pool2d(x, (kh, kw), (sh, sw), (ph, pw), mode)
    assert got.shape == ref.shape
    if mode == "max":
        assert np.array_equal(got, ref)
    else:
        assert np.all(np.abs(got - ref) <= 1e-5 * np.abs(ref) + 1e-6)


@pytest.mark.parametrize("th", [1, 3, 4, 7, 8, 14, 28])
def test_pool_tile_override(mb, th):
    rng = np.random.default_rng(th)
    x = rng.standard_normal((1, 3, 112, 112)).astype(np.float32)
    for is_avg, mode in ((0, "max"), (1, "avg")):
        plan = mb.merit_plan_pool2d(1, 3, 112, 112, 3, 3, 2, 2, 1, 1, is_avg).set_tile((0, 0, th))
        print("pool tile", th, plan.launch_info(), flush=True)
        got = mb.merit_pool2d(plan, dev(x)).cpu().numpy()
        ref = oracle.pool2d(x, (3, 3), (2, 2), (1, 1), mode)
        if mode == "max":
            assert np.array_equal(got, ref)
        else:
            assert bool(np.all(np.abs(got - ref) <= 1e-5 * np.abs(ref) + 1e-6))


@pytest.mark.parametrize("th", [4, 9])
def test_pool_stride_1_row_strips_on_request(mb, th):
    # 3x3 / stride 1 / padding 1: the planner takes the two-columns-per-lane kernel; a strip height asks for the row-strip one
    rng = np.random.default_rng(40 + th)
    x = rng.standard_normal((2, 3, 20, 24)).astype(np.float32)
    for is_avg, mode in ((0, "max"), (1, "avg")):
        assert mb.merit_plan_pool2d(2, 3, 20, 24, 3, 3, 1, 1, 1, 1, is_avg).launch_info()["kernel"].startswith("merit_pool2d_lanes2_s2")
        plan = mb.merit_plan_pool2d(2, 3, 20, 24, 3, 3, 1, 1, 1, 1, is_avg).set_tile((0, 0, th))
        assert plan.launch_info()["kernel"].startswith("merit_pool2d_rows<3,3,1,1,1")
        got = mb.merit_pool2d(plan, dev(x)).cpu().numpy()
        ref = oracle.pool2d(x, (3, 3), (1, 1), (1, 1), mode)
        if mode == "max":
            assert np.array_equal(got, ref)
        else:
            assert bool(np.all(np.abs(got - ref) <= 1e-5 * np.abs(ref) + 1e-6))


@pytest.mark.parametrize("mode", ["max", "avg"])
def test_pool_full_workload(mb, mode):
    c = wl.CFG1_POOL
    x = wl.make_pool_input(c)
    plan = mb.merit_plan_pool2d(c.N, c.C, c.H, c.W, c.kh, c.kw, c.sh, c.sw, c.ph, c.pw, mode == "avg")
    print("pool full", mode, plan.launch_info(), flush=True)
    got = mb.merit_pool2d(plan, dev(x)).cpu().numpy()
    ref = oracle.pool2d(x, (c.kh, c.kw), (c.sh, c.sw), (c.ph, c.pw), mode)
    assert got.shape == (16, 64, 56, 56)
    if mode == "max":
        assert np.array_equal(got, ref)
    else:
        assert np.all(np.abs(got - ref) <= 1e-5 * np.abs(ref) + 1e-6)


def test_pool_constant_and_negative_planes(mb):
    x = np.full((1, 2, 16, 16), -3.0, np.float32)
    for mode, is_avg in (("max", 0), ("avg", 1)):
        plan = mb.merit_plan_pool2d(1, 2, 16, 16, 3, 3, 2, 2, 1, 1, is_avg)
        assert np.all(mb.merit_pool2d(plan, dev(x)).cpu().numpy() == -3.0), mode


def test_pool_empty_batch(mb):
    plan = mb.merit_plan_pool2d(0, 4, 16, 16, 3, 3, 2, 2, 1, 1, 0)
    y = mb.merit_pool2d(plan, torch.empty((0, 4, 16, 16), device="cuda:0"))
    torch.cuda.synchronize()
    assert tuple(y.shape) == (0, 4, 8, 8)


# ----------------------------------------------------------- block matching
def _sad_check(mb, cur, ref, B, R, tile=None):
    H, W = cur.shape
    plan = mb.merit_plan_sad(H, W, B, R)
    if tile is not None:
        plan.set_tile(tile)
    print("sad", (H, W, B, R), plan.launch_info(), flush=True)
    nby, nbx = plan.out_shape()
    bs, sad, p1 = guarded_empty((nby, nbx), torch.int32, -77)
    bm, mv, p2 = guarded_empty((nby, nbx, 2), torch.int32, -77)
    mb.merit_sad_search(plan, dev(cur), dev(ref), sad, mv)
    torch.cuda.synchronize()
    check_canary(bs, p1, -77)
    check_canary(bm, p2, -77)
    osad, omv = oracle.sad_search(cur, ref, B, R)
    assert np.array_equal(sad.cpu().numpy(), osad)
    assert np.array_equal(mv.cpu().numpy(), omv)


SAD_CASES = [(16, 16, 4, 2), (32, 48, 8, 4), (24, 40, 8, 3), (64, 96, 16, 8), (32, 32, 16, 5),
             (48, 64, 16, 32), (8, 8, 8, 1), (40, 24, 4, 0), (64, 64, 32, 3),
             # row-scan kernel (16x16 blocks, R = 16 / 32): ragged last group of blocks, one block row
             (64, 96, 16, 16), (80, 112, 16, 32), (16, 16, 16, 32), (32, 80, 16, 16),
             # two blocks per wavefront (8x8 blocks, R = 8 / 16): full and ragged groups of eight blocks
             (32, 64, 8, 16), (24, 88, 8, 16), (8, 8, 8, 16), (40, 72, 8, 8), (16, 136, 8, 8)]


@pytest.mark.parametrize("H,W,B,R", SAD_CASES)
def test_sad_small_random(mb, H, W, B, R):
    rng = np.random.default_rng(H * 1000 + W * 10 + R)
    cur = rng.integers(0, 256, size=(H, W), dtype=np.uint8)
    ref = rng.integers(0, 256, size=(H, W), dtype=np.uint8)
    print("sad", (H, W, B, R), flush=True)
    _sad_check(mb, cur, ref, B, R)
    # few distinct values (including 0x00 bytes): many exact ties, exercises the tie-break
    _sad_check(mb, cur & 0x3, ref & 0x3, B, R)


def test_sad_degenerate_frames(mb):
    const = np.full((32, 32), 77, np.uint8)
    _sad_check(mb, const, const, 8, 4)                      # every candidate ties: (-R,-R)
    rng = np.random.default_rng(9)
    f = rng.integers(0, 256, size=(32, 32), dtype=np.uint8)
    _sad_check(mb, f, f, 8, 4)                              # zero motion
    _sad_check(mb, np.zeros((32, 32), np.uint8), np.full((32, 32), 255, np.uint8), 16, 4)   # max SAD
    rows = np.tile(rng.permutation(256)[:32].astype(np.uint8), (32, 1))
    _sad_check(mb, rows, rows, 8, 4)                        # all dy tie
    _sad_check(mb, np.ascontiguousarray(rows.T), np.ascontiguousarray(rows.T), 8, 4)


def test_sad_generic_kernel_on_rowscan_shape(mb):
    """One block per workgroup selects the generic kernel for a shape the row-scan kernel covers."""
    rng = np.random.default_rng(21)
    cur = rng.integers(0, 256, size=(48, 64), dtype=np.uint8)
    ref = rng.integers(0, 256, size=(48, 64), dtype=np.uint8)
    _sad_check(mb, cur, ref, 16, 32, tile=(0, 1))
    _sad_check(mb, cur & 0x1, ref & 0x1, 16, 32)


def test_sad_pair_kernel(mb):
    """The two-blocks-per-wavefront kernel: the default for 8x8 blocks and for 16x16 blocks
    with R = 16 (four blocks per workgroup keep the one-block-per-wavefront kernel there);
    ties and clamping included."""
    assert mb.merit_plan_sad(720, 1280, 8, 16).launch_info()["kernel"] == "merit_sad_rowscan_pair<8,16>"
    assert mb.merit_plan_sad(64, 64, 16, 16).launch_info()["kernel"] == "merit_sad_rowscan_pair<16,16>"
    rng = np.random.default_rng(22)
    cur = rng.integers(0, 256, size=(48, 208), dtype=np.uint8)
    ref = rng.integers(0, 256, size=(48, 208), dtype=np.uint8)
    _sad_check(mb, cur, ref, 16, 16)
    _sad_check(mb, cur & 0x1, ref & 0x1, 16, 16)
    plan = mb.merit_plan_sad(48, 208, 16, 16)
    plan.set_tile((0, 4))
    assert plan.launch_info()["kernel"] == "merit_sad_rowscan16<16>"
    _sad_check(mb, cur, ref, 16, 16, tile=(0, 4))
    _sad_check(mb, cur & 0x1, ref & 0x1, 16, 16, tile=(0, 4))
    _sad_check(mb, cur, ref, 8, 16, tile=(0, 1))            # generic kernel on the same frames
    const = np.full((16, 64), 200, np.uint8)
    _sad_check(mb, const, const, 8, 16)                     # every candidate ties: (-R,-R)
    rows = np.tile(rng.permutation(256)[:64].astype(np.uint8), (16, 1))
    _sad_check(mb, rows, rows, 8, 16)                       # all dy tie
    _sad_check(mb, np.ascontiguousarray(rows[:, :16].T.repeat(4, 1)), np.ascontiguousarray(rows[:, :16].T.repeat(4, 1)), 8, 8)


def test_sad_720p_workload(mb):
    c = wl.CFG_ME_720P
    cur, ref, planted = wl.make_sad_frames(c)
    plan = mb.merit_plan_sad(c.H, c.W, c.block, c.search)
    print("sad 720p", plan.launch_info(), flush=True)
    sad, mv = mb.merit_sad_search(plan, dev(cur), dev(ref))
    sad, mv = sad.cpu().numpy(), mv.cpu().numpy()
    assert sad.shape == (90, 160) and np.all(sad == 0)      # planted copies are exact
    osad, omv = oracle.sad_search(cur, ref, c.block, c.search)
    assert np.array_equal(sad, osad)
    assert np.array_equal(mv, omv)


def test_sad_cfg0(mb):
    cur, ref, planted = wl.make_sad_frames(wl.CFG0_ME_SMALL)
    _sad_check(mb, cur, ref, 8, 4)


RAGGED_SAD_CASES = [
    # H   W   B  R  tile      kernel                       (frames the block does not divide)
    (30, 29, 8, 2, None, "merit_sad_generic"),              # both extents ragged, W not a multiple of 4
    (27, 40, 8, 3, None, "merit_sad_generic"),              # ragged height only
    (32, 46, 8, 8, None, "merit_sad_generic"),              # rows that are not whole dwords keep the row-scan kernels out
    (32, 44, 8, 8, None, "merit_sad_rowscan_pair<8,8>"),    # last block column: 4 of 8 columns inside
    (50, 100, 16, 16, None, "merit_sad_rowscan_pair<16,16>"),  # 6.25 x 3.125 blocks
    (50, 100, 16, 16, (0, 4), "merit_sad_rowscan16<16>"),
    (40, 72, 16, 32, None, "merit_sad_rowscan16<32>"),      # 4.5 block columns
    (5, 7, 8, 1, None, "merit_sad_generic"),                # frame smaller than one block
    (36, 64, 8, 8, None, "merit_sad_rowscan_pair<8,8>"),    # last block row: 4 of 8 rows inside
    (41, 96, 16, 16, None, "merit_sad_rowscan_pair<16,16>"),  # last block row: 9 of 16 rows inside
    (41, 96, 16, 16, (0, 4), "merit_sad_rowscan16<16>"),
    (56, 80, 16, 32, None, "merit_sad_rowscan16<32>"),
]


@pytest.mark.parametrize("H,W,B,R,tile,kernel", RAGGED_SAD_CASES)
def test_sad_frames_the_block_does_not_divide(mb, H, W, B, R, tile, kernel):
    rng = np.random.default_rng(H * 1000 + W * 10 + R)
    ref = rng.integers(0, 256, size=(H, W), dtype=np.uint8)
    cur = np.roll(ref, (1, -2), axis=(0, 1))                 # a real minimum away from the origin
    cur[::3] = rng.integers(0, 256, size=cur[::3].shape, dtype=np.uint8)
    plan = mb.merit_plan_sad(H, W, B, R)
    if tile is not None:
        plan.set_tile(tile)
    assert plan.launch_info()["kernel"] == kernel
    _sad_check(mb, cur, ref, B, R, tile)
    _sad_check(mb, cur & 3, ref & 3, B, R, tile)             # many ties


def test_sad_1080p_workload(mb):
    """Full HD at its real height (67.5 block rows): every block against the oracle."""
    c = wl.CFG_ME_1080P
    cur, ref, planted = wl.make_sad_frames(c)
    plan = mb.merit_plan_sad(c.H, c.W, c.block, c.search)
    assert plan.launch_info()["kernel"] == "merit_sad_rowscan16<32>" and plan.out_shape() == (68, 120)
    sad, mv = mb.merit_sad_search(plan, dev(cur), dev(ref))
    torch.cuda.synchronize()
    sad, mv = sad.cpu().numpy(), mv.cpu().numpy()
    assert np.all(sad[:67] == 0)                             # planted copies are exact inside the frame
    osad, omv = oracle.sad_search(cur, ref, c.block, c.search)
    assert np.array_equal(sad, osad) and np.array_equal(mv, omv)


def test_sad_full_hd_workload(mb):
    c = wl.CFG3_ME_FHD
    cur, ref, planted = wl.make_sad_frames(c)
    plan = mb.merit_plan_sad(c.H, c.W, c.block, c.search)
    print("sad full", plan.launch_info(), flush=True)
    sad, mv = mb.merit_sad_search(plan, dev(cur), dev(ref))
    torch.cuda.synchronize()
    sad, mv = sad.cpu().numpy(), mv.cpu().numpy()
    # properties that hold at any size: planted copies are exact, so the minimum is 0
    assert sad.shape == (68, 120) and np.all(sad == 0)
    osad, omv = oracle.sad_search(cur, ref, c.block, c.search)
    assert np.array_equal(sad, osad)
    assert np.array_equal(mv, omv)


# -------------------------------------------------- depthwise convolution
DW_CASES = [
    # N  C   H   W  kh kw sh sw ph pw tile
    (1, 3, 9, 16, 3, 3, 1, 1, 1, 1, None),       # row kernel, one strip
    (2, 5, 70, 64, 3, 3, 1, 1, 1, 1, None),      # row kernel, two strips, the second ragged
    (1, 2, 12, 136, 3, 3, 1, 1, 1, 1, None),     # row kernel, wide rows
    (2, 5, 70, 64, 3, 3, 1, 1, 1, 1, (0, 0, 16)),  # generic kernel on the same shape
    (1, 4, 11, 13, 3, 3, 2, 2, 1, 1, None),      # generic: stride 2, odd sizes
    (2, 3, 17, 10, 5, 3, 1, 2, 2, 0, None),      # generic: rectangular window, mixed stride / padding
    (1, 1, 8, 8, 1, 1, 1, 1, 0, 0, None),        # pointwise scale
    (1, 1, 40, 1200, 31, 3, 1, 1, 15, 1, None),  # generic: tall window on wide rows, more than 64 KB of LDS
    (1, 2, 12, 2800, 3, 3, 1, 1, 1, 1, None),    # row kernel, rows so wide that a strip needs more than 64 KB
]


@pytest.mark.parametrize("case", DW_CASES)
def test_depthwise(mb, case):
    N, C, H, W, kh, kw, sh, sw, ph, pw, tile = case
    rng = np.random.default_rng(abs(hash(case[:10])) % 2 ** 31)
    x = rng.standard_normal((N, C, H, W)).astype(np.float16)
    w = (rng.standard_normal((C, kh, kw)) / np.sqrt(kh * kw)).astype(np.float16)
    plan = mb.merit_plan_conv2d_depthwise(N, C, H, W, kh, kw, sh, sw, ph, pw)
    if tile is not None:
        plan.set_tile(tile)
    print("dwconv", case, plan.launch_info(), flush=True)
    buf, y, pad = guarded_empty(plan.out_shape(), torch.float16, 777.0)
    mb.merit_conv2d_depthwise(plan, dev(x), dev(w), y)
    torch.cuda.synchronize()
    check_canary(buf, pad, 777.0)
    got = y.cpu().numpy().astype(np.float64)
    ref = oracle.conv2d_depthwise(x, w, (sh, sw), (ph, pw)).astype(np.float64)
    assert got.shape == ref.shape
    assert np.all(np.abs(got - ref) <= 2e-2 * np.abs(ref) + 1e-3)


def test_depthwise_one_hot_taps_are_exact(mb):
    rng = np.random.default_rng(7)
    x = rng.standard_normal((1, 2, 16, 24)).astype(np.float16)
    w = np.zeros((2, 3, 3), np.float16)
    w[0, 0, 2] = 1.0
    w[1, 1, 1] = 1.0
    y = mb.merit_conv2d_depthwise(mb.merit_plan_conv2d_depthwise(1, 2, 16, 24, 3, 3, 1, 1, 1, 1), dev(x), dev(w))
    y = y.cpu().numpy()
    want = np.zeros((16, 24), np.float16)
    want[1:, :-1] = x[0, 0, :-1, 1:]
    assert np.array_equal(y[0, 1], x[0, 1]) and np.array_equal(y[0, 0], want)


def test_depthwise_workload(mb):
    c = wl.CFG_DEPTHWISE
    x, w = wl.make_depthwise_inputs(c)
    plan = mb.merit_plan_conv2d_depthwise(c.N, c.C, c.H, c.W, c.kh, c.kw, c.sh, c.sw, c.ph, c.pw)
    assert plan.launch_info()["kernel"] == "merit_dwconv_rows_k3s1p1"
    y = mb.merit_conv2d_depthwise(plan, dev(x), dev(w)).cpu().numpy().astype(np.float64)
    ref = oracle.conv2d_depthwise(x, w, (c.sh, c.sw), (c.ph, c.pw)).astype(np.float64)
    assert np.all(np.abs(y - ref) <= 2e-2 * np.abs(ref) + 1e-3)


# ------------------------------------------------------- correlation layer
CORR_CASES = [
    # N  C   H   W   R  sd
    (1, 8, 8, 8, 1, 1),
    (2, 20, 9, 24, 2, 1),        # channels not a multiple of 8
    (1, 64, 12, 72, 5, 2),       # two pixel chunks, the second ragged
    (1, 130, 6, 64, 3, 3),       # two channel passes
    (1, 16, 10, 16, 0, 1),       # zero range: the per-pixel dot product
    (1, 32, 5, 40, 15, 1),       # widest range: 31 displacements, three column blocks per pixel block
    (1, 40, 7, 128, 8, 1),       # two column blocks exactly (16 + 2R = 32); channel groups padded to 8
    (1, 24, 20, 64, 9, 2),       # three column blocks with two residue classes
    (2, 72, 9, 80, 2, 4),        # four residue classes
    (1, 16, 30, 64, 4, 5),       # classes of unequal size (13, 13, 13, 13, 12): five pixel blocks
    (1, 48, 44, 72, 2, 8),       # eight classes: two pixel blocks per wavefront
    (1, 264, 23, 64, 5, 3),      # three channel passes, classes of 22, 21, 21 pixels in two blocks each
]


@pytest.mark.parametrize("case", CORR_CASES)
def test_correlation(mb, case):
    N, C, H, W, R, sd = case
    rng = np.random.default_rng(abs(hash(case)) % 2 ** 31)
    x1 = (rng.standard_normal((N, C, H, W)) / np.sqrt(C)).astype(np.float16)
    x2 = rng.standard_normal((N, C, H, W)).astype(np.float16)
    plan = mb.merit_plan_correlation(N, C, H, W, R, sd)
    print("corr", case, plan.launch_info(), flush=True)
    buf, y, pad = guarded_empty(plan.out_shape(), torch.float16, 777.0)
    mb.merit_correlation(plan, dev(x1), dev(x2), y)
    torch.cuda.synchronize()
    check_canary(buf, pad, 777.0)
    got = y.cpu().numpy().astype(np.float64)
    ref = oracle.correlation(x1, x2, R, sd).astype(np.float64)
    assert np.all(np.abs(got - ref) <= 2e-2 * np.abs(ref) + 1e-3)
    if R > 0:                                                       # displaced above the first row: exact zeros
        assert np.all(got[:, 0, :, 0, :] == 0) and np.all(ref[:, 0, :, 0, :] == 0)


def test_correlation_delta_images(mb):
    """One-hot tensors answer at exactly one pixel and displacement."""
    H, W, R, sd = 16, 24, 3, 2
    x1 = np.zeros((1, 8, H, W), np.float16)
    x2 = np.zeros((1, 8, H, W), np.float16)
    x1[0, 5, 6, 7] = 2.0
    x2[0, 5, 10, 3] = 3.0                                           # displacement (+4, -4) = (+2, -2) * sd
    y = mb.merit_correlation(mb.merit_plan_correlation(1, 8, H, W, R, sd), dev(x1), dev(x2)).cpu().numpy()
    want = np.zeros((1, H, W, 7, 7), np.float16)
    want[0, 6, 7, R + 2, R - 2] = 6.0
    assert np.array_equal(y, want)


def test_correlation_paper_shape(mb):
    c = wl.CFG_CORRELATION
    x1, x2 = wl.make_correlation_inputs(c)
    plan = mb.merit_plan_correlation(c.N, c.C, c.H, c.W, c.search, c.stride)
    y = mb.merit_correlation(plan, dev(x1), dev(x2)).cpu().numpy().astype(np.float64)
    ref = oracle.correlation(x1, x2, c.search, c.stride).astype(np.float64)
    assert y.shape == (1, 64, 64, 11, 11)
    assert np.all(np.abs(y - ref) <= 2e-2 * np.abs(ref) + 1e-3)


# ------------------------------------------------------------- convolution
def _conv_check(mb, x, w, stride, pad, tile=None, relu=False, dilation=(1, 1)):
    N, Cin, H, W = x.shape
    Cout, _, kh, kw = w.shape
    if dilation != (1, 1):
        plan = mb.merit_plan_conv2d_dilated(N, Cin, H, W, Cout, kh, kw, *stride, *pad, *dilation, int(relu))
    else:
        make = mb.merit_plan_conv2d_relu if relu else mb.merit_plan_conv2d
        plan = make(N, Cin, H, W, Cout, kh, kw, *stride, *pad)
    if tile is not None:
        plan.set_tile(tile)
    print("conv", x.shape, w.shape, stride, pad, plan.launch_info(), flush=True)
    buf, y, p = guarded_empty(plan.out_shape(), torch.float16, 777.0)
    mb.merit_conv2d(plan, dev(x), dev(w), y)
    torch.cuda.synchronize()
    check_canary(buf, p, 777.0)
    got = y.cpu().numpy().astype(np.float64)
    ref = oracle.conv2d(x, w, stride, pad, relu=relu, dilation=dilation).astype(np.float64)
    assert got.shape == ref.shape
    if relu:                                       # clipped at +0: no negative value, no -0
        assert not np.signbit(got).any()
    err = np.abs(got - ref)
    tol = 2e-2 * np.abs(ref) + 1e-3
    ok = bool(np.all(err <= tol))
    assert ok, f"max excess {np.max(err - tol)} at {np.unravel_index(np.argmax(err - tol), err.shape)}"
    return got, ref


CONV_CASES = [
    # N Cin H   W  Cout kh kw sh sw ph pw
    (1, 3, 20, 24, 64, 7, 7, 2, 2, 3, 3),      # planar, stride 2
    (2, 3, 17, 19, 40, 7, 7, 2, 2, 3, 3),      # planar, odd sizes, ragged channels
    (1, 1, 12, 16, 8, 3, 3, 1, 1, 1, 1),       # planar, odd stride alignment
    (1, 4, 9, 40, 33, 5, 5, 1, 2, 2, 2),       # planar, even group count, mixed strides
    (1, 3, 30, 30, 16, 1, 8, 1, 1, 0, 4),      # planar, 8-wide window
    (1, 16, 12, 16, 32, 3, 3, 1, 1, 1, 1),     # channel-block, vector staging
    (2, 64, 14, 16, 64, 3, 3, 1, 1, 1, 1),     # channel-block, the 3x3 workload's shape class
    (1, 24, 10, 12, 48, 3, 3, 2, 2, 1, 1),     # channel-block, padded channel group, stride 2
    (1, 20, 9, 11, 10, 2, 3, 1, 1, 0, 1),      # channel-block, scalar staging everywhere
    (1, 32, 8, 8, 96, 1, 1, 1, 1, 0, 0),       # channel-block, 1x1, three channel blocks
    (1, 8, 40, 40, 16, 5, 5, 1, 1, 2, 2),      # channel-block, many tiles per image
    # layers whose operands do not fit LDS at once: the channels go through in passes
    (1, 200, 14, 14, 70, 3, 3, 1, 1, 1, 1),    # passes, vector weight staging, three channel blocks
    (2, 35, 12, 18, 52, 7, 5, 1, 1, 3, 3),     # passes, scalar weight staging, ragged channels
    (1, 96, 27, 27, 40, 5, 5, 1, 1, 2, 2),     # passes, the 5x5 / 96-channel layer class
    (1, 520, 9, 16, 64, 1, 1, 1, 1, 0, 0),     # passes, 1x1 over many channels
    (1, 64, 20, 120, 32, 3, 3, 1, 1, 1, 1),    # passes because the rows are wide
    (1, 128, 21, 23, 64, 3, 3, 2, 2, 1, 1),    # passes, stride 2, odd sizes
    # passes on the vector staging paths (3x3 or 1x1, Cin % 8 = 0, W % 8 = 0)
    (1, 256, 20, 56, 64, 3, 3, 1, 1, 1, 1),    # 3x3 passes, two channel blocks
    (2, 136, 9, 24, 40, 3, 3, 1, 1, 1, 1),     # last pass padded with zero channels, ragged blocks
    (1, 128, 24, 24, 64, 3, 3, 2, 2, 1, 1),    # 3x3 passes, stride 2
    (1, 512, 16, 64, 64, 1, 1, 1, 1, 0, 0),    # 1x1 passes
    (1, 520, 12, 64, 96, 1, 1, 1, 1, 0, 0),    # 1x1 passes, three channel blocks in two groups
    # the same kernels with 64-channel blocks (grids of more than 128 workgroups keep them)
    (70, 35, 12, 18, 52, 7, 5, 1, 1, 3, 3),    # passes, scalar weight staging
    (33, 200, 14, 14, 70, 3, 3, 1, 1, 1, 1),   # passes, 3x3, one-pixel input units
    (17, 256, 20, 56, 64, 3, 3, 1, 1, 1, 1),   # passes, 3x3, 8-pixel input units
    (20, 520, 12, 64, 96, 1, 1, 1, 1, 0, 0),   # passes, 1x1
    # planar, window rows of 9 to 16 taps: two 8-slot fragments per row
    (1, 3, 67, 67, 48, 11, 11, 4, 4, 5, 5),    # the paper's strided example: x = 4p + a - 5, 11x11 window
    (2, 5, 30, 41, 7, 9, 12, 2, 3, 4, 6),      # odd column stride: funnel-shifted fragments
    (3, 3, 44, 48, 40, 11, 11, 4, 4, 5, 5),    # W % 8 == 0: vector staging with prefetch, several tiles
    (2, 1, 20, 64, 33, 1, 16, 1, 2, 0, 8),     # one channel, one window row of 16 taps, widest padding
    (1, 2, 25, 37, 16, 3, 9, 1, 2, 1, 4),      # 9 taps, even stride, even start: no front slot
    (1, 4, 23, 31, 20, 2, 15, 2, 2, 1, 7),     # 15 taps + the front slot: all 16 slots
    (9, 3, 40, 40, 64, 9, 9, 1, 1, 4, 4),      # stride 1, several tiles per workgroup
    (1, 1, 22, 17, 53, 1, 7, 3, 3, 0, 1),      # the weight tensor ends in the middle of a 16-byte vector
    (9, 2, 150, 131, 144, 9, 9, 3, 3, 2, 3),   # more 128-pixel tiles than compute units: 256-pixel tiles on 8 wavefronts
    (2, 3, 29, 30, 37, 7, 7, 2, 2, 3, 3),      # W % 4 == 2, 225 pixels per output plane: every alignment of a plane's start
    (3, 3, 30, 29, 37, 5, 5, 1, 1, 1, 1),      # odd W, 756 pixels per plane (8-byte aligned planes), several tiles
    (5, 1, 19, 23, 9, 3, 3, 1, 1, 0, 0),       # planes of 357 pixels on 9 channels: runs shorter than a unit's reach at the ends
    # neither MFMA kernel: the one-element-per-thread kernel
    (1, 3, 40, 44, 10, 5, 17, 2, 2, 2, 8),     # 17 taps per window row on few channels
    (2, 5, 30, 41, 7, 9, 12, 2, 3, 4, 9),      # padding wider than the staged left margin
]


@pytest.mark.parametrize("case", CONV_CASES)
def test_conv_small(mb, case):
    N, Cin, H, W, Cout, kh, kw, sh, sw, ph, pw = case
    rng = np.random.default_rng(abs(hash(case)) % 2 ** 31)
    x = rng.standard_normal((N, Cin, H, W)).astype(np.float16)
    w = (rng.standard_normal((Cout, Cin, kh, kw)) / np.sqrt(Cin * kh * kw)).astype(np.float16)
    _conv_check(mb, x, w, (sh, sw), (ph, pw))


@pytest.mark.parametrize("tile", [(0, 0, 4, 32), (0, 0, 4, 64)])
def test_conv_tile_override(mb, tile):
    rng = np.random.default_rng(3)
    x = rng.standard_normal((1, 16, 24, 24)).astype(np.float16)
    w = (rng.standard_normal((32, 16, 3, 3)) / 12).astype(np.float16)
    _conv_check(mb, x, w, (1, 1), (1, 1), tile)


@pytest.mark.parametrize("tile", [(0, 0, 4, 32), (0, 0, 4, 64), (0, 0, 8, 32), (0, 0, 8, 64)])
def test_conv_tile_override_few_channels(mb, tile):
    rng = np.random.default_rng(5)
    x = rng.standard_normal((2, 3, 40, 48)).astype(np.float16)
    w = (rng.standard_normal((40, 3, 7, 7)) / 12).astype(np.float16)
    _conv_check(mb, x, w, (2, 2), (3, 3), tile)


@pytest.mark.parametrize("tile", [None, (0, 0, 8, 32), (0, 0, 4, 64)])
def test_conv_two_fragment_rows_tilings(mb, tile):
    # window rows of 11 taps (two 8-slot fragments) on every tiling of the planar kernel; the planner
    # itself takes 8 wavefronts when the layer has more 128-pixel tiles than the chip has compute units
    big = mb.merit_plan_conv2d(9, 2, 150, 131, 144, 9, 9, 3, 3, 2, 3).launch_info()
    assert big["kernel"] == "merit_conv2d_planar" and big["block"][0] == 512
    rng = np.random.default_rng(17)
    x = rng.standard_normal((3, 3, 75, 83)).astype(np.float16)
    w = (rng.standard_normal((56, 3, 11, 11)) / 19).astype(np.float16)
    _conv_check(mb, x, w, (4, 4), (2, 0), tile)


WS_CASES = [
    # wave-specialised kernel (tile 8 x 64): one tile, several tiles per workgroup, ragged ends
    (1, 3, 20, 24, 64, 7, 7, 2, 2, 3, 3),
    (3, 3, 64, 72, 40, 7, 7, 2, 2, 3, 3),
    (2, 1, 33, 40, 8, 3, 3, 1, 1, 1, 1),
    (300, 3, 32, 32, 64, 7, 7, 2, 2, 3, 3),    # 300 tiles on 256 workgroups: 1 or 2 tiles each
    (1100, 3, 32, 32, 64, 7, 7, 2, 2, 3, 3),   # 4 or 5 tiles each: both LDS buffers reused
    (1, 4, 96, 160, 33, 5, 5, 1, 2, 2, 2),
]


WS_UNALIGNED_CASES = [
    # the same kernel where image rows or output planes start on any element
    (1, 3, 61, 67, 40, 7, 7, 2, 2, 3, 3),      # odd width, odd element count (the tensor's last unit crosses its end), planes of 1054 pixels
    (3, 3, 61, 67, 40, 7, 7, 2, 2, 3, 3),      # every parity of an image's start
    (2, 3, 40, 48, 33, 3, 3, 1, 1, 0, 0),      # W % 8 == 0, planes of 1748 pixels: only the stores are off the grid
    (2, 3, 34, 36, 33, 5, 5, 1, 1, 2, 2),      # W % 8 == 4, planes of 1224 pixels: only the rows are
    (300, 3, 31, 33, 64, 7, 7, 2, 2, 3, 3),    # 600 tiles on 256 workgroups: both LDS buffers reused
    (2, 1, 37, 45, 9, 3, 3, 1, 1, 1, 1),       # one channel, 9 output channels, planes of 1665 pixels
    (5, 2, 23, 19, 70, 4, 4, 1, 1, 0, 0),      # planes of 320 pixels behind an odd width; three 32-channel blocks in two groups
    (64, 3, 32, 36, 16, 3, 3, 1, 1, 0, 0),     # planes of 1020 pixels, 256 tiles: overlapping tiles would need a second round, so every tile has loose ends
]


@pytest.mark.parametrize("case", WS_UNALIGNED_CASES)
def test_conv_wave_specialised_unaligned(mb, case):
    N, Cin, H, W, Cout, kh, kw, sh, sw, ph, pw = case
    rng = np.random.default_rng(abs(hash(case)) % 2 ** 31)
    x = rng.standard_normal((N, Cin, H, W)).astype(np.float16)
    w = (rng.standard_normal((Cout, Cin, kh, kw)) / np.sqrt(Cin * kh * kw)).astype(np.float16)
    plan = mb.merit_plan_conv2d(N, Cin, H, W, Cout, kh, kw, sh, sw, ph, pw)
    plan.set_tile((0, 0, 8, 64))
    assert plan.launch_info()["kernel"] == "merit_conv2d_planar_ws"
    _conv_check(mb, x, w, (sh, sw), (ph, pw), (0, 0, 8, 64))


@pytest.mark.parametrize("case", WS_CASES)
def test_conv_wave_specialised(mb, case):
    N, Cin, H, W, Cout, kh, kw, sh, sw, ph, pw = case
    rng = np.random.default_rng(abs(hash(case)) % 2 ** 31)
    x = rng.standard_normal((N, Cin, H, W)).astype(np.float16)
    w = (rng.standard_normal((Cout, Cin, kh, kw)) / np.sqrt(Cin * kh * kw)).astype(np.float16)
    plan = mb.merit_plan_conv2d(N, Cin, H, W, Cout, kh, kw, sh, sw, ph, pw)
    plan.set_tile((0, 0, 8, 64))
    assert plan.launch_info()["kernel"] == "merit_conv2d_planar_ws"
    _conv_check(mb, x, w, (sh, sw), (ph, pw), (0, 0, 8, 64))


RELU_CASES = [
    # the fused-ReLU product function on each kernel: wave-specialised planar, planar, channel-block
    ((300, 3, 32, 32, 64, 7, 7, 2, 2, 3, 3), (0, 0, 8, 64), "merit_conv2d_planar_ws"),
    ((2, 3, 17, 19, 40, 7, 7, 2, 2, 3, 3), None, "merit_conv2d_planar"),
    ((1, 16, 12, 16, 32, 3, 3, 1, 1, 1, 1), None, "merit_conv2d_chblock"),
    ((2, 64, 28, 28, 64, 3, 3, 1, 1, 1, 1), (0, 0, 4, 32), "merit_conv2d_chblock"),
    ((2, 64, 28, 28, 64, 3, 3, 1, 1, 1, 1), None, "merit_conv2d_chws"),
]


@pytest.mark.parametrize("case,tile,kernel", RELU_CASES)
def test_conv_relu_product_function(mb, case, tile, kernel):
    N, Cin, H, W, Cout, kh, kw, sh, sw, ph, pw = case
    plan = mb.merit_plan_conv2d_relu(N, Cin, H, W, Cout, kh, kw, sh, sw, ph, pw)
    if tile is not None:
        plan.set_tile(tile)
    assert plan.launch_info()["kernel"] == kernel
    rng = np.random.default_rng(abs(hash(case)) % 2 ** 31)
    x = rng.standard_normal((N, Cin, H, W)).astype(np.float16)
    w = (rng.standard_normal((Cout, Cin, kh, kw)) / np.sqrt(Cin * kh * kw)).astype(np.float16)
    got, ref = _conv_check(mb, x, w, (sh, sw), (ph, pw), tile, relu=True)
    assert (ref == 0).mean() > 0.3 and (ref > 0).mean() > 0.3      # both branches exercised


def test_conv_relu_identity_kernel_clips_exactly(mb):
    rng = np.random.default_rng(5)
    C = 16
    x = rng.standard_normal((1, C, 12, 16)).astype(np.float16)
    x[0, 0, 0, :2] = [-0.0, -6.1e-5]
    w = np.zeros((C, C, 3, 3), np.float16)
    for c in range(C):
        w[c, c, 1, 1] = 1.0
    got, ref = _conv_check(mb, x, w, (1, 1), (1, 1), relu=True)
    assert np.array_equal(got, np.maximum(x.astype(np.float64), 0.0))


_CFG4_ORACLE = {}


def cfg4_oracle(relu):
    """The oracle on the whole batch of the 7x7 workload (every image, every output), computed
    once per test session and clipping mode (about 10-20 s of host time each)."""
    if relu not in _CFG4_ORACLE:
        c = wl.CFG4_CONV7
        x, w = wl.make_conv_inputs(c)
        print("oracle: 7x7 workload, whole batch, relu =", relu, flush=True)
        _CFG4_ORACLE[relu] = oracle.conv2d(x, w, (c.sh, c.sw), (c.ph, c.pw), relu=relu)
    return _CFG4_ORACLE[relu]


def test_conv_7x7_workload_relu_every_image(mb):
    """Full-size launch with the clipped product function; the oracle checks every output of
    every image."""
    c = wl.CFG4_CONV7
    x, w = wl.make_conv_inputs(c)
    plan = mb.merit_plan_conv2d_relu(c.N, c.Cin, c.H, c.W, c.Cout, c.kh, c.kw, c.sh, c.sw, c.ph, c.pw)
    assert plan.launch_info()["kernel"] == "merit_conv2d_planar_ws"
    y = mb.merit_conv2d(plan, dev(x), dev(w))
    got = y.cpu().numpy().astype(np.float64)
    ref = cfg4_oracle(True).astype(np.float64)
    assert not np.signbit(got).any()
    assert np.all(np.abs(got - ref) <= 2e-2 * np.abs(ref) + 1e-3)
    plain = mb.merit_conv2d(mb.merit_plan_conv2d(c.N, c.Cin, c.H, c.W, c.Cout, c.kh, c.kw, c.sh, c.sw, c.ph, c.pw),
                            dev(x), dev(w))
    assert torch.equal(y, torch.clamp_min(plain, 0.0) + 0.0)      # same products, clipped; "+ 0.0" folds -0


POOLFUSE_CASES = [
    # N Cin H   W  Cout kh kw sh sw ph pw relu
    (2, 3, 64, 64, 64, 7, 7, 2, 2, 3, 3, 1),    # 4 bands of 4 pooled rows per image
    (3, 3, 40, 64, 40, 3, 3, 1, 1, 1, 1, 0),    # ragged channels, no clipping, odd window alignment
    (1, 3, 44, 32, 64, 3, 3, 1, 1, 1, 1, 1),    # last band shorter than the others
    (2, 1, 16, 128, 32, 5, 5, 1, 1, 2, 2, 0),   # widest row pair (2 x 128 = the whole tile), one channel block
    (300, 3, 32, 32, 64, 7, 7, 2, 2, 3, 3, 1),  # more images than compute units: one band per image
    (1, 2, 8, 16, 8, 3, 3, 1, 1, 1, 1, 1),      # smallest: one unit per pooled row
]

# the same fusion on many input channels: the wave-specialised multi-pass kernel pools its staging area
POOLFUSE_CHWS_CASES = [
    # N Cin H   W  Cout kh kw sh sw ph pw relu, tile request
    (8, 64, 56, 56, 64, 3, 3, 1, 1, 1, 1, 1, None),       # the 56x56 / 64-channel layer: 3-row tiles (the row above computed), one pooled row each
    (2, 64, 56, 56, 64, 3, 3, 1, 1, 1, 1, 0, (0, 0, 8, 64)),  # the same tiling on request; no clipping
    (1, 16, 12, 20, 64, 3, 3, 1, 1, 1, 1, 0, None),       # W % 8 != 0: one-pixel staging; 10 pooled columns: 2-byte stores
    (2, 32, 28, 28, 96, 3, 3, 1, 1, 1, 1, 1, None),       # 14 pooled columns, second channel block half empty
    (1, 64, 16, 112, 64, 3, 3, 1, 1, 1, 1, 1, (0, 0, 8, 64)),  # widest rows the 256-pixel tile takes two of (on request: the planner would take two launches here)
    (3, 24, 36, 40, 64, 3, 3, 1, 1, 1, 1, 0, (0, 0, 8, 64)),  # 6 rows per tile, padded last pass (24 channels)
    (1, 16, 48, 48, 64, 3, 3, 2, 2, 1, 1, 1, None),       # stride-2 convolution below the pooling
    (150, 16, 16, 16, 64, 3, 3, 1, 1, 1, 1, 1, None),     # more bands than compute units: several items per workgroup
    (1, 40, 8, 8, 70, 3, 3, 1, 1, 1, 1, 0, None),         # smallest image here: whole image in one tile, ragged channels
    (2, 64, 56, 56, 64, 3, 3, 1, 1, 1, 1, 1, (0, 0, 8, 32)),  # 128-pixel tiles: the row above carried, a warm-up tile per band
    (2, 32, 28, 56, 160, 3, 3, 1, 1, 1, 1, 1, (0, 0, 12, 64)),  # 128-channel tiles on 12 wavefronts (second block: 32 channels), the row above computed
    (1, 32, 16, 112, 128, 3, 3, 1, 1, 1, 1, 0, (0, 0, 12, 64)),  # the same tiling, two rows of 112: the row above carried
    (32, 16, 24, 56, 64, 3, 3, 1, 1, 1, 1, 1, (0, 0, 8, 64)),  # many images: 256-pixel tiles of 4 rows, carried row, 6 bands per image
]


def _window_max_abs(a):
    """max |a| over the 3x3 / stride 2 / padding 1 window of every pooled position."""
    return oracle.pool2d(np.abs(a).astype(np.float32), (3, 3), (2, 2), (1, 1), "max").astype(np.float64)


@pytest.mark.parametrize("case", POOLFUSE_CASES + POOLFUSE_CHWS_CASES)
def test_conv_pool_fused(mb, case):
    N, Cin, H, W, Cout, kh, kw, sh, sw, ph, pw, relu = case[:12]
    tile = case[12] if len(case) > 12 else None
    rng = np.random.default_rng(abs(hash(case[:12])) % 2 ** 31)
    x = rng.standard_normal((N, Cin, H, W)).astype(np.float16)
    w = (rng.standard_normal((Cout, Cin, kh, kw)) / np.sqrt(Cin * kh * kw)).astype(np.float16)
    plan = mb.merit_plan_conv2d_pool(N, Cin, H, W, Cout, kh, kw, sh, sw, ph, pw, relu)
    if tile is not None:
        plan.set_tile(tile)
    info = plan.launch_info()
    print("conv+pool", case, info, flush=True)
    assert info["kernel"] == ("merit_conv2d_planar_ws_pool" if Cin < 8 else "merit_conv2d_chws_pool")
    buf, y, p = guarded_empty(plan.out_shape(), torch.float16, 777.0)
    mb.merit_conv2d(plan, dev(x), dev(w), y)
    torch.cuda.synchronize()
    check_canary(buf, p, 777.0)
    got = y.cpu().numpy().astype(np.float64)
    # (1) against the oracle: max is 1-Lipschitz, so the convolution's tolerance carries over with
    # the largest magnitude in the window in place of the element's own
    conv_ref = oracle.conv2d(x, w, (sh, sw), (ph, pw), relu=bool(relu))
    ref = oracle.conv2d_pool(x, w, (sh, sw), (ph, pw), relu=bool(relu)).astype(np.float64)
    assert got.shape == ref.shape
    tol = 2e-2 * _window_max_abs(conv_ref) + 1e-3
    err = np.abs(got - ref)
    assert np.all(err <= tol), f"max excess {np.max(err - tol)} at {np.unravel_index(np.argmax(err - tol), err.shape)}"
    # (2) exactly the pooled maximum of what the unfused kernel rounds to
    # (the unfused plan on the same kernel family: the same order of summation.  The single-pass kernel,
    # which the planner prefers for fewer than 32 input channels, rounds a few sums per 10^4 the other way.)
    make = mb.merit_plan_conv2d_relu if relu else mb.merit_plan_conv2d
    unfused = make(N, Cin, H, W, Cout, kh, kw, sh, sw, ph, pw)
    if Cin >= 8:
        unfused.set_tile((0, 0, 8, 64))
        assert unfused.launch_info()["kernel"] == "merit_conv2d_chws"
    plain = mb.merit_conv2d(unfused, dev(x), dev(w)).cpu().numpy()
    exact = oracle.pool2d(plain.astype(np.float32), (3, 3), (2, 2), (1, 1), "max").astype(np.float64)
    assert np.array_equal(got, exact)


TWO_LAUNCH_POOL_CASES = [
    # W, pooled rows odd?, relu: 4 images of 256 -> 256 channels; the height is the first of a few for which
    # the planner takes the plain convolution + the pooling kernel (its estimate moves with the tilings)
    (56, False, 1),      # 16-byte pooling loads (OW % 8 == 0), even pooled row count
    (60, False, 0),      # 8-byte loads (OW % 4 == 0), no clipping
    (56, True, 1),       # odd number of pooled rows: a plane's last thread row makes one pooled row
    (54, False, 1),      # OW % 4 == 2: two pooled pixels per thread, odd pooled width
]


@pytest.mark.parametrize("case", TWO_LAUNCH_POOL_CASES)
def test_conv_pool_in_two_launches(mb, case):
    """Convolution + pooling plans the planner runs as two launches (compute-bound layers on few
    images): against the oracle, exactly equal to the fused kernel's result on request, and the
    second call reuses the stream's temporary."""
    W, odd, relu = case
    N, Cin, Cout = 4, 256, 256
    H = None
    for h in ((38, 42, 46, 34) if odd else (36, 40, 44, 48)):
        if mb.merit_plan_conv2d_pool(N, Cin, h, W, Cout, 3, 3, 1, 1, 1, 1, relu).launch_info()["kernel"].endswith("maxpool_f16"):
            H = h
            break
    assert H is not None, "no candidate height gives a two-launch plan"
    rng = np.random.default_rng(abs(hash(case)) % 2 ** 31)
    x = rng.standard_normal((N, Cin, H, W)).astype(np.float16)
    w = (rng.standard_normal((Cout, Cin, 3, 3)) / np.sqrt(Cin * 9)).astype(np.float16)
    plan = mb.merit_plan_conv2d_pool(N, Cin, H, W, Cout, 3, 3, 1, 1, 1, 1, relu)
    assert plan.launch_info()["kernel"] == "merit_conv2d_chws+merit_maxpool_f16", plan.launch_info()
    buf, y, p = guarded_empty(plan.out_shape(), torch.float16, 777.0)
    mb.merit_conv2d(plan, dev(x), dev(w), y)
    torch.cuda.synchronize()
    check_canary(buf, p, 777.0)
    got = y.cpu().numpy().astype(np.float64)
    conv_ref = oracle.conv2d(x, w, (1, 1), (1, 1), relu=bool(relu))
    ref = oracle.conv2d_pool(x, w, (1, 1), (1, 1), relu=bool(relu)).astype(np.float64)
    assert got.shape == ref.shape
    assert np.all(np.abs(got - ref) <= 2e-2 * _window_max_abs(conv_ref) + 1e-3)
    fused = mb.merit_plan_conv2d_pool(N, Cin, H, W, Cout, 3, 3, 1, 1, 1, 1, relu)
    fused.set_tile((0, 0, 8, 64))
    assert fused.launch_info()["kernel"] == "merit_conv2d_chws_pool"
    assert torch.equal(mb.merit_conv2d(fused, dev(x), dev(w)), y)
    # a second input through the same plan (its buffer is reused)
    x2 = rng.standard_normal((N, Cin, H, W)).astype(np.float16)
    y2 = mb.merit_conv2d(plan, dev(x2), dev(w))
    assert torch.equal(mb.merit_conv2d(fused, dev(x2), dev(w)), y2)


def test_conv_pool_fused_7x7_workload(mb):
    """Full-size launch of the 7x7 stride-2 layer with clipping and pooling fused; the oracle
    checks every pooled output of every image (the comparison with the library's own unfused
    result below is a second, exact check and not what parity rests on)."""
    c = wl.CFG4_CONV7
    x, w = wl.make_conv_inputs(c)
    plan = mb.merit_plan_conv2d_pool(c.N, c.Cin, c.H, c.W, c.Cout, c.kh, c.kw, c.sh, c.sw, c.ph, c.pw, 1)
    info = plan.launch_info()
    assert info["kernel"] == "merit_conv2d_planar_ws_pool" and info["grid"][0] == 256
    assert plan.out_shape() == (32, 64, 56, 56)
    y = mb.merit_conv2d(plan, dev(x), dev(w))
    torch.cuda.synchronize()
    got = y.cpu().numpy().astype(np.float64)
    conv_ref = cfg4_oracle(True)
    # oracle.conv2d_pool is the oracle's pooling applied to the oracle's clipped convolution:
    # the same two calls here, the convolution taken from the cache
    ref = oracle.pool2d(conv_ref.astype(np.float32), (3, 3), (2, 2), (1, 1), "max").astype(np.float64)
    n0 = 5
    assert np.array_equal(ref[n0], oracle.conv2d_pool(x[n0:n0 + 1], w, (c.sh, c.sw), (c.ph, c.pw),
                                                      relu=True)[0].astype(np.float64))
    tol = 2e-2 * _window_max_abs(conv_ref) + 1e-3
    assert np.all(np.abs(got - ref) <= tol)
    plain = mb.merit_conv2d(mb.merit_plan_conv2d_relu(c.N, c.Cin, c.H, c.W, c.Cout, c.kh, c.kw, c.sh, c.sw, c.ph,
                                                      c.pw), dev(x), dev(w))
    pooled = torch.nn.functional.max_pool2d(plain.float(), 3, 2, 1).half()
    assert torch.equal(y, pooled)


RESIDUAL_CASES = [
    # N Cin H   W  Cout kh kw sh sw ph pw relu   (one per kernel and staging path)
    (2, 64, 28, 28, 64, 3, 3, 1, 1, 1, 1, 1),   # the residual block's shape class
    (1, 16, 12, 16, 40, 3, 3, 1, 1, 1, 1, 0),   # channel-block, ragged channels, no clip
    (1, 20, 9, 11, 10, 2, 3, 1, 1, 0, 1, 1),    # channel-block, OH*OW % 8 != 0: scalar staging of r
    (2, 3, 32, 32, 64, 7, 7, 2, 2, 3, 3, 1),    # planar with prefetch
    (2, 3, 17, 19, 40, 7, 7, 2, 2, 3, 3, 0),    # planar, odd sizes
    (40, 3, 64, 64, 64, 7, 7, 2, 2, 3, 3, 1),   # planar, several tiles per workgroup
    (1, 136, 10, 16, 64, 3, 3, 1, 1, 1, 1, 1),  # channels in passes, the last one half empty
    (1, 256, 12, 56, 64, 3, 3, 1, 1, 1, 1, 1),  # passes on the vector staging path
    (22, 256, 12, 56, 64, 3, 3, 1, 1, 1, 1, 1), # the same with 64-channel blocks (more than 128 workgroups)
    (1, 3, 45, 45, 6, 11, 11, 4, 4, 0, 0, 1),   # planar, two fragments per window row
    (1, 3, 45, 45, 6, 11, 17, 4, 4, 0, 0, 1),   # one element per thread
    # the wave-specialised multi-pass kernel (3x3, at least 32 input channels): r read in the accumulators' layout
    (1, 32, 9, 11, 70, 3, 3, 1, 1, 1, 1, 1),    # 99 output pixels: 2-byte loads of r; ragged channel block; one-pixel staging
    (3, 96, 20, 24, 128, 3, 3, 1, 1, 1, 1, 0),  # two channel blocks, several tiles per image, no clip
    (300, 32, 8, 8, 64, 3, 3, 1, 1, 1, 1, 1),   # more work items than workgroups
    (2, 64, 30, 32, 64, 3, 3, 2, 2, 1, 1, 1),   # stride 2
]


def _residual_check(mb, case, tile=None, in_place=False):
    N, Cin, H, W, Cout, kh, kw, sh, sw, ph, pw, relu = case
    rng = np.random.default_rng(abs(hash(case)) % 2 ** 31)
    x = rng.standard_normal((N, Cin, H, W)).astype(np.float16)
    w = (rng.standard_normal((Cout, Cin, kh, kw)) / np.sqrt(Cin * kh * kw)).astype(np.float16)
    plan = mb.merit_plan_conv2d_residual(N, Cin, H, W, Cout, kh, kw, sh, sw, ph, pw, relu)
    if tile is not None:
        plan.set_tile(tile)
    r = rng.standard_normal(plan.out_shape()).astype(np.float16)
    print("conv+residual", case, plan.launch_info(), flush=True)
    buf, y, p = guarded_empty(plan.out_shape(), torch.float16, 777.0)
    if in_place:
        y.copy_(dev(r))
        mb.merit_conv2d_residual(plan, dev(x), dev(w), y, y)
    else:
        mb.merit_conv2d_residual(plan, dev(x), dev(w), dev(r), y)
    torch.cuda.synchronize()
    check_canary(buf, p, 777.0)
    got = y.cpu().numpy().astype(np.float64)
    ref = oracle.conv2d_residual(x, w, r, (sh, sw), (ph, pw), relu=bool(relu)).astype(np.float64)
    # one rounding of (sum + r): the convolution's bar holds on the result itself, also where
    # the two terms cancel
    err = np.abs(got - ref)
    tol = 2e-2 * np.abs(ref) + 1e-3
    assert np.all(err <= tol), f"max excess {np.max(err - tol)} at {np.unravel_index(np.argmax(err - tol), err.shape)}"
    if relu:
        assert not np.signbit(got).any()
    return got, ref


@pytest.mark.parametrize("case", RESIDUAL_CASES)
def test_conv_residual(mb, case):
    _residual_check(mb, case)


@pytest.mark.parametrize("case", [c for c in RESIDUAL_CASES if c[1] >= 32 and c[5] == 3])
@pytest.mark.parametrize("tile", [(0, 0, 4, 32), (0, 0, 8, 64), (0, 0, 8, 32)])
def test_conv_residual_many_channels_every_kernel(mb, case, tile):
    """The many-channel cases on the plain kernels (4 x 32: single- or multi-pass) and on both
    64-channel tilings of the wave-specialised kernel."""
    _residual_check(mb, case, tile=tile)


def test_conv_residual_in_place_and_big_tiles(mb):
    _residual_check(mb, RESIDUAL_CASES[0], in_place=True)
    _residual_check(mb, RESIDUAL_CASES[0], tile=(0, 0, 4, 64))
    _residual_check(mb, RESIDUAL_CASES[3], tile=(0, 0, 4, 64), in_place=True)
    _residual_check(mb, RESIDUAL_CASES[3], tile=(0, 0, 8, 32))


def test_conv_residual_single_rounding(mb):
    """sum = 2049 is a binary16 tie (alone it rounds to 2048); with r = 1 the exact 2050 is
    representable, and r = -2048 leaves exactly 1: both need the addition before the rounding."""
    Cin = 16
    x = np.zeros((1, Cin, 8, 8), np.float16)
    x[0, 0], x[0, 1] = 2048.0, 1.0
    w = np.zeros((32, Cin, 1, 1), np.float16)
    w[:, 0], w[:, 1] = 1.0, 1.0
    plan = mb.merit_plan_conv2d_residual(1, Cin, 8, 8, 32, 1, 1, 1, 1, 0, 0, 0)
    r = np.ones(plan.out_shape(), np.float16)
    r[0, :, 4:] = -2048.0
    y = mb.merit_conv2d_residual(plan, dev(x), dev(w), dev(r)).cpu().numpy().astype(np.float64)
    assert np.all(y[0, :, :4] == 2050.0) and np.all(y[0, :, 4:] == 1.0)
    assert np.array_equal(y, oracle.conv2d_residual(x, w, r).astype(np.float64))
    # the same on the wave-specialised multi-pass kernel: a 3x3 window whose centre tap does it
    Cin = 32
    x = np.zeros((1, Cin, 8, 8), np.float16)
    x[0, 0], x[0, 1] = 2048.0, 1.0
    w = np.zeros((64, Cin, 3, 3), np.float16)
    w[:, 0, 1, 1], w[:, 1, 1, 1] = 1.0, 1.0
    plan = mb.merit_plan_conv2d_residual(1, Cin, 8, 8, 64, 3, 3, 1, 1, 1, 1, 0)
    assert plan.launch_info()["kernel"] == "merit_conv2d_chws"
    r = np.ones(plan.out_shape(), np.float16)
    r[0, :, 4:] = -2048.0
    y = mb.merit_conv2d_residual(plan, dev(x), dev(w), dev(r)).cpu().numpy().astype(np.float64)
    assert np.all(y[0, :, :4] == 2050.0) and np.all(y[0, :, 4:] == 1.0)
    assert np.array_equal(y, oracle.conv2d_residual(x, w, r, (1, 1), (1, 1)).astype(np.float64))


def test_conv_residual_3x3_workload(mb):
    """The 3x3 / 64-channel layer as a residual block's second convolution, full size."""
    c = wl.CFG2_CONV3
    x, w = wl.make_conv_inputs(c)
    plan = mb.merit_plan_conv2d_residual(c.N, c.Cin, c.H, c.W, c.Cout, c.kh, c.kw, c.sh, c.sw, c.ph, c.pw, 1)
    assert plan.launch_info()["kernel"] == "merit_conv2d_chws"
    r = np.random.default_rng(wl.BASE_SEED + 77).standard_normal(plan.out_shape()).astype(np.float16)
    y = mb.merit_conv2d_residual(plan, dev(x), dev(w), dev(r)).cpu().numpy().astype(np.float64)
    ref = oracle.conv2d_residual(x, w, r, (c.sh, c.sw), (c.ph, c.pw), relu=True).astype(np.float64)
    assert np.all(np.abs(y - ref) <= 2e-2 * np.abs(ref) + 1e-3)
    assert (ref == 0).mean() > 0.2 and (ref > 0).mean() > 0.2


DILATED_CASES = [
    # N Cin H   W  Cout kh kw sh sw ph pw dh dw relu
    (1, 32, 64, 64, 32, 3, 3, 1, 1, 2, 2, 2, 2, 0),   # the dilated layer of the paper's table: 64x64x32 out
    (2, 16, 21, 19, 40, 3, 3, 1, 1, 2, 2, 2, 2, 1),   # odd sizes, ragged channels, clipped product
    (1, 64, 30, 34, 64, 3, 3, 2, 1, 3, 0, 3, 1, 0),   # mixed dilation and stride
    (2, 3, 33, 40, 8, 3, 3, 1, 1, 2, 2, 2, 2, 0),     # few input channels (padded to 16)
    (1, 8, 18, 24, 16, 2, 5, 1, 2, 0, 4, 4, 2, 0),    # even window, wide dilation
    (1, 144, 20, 40, 32, 3, 3, 1, 1, 2, 2, 2, 2, 1),  # channels in passes
    (1, 3, 50, 50, 8, 11, 11, 2, 2, 10, 10, 2, 2, 1), # one element per thread, dilated and clipped
]


@pytest.mark.parametrize("case", DILATED_CASES)
def test_conv_dilated(mb, case):
    N, Cin, H, W, Cout, kh, kw, sh, sw, ph, pw, dh, dw, relu = case
    rng = np.random.default_rng(abs(hash(case)) % 2 ** 31)
    x = rng.standard_normal((N, Cin, H, W)).astype(np.float16)
    w = (rng.standard_normal((Cout, Cin, kh, kw)) / np.sqrt(Cin * kh * kw)).astype(np.float16)
    _conv_check(mb, x, w, (sh, sw), (ph, pw), relu=bool(relu), dilation=(dh, dw))


def test_conv_channel_passes_and_wide_window_workloads_sampled(mb):
    """Full-size launches of the two layers beyond the MFMA single-pass kernels; the oracle
    checks one image of the 256-channel layer and all of the 11 x 11 layer."""
    c = wl.CFG_CONV256
    x, w = wl.make_conv_inputs(c)
    plan = mb.merit_plan_conv2d(c.N, c.Cin, c.H, c.W, c.Cout, c.kh, c.kw, c.sh, c.sw, c.ph, c.pw)
    assert plan.launch_info()["kernel"] == "merit_conv2d_chws"
    y = mb.merit_conv2d(plan, dev(x), dev(w)).cpu().numpy().astype(np.float64)
    n = 5
    ref = oracle.conv2d(x[n:n + 1], w, (c.sh, c.sw), (c.ph, c.pw)).astype(np.float64)
    assert np.all(np.abs(y[n:n + 1] - ref) <= 2e-2 * np.abs(ref) + 1e-3)
    c = wl.CFG_CONV11
    x, w = wl.make_conv_inputs(c)
    plan = mb.merit_plan_conv2d(c.N, c.Cin, c.H, c.W, c.Cout, c.kh, c.kw, c.sh, c.sw, c.ph, c.pw)
    assert plan.launch_info()["kernel"] == "merit_conv2d_planar" and plan.out_shape() == (8, 48, 55, 55)
    y = mb.merit_conv2d(plan, dev(x), dev(w)).cpu().numpy().astype(np.float64)
    ref = oracle.conv2d(x, w, (c.sh, c.sw), (c.ph, c.pw)).astype(np.float64)
    assert np.all(np.abs(y - ref) <= 2e-2 * np.abs(ref) + 1e-3)


def test_conv_dilated_one_hot_tap_shifts_the_input_exactly(mb):
    """x = p + 2a (Section III-C): a one-hot kernel returns the input shifted by twice the tap."""
    rng = np.random.default_rng(6)
    C = 16
    x = rng.standard_normal((1, C, 20, 24)).astype(np.float16)
    w = np.zeros((C, C, 3, 3), np.float16)
    for c in range(C):
        w[c, c, 2, 1] = 1.0
    got, ref = _conv_check(mb, x, w, (1, 1), (0, 0), dilation=(2, 2))
    assert np.array_equal(got, x[:, :, 4:4 + 16, 2:2 + 20].astype(np.float64))


def test_conv_identity_kernel_is_exact(mb):
    rng = np.random.default_rng(4)
    C = 16
    x = rng.standard_normal((1, C, 12, 16)).astype(np.float16)
    w = np.zeros((C, C, 3, 3), np.float16)
    for c in range(C):
        w[c, c, 1, 1] = 1.0
    got, ref = _conv_check(mb, x, w, (1, 1), (1, 1))
    assert np.array_equal(got, x.astype(np.float64))


def _ulp_distance(a16, b16):
    """Distance in binary16 units in the last place (values mapped to ordered integers)."""
    def ordered(h):
        u = np.ascontiguousarray(h, np.float16).view(np.uint16).astype(np.int32)
        return np.where(u & 0x8000, -(u & 0x7FFF), u)
    return np.abs(ordered(a16) - ordered(b16))


def _report_ulps(name, got16, ref16):
    """Next to the tolerance test: how far the kernel's fp32 accumulation and single rounding
    end up from the oracle's double sum rounded once.  Away from cancellations the two differ
    by at most one binary16 unit in the last place; near zero a difference of 1e-6 is many
    units, which is what the absolute term of the tolerance is for."""
    d = _ulp_distance(got16, ref16)
    big = np.abs(ref16.astype(np.float64)) >= 2.0 ** -6
    print(f"{name}: ulp distance max {d.max()}, 99.9th percentile {np.percentile(d, 99.9):.1f}, "
          f"max where |ref| >= 2^-6: {d[big].max()}, equal {np.mean(d == 0):.4f}", flush=True)
    assert d[big].max() <= 1 and np.percentile(d, 99.9) <= 1


def test_conv_3x3_workload(mb):
    c = wl.CFG2_CONV3
    x, w = wl.make_conv_inputs(c)
    got, ref = _conv_check(mb, x, w, (c.sh, c.sw), (c.ph, c.pw))
    _report_ulps("conv 3x3 workload", got.astype(np.float16), ref.astype(np.float16))


def test_conv_7x7_workload_kernels_agree(mb):
    """Every output of the full-size launch, from the wave-specialised kernel and from the
    one-role kernel (same products, same order): guards the hand-over of the LDS buffers
    between wavefronts, which a sampled comparison could miss."""
    c = wl.CFG4_CONV7
    x, w = wl.make_conv_inputs(c)
    dx, dw = dev(x), dev(w)
    outs = []
    for tile in (None, (0, 0, 4, 64)):
        plan = mb.merit_plan_conv2d(c.N, c.Cin, c.H, c.W, c.Cout, c.kh, c.kw, c.sh, c.sw, c.ph, c.pw)
        if tile:
            plan.set_tile(tile)
        outs.append((plan.launch_info()["kernel"], mb.merit_conv2d(plan, dx, dw)))
    assert outs[0][0] == "merit_conv2d_planar_ws" and outs[1][0] == "merit_conv2d_planar"
    for rep in range(3):                                  # repeated: a race shows up sporadically
        plan = mb.merit_plan_conv2d(c.N, c.Cin, c.H, c.W, c.Cout, c.kh, c.kw, c.sh, c.sw, c.ph, c.pw)
        again = mb.merit_conv2d(plan, dx, dw)
        assert torch.equal(again, outs[0][1]), rep
    a, b = outs[0][1].float(), outs[1][1].float()
    assert bool(torch.all((a - b).abs() <= 2e-3 * b.abs() + 1e-3))


def test_conv_7x7_workload_every_image(mb):
    """Full-size launch; the oracle checks every output of every image of the batch."""
    c = wl.CFG4_CONV7
    x, w = wl.make_conv_inputs(c)
    plan = mb.merit_plan_conv2d(c.N, c.Cin, c.H, c.W, c.Cout, c.kh, c.kw, c.sh, c.sw, c.ph, c.pw)
    print("conv7 full", plan.launch_info(), flush=True)
    y = mb.merit_conv2d(plan, dev(x), dev(w))
    torch.cuda.synchronize()
    got = y.cpu().numpy().astype(np.float64)
    assert got.shape == (32, 64, 112, 112) and np.all(np.isfinite(got))
    ref_all = cfg4_oracle(False).astype(np.float64)
    for n in range(c.N):
        ref = ref_all[n]
        err = np.abs(got[n] - ref)
        assert np.all(err <= 2e-2 * np.abs(ref) + 1e-3), n
    for n in (0, 17, 31):
        _report_ulps(f"conv 7x7 workload, image {n}", got[n].astype(np.float16), ref_all[n].astype(np.float16))


def test_misaligned_pointer_is_rejected(mb):
    plan = mb.merit_plan_pool2d(1, 1, 8, 8, 2, 2, 2, 2, 0, 0, 0)
    x = torch.zeros(8 * 8 + 4, device="cuda:0")[1:65].view(1, 1, 8, 8)
    with pytest.raises(mb.MeritError) as e:
        mb.merit_pool2d(plan, x)
    assert e.value.status == mb.MERIT_ERR_ALIGNMENT


# -------------------------------------------------- separable filter
SEP_CASES = [
    # N  H    W    k  staged rows
    (1, 40, 70, 3, 32),          # ragged tiles in both directions
    (2, 133, 129, 5, None),      # one column past two tiles, three tiles down
    (1, 64, 64, 1, None),        # single tap: a scaled copy
    (1, 17, 23, 4, None),        # even window: one tap further back than forward
    (1, 100, 130, 30, None),     # the long window of the paper's table, 64-row tiles
    (1, 100, 130, 30, 64),       # the same on 32-row tiles
    (1, 9, 9, 32, None),         # window much larger than the image: everything clamps
    (2, 50, 66, 7, None),        # width not a multiple of 4: scalar staging and stores
    (3, 32, 64, 9, 64),          # tile taller than the image
    (2, 37, 300, 3, None),       # several column tiles, the last ragged
    (1, 50, 1032, 9, None),      # seventeen column tiles
    (1, 9, 12, 8, None),         # three column groups: everything near an edge
    (3, 16, 256, 6, None),       # exactly four column tiles
    (1, 5, 4, 5, None),          # a single column group, window wider than the image
]


def _sep_tol(x, kx, ky):
    # fp32 multiply-adds, 2k of them per output, each rounding at most 2^-24 of the running
    # magnitude, which sum|kx| sum|ky| max|x| bounds
    return 1e-5 * float(np.abs(kx).sum() * np.abs(ky).sum() * np.abs(x).max()) + 1e-30


@pytest.mark.parametrize("N,H,W,k,tile", SEP_CASES)
def test_sepfilter(mb, N, H, W, k, tile):
    rng = np.random.default_rng(N * 1000 + H * 10 + k)
    x = rng.standard_normal((N, H, W)).astype(np.float32)
    kx = rng.standard_normal(k).astype(np.float32)
    ky = rng.standard_normal(k).astype(np.float32)
    plan = mb.merit_plan_sepfilter(N, H, W, k)
    if tile is not None:
        plan.set_tile((0, tile))
    print("sepfilter", (N, H, W, k), plan.launch_info(), flush=True)
    buf, y, p = guarded_empty((N, H, W), torch.float32, 777.0)
    mb.merit_sepfilter(plan, dev(x), dev(kx), dev(ky), y)
    torch.cuda.synchronize()
    check_canary(buf, p, 777.0)
    got = y.cpu().numpy().astype(np.float64)
    ref = oracle.sepfilter(x, kx, ky).astype(np.float64)
    err = np.abs(got - ref)
    assert np.all(err <= _sep_tol(x, kx, ky)), f"max err {err.max()} at {np.unravel_index(err.argmax(), err.shape)}"


@pytest.mark.parametrize("k", range(1, 33))
def test_sepfilter_every_window_length(mb, k):
    """Every window length is a kernel instantiation of its own (taps and windows unrolled):
    each is checked on an image of three column tiles, the last ragged, two tiles down."""
    N, H, W = 2, 101, 136
    rng = np.random.default_rng(4000 + k)
    x = rng.uniform(0, 255, (N, H, W)).astype(np.float32)
    kx = rng.standard_normal(k).astype(np.float32)
    ky = rng.standard_normal(k).astype(np.float32)
    plan = mb.merit_plan_sepfilter(N, H, W, k)
    print("sepfilter k", k, plan.launch_info(), flush=True)
    buf, y, p = guarded_empty((N, H, W), torch.float32, 777.0)
    mb.merit_sepfilter(plan, dev(x), dev(kx), dev(ky), y)
    torch.cuda.synchronize()
    check_canary(buf, p, 777.0)
    err = np.abs(y.cpu().numpy().astype(np.float64) - oracle.sepfilter(x, kx, ky).astype(np.float64))
    assert np.all(err <= _sep_tol(x, kx, ky)), f"k={k}: max err {err.max()} at {np.unravel_index(err.argmax(), err.shape)}"


def test_sepfilter_impulse_is_exact(mb):
    """Small-integer taps and one impulse: every product is exact in fp32, so the result must
    equal the oracle bit for bit, and shows the unflipped, -k/2-centred window."""
    H, W, k = 70, 75, 6
    x = np.zeros((1, H, W), np.float32)
    x[0, 33, 64] = 1.0                                       # next to a tile boundary
    x[0, 0, 0] = 2.0                                         # in the corner: clamped copies pile up
    kx = (np.arange(k) + 1).astype(np.float32)
    ky = (10 * (np.arange(k) + 1)).astype(np.float32)
    y = mb.merit_sepfilter(mb.merit_plan_sepfilter(1, H, W, k), dev(x), dev(kx), dev(ky)).cpu().numpy()
    assert np.array_equal(y, oracle.sepfilter(x, kx, ky))
    assert y[0, 33 - 0 + 3, 64 - 5 + 3] == ky[0] * kx[5]
    # the same on a width that is a multiple of 4 (aligned 16-byte staging), impulses at a tile
    # boundary (column 255 | 256) and in the corners
    W = 520
    x = np.zeros((1, H, W), np.float32)
    x[0, 33, 255] = 1.0
    x[0, 40, 256] = 3.0
    x[0, 0, 0] = 2.0
    x[0, H - 1, W - 1] = 5.0
    y = mb.merit_sepfilter(mb.merit_plan_sepfilter(1, H, W, k), dev(x), dev(kx), dev(ky)).cpu().numpy()
    assert np.array_equal(y, oracle.sepfilter(x, kx, ky))


def test_sepfilter_workloads_every_image(mb):
    """Full-size launches (k = 3 and k = 30); the oracle checks every pixel of every image."""
    for c in (wl.CFG_SEP_K3, wl.CFG_SEP_K30):
        x, kx, ky = wl.make_sepfilter_inputs(c)
        plan = mb.merit_plan_sepfilter(c.N, c.H, c.W, c.k)
        y = mb.merit_sepfilter(plan, dev(x), dev(kx), dev(ky))
        torch.cuda.synchronize()
        ref = oracle.sepfilter(x, kx, ky).astype(np.float64)
        got = y.cpu().numpy().astype(np.float64)
        assert got.shape == ref.shape == (c.N, c.H, c.W)
        assert np.all(np.abs(got - ref) <= _sep_tol(x, kx, ky))
        # a normalised positive window keeps the range and (up to the borders) the mean
        assert got.min() >= 0.0 and got.max() <= 255.0 + 1e-3


# -------------------------------------------------- bilateral filter
BILATERAL_CASES = [
    # N  H   W   k  sigma_r
    (1, 40, 70, 5, 20.0),        # ragged tiles
    (2, 33, 129, 9, 25.0),       # one column past two tiles
    (1, 16, 64, 1, 10.0),        # single tap: the input itself
    (1, 23, 30, 4, 40.0),        # even window, width not a multiple of 4
    (1, 50, 66, 31, 30.0),       # window larger than a tile
    (1, 20, 64, 7, 2.0),         # sharp range term: most weights underflow
]


def _bilateral_tol(x, k):
    # weights carry a relative error of a few 1e-6 (two fp32 products in the exponent, the
    # hardware exponential), which moves a weighted mean by at most twice that times the range
    # of the window; k*k fp32 additions add k*k * 2^-24 of it.  The range is taken per output
    # pixel over its own (clamped) k x k window; the last term is what is left when the range
    # is zero (k = 1, flat areas): the fp32 roundings of the product w*v, of the quotient and of
    # the oracle's own result, 4 * 2^-24 of the largest magnitude in the window.
    x = np.asarray(x, np.float64)
    N, H, W = x.shape
    c = k // 2
    lo = np.full_like(x, np.inf)
    hi = np.full_like(x, -np.inf)
    rows = np.arange(H)
    cols = np.arange(W)
    for a1 in range(k):
        yy = np.clip(rows + a1 - c, 0, H - 1)
        for a2 in range(k):
            xx = np.clip(cols + a2 - c, 0, W - 1)
            v = x[:, yy][:, :, xx]
            lo = np.minimum(lo, v)
            hi = np.maximum(hi, v)
    return (2e-5 + 1.2e-7 * k * k) * (hi - lo) + 2.4e-7 * np.maximum(np.abs(lo), np.abs(hi)) + 1e-30


@pytest.mark.parametrize("N,H,W,k,sigma_r", BILATERAL_CASES)
def test_bilateral(mb, N, H, W, k, sigma_r):
    rng = np.random.default_rng(N * 1000 + H * 10 + k)
    x = (rng.integers(0, 3, size=(N, H, W)) * 80.0 + rng.normal(0, 6.0, size=(N, H, W))).astype(np.float32)
    gx = np.exp(-0.5 * ((np.arange(k) - k // 2) / max(k / 4.0, 0.5)) ** 2).astype(np.float32)
    gy = rng.uniform(0.3, 1.0, k).astype(np.float32)         # a different table per axis
    norm = -1.0 / (2 * sigma_r * sigma_r)
    plan = mb.merit_plan_bilateral(N, H, W, k)
    print("bilateral", (N, H, W, k), plan.launch_info(), flush=True)
    buf, y, p = guarded_empty((N, H, W), torch.float32, 777.0)
    mb.merit_bilateral(plan, dev(x), dev(gx), dev(gy), norm, y)
    torch.cuda.synchronize()
    check_canary(buf, p, 777.0)
    got = y.cpu().numpy().astype(np.float64)
    ref = oracle.bilateral(x, gx, gy, norm).astype(np.float64)
    err = np.abs(got - ref)
    assert np.all(err <= _bilateral_tol(x, k)), f"max err {err.max()} at {np.unravel_index(err.argmax(), err.shape)}"


@pytest.mark.parametrize("k", range(1, 19))
def test_bilateral_every_window_length(mb, k):
    """k <= 16 are instantiations of the row kernel, above that the tile kernel takes over."""
    N, H, W = 1, 37, 132
    rng = np.random.default_rng(5000 + k)
    x = (rng.integers(0, 3, size=(N, H, W)) * 80.0 + rng.normal(0, 6.0, size=(N, H, W))).astype(np.float32)
    gx = np.exp(-0.5 * ((np.arange(k) - k // 2) / max(k / 4.0, 0.5)) ** 2).astype(np.float32)
    gy = rng.uniform(0.3, 1.0, k).astype(np.float32)
    norm = -1.0 / (2 * 25.0 * 25.0)
    plan = mb.merit_plan_bilateral(N, H, W, k)
    print("bilateral k", k, plan.launch_info(), flush=True)
    buf, y, p = guarded_empty((N, H, W), torch.float32, 777.0)
    mb.merit_bilateral(plan, dev(x), dev(gx), dev(gy), norm, y)
    torch.cuda.synchronize()
    check_canary(buf, p, 777.0)
    err = np.abs(y.cpu().numpy().astype(np.float64) - oracle.bilateral(x, gx, gy, norm).astype(np.float64))
    assert np.all(err <= _bilateral_tol(x, k)), f"k={k}: max err {err.max()}"


def test_bilateral_positive_constant(mb):
    """The constant is used as given (the listing passes a positive one): weights grow with the
    difference."""
    rng = np.random.default_rng(31)
    x = rng.uniform(0, 100, (1, 30, 70)).astype(np.float32)
    g = np.exp(-0.5 * ((np.arange(5) - 2) / 1.5) ** 2).astype(np.float32)
    y = mb.merit_bilateral(mb.merit_plan_bilateral(1, 30, 70, 5), dev(x), dev(g), dev(g), 2e-4).cpu().numpy()
    ref = oracle.bilateral(x, g, g, 2e-4)
    assert np.all(np.abs(y.astype(np.float64) - ref) <= _bilateral_tol(x, 5))
    assert np.abs(ref - oracle.bilateral(x, g, g, -2e-4)).max() > 1.0       # the sign matters


def test_bilateral_without_range_term_is_the_normalised_separable_filter(mb):
    """norm = 0: both kernels of the library must agree (up to fp32 rounding)."""
    rng = np.random.default_rng(12)
    x = rng.uniform(0, 255, (1, 45, 80)).astype(np.float32)
    g = np.exp(-0.5 * ((np.arange(7) - 3) / 2.0) ** 2).astype(np.float32)
    yb = mb.merit_bilateral(mb.merit_plan_bilateral(1, 45, 80, 7), dev(x), dev(g), dev(g), 0.0).cpu().numpy()
    ys = mb.merit_sepfilter(mb.merit_plan_sepfilter(1, 45, 80, 7), dev(x), dev(g), dev(g)).cpu().numpy()
    assert np.allclose(yb, ys / float(g.sum()) ** 2, rtol=1e-5, atol=1e-3)


def test_bilateral_workload(mb):
    """Full-size launch; the oracle checks the whole (single) image."""
    c = wl.CFG_BILATERAL
    x, g = wl.make_bilateral_inputs(c)
    y = mb.merit_bilateral(mb.merit_plan_bilateral(c.N, c.H, c.W, c.k), dev(x), dev(g), dev(g), c.norm)
    torch.cuda.synchronize()
    got = y.cpu().numpy().astype(np.float64)
    ref = oracle.bilateral(x, g, g, c.norm).astype(np.float64)
    assert np.all(np.abs(got - ref) <= _bilateral_tol(x, c.k))
    assert got.min() >= x.min() and got.max() <= x.max()
    # it denoises: closer to the noise-free steps than the input on flat areas
    assert np.abs(np.diff(got, axis=2)).mean() < 0.5 * np.abs(np.diff(x.astype(np.float64), axis=2)).mean()


# -------------------------------------------------- peak probes
def test_probe_copy_and_alu_loops(mb):
    src = torch.arange(4 * 1000 + 4, dtype=torch.float32, device="cuda:0")       # not a multiple of the step
    buf, dst, p = guarded_empty((src.numel(),), torch.float32, 777.0)
    mb.merit_probe_copy(src, dst)
    torch.cuda.synchronize()
    check_canary(buf, p, 777.0)
    assert torch.equal(dst, src)
    sink = torch.full((3 * 256,), -1, dtype=torch.int32, device="cuda:0")
    for which in (mb.MERIT_PROBE_MFMA_F16, mb.MERIT_PROBE_FMA_F32, mb.MERIT_PROBE_SAD_U8, mb.MERIT_PROBE_EXP2_F32):
        sink.fill_(-1)
        mb.merit_probe_alu(which, 3, 5, sink)
        torch.cuda.synchronize()
        assert not bool((sink == -1).all())
    # v_sad_u8 chain c after 5 steps: c + 5 * sum_bytes |(p + c) - q|, p = lane seed, q = p ^ 0x5a5a5a5a
    mb.merit_probe_alu(mb.MERIT_PROBE_SAD_U8, 1, 5, sink)
    torch.cuda.synchronize()
    t = 7
    pz = (t * 2654435761 + 0) & 0xFFFFFFFF
    q = pz ^ 0x5A5A5A5A
    want = 0
    for c in range(8):
        a = (pz + c) & 0xFFFFFFFF
        want += c + 5 * sum(abs(((a >> (8 * b)) & 255) - ((q >> (8 * b)) & 255)) for b in range(4))
    assert int(sink[t].item()) & 0xFFFFFFFF == want & 0xFFFFFFFF


# -------------------------------------------------- streams
def test_launches_follow_the_given_stream(mb):
    """Every entry point enqueues on the stream it is handed (default priority) and returns:
    work queued behind a producer on a side stream sees the producer's output, and the plan can
    be shared by two streams."""
    side = torch.cuda.Stream()
    c = wl.CFG1_POOL
    x = wl.make_pool_input(c, N=2)
    plan = mb.merit_plan_pool2d(2, c.C, c.H, c.W, c.kh, c.kw, c.sh, c.sw, c.ph, c.pw, 0)
    dx = torch.empty(x.shape, dtype=torch.float32, device="cuda:0")
    host = torch.empty(x.shape, dtype=torch.float32, pin_memory=True)      # freshly allocated pinned memory
    host.copy_(torch.from_numpy(x))
    with torch.cuda.stream(side):
        dx.copy_(host, non_blocking=True)                   # producer on the side stream
        y_side = mb.merit_pool2d(plan, dx, stream=side)     # consumer behind it, same stream
        sep = mb.merit_plan_sepfilter(2 * c.C, c.H, c.W, 3)
        taps = torch.tensor([0.25, 0.5, 0.25], device="cuda:0")
        z_side = mb.merit_sepfilter(sep, dx.view(2 * c.C, c.H, c.W), taps, taps, stream=side)
    side.synchronize()
    y_main = mb.merit_pool2d(plan, dx)                      # the same plan on the current stream
    torch.cuda.synchronize()
    ref = oracle.pool2d(x, (c.kh, c.kw), (c.sh, c.sw), (c.ph, c.pw), "max")
    assert np.array_equal(y_side.cpu().numpy(), ref) and np.array_equal(y_main.cpu().numpy(), ref)
    zr = oracle.sepfilter(x.reshape(2 * c.C, c.H, c.W), np.array([0.25, 0.5, 0.25], np.float32),
                          np.array([0.25, 0.5, 0.25], np.float32))
    assert np.allclose(z_side.cpu().numpy(), zr, rtol=0, atol=1e-5 * float(np.abs(x).max()))


def test_launches_can_be_captured_in_a_graph(mb):
    """The entry points neither allocate nor synchronise, so a stream capture records them
    (after one eager call per kernel instance, which raises that instance's LDS limit).  The
    graph is replayed several times with eager work in between and every replay is checked."""
    rng = np.random.default_rng(77)
    shape = (2, 8, 30, 36)
    pmax = mb.merit_plan_pool2d(*shape, 3, 3, 2, 2, 1, 1, 0)
    pavg = mb.merit_plan_pool2d(*shape, 3, 3, 2, 2, 1, 1, 1)
    conv = mb.merit_plan_conv2d_relu(2, 16, 30, 36, 32, 3, 3, 1, 1, 1, 1)
    x = torch.zeros(shape, dtype=torch.float32, device="cuda:0")
    xh = torch.zeros((2, 16, 30, 36), dtype=torch.float16, device="cuda:0")
    w = rng.standard_normal((32, 16, 3, 3)).astype(np.float16) / 12
    dw = dev(w)
    ymax = torch.empty(pmax.out_shape(), dtype=torch.float32, device="cuda:0")
    yavg = torch.empty(pavg.out_shape(), dtype=torch.float32, device="cuda:0")
    yc = torch.empty(conv.out_shape(), dtype=torch.float16, device="cuda:0")
    mb.merit_pool2d(pmax, x, ymax); mb.merit_pool2d(pavg, x, yavg); mb.merit_conv2d(conv, xh, dw, yc)   # eager first
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        mb.merit_pool2d(pmax, x, ymax)
        mb.merit_pool2d(pavg, x, yavg)
        mb.merit_conv2d(conv, xh, dw, yc)
    for rep in range(3):
        xv = rng.standard_normal(shape).astype(np.float32)
        xc = rng.standard_normal((2, 16, 30, 36)).astype(np.float16)
        x.copy_(torch.from_numpy(xv)); xh.copy_(torch.from_numpy(xc))          # eager work between replays
        ymax.fill_(-7.0); yavg.fill_(-7.0); yc.fill_(-7.0)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert np.array_equal(ymax.cpu().numpy(), oracle.pool2d(xv, (3, 3), (2, 2), (1, 1), "max")), rep
        ra = oracle.pool2d(xv, (3, 3), (2, 2), (1, 1), "avg")
        assert np.all(np.abs(yavg.cpu().numpy() - ra) <= 1e-5 * np.abs(ra) + 1e-6), rep
        rc = oracle.conv2d(xc, w, (1, 1), (1, 1), relu=True).astype(np.float64)
        assert np.all(np.abs(yc.cpu().numpy().astype(np.float64) - rc) <= 2e-2 * np.abs(rc) + 1e-3), rep


def test_more_launches_can_be_captured_in_a_graph(mb):
    """The same for the kernels with more host-side work in their launchers: the long-window
    separable filter (its persistent grid is sized by an occupancy query), the multi-pass and
    the one-element-per-thread convolution, the lane-per-column and per-plane pooling, and the
    correlation layer.  One eager call each, then capture, then replays with eager work between."""
    rng = np.random.default_rng(78)
    sep = mb.merit_plan_sepfilter(1, 70, 136, 30)
    kx = rng.standard_normal(30).astype(np.float32); ky = rng.standard_normal(30).astype(np.float32)
    xs = torch.zeros((1, 70, 136), dtype=torch.float32, device="cuda:0"); ys = torch.empty_like(xs)
    cp = mb.merit_plan_conv2d(1, 260, 10, 16, 40, 5, 5, 1, 1, 2, 2)
    cd = mb.merit_plan_conv2d(1, 3, 45, 45, 6, 11, 17, 4, 4, 0, 0)
    assert cp.launch_info()["kernel"] == "merit_conv2d_chpass" and cd.launch_info()["kernel"] == "merit_conv2d_direct"
    wp = (rng.standard_normal((40, 260, 5, 5)) / 81).astype(np.float16)
    wd = (rng.standard_normal((6, 3, 11, 17)) / 24).astype(np.float16)
    xp = torch.zeros((1, 260, 10, 16), dtype=torch.float16, device="cuda:0")
    xd = torch.zeros((1, 3, 45, 45), dtype=torch.float16, device="cuda:0")
    yp = torch.empty(cp.out_shape(), dtype=torch.float16, device="cuda:0")
    yd = torch.empty(cd.out_shape(), dtype=torch.float16, device="cuda:0")
    pl = mb.merit_plan_pool2d(2, 5, 27, 27, 3, 3, 2, 2, 0, 0, 0)
    pg = mb.merit_plan_pool2d(2, 5, 27, 27, 27, 27, 1, 1, 0, 0, 1)
    xq = torch.zeros((2, 5, 27, 27), dtype=torch.float32, device="cuda:0")
    yl = torch.empty(pl.out_shape(), dtype=torch.float32, device="cuda:0")
    yg = torch.empty(pg.out_shape(), dtype=torch.float32, device="cuda:0")
    co = mb.merit_plan_correlation(1, 24, 12, 24, 3, 2)
    x1 = torch.zeros((1, 24, 12, 24), dtype=torch.float16, device="cuda:0"); x2 = torch.zeros_like(x1)
    yo = torch.empty(co.out_shape(), dtype=torch.float16, device="cuda:0")
    dkx, dky, dwp, dwd = dev(kx), dev(ky), dev(wp), dev(wd)

    def launch_all():
        mb.merit_sepfilter(sep, xs, dkx, dky, ys)
        mb.merit_conv2d(cp, xp, dwp, yp)
        mb.merit_conv2d(cd, xd, dwd, yd)
        mb.merit_pool2d(pl, xq, yl)
        mb.merit_pool2d(pg, xq, yg)
        mb.merit_correlation(co, x1, x2, yo)

    launch_all()                                                    # eager first
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        launch_all()
    for rep in range(2):
        a = rng.uniform(0, 255, (1, 70, 136)).astype(np.float32)
        b = rng.standard_normal((1, 260, 10, 16)).astype(np.float16)
        c = rng.standard_normal((1, 3, 45, 45)).astype(np.float16)
        d = rng.standard_normal((2, 5, 27, 27)).astype(np.float32)
        e1 = (rng.standard_normal((1, 24, 12, 24)) / 5).astype(np.float16)
        e2 = rng.standard_normal((1, 24, 12, 24)).astype(np.float16)
        for t, v in ((xs, a), (xp, b), (xd, c), (xq, d), (x1, e1), (x2, e2)):
            t.copy_(torch.from_numpy(v))                            # eager work between replays
        for t in (ys, yp, yd, yl, yg, yo):
            t.fill_(-7.0)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert np.all(np.abs(ys.cpu().numpy() - oracle.sepfilter(a, kx, ky)) <= _sep_tol(a, kx, ky)), rep
        for got, ref in ((yp, oracle.conv2d(b, wp, (1, 1), (2, 2))), (yd, oracle.conv2d(c, wd, (4, 4), (0, 0))),
                         (yo, oracle.correlation(e1, e2, 3, 2))):
            gg, rr = got.cpu().numpy().astype(np.float64), ref.astype(np.float64)
            assert np.all(np.abs(gg - rr) <= 2e-2 * np.abs(rr) + 1e-3), rep
        assert np.array_equal(yl.cpu().numpy(), oracle.pool2d(d, (3, 3), (2, 2), (0, 0), "max")), rep
        rg = oracle.pool2d(d, (27, 27), (1, 1), (0, 0), "avg")
        assert np.all(np.abs(yg.cpu().numpy() - rg) <= 1e-5 * np.abs(rg) + 1e-6), rep
