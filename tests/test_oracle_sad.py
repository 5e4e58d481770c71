"""Pins for the block-matching oracle (no GPU)."""
import numpy as np
import pytest

import oracle
from oracle import merit_literal as lit
from paper_1911_03458_amd import workloads as wl


def test_identical_random_frames_give_zero_at_origin():
    rng = np.random.default_rng(1)
    f = rng.integers(0, 256, size=(32, 48), dtype=np.uint8)
    sad, mv = oracle.sad_search(f, f, 8, 4)
    assert sad.shape == (4, 6) and mv.shape == (4, 6, 2)
    assert np.all(sad == 0)
    assert np.all(mv == 0)


def test_constant_frames_tie_to_lowest_raster_index():
    f = np.full((16, 16), 77, np.uint8)
    for R in (1, 2, 4):
        sad, mv = oracle.sad_search(f, f, 4, R)
        assert np.all(sad == 0)
        assert np.all(mv == -R), "all candidates tie at 0: the first one scanned is (-R,-R)"


def test_tie_break_is_dy_major():
    """Rows all equal => every dy ties for a given dx; columns distinct => only
    dx=0 reaches 0.  The answer must be (dy,dx) = (-R, 0), not (0,0) or (0,-R)."""
    rng = np.random.default_rng(2)
    row = rng.permutation(256)[:24].astype(np.uint8)       # distinct values
    f = np.tile(row, (16, 1))
    sad, mv = oracle.sad_search(f, f, 8, 2)
    assert np.all(sad == 0)
    # interior block columns: only dx = 0 matches; every dy ties
    assert mv[0, 1].tolist() == [-2, 0] and mv[1, 1].tolist() == [-2, 0]
    # transpose: columns all equal => every dx ties, dy = 0 only
    sad, mv = oracle.sad_search(np.ascontiguousarray(f.T), np.ascontiguousarray(f.T), 8, 2)
    assert mv[1, 0].tolist() == [0, -2] and mv[1, 1].tolist() == [0, -2]


def test_clamped_border_creates_ties():
    """Top block, flat top rows: dy=-2 and dy=-1 read the same (clamped) rows."""
    rng = np.random.default_rng(3)
    f = rng.integers(0, 256, size=(16, 16), dtype=np.uint8)
    s = oracle.sad_surface(f, f, 8, 2, 0, 0)
    # candidate (dy,dx) = (0,0) is exact
    assert s[2, 2] == 0
    # reading above the frame clamps to row 0: build it by hand for dy=-2, dx=0
    want = 0
    for i in range(8):
        for j in range(8):
            want += abs(int(f[i, j]) - int(f[max(i - 2, 0), j]))
    assert s[0, 2] == want
    # and to the left for dx=-1
    want = sum(abs(int(f[i, j]) - int(f[i, max(j - 1, 0)])) for i in range(8) for j in range(8))
    assert s[2, 1] == want


def test_displacement_sign_ref_equals_cur_plus_d():
    """cur block = ref block displaced by (+2,-1) => the search reports (+2,-1)."""
    rng = np.random.default_rng(4)
    ref = rng.integers(0, 256, size=(32, 32), dtype=np.uint8)
    cur = np.zeros_like(ref)
    vy, vx = 2, -1
    for y in range(32):
        for x in range(32):
            cur[y, x] = ref[min(max(y + vy, 0), 31), min(max(x + vx, 0), 31)]
    sad, mv = oracle.sad_search(cur, ref, 8, 3)
    assert np.all(sad == 0)
    assert mv[1, 1].tolist() == [vy, vx] and mv[2, 2].tolist() == [vy, vx]


def test_triangle_lower_bound_and_surface_minimum():
    rng = np.random.default_rng(5)
    cur = rng.integers(0, 256, size=(16, 24), dtype=np.uint8)
    ref = rng.integers(0, 256, size=(16, 24), dtype=np.uint8)
    sad, mv = oracle.sad_search(cur, ref, 8, 3)
    for by in range(2):
        for bx in range(3):
            s = oracle.sad_surface(cur, ref, 8, 3, by, bx)
            assert s.min() == sad[by, bx]
            k = int(np.argmin(s))                          # first minimum, raster order
            assert [k // 7 - 3, k % 7 - 3] == mv[by, bx].tolist()
            # |sum cur - sum ref| <= SAD for the zero-displacement candidate
            cb = cur[by * 8:by * 8 + 8, bx * 8:bx * 8 + 8].astype(int)
            rb = ref[by * 8:by * 8 + 8, bx * 8:bx * 8 + 8].astype(int)
            assert abs(cb.sum() - rb.sum()) <= s[3, 3] == np.abs(cb - rb).sum()


@pytest.mark.parametrize("H,W,B,R", [(16, 16, 4, 2), (8, 24, 8, 3), (12, 8, 4, 1), (16, 32, 16, 2),
                                     (13, 24, 8, 3), (16, 21, 8, 2), (9, 10, 4, 1)])
def test_matches_literal_transform_evaluator(H, W, B, R):
    rng = np.random.default_rng(H * W + B + R)
    cur = rng.integers(0, 256, size=(H, W), dtype=np.uint8)
    ref = rng.integers(0, 256, size=(H, W), dtype=np.uint8)
    # low-entropy variant produces many ties, exercising the tie-break
    for c, r in [(cur, ref), (cur & 0x3, ref & 0x3)]:
        a_sad, a_mv = oracle.sad_search(c, r, B, R)
        b_sad, b_mv = lit.sad_search(c, r, B, R)
        assert np.array_equal(a_sad, b_sad)
        assert np.array_equal(a_mv, b_mv)


@pytest.mark.parametrize("H,W,B,R", [(27, 40, 8, 3), (32, 45, 16, 4), (30, 29, 8, 2), (5, 7, 8, 1)])
def test_frames_the_block_does_not_divide_equal_edge_padded_frames(H, W, B, R):
    """Blocks that reach past the edge read both frames with clamped coordinates: the same
    as replicating the border out to a multiple of the block first (numpy's edge padding) and
    running the search the block divides.  A clamp missing on either frame, or the clamp
    applied before the displacement is added, fails here."""
    rng = np.random.default_rng(H * 100 + W)
    cur = rng.integers(0, 256, size=(H, W), dtype=np.uint8)
    ref = rng.integers(0, 256, size=(H, W), dtype=np.uint8)
    Hp, Wp = -(-H // B) * B, -(-W // B) * B
    pad = ((0, Hp - H), (0, Wp - W))
    sad, mv = oracle.sad_search(cur, ref, B, R)
    psad, pmv = oracle.sad_search(np.pad(cur, pad, mode="edge"), np.pad(ref, pad, mode="edge"), B, R)
    assert sad.shape == (Hp // B, Wp // B)
    assert np.array_equal(sad, psad) and np.array_equal(mv, pmv)
    # one partial block by brute force
    by, bx = sad.shape[0] - 1, sad.shape[1] - 1
    surf = oracle.sad_surface(cur, ref, B, R, by, bx)
    ys = np.clip(np.arange(by * B, by * B + B), 0, H - 1)
    xs = np.clip(np.arange(bx * B, bx * B + B), 0, W - 1)
    cb = cur[np.ix_(ys, xs)].astype(np.int64)
    for dy in (-R, 0, R):
        for dx in (-R, 1):
            ry = np.clip(np.arange(by * B, by * B + B) + dy, 0, H - 1)
            rx = np.clip(np.arange(bx * B, bx * B + B) + dx, 0, W - 1)
            assert surf[dy + R, dx + R] == np.abs(cb - ref[np.ix_(ry, rx)].astype(np.int64)).sum()
    assert sad[by, bx] == surf.min()


def test_cfg0_planted_vectors_and_noise_bound():
    cur, ref, planted = wl.make_sad_frames(wl.CFG0_ME_SMALL)
    sad, mv = oracle.sad_search(cur, ref, 8, 4)
    assert sad.max() <= 3 * 64, "noise is at most 3 per pixel"
    # random texture: the planted candidate is (with overwhelming probability) the unique best
    assert np.array_equal(mv, planted)


def test_cfg3_generator_plants_exact_copies_on_a_crop():
    """Same recipe as the full-HD workload on a small frame: planted SAD is 0."""
    small = wl.SadWorkload("crop", 96, 128, 16, 8, 0, "sinusoid")
    cur, ref, planted = wl.make_sad_frames(small, seed=1914)
    sad, mv = oracle.sad_search(cur, ref, 16, 8)
    assert np.all(sad == 0)
    for by in range(6):
        for bx in range(8):
            s = oracle.sad_surface(cur, ref, 16, 8, by, bx)
            zeros = np.flatnonzero(s.ravel() == 0)
            pk = (planted[by, bx, 0] + 8) * 17 + planted[by, bx, 1] + 8
            assert pk in zeros
            assert (mv[by, bx, 0] + 8) * 17 + mv[by, bx, 1] + 8 == zeros[0]
