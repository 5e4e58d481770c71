"""Pins for the literal transform evaluator against values the paper prints."""
import os

import numpy as np

from oracle import merit_literal as lit

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _read(name):
    rows = {}
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            parts = line.split()
            rows.setdefault(parts[0], []).append(parts[1:])
    return rows


def test_footprint_worked_example():
    g = _read("footprint_example.txt")
    tp = [int(v) for v in g["tile_p"][0]]
    ta = [int(v) for v in g["tile_a"][0]]
    sp = [int(v) for v in g["stride_p"][0]]
    sa = [int(v) for v in g["stride_a"][0]]
    want = tuple(int(v) for v in g["footprint"][0])
    t = lit.Transform(axis=(0, 1, 0, 1), stride=tuple(sp + sa), offset=(0, 0, -2, -2))
    assert lit.footprint(tp + ta, t, 2) == want == (20, 12)
    # and it really is the extent of the coordinates the tile touches
    x = lit.coordinates(tp + ta, t, 2)
    assert (x[0].max() - x[0].min() + 1, x[1].max() - x[1].min() + 1) == want


def test_footprint_with_strides_matches_touched_extent():
    # stride-2 7x7 window (the small-Cin convolution workload), tile of 4x8 outputs
    ranges, n_par, tx, tw = lit.conv2d_desc(1, 3, 64, 64, 8, 7, 7, 2, 2, 3, 3)
    tile = (1, 8, 4, 8, 3, 7, 7)
    fp = lit.footprint(tile, tx, 4)
    assert fp == (1, 3, 2 * 3 + 7, 2 * 7 + 7)
    x = lit.coordinates(tile, tx, 4)
    assert tuple(int(x[i].max() - x[i].min() + 1) for i in range(4)) == fp
    # the weight operand of the same tile: all taps of 8 output channels
    assert lit.footprint(tile, tw, 4) == (8, 3, 7, 7)


def test_alexnet_conv1_index_expression():
    g = _read("alexnet_conv1_index.txt")
    nd = tuple(int(v) for v in g["ndrange"][0])
    s = int(g["input_stride"][0][0])
    o = int(g["input_offset"][0][0])
    assert nd == (48, 55, 55, 3, 11, 11)
    # single image: drop the batch index of conv2d_desc by using N=1
    _, n_par, tx, tw = lit.conv2d_desc(1, 3, 227, 227, 48, 11, 11, s, s, -o, -o)
    ranges = (1,) + nd                                      # the printed NDRange, one image
    x = lit.coordinates(ranges, tx, 4)
    k = np.indices(ranges)
    assert np.array_equal(x[1], k[4])                       # channel  = a1
    assert np.array_equal(x[2], s * k[2] + k[5] + o)        # row      = 4 p2 + a2 - 5
    assert np.array_equal(x[3], s * k[3] + k[6] + o)        # column   = 4 p3 + a3 - 5
    xw = lit.coordinates(ranges, tw, 4)
    assert g["weight_index"][0] == ["p1", "a1", "a2", "a3"]
    for axis, kk in zip(range(4), (k[1], k[4], k[5], k[6])):
        assert np.array_equal(xw[axis], kk)


def test_transformed_tensor_sizes():
    g = _read("transformed_sizes.txt")
    assert g["conv"][0] == ["p", "h", "w", "a", "k", "k"]
    assert g["gemm"][0] == ["p", "m", "n", "a", "k"]
    h, w, k = 6, 7, 3
    # single-channel k x k convolution with 'same' padding: M(A) is ((h,w),(k,k))
    ranges, n_par, tx, tw = lit.conv2d_desc(1, 1, h, w, 1, k, k, 1, 1, k // 2, k // 2)
    A = np.arange(h * w, dtype=np.float64).reshape(1, 1, h, w)
    MA, _ = lit.transform(A, ranges, tx, n_par, "zero")
    assert MA.shape == (h * w, k * k)
    # GEMM in the same notation: C[m,n] = sum_k A[m,k] B[k,n]; M(A) repeats rows, M(B) columns
    m, n, kk = 3, 4, 5
    rng = np.random.default_rng(0)
    Amat, Bmat = rng.standard_normal((m, kk)), rng.standard_normal((kk, n))
    ta = lit.Transform(axis=(0, lit.UNUSED, 1), stride=(1, 0, 1), offset=(0, 0, 0))
    tb = lit.Transform(axis=(lit.UNUSED, 1, 0), stride=(0, 1, 1), offset=(0, 0, 0))
    MA, _ = lit.transform(Amat, (m, n, kk), ta, 2, "zero")
    MB, _ = lit.transform(Bmat, (m, n, kk), tb, 2, "zero")
    assert MA.shape == MB.shape == (m * n, kk)
    assert np.allclose((MA * MB).sum(axis=1).reshape(m, n), Amat @ Bmat)


def test_dilated_index_expression():
    """I[a1, p2 + 2 a2, p3 + 2 a3]: the window indices move two input pixels per step."""
    g = _read("dilated_index.txt")
    assert g["row"][0] == ["p2", "1", "a2", "2"] and g["column"][0] == ["p3", "1", "a3", "2"]
    ranges, n_par, tx, tw = lit.conv2d_desc(1, 3, 20, 22, 4, 3, 3, 1, 1, 0, 0, 2, 2)
    x = lit.coordinates(ranges, tx, 4)
    k = np.indices(ranges)
    assert np.array_equal(x[1], k[4])
    assert np.array_equal(x[2], k[2] + 2 * k[5]) and np.array_equal(x[3], k[3] + 2 * k[6])
    assert ranges[2:4] == (20 - 4, 22 - 4)                  # extent of the dilated window: 2 (k - 1) + 1


def test_correlation_index_expression():
    """Eq. 8 with the displacement indices centred (p3 - R) and strided as the workload needs;
    at R = 0 offsets and stride 1 it is the printed expression."""
    g = _read("correlation_index.txt")
    assert ["row", "p1", "p3"] in g["i2"] and ["column", "p2", "p4"] in g["i2"] and ["row", "p1"] in g["i1"]
    ranges, n_par, t1, t2 = lit.correlation_desc(1, 4, 6, 7, 2, 1)
    k = np.indices(ranges)                                  # (n, p1, p2, p3, p4 | a1)
    x1 = lit.coordinates(ranges, t1, 4)
    x2 = lit.coordinates(ranges, t2, 4)
    assert np.array_equal(x1[1], k[5]) and np.array_equal(x1[2], k[1]) and np.array_equal(x1[3], k[2])
    assert np.array_equal(x2[1], k[5])
    assert np.array_equal(x2[2], k[1] + k[3] - 2) and np.array_equal(x2[3], k[2] + k[4] - 2)


def test_bilateral_call_descriptor():
    """Listing 3: window indices on the two image axes at offset -k/2, stride 1; 16 x 16 tiles."""
    g = _read("bilateral_call.txt")
    assert g["acc"] == [["0", "-k/2", "1"], ["1", "-k/2", "1"]] and g["tile"][0] == ["16", "16"]
    k = 5
    ranges, n_par, t_row, t_col, t_ker = lit.sepfilter_desc(1, 9, 10, k)
    # the row pass carries the a2 triple {1,-k/2,1}, the column pass the a1 triple {0,-k/2,1}
    # (image axes 1 and 2 here: axis 0 is the batch)
    assert (t_col.axis[3], t_col.offset[3], t_col.stride[3]) == (1, -(k // 2), 1)
    assert (t_row.axis[3], t_row.offset[3], t_row.stride[3]) == (2, -(k // 2), 1)
    # a 16 x 16 tile of outputs with the k x k window covers (16 + k - 1)^2 pixels (Eq. 9)
    both = lit.Transform(axis=(0, 1, 2, 1, 2), stride=(1,) * 5, offset=(0, 0, 0, -(k // 2), -(k // 2)))
    assert lit.footprint((1, 16, 16, k, k), both, 3) == (1, 16 + k - 1, 16 + k - 1)


def test_workload_table_shapes_are_the_synthetic_workloads():
    from paper_1911_03458_amd import workloads as wl
    g = _read("workload_table.txt")
    assert [int(v) for v in g["dilated"][0]] == [wl.CFG_DILATED.OH, wl.CFG_DILATED.OW, wl.CFG_DILATED.Cout]
    c = wl.CFG_CORRELATION
    assert [int(v) for v in g["correlation"][0]] == [c.H, c.W, 2 * c.search + 1, 2 * c.search + 1]
    d = wl.CFG_DEPTHWISE
    assert [int(v) for v in g["depthwise"][0]] == [d.H, d.W, d.C]
    m = wl.CFG_ME_720P
    assert g["motion_estimation"][0] == ["720p", "8", "8"] and (m.H, m.W, m.block) == (720, 1280, 8)
