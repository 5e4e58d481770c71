"""Host-only checks of the C ABI: the library loads, exports every declared symbol,
and the plan logic (validation, output shapes, footprint rule) behaves.  No GPU."""
import ctypes
import os
import re

import pytest

from oracle import merit_literal as lit
from paper_1911_03458_amd import binding as mb

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    names = set()
    inc = os.path.join(ROOT, "include")
    for header in sorted(os.listdir(inc)):                  # every header of the boundary
        if not header.endswith(".h"):
            continue
        text = open(os.path.join(inc, header)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names |= set(re.findall(r"\b(merit_[a-z0-9_]+)\s*\(", text))
    return sorted(names)


def test_library_exports_every_declared_symbol():
    L = mb.lib()
    names = _declared_symbols()
    assert {"merit_plan_create", "merit_plan_destroy", "merit_conv2d", "merit_pool2d",
            "merit_sad_search", "merit_status_string", "merit_probe_copy", "merit_probe_alu"} <= set(names)
    for n in names:
        assert hasattr(L, n), n


def test_status_strings():
    L = mb.lib()
    seen = {L.merit_status_string(i).decode() for i in range(8)}
    assert len(seen) == 8 and "ok" in seen


def test_struct_layout_matches_header_sizes():
    # int32 + 6*int64 + 12*int32 + 2*12*int64, natural alignment
    assert ctypes.sizeof(mb.merit_operand) == 8 + 48 + 48 + 96 + 96
    assert ctypes.sizeof(mb.merit_plan_desc) == 24 + 96 + 2 * ctypes.sizeof(mb.merit_operand)


# ------------------------------------------------------------ descriptors
def _triples(op, n):
    return [(op.axis[j], op.stride[j], op.offset[j]) for j in range(n)]


def test_conv_plan_descriptor_is_the_papers_transform():
    plan = mb.merit_plan_conv2d(2, 3, 224, 224, 64, 7, 7, 2, 2, 3, 3)
    d = plan.desc()
    ranges, n_par, tx, tw = lit.conv2d_desc(2, 3, 224, 224, 64, 7, 7, 2, 2, 3, 3)
    assert (d.n_par, d.n_acc) == (4, 3)
    assert tuple(d.range[:7]) == ranges
    for got, want in ((d.a, tx), (d.b, tw)):
        for j in range(7):
            assert got.axis[j] == want.axis[j]
            if want.axis[j] != lit.UNUSED:
                assert (got.stride[j], got.offset[j]) == (want.stride[j], want.offset[j])
    assert plan.out_shape() == (2, 64, 112, 112)


def test_relu_plan_differs_only_in_the_product_function():
    a = mb.merit_plan_conv2d(2, 3, 32, 32, 8, 7, 7, 2, 2, 3, 3)
    b = mb.merit_plan_conv2d_relu(2, 3, 32, 32, 8, 7, 7, 2, 2, 3, 3)
    da, db = a.desc(), b.desc()
    assert (da.op, db.op) == (mb.MERIT_OP_CONV_DOT, mb.MERIT_OP_CONV_DOT_RELU)
    assert tuple(da.range) == tuple(db.range) and a.out_shape() == b.out_shape()
    assert a.launch_info() == b.launch_info()
    # the generic constructor accepts the same descriptor
    assert mb.merit_plan_create(db).desc().op == mb.MERIT_OP_CONV_DOT_RELU
    db.pad = mb.MERIT_PAD_CLAMP                      # border replication: no specialised kernel, the definition kernel
    assert mb.merit_plan_create(db).launch_info()["kernel"] == "merit_generic<dot>"
    db.pad = mb.MERIT_PAD_NEG_INF                    # not a rule a dot product can have
    with pytest.raises(mb.MeritError):
        mb.merit_plan_create(db)


def test_dilated_plan_is_the_papers_expression():
    """I[a1, p2 + 2 a2, p3 + 2 a3] (Section III-C): stride 2 on the window indices."""
    plan = mb.merit_plan_conv2d_dilated(1, 32, 64, 64, 32, 3, 3, 1, 1, 2, 2, 2, 2, 0)
    d = plan.desc()
    ranges, n_par, tx, tw = lit.conv2d_desc(1, 32, 64, 64, 32, 3, 3, 1, 1, 2, 2, 2, 2)
    assert tuple(d.range[:7]) == ranges and plan.out_shape() == (1, 32, 64, 64)
    assert (d.a.stride[5], d.a.stride[6], d.a.offset[5], d.a.offset[6]) == (2, 2, -2, -2)
    assert plan.launch_info()["kernel"] == "merit_conv2d_chblock"
    assert plan.footprint(0, (1, 1, 8, 8, 32, 3, 3)) == lit.footprint((1, 1, 8, 8, 32, 3, 3), tx, 4)
    # few input channels: the adjacent-tap kernels do not apply, the channel-block one does
    assert mb.merit_plan_conv2d_dilated(2, 3, 32, 32, 8, 3, 3, 1, 1, 2, 2, 2, 2, 1).launch_info()["kernel"] == \
        "merit_conv2d_chblock"


def test_fused_pooling_plan():
    """Convolution + clipping + 3x3/s2/p1 max pooling as one launch: the descriptor is the
    convolution's, the output shape the pooled tensor's."""
    plan = mb.merit_plan_conv2d_pool(32, 3, 224, 224, 64, 7, 7, 2, 2, 3, 3, 1)
    conv = mb.merit_plan_conv2d_relu(32, 3, 224, 224, 64, 7, 7, 2, 2, 3, 3)
    d = plan.desc()
    assert d.op == mb.MERIT_OP_CONV_DOT_RELU_POOLMAX and tuple(d.range) == tuple(conv.desc().range)
    assert conv.out_shape() == (32, 64, 112, 112) and plan.out_shape() == (32, 64, 56, 56)
    li = plan.launch_info()
    assert li["kernel"] == "merit_conv2d_planar_ws_pool" and li["block"][0] == 512
    # 32 images x 8 bands of 7 pooled rows; a band computes 8 convolution row pairs
    assert li["grid"][:2] == (256, 1) and li["tile"][2] == 16
    assert li["lds_bytes"] <= 160 * 1024
    assert mb.merit_plan_conv2d_pool(32, 3, 224, 224, 64, 7, 7, 2, 2, 3, 3, 0).desc().op == \
        mb.MERIT_OP_CONV_DOT_POOLMAX
    assert mb.merit_plan_create(d).out_shape() == (32, 64, 56, 56)
    plan.set_tile((0, 0, 8, 64))                           # the kernel it already uses
    with pytest.raises(mb.MeritError):
        plan.set_tile((0, 0, 4, 32))
    # few bands for a single image: at least 4 pooled rows each
    one = mb.merit_plan_conv2d_pool(1, 3, 44, 32, 64, 3, 3, 1, 1, 1, 1, 1).launch_info()
    assert one["grid"][0] == 5 and one["tile"][2] == 12
    for bad in ((2, 3, 62, 62, 8, 7, 7, 2, 2, 3, 3),        # 31 x 31 result: odd height
                (2, 3, 64, 48, 8, 7, 7, 2, 2, 3, 3),        # 24 columns: not a multiple of 16
                (2, 3, 32, 256, 8, 3, 3, 1, 1, 1, 1),       # a row pair does not fit a tile
                (2, 16, 32, 32, 8, 3, 3, 1, 1, 1, 1),       # many input channels, fewer than 33 output channels
                (2, 16, 32, 32, 64, 5, 5, 1, 1, 2, 2),      # many input channels: 3x3 windows only
                (2, 16, 31, 33, 64, 3, 3, 1, 1, 1, 1),      # odd result
                (2, 64, 8, 224, 64, 3, 3, 1, 1, 1, 1)):     # a row pair does not fit the largest tile
        with pytest.raises(mb.MeritError) as e:
            mb.merit_plan_conv2d_pool(*bad, 1)
        assert e.value.status == mb.MERIT_ERR_UNSUPPORTED


def test_small_launches_get_32_channel_tiles():
    """A launch whose 128-pixel x 64-channel tiles would leave half the chip idle takes 128 x 32
    tiles (twice the work items, each 0.7 of the time); with enough items for every compute unit
    the 64-channel tiles stay."""
    small = mb.merit_plan_conv2d(8, 512, 14, 14, 512, 3, 3, 1, 1, 1, 1).launch_info()
    assert small["kernel"] == "merit_conv2d_chws" and small["tile"][1] == 32 and small["grid"][0] == 256
    one = mb.merit_plan_conv2d(1, 256, 56, 56, 256, 3, 3, 1, 1, 1, 1).launch_info()
    assert one["tile"][1] == 32 and one["grid"][0] == 200
    full = mb.merit_plan_conv2d(8, 64, 56, 56, 64, 3, 3, 1, 1, 1, 1).launch_info()
    assert full["tile"][1] == 64 and full["grid"][0] == 200
    # an added tensor keeps the 64-channel tiles (the residual instance)
    res = mb.merit_plan_conv2d_residual(1, 256, 56, 56, 256, 3, 3, 1, 1, 1, 1, 1).launch_info()
    assert res["kernel"] == "merit_conv2d_chws" and res["tile"][1] == 64


def test_wide_images_get_tiles_of_whole_rows():
    """64 -> 64 on 224x224: a 256-pixel run would start anywhere in a row and stage 5 rows for
    1.14 rows of results; a tile of one whole row (224 pixels) stages 3.  56-wide layers keep the
    runs (a fifth less staging does not pay for the idle eighth of the tile)."""
    wide = mb.merit_plan_conv2d(8, 64, 224, 224, 64, 3, 3, 1, 1, 1, 1).launch_info()
    assert wide["kernel"] == "merit_conv2d_chws" and wide["tile"][2] == 1 and wide["tile"][3] == 224
    mid = mb.merit_plan_conv2d(8, 128, 112, 112, 128, 3, 3, 1, 1, 1, 1).launch_info()
    assert mid["kernel"] == "merit_conv2d_chws" and mid["tile"][2] == 2
    narrow = mb.merit_plan_conv2d(8, 256, 56, 56, 256, 3, 3, 1, 1, 1, 1).launch_info()
    assert narrow["tile"][2] == 6 and narrow["grid"][0] == 208


def test_pooling_plan_in_two_launches_where_fusion_would_cost_more():
    """Compute-bound layers on few images (256 -> 256 on 56x56, batch 8): the plan runs the plain
    convolution and then the binary16 pooling kernel; a tile request names a fused tiling and keeps
    the plan fused, an empty request gives the choice back to the planner."""
    plan = mb.merit_plan_conv2d_pool(8, 256, 56, 56, 256, 3, 3, 1, 1, 1, 1, 1)
    assert plan.out_shape() == (8, 256, 28, 28)
    li = plan.launch_info()
    assert li["kernel"] == "merit_conv2d_chws+merit_maxpool_f16" and li["block"][0] == 768 and li["tile"][1] == 128
    plan.set_tile((0, 0, 8, 64))
    assert plan.launch_info()["kernel"] == "merit_conv2d_chws_pool"
    plan.set_tile((0,) * 12)
    assert plan.launch_info()["kernel"] == "merit_conv2d_chws+merit_maxpool_f16"
    # memory-bound and small layers, launches that leave most of the chip idle, and launches with enough
    # images to fill the chip with long bands stay fused
    for shape in ((8, 64, 56, 56, 64), (8, 256, 28, 28, 512), (1, 256, 56, 56, 256), (32, 256, 56, 56, 256), (8, 128, 112, 112, 128)):
        N, Cin, H, W, Cout = shape
        assert mb.merit_plan_conv2d_pool(N, Cin, H, W, Cout, 3, 3, 1, 1, 1, 1, 1).launch_info()["kernel"] == "merit_conv2d_chws_pool"


def test_fused_pooling_plan_many_channels():
    """The same fusion on the wave-specialised multi-pass kernel (3x3 layers with at least 16
    input and 33 output channels): work items are bands of pooled rows, tiles whole rows."""
    plan = mb.merit_plan_conv2d_pool(8, 64, 56, 56, 64, 3, 3, 1, 1, 1, 1, 1)
    assert plan.desc().op == mb.MERIT_OP_CONV_DOT_RELU_POOLMAX and plan.out_shape() == (8, 64, 28, 28)
    li = plan.launch_info()
    # 256-pixel tiles of 3 rows = the row above + 1 pooled row; 8 images x 28 tiles
    assert li["kernel"] == "merit_conv2d_chws_pool" and li["block"][0] == 512 and li["tile"][1] == 64
    assert li["grid"][:2] == (224, 1) and li["tile"][2] == 3 and li["lds_bytes"] <= 160 * 1024
    plan.set_tile((0, 0, 8, 32))       # 128-pixel tiles: 2 rows, the row above carried from the tile before; a band below the top computes that tile too
    li = plan.launch_info()
    assert li["kernel"] == "merit_conv2d_chws_pool" and li["grid"][0] == 8 * 28 and li["tile"][2] == 4
    plan.set_tile((0, 0, 8, 64))
    assert plan.launch_info()["tile"][2] == 3
    with pytest.raises(mb.MeritError):
        plan.set_tile((0, 0, 12, 64))
    with pytest.raises(mb.MeritError):
        mb.merit_plan_packed_weights_bytes(plan)           # the pooling kernel reads the caller's weights
    # many images: bands of 2 pooled rows, 4-row tiles with the row above carried
    many = mb.merit_plan_conv2d_pool(32, 16, 24, 56, 64, 3, 3, 1, 1, 1, 1, 1)
    many.set_tile((0, 0, 8, 64))
    li = many.launch_info()
    assert li["grid"][0] == 32 * 6 and li["tile"][2] == 2 * 2 + 4
    wide = mb.merit_plan_conv2d_pool(8, 128, 112, 112, 128, 3, 3, 1, 1, 1, 1, 0)
    li = wide.launch_info()
    # 128 output channels: 256 x 128 tiles on 12 wavefronts; two rows of 112 per tile, 8 images x 28 bands of 2 pooled rows
    assert li["kernel"] == "merit_conv2d_chws_pool" and li["block"][0] == 768 and li["tile"][1] == 128
    assert li["grid"][0] == 224 and li["tile"][2] == 6 and li["lds_bytes"] <= 160 * 1024
    assert wide.out_shape() == (8, 128, 56, 56)
    wide.set_tile((0, 0, 8, 64))                           # 64-channel tiles on request
    assert wide.launch_info()["tile"][1] == 64 and wide.launch_info()["block"][0] == 512


def test_residual_plan():
    """The residual layer keeps the convolution's descriptor; only the multiply-and-store kernels
    take the added tensor; of the wave-specialised ones only the many-channel kernel does."""
    args = (32, 3, 224, 224, 64, 7, 7, 2, 2, 3, 3)
    plan = mb.merit_plan_conv2d_residual(*args, 1)
    conv = mb.merit_plan_conv2d(*args)
    assert plan.desc().op == mb.MERIT_OP_CONV_DOT_ADD_RELU and tuple(plan.desc().range) == tuple(conv.desc().range)
    assert mb.merit_plan_conv2d_residual(*args, 0).desc().op == mb.MERIT_OP_CONV_DOT_ADD
    assert plan.out_shape() == conv.out_shape()
    assert conv.launch_info()["kernel"] == "merit_conv2d_planar_ws"
    assert plan.launch_info()["kernel"] == "merit_conv2d_planar"
    with pytest.raises(mb.MeritError):
        plan.set_tile((0, 0, 8, 64))
    plan.set_tile((0, 0, 4, 64))
    assert plan.launch_info()["kernel"] == "merit_conv2d_planar"
    # many channels, 3x3: the wave-specialised multi-pass kernel adds the tensor in its accumulators' layout
    res = mb.merit_plan_conv2d_residual(8, 64, 56, 56, 64, 3, 3, 1, 1, 1, 1, 1)
    plain = mb.merit_plan_conv2d(8, 64, 56, 56, 64, 3, 3, 1, 1, 1, 1)
    assert res.launch_info()["kernel"] == "merit_conv2d_chws" and res.launch_info() == plain.launch_info()
    assert mb.merit_plan_create(res.desc()).desc().op == mb.MERIT_OP_CONV_DOT_ADD_RELU
    res.set_tile((0, 0, 4, 32))                                       # the plain kernel on request
    assert res.launch_info()["kernel"] == "merit_conv2d_chblock"
    with pytest.raises(mb.MeritError):
        res.set_tile((0, 0, 12, 64))                                  # not the 128-channel tilings
    # 256 channels: the 64-channel tiles (the plain plan takes 128-channel ones)
    big = mb.merit_plan_conv2d_residual(8, 256, 56, 56, 256, 3, 3, 1, 1, 1, 1, 0).launch_info()
    assert big["kernel"] == "merit_conv2d_chws" and big["tile"][1] == 64 and big["block"][0] == 512
    # other windows: the plain kernels
    assert mb.merit_plan_conv2d_residual(1, 64, 28, 28, 64, 5, 5, 1, 1, 2, 2, 1).launch_info()["kernel"] in (
        "merit_conv2d_chblock", "merit_conv2d_chpass")


def test_sepfilter_plan():
    plan = mb.merit_plan_sepfilter(4, 1080, 1920, 30)
    d = plan.desc()
    ranges, n_par, t_row, t_col, t_ker = lit.sepfilter_desc(4, 1080, 1920, 30)
    assert (d.op, d.n_par, d.n_acc, d.dtype, d.pad) == (mb.MERIT_OP_SEPFILTER_DOT, 3, 2, mb.MERIT_F32,
                                                      mb.MERIT_PAD_CLAMP)
    assert tuple(d.range[:5]) == (4, 1080, 1920, 30, 30) and plan.out_shape() == (4, 1080, 1920)
    # the window indices sit on the image axes at offset -k/2, as in the two 1-D passes
    assert (d.a.axis[3], d.a.offset[3]) == (t_col.axis[3], t_col.offset[3]) == (1, -15)
    assert (d.a.axis[4], d.a.offset[4]) == (t_row.axis[3], t_row.offset[3]) == (2, -15)
    li = plan.launch_info()
    assert li["kernel"] == "merit_sepfilter_tile" and li["tile"][1:3] == (64, 64)
    assert li["grid"][0] == 1024 and li["lds_bytes"] <= 160 * 1024       # persistent: 4 workgroups (37 KB each) per CU for 2040 tiles
    # Eq. 9: a 64 x 64 tile of outputs with a 30 x 30 window covers 93 x 93 pixels
    assert plan.footprint(0, (1, 64, 64, 30, 30)) == (1, 93, 93)
    # output rows: a multiple of 4 that keeps the staged rows (output rows + k - 1) within the request
    small = mb.merit_plan_sepfilter(1, 40, 70, 3)
    assert small.launch_info()["tile"][1] == 60
    small.set_tile((0, 32))
    assert small.launch_info()["tile"][1] == 28
    with pytest.raises(mb.MeritError):
        small.set_tile((0, 5))                              # no room for four output rows
    with pytest.raises(mb.MeritError):
        plan.set_tile((0, 32))                              # not above the 30-tap window
    with pytest.raises(mb.MeritError) as e:
        mb.merit_plan_sepfilter(1, 40, 70, 33)
    assert e.value.status == mb.MERIT_ERR_UNSUPPORTED
    with pytest.raises(mb.MeritError):
        mb.merit_plan_sepfilter(1, 0, 70, 3)


def test_bilateral_plan():
    plan = mb.merit_plan_bilateral(1, 1080, 1920, 9)
    d = plan.desc()
    assert (d.op, d.n_par, d.n_acc, d.dtype, d.pad) == (mb.MERIT_OP_BILATERAL, 3, 2, mb.MERIT_F32, mb.MERIT_PAD_CLAMP)
    assert tuple(d.range[:5]) == (1, 1080, 1920, 9, 9) and plan.out_shape() == (1, 1080, 1920)
    assert (d.a.offset[3], d.a.offset[4]) == (-4, -4)            # Listing 3: {0,-k/2,1}, {1,-k/2,1}
    li = plan.launch_info()
    assert li["kernel"] == "merit_bilateral_rows" and li["tile"][1:3] == (16, 64)      # the listing's 16-row tiles
    assert mb.merit_plan_bilateral(1, 64, 64, 21).launch_info()["kernel"] == "merit_bilateral_tile"
    assert li["grid"][0] == 68 * 30
    assert plan.footprint(0, (1, 16, 64, 9, 9)) == (1, 24, 72)
    with pytest.raises(mb.MeritError) as e:
        mb.merit_plan_bilateral(1, 64, 64, 33)
    assert e.value.status == mb.MERIT_ERR_UNSUPPORTED


def test_depthwise_plan():
    plan = mb.merit_plan_conv2d_depthwise(32, 32, 64, 64, 3, 3, 1, 1, 1, 1)
    d = plan.desc()
    ranges, n_par, tx, tw = lit.depthwise_desc(32, 32, 64, 64, 3, 3, 1, 1, 1, 1)
    assert (d.op, d.n_par, d.n_acc) == (mb.MERIT_OP_DWCONV_DOT, 4, 2)
    assert tuple(d.range[:6]) == ranges and plan.out_shape() == (32, 32, 64, 64)
    assert _triples(d.a, 6) == list(zip(tx.axis, tx.stride, tx.offset))
    for j in range(6):
        assert d.b.axis[j] == tw.axis[j]
    li = plan.launch_info()
    assert li["kernel"] == "merit_dwconv_rows_k3s1p1" and li["grid"][0] == 32 * 32 * (64 // li["tile"][2])
    assert plan.footprint(0, (1, 1, li["tile"][2], 64, 3, 3))[2:] == (li["tile"][2] + 2, 66)
    plan.set_tile((0, 0, 8))
    assert plan.launch_info()["kernel"] == "merit_dwconv_tile"
    assert mb.merit_plan_conv2d_depthwise(1, 3, 9, 11, 5, 3, 2, 1, 2, 0).launch_info()["kernel"] == "merit_dwconv_tile"
    d.b.shape[0] = 31                                                # one kernel per channel
    with pytest.raises(mb.MeritError) as e:
        mb.merit_plan_create(d)
    assert e.value.status == mb.MERIT_ERR_SHAPE


def test_correlation_plan_is_eq8():
    """M(I2) = I2[a1, p1 + p3, p2 + p4] (Section III-C, Eq. 8): two indices on one axis."""
    plan = mb.merit_plan_correlation(1, 256, 64, 64, 5, 2)
    d = plan.desc()
    ranges, n_par, t1, t2 = lit.correlation_desc(1, 256, 64, 64, 5, 2)
    assert (d.op, d.n_par, d.n_acc) == (mb.MERIT_OP_CORR_DOT, 5, 1)
    assert tuple(d.range[:6]) == ranges == (1, 64, 64, 11, 11, 256)
    assert _triples(d.b, 6) == list(zip(t2.axis, t2.stride, t2.offset))
    for j in range(6):
        assert d.a.axis[j] == t1.axis[j]
    assert plan.out_shape() == (1, 64, 64, 11, 11)                  # the paper's 64 x 64 x 11 x 11
    # footprint of a (1 row x 64 pixels x 1 x 11 displacements) tile of the second tensor
    assert plan.footprint(1, (1, 1, 64, 1, 11, 256)) == lit.footprint((1, 1, 64, 1, 11, 256), t2, 4)
    assert plan.footprint(1, (1, 1, 64, 1, 11, 256))[3] == 64 + 10 * 2
    li = plan.launch_info()
    assert li["kernel"] == "merit_corr_mfma" and li["grid"][0] == 64 * 11 and li["lds_bytes"] <= 160 * 1024
    assert mb.merit_plan_create(d).out_shape() == (1, 64, 64, 11, 11)
    d.b.offset[3] = -9                                              # not centred: the definition kernel
    off = mb.merit_plan_create(d)
    assert off.launch_info()["kernel"] == "merit_generic<dot>" and off.out_shape() == (1, 64, 64, 11, 11)
    odd = mb.merit_plan_correlation(1, 8, 16, 20, 2, 1)             # W not a multiple of 8: the same
    assert odd.launch_info()["kernel"] == "merit_generic<dot>" and odd.out_shape() == (1, 16, 20, 5, 5)
    assert odd.launch_info()["grid"][0] == -(-16 * 20 * 25 // 256) and odd.launch_info()["lds_bytes"] == 0
    with pytest.raises(mb.MeritError):
        odd.set_tile((0, 4))                                        # nothing to choose there
    L = mb.lib()
    assert L.merit_correlation(plan.handle, None, 16, 16, None) == mb.MERIT_ERR_NULL
    assert L.merit_conv2d(plan.handle, 16, 16, 16, None) == mb.MERIT_ERR_INVALID_ARG


def test_pool_and_sad_plan_descriptors():
    plan = mb.merit_plan_pool2d(16, 64, 112, 112, 3, 3, 2, 2, 1, 1, 0)
    d = plan.desc()
    ranges, n_par, tx = lit.pool2d_desc(16, 64, 112, 112, 3, 3, 2, 2, 1, 1)
    assert tuple(d.range[:6]) == ranges and d.b.ndim == 0
    assert _triples(d.a, 6) == list(zip(tx.axis, tx.stride, tx.offset))
    assert plan.out_shape() == (16, 64, 56, 56)

    plan = mb.merit_plan_sad(1088, 1920, 16, 32)
    d = plan.desc()
    ranges, n_par, tref, tcur = lit.sad_desc(1088, 1920, 16, 32)
    assert tuple(d.range[:6]) == ranges == (68, 120, 65, 65, 16, 16)
    assert _triples(d.a, 6) == list(zip(tref.axis, tref.stride, tref.offset))
    for j in range(6):
        assert d.b.axis[j] == tcur.axis[j]
    assert plan.out_shape() == (68, 120)


# -------------------------------------------------------------- footprint
def test_footprint_worked_example_through_the_abi():
    """16x8 outputs of a 5x5 window need a 20x12 input sub-tensor (Section IV-A)."""
    plan = mb.merit_plan_conv2d(1, 1, 64, 64, 1, 5, 5, 1, 1, 2, 2)
    assert plan.footprint(0, (1, 1, 16, 8, 1, 5, 5)) == (1, 1, 20, 12)
    assert plan.footprint(1, (1, 1, 16, 8, 1, 5, 5)) == (1, 1, 5, 5)


@pytest.mark.parametrize("tile", [(1, 8, 4, 8, 3, 7, 7), (2, 64, 1, 112, 3, 7, 7), (1, 1, 3, 5, 1, 2, 1)])
def test_footprint_matches_literal_evaluator(tile):
    plan = mb.merit_plan_conv2d(2, 3, 224, 224, 64, 7, 7, 2, 2, 3, 3)
    ranges, n_par, tx, tw = lit.conv2d_desc(2, 3, 224, 224, 64, 7, 7, 2, 2, 3, 3)
    assert plan.footprint(0, tile) == lit.footprint(tile, tx, 4)
    assert plan.footprint(1, tile) == lit.footprint(tile, tw, 4)


def test_sad_search_window_is_block_plus_twice_range():
    plan = mb.merit_plan_sad(1088, 1920, 16, 32)
    assert plan.footprint(0, (1, 1, 65, 65, 16, 16)) == (80, 80)
    assert plan.footprint(1, (1, 1, 65, 65, 16, 16)) == (16, 16)
    # four horizontally adjacent blocks share one 80 x 128 window
    assert plan.footprint(0, (1, 4, 65, 65, 16, 16)) == (80, 128)


def test_launch_info_tiles_cover_the_output():
    plan = mb.merit_plan_pool2d(16, 64, 112, 112, 3, 3, 2, 2, 1, 1, 0)
    li = plan.launch_info()
    th = li["tile"][2]
    # default: register-streaming kernel, 28 lanes (a 32-lane group) per (plane, strip)
    assert li["kernel"].startswith("merit_pool2d_stream") and li["lds_bytes"] == 0
    assert 56 % th == 0 and li["grid"][0] == 16 * 64 * (56 // th) // 8
    # rows a lane holds per strip = footprint rule on the row axis
    assert plan.footprint(0, (1, 1, th, 56, 3, 3))[2] == 2 * th + 1
    # a strip height the streaming kernel has no instance for selects the LDS row-strip kernel
    plan.set_tile((0, 0, 14))
    li = plan.launch_info()
    assert li["kernel"].startswith("merit_pool2d_rows") and li["tile"][2] == 14
    assert li["grid"][0] == 1024 * 4
    assert li["lds_bytes"] == (13 * 2 + 3) * (112 + 8) * 4 <= 160 * 1024


def test_block_matching_plan_for_frames_the_block_does_not_divide():
    """ceil(H/B) x ceil(W/B) blocks; the row-scan kernels need rows of whole dwords
    (W % 4 == 0) but any height; otherwise the one-block-per-workgroup kernel runs."""
    full_hd = mb.merit_plan_sad(1080, 1920, 16, 32)             # 1080 = 67.5 blocks
    assert full_hd.out_shape() == (68, 120)
    assert tuple(full_hd.desc().range[:2]) == (68, 120)
    li = full_hd.launch_info()
    assert li["kernel"] == "merit_sad_rowscan16<32>" and li["grid"][0] == 68 * 30
    odd_w = mb.merit_plan_sad(64, 60, 8, 4)
    assert odd_w.out_shape() == (8, 8) and odd_w.launch_info()["kernel"] == "merit_sad_generic"   # no kernel for R = 4
    assert mb.merit_plan_sad(90, 100, 16, 16).launch_info()["kernel"].startswith("merit_sad_rowscan_pair")  # 6.25 blocks
    assert mb.merit_plan_sad(90, 98, 16, 16).launch_info()["kernel"] == "merit_sad_generic"    # rows of 24.5 dwords
    assert mb.merit_plan_sad(90, 96, 16, 16).launch_info()["kernel"].startswith("merit_sad_rowscan_pair")
    d = odd_w.desc()
    d.range[1] = 7                                              # the floor: a block column missing
    with pytest.raises(mb.MeritError) as e:
        mb.merit_plan_create(d)
    assert e.value.status == mb.MERIT_ERR_SHAPE


# ------------------------------------------------------------- validation
def test_invalid_arguments_are_rejected():
    with pytest.raises(mb.MeritError) as e:
        mb.merit_plan_pool2d(1, 1, 0, 8, 3, 3, 2, 2, 1, 1, 0)
    assert e.value.status == mb.MERIT_ERR_INVALID_ARG
    with pytest.raises(mb.MeritError) as e:
        mb.merit_plan_conv2d(1, 3, 4, 4, 8, 7, 7, 1, 1, 0, 0)   # window larger than the image
    assert e.value.status == mb.MERIT_ERR_SHAPE
    with pytest.raises(mb.MeritError) as e:
        mb.merit_plan_sad(60, 60, 6, 4)             # block not a multiple of 4
    assert e.value.status == mb.MERIT_ERR_UNSUPPORTED


def test_generic_descriptor_patterns():
    d = mb.merit_plan_conv2d(1, 8, 16, 16, 8, 3, 3, 1, 1, 1, 1).desc()
    assert mb.merit_plan_create(d).out_shape() == (1, 8, 16, 16)
    d.a.stride[5] = 2                                # dilation on the window row index ...
    with pytest.raises(mb.MeritError) as e:
        mb.merit_plan_create(d)
    assert e.value.status == mb.MERIT_ERR_SHAPE      # ... shrinks the output: (16 + 2 - 5) + 1
    d.range[2] = 14
    plan = mb.merit_plan_create(d)
    assert plan.out_shape() == (1, 8, 14, 16) and plan.launch_info()["kernel"] == "merit_conv2d_chblock"
    assert plan.footprint(0, (1, 1, 4, 4, 8, 3, 3))[2:] == (8, 6)   # rows 1 + 3 + 2*2, columns 1 + 3 + 2
    d.a.stride[5] = 1
    d.range[2] = 16
    dp = mb.merit_plan_pool2d(1, 1, 16, 16, 3, 3, 2, 2, 1, 1, 0).desc()
    dp.a.stride[4] = 2                               # a dilated pooling window: none of the pooling kernels, ...
    gp = mb.merit_plan_create(dp)                    # ... but still a ranged maximum: the definition kernel
    assert gp.launch_info()["kernel"] == "merit_generic<max>" and gp.out_shape() == (1, 1, 8, 8)
    dp.dtype = mb.MERIT_F16
    with pytest.raises(mb.MeritError) as e:
        mb.merit_plan_create(dp)
    assert e.value.status == mb.MERIT_ERR_UNSUPPORTED
    d.range[2] = 17                                  # output extent that the input cannot supply
    with pytest.raises(mb.MeritError) as e:
        mb.merit_plan_create(d)
    assert e.value.status == mb.MERIT_ERR_SHAPE
    d.range[2] = 16
    d.pad = mb.MERIT_PAD_EXCLUDE                     # wrong padding rule for a dot product
    with pytest.raises(mb.MeritError) as e:
        mb.merit_plan_create(d)
    assert e.value.status == mb.MERIT_ERR_UNSUPPORTED


def test_null_and_misuse_without_gpu():
    L = mb.lib()
    assert L.merit_plan_destroy(None) == mb.MERIT_ERR_NULL
    plan = mb.merit_plan_pool2d(1, 1, 8, 8, 2, 2, 2, 2, 0, 0, 0)
    # wrong op for the entry point, NULL and misaligned pointers: all rejected before any launch
    assert L.merit_conv2d(plan.handle, 16, 16, 16, None) == mb.MERIT_ERR_INVALID_ARG
    assert L.merit_pool2d(plan.handle, None, 16, None) == mb.MERIT_ERR_NULL
    assert L.merit_pool2d(plan.handle, 16, 20, None) == mb.MERIT_ERR_ALIGNMENT
    # the entry points of the widened operations reject the same things in the same order
    import ctypes
    res = mb.merit_plan_conv2d_residual(1, 16, 8, 8, 32, 3, 3, 1, 1, 1, 1, 1)
    assert L.merit_conv2d(res.handle, 16, 16, 16, None) == mb.MERIT_ERR_INVALID_ARG        # needs the added tensor
    assert L.merit_conv2d_residual(res.handle, 16, 16, None, 16, None) == mb.MERIT_ERR_NULL
    assert L.merit_conv2d_residual(res.handle, 16, 16, 24, 16, None) == mb.MERIT_ERR_ALIGNMENT
    assert L.merit_conv2d_residual(plan.handle, 16, 16, 16, 16, None) == mb.MERIT_ERR_INVALID_ARG
    fused = mb.merit_plan_conv2d_pool(1, 3, 32, 32, 8, 3, 3, 1, 1, 1, 1, 1)
    assert L.merit_conv2d(fused.handle, 16, None, 16, None) == mb.MERIT_ERR_NULL
    sep = mb.merit_plan_sepfilter(1, 8, 8, 3)
    assert L.merit_sepfilter(sep.handle, 16, None, 4, 16, None) == mb.MERIT_ERR_NULL
    assert L.merit_sepfilter(sep.handle, 16, 6, 4, 16, None) == mb.MERIT_ERR_ALIGNMENT     # taps: 4-byte aligned
    assert L.merit_sepfilter(sep.handle, 24, 4, 4, 16, None) == mb.MERIT_ERR_ALIGNMENT     # image: 16-byte aligned
    assert L.merit_sepfilter(plan.handle, 16, 4, 4, 16, None) == mb.MERIT_ERR_INVALID_ARG
    bil = mb.merit_plan_bilateral(1, 8, 8, 3)
    norm = ctypes.c_double(-0.01)
    assert L.merit_bilateral(bil.handle, 16, 4, None, norm, 16, None) == mb.MERIT_ERR_NULL
    assert L.merit_bilateral(bil.handle, 16, 4, 4, ctypes.c_double(float("nan")), 16, None) == mb.MERIT_ERR_INVALID_ARG
    assert L.merit_bilateral(sep.handle, 16, 4, 4, norm, 16, None) == mb.MERIT_ERR_INVALID_ARG
    dw = mb.merit_plan_conv2d_depthwise(1, 4, 8, 8, 3, 3, 1, 1, 1, 1)
    assert L.merit_conv2d_depthwise(dw.handle, 16, 16, None, None) == mb.MERIT_ERR_NULL
    # an empty batch is a no-op, whatever the pointers
    assert L.merit_sepfilter(mb.merit_plan_sepfilter(0, 8, 8, 3).handle, None, None, None, None, None) == mb.MERIT_OK
    assert L.merit_bilateral(mb.merit_plan_bilateral(0, 8, 8, 3).handle, None, None, None, norm, None, None) == mb.MERIT_OK


def test_conv_variant_selection():
    assert mb.merit_plan_conv2d(32, 3, 224, 224, 64, 7, 7, 2, 2, 3, 3).launch_info()["kernel"].startswith("merit_conv2d_planar")
    # the 3x3 workload: the wave-specialised kernel on 128-pixel tiles (200 workgroups), 32 channels per pass
    li = mb.merit_plan_conv2d(8, 64, 56, 56, 64, 3, 3, 1, 1, 1, 1).launch_info()
    assert li["kernel"] == "merit_conv2d_chws" and li["grid"][0] == 200 and li["block"][0] == 512
    assert li["lds_bytes"] <= 160 * 1024
    # fewer than 32 input channels, or fewer than 64 output channels: the single-pass channel-block kernel
    assert mb.merit_plan_conv2d(8, 16, 56, 56, 64, 3, 3, 1, 1, 1, 1).launch_info()["kernel"] == "merit_conv2d_chblock"
    assert mb.merit_plan_conv2d(8, 64, 56, 56, 32, 3, 3, 1, 1, 1, 1).launch_info()["kernel"] == "merit_conv2d_chblock"


def test_plans_for_extreme_shapes_are_sane_or_refused():
    """Planning is host arithmetic only: very large or degenerate shapes must come back as a plan
    whose launch fits the chip (grid > 0, LDS <= 160 KB) or as a clean refusal, never anything else."""
    def ok(make, *a):
        try:
            plan = make(*a)
        except mb.MeritError as e:
            assert e.status in (mb.MERIT_ERR_UNSUPPORTED, mb.MERIT_ERR_SHAPE, mb.MERIT_ERR_INVALID_ARG), (a, e.status)
            return None
        li = plan.launch_info()
        assert 0 <= li["lds_bytes"] <= 160 * 1024, (a, li)
        assert all(g >= 0 for g in li["grid"]) and li["block"][0] in (256, 512), (a, li)
        n_out = 1
        for e in plan.out_shape():
            n_out *= e
        assert (n_out == 0) == (li["grid"][0] == 0) or li["grid"][0] > 0, (a, li)
        return plan
    for a in [(1 << 16, 3, 224, 224, 64, 7, 7, 2, 2, 3, 3),         # 4 GiB of input: no 32-bit buffer offsets
              (1, 3, 4096, 4096, 64, 7, 7, 2, 2, 3, 3),             # very wide rows
              (1, 4096, 8, 8, 4096, 3, 3, 1, 1, 1, 1),              # many channels, tiny image
              (1, 64, 1024, 1024, 64, 3, 3, 1, 1, 1, 1),            # staged rows beyond LDS?
              (0, 3, 32, 32, 8, 3, 3, 1, 1, 1, 1),                  # empty batch
              (2, 5, 7, 9, 3, 7, 9, 3, 2, 3, 4)]:                   # window as large as the padded image
        ok(mb.merit_plan_conv2d, *a)
        ok(mb.merit_plan_conv2d_relu, *a)
        ok(lambda *b: mb.merit_plan_conv2d_residual(*b, 1), *a)
        ok(lambda *b: mb.merit_plan_conv2d_pool(*b, 1), *a)
    for a in [(1 << 14, 256, 112, 112, 3, 3, 2, 2, 1, 1, 0), (1, 1, 1, 1, 3, 3, 2, 2, 1, 1, 1),
              (4, 4, 8192, 8192, 2, 2, 2, 2, 0, 0, 0), (0, 8, 16, 16, 3, 3, 2, 2, 1, 1, 0)]:
        ok(mb.merit_plan_pool2d, *a)
    for a in [(4320, 7680, 16, 32), (16, 16, 16, 63), (17, 33, 32, 0), (8, 8, 8, 64), (1, 1, 4, 1)]:
        ok(mb.merit_plan_sad, *a)
    for a in [(1 << 12, 1080, 1920, 3), (1, 1, 1, 32), (1, 100000, 8, 5), (0, 64, 64, 9)]:
        ok(mb.merit_plan_sepfilter, *a)
        ok(mb.merit_plan_bilateral, *a)
    for a in [(64, 1024, 64, 64, 15, 8), (1, 1, 8, 8, 0, 1), (1, 256, 64, 60, 5, 2)]:
        ok(mb.merit_plan_correlation, *a)
    for a in [(1 << 10, 1024, 112, 112, 3, 3, 1, 1, 1, 1), (1, 1, 3, 8192, 5, 5, 2, 2, 2, 2)]:
        ok(mb.merit_plan_conv2d_depthwise, *a)


def test_conv_plans_for_layers_that_do_not_fit_lds_at_once():
    """Channel passes for many-channel layers; the one-element-per-thread kernel when a wide
    window on few channels fits neither MFMA layout; the tile request and the fused pooling
    stay with the MFMA kernels."""
    for shape, kernel in (((1, 512, 14, 14, 512, 3, 3, 1, 1, 1, 1), "merit_conv2d_chws"),
                          ((1, 96, 27, 27, 256, 5, 5, 1, 1, 2, 2), "merit_conv2d_chws"),        # 5x5 window on a multiple of 8 channels
                              ((1, 100, 27, 27, 256, 5, 5, 1, 1, 2, 2), "merit_conv2d_chpass"),     # 5x5, Cin % 8 != 0
                              ((1, 96, 27, 27, 256, 7, 7, 1, 1, 3, 3), "merit_conv2d_chpass"),      # 7x7 window on many channels
                          ((1, 512, 7, 7, 512, 3, 3, 1, 1, 1, 1), "merit_conv2d_chws"),         # 49 pixels on a 128-pixel tile: still the faster kernel
                          ((1, 300, 56, 56, 64, 3, 3, 1, 1, 1, 1), "merit_conv2d_chpass"),      # Cin % 8 != 0
                          ((1, 64, 224, 224, 64, 3, 3, 1, 1, 1, 1), "merit_conv2d_chws"),
                          ((8, 256, 56, 56, 256, 3, 3, 1, 1, 1, 1), "merit_conv2d_chws"),
                          ((8, 256, 56, 56, 64, 1, 1, 1, 1, 0, 0), "merit_conv2d_chws"),         # 1x1
                          ((8, 260, 56, 56, 64, 1, 1, 1, 1, 0, 0), "merit_conv2d_chpass")):       # 1x1, Cin % 8 != 0: larger passes
        li = mb.merit_plan_conv2d(*shape).launch_info()
        assert li["kernel"] == kernel and 0 < li["lds_bytes"] <= 160 * 1024, (shape, li)
        if kernel == "merit_conv2d_chws":
            # 4 moving wavefronts + 8 multiplying ones on 128-channel tiles, 4 on 64-channel tiles
            assert li["block"][0] == (768 if li["tile"][1] == 128 else 512), li
            assert li["grid"][0] <= 256 and li["grid"][1] == 1
    # the wave-specialised kernel on request: 8 wavefronts, 128 or 64 pixels per multiplying wavefront
    p = mb.merit_plan_conv2d(8, 64, 56, 56, 64, 3, 3, 1, 1, 1, 1)
    p.set_tile((0, 0, 8, 64))
    assert p.launch_info()["kernel"] == "merit_conv2d_chws" and p.launch_info()["tile"][1] == 64
    assert mb.merit_plan_packed_weights_bytes(p) == 64 * 64 * 9 * 2           # nothing padded here
    p = mb.merit_plan_conv2d(8, 256, 56, 56, 256, 3, 3, 1, 1, 1, 1)
    assert p.launch_info()["tile"][1] == 128 and mb.merit_plan_packed_weights_bytes(p) == 256 * 256 * 9 * 2
    with pytest.raises(mb.MeritError):                                          # 5x5: no such instance
        mb.merit_plan_conv2d(1, 96, 27, 27, 256, 5, 5, 1, 1, 2, 2).set_tile((0, 0, 8, 128))
    with pytest.raises(mb.MeritError):                                          # packed weights: only that kernel
        mb.merit_plan_packed_weights_bytes(mb.merit_plan_conv2d(1, 3, 32, 32, 16, 7, 7, 2, 2, 3, 3))
    alex1 = (1, 3, 227, 227, 96, 11, 11, 4, 4, 0, 0)
    p = mb.merit_plan_conv2d(*alex1)
    li = p.launch_info()
    # 11 taps per window row: two 8-slot fragments per row in the few-channel MFMA kernel
    assert li["kernel"] == "merit_conv2d_planar" and p.out_shape() == (1, 96, 55, 55)
    p.set_tile((0, 0, 4, 32))
    assert p.launch_info()["kernel"] == "merit_conv2d_planar"
    # 17 taps: neither MFMA layout holds the window
    p = mb.merit_plan_conv2d(1, 3, 227, 227, 96, 11, 17, 4, 4, 0, 0)
    li = p.launch_info()
    assert li["kernel"] == "merit_conv2d_direct" and li["lds_bytes"] == 32 * 1024
    assert p.out_shape() == (1, 96, 55, 53) and li["grid"][:2] == (12 * -(-55 * 53 // 256), 1)   # 8 channels x 256 pixels
    with pytest.raises(mb.MeritError):
        p.set_tile((0, 0, 4, 32))
    with pytest.raises(mb.MeritError):
        mb.merit_plan_conv2d_pool(1, 3, 224, 224, 64, 11, 11, 2, 2, 5, 5)


def test_pool_plan_one_output_per_plane():
    li = mb.merit_plan_pool2d(32, 512, 7, 7, 7, 7, 1, 1, 0, 0, 1).launch_info()
    # 49 elements per plane: 16 lanes each, four planes per wavefront, sixteen per workgroup
    assert li["kernel"] == "merit_pool2d_plane<avg>" and li["grid"][0] == 32 * 512 // 16 and li["lds_bytes"] == 0
    assert mb.merit_plan_pool2d(2, 10, 40, 40, 40, 40, 1, 1, 0, 0, 0).launch_info()["grid"][0] == 5     # 1600 elements: a wavefront per plane
    p = mb.merit_plan_pool2d(1, 3, 5, 6, 7, 8, 1, 1, 1, 1, 0)
    assert p.out_shape() == (1, 3, 1, 1) and p.launch_info()["kernel"] == "merit_pool2d_plane<max>"
    p.set_tile((0, 0, 1, 1))                               # a tile request names the generic kernel
    assert p.launch_info()["kernel"] == "merit_pool2d_tile<max>"


def test_pool_plan_lane_per_column_for_odd_widths():
    li = mb.merit_plan_pool2d(32, 96, 55, 55, 3, 3, 2, 2, 0, 0, 0).launch_info()
    assert li["kernel"] == "merit_pool2d_lanes2_s2<max,3>" and li["lds_bytes"] == 0    # two output columns per lane
    assert li["grid"][0] == -(-(32 * 96 * 7) // 16)         # 7 strips of 4 rows, 27 columns on 16 lanes: four items per wavefront
    li = mb.merit_plan_pool2d(2, 3, 27, 27, 3, 3, 2, 2, 0, 0, 1).launch_info()         # 13 columns on 8 lanes: eight items per wavefront
    assert li["kernel"] == "merit_pool2d_lanes2_s2<avg,3>" and li["grid"][0] == -(-(2 * 3 * 4) // 32)
    li = mb.merit_plan_pool2d(2, 3, 9, 7, 3, 3, 2, 2, 1, 1, 1).launch_info()           # narrower than 8: a lane per column
    assert li["kernel"] == "merit_pool2d_lanes_k3s2<avg>"
    li = mb.merit_plan_pool2d(2, 3, 40, 301, 3, 3, 2, 2, 0, 0, 0).launch_info()        # 150 output columns: two chunks of 128
    assert li["kernel"] == "merit_pool2d_lanes2_s2<max,3>" and li["grid"][0] == -(-(2 * 3 * 2 * 5) // 4)
    # 3x3 / stride 1 on widths the row kernel does not take (the pooling branch of an inception module)
    li = mb.merit_plan_pool2d(32, 288, 35, 35, 3, 3, 1, 1, 1, 1, 1).launch_info()
    assert li["kernel"] == "merit_pool2d_lanes2_s2<avg,3,1>" and li["grid"][0] == -(-(32 * 288 * 5) // 8)   # 5 strips of 8 rows, 32 lanes each
    assert mb.merit_plan_pool2d(32, 192, 28, 28, 3, 3, 1, 1, 1, 1, 0).launch_info()["kernel"] == "merit_pool2d_lanes2_s2<max,3,1>"
    assert mb.merit_plan_pool2d(32, 192, 28, 28, 3, 3, 1, 1, 1, 1, 0).set_tile((0, 0, 7)).launch_info()["kernel"].startswith("merit_pool2d_rows<3,3,1,1,1")
    # 2x2 / stride 2 where the output rows are not whole 16-byte vectors (28 -> 14, 14 -> 7)
    li = mb.merit_plan_pool2d(8, 512, 28, 28, 2, 2, 2, 2, 0, 0, 0).launch_info()
    assert li["kernel"] == "merit_pool2d_lanes2_s2<max,2>" and li["grid"][0] == -(-(8 * 512 * 4) // 32)
    assert mb.merit_plan_pool2d(8, 64, 224, 224, 2, 2, 2, 2, 0, 0, 0).launch_info()["kernel"].startswith("merit_pool2d_rows")
    # the 16-byte kernels keep the shapes they take
    assert mb.merit_plan_pool2d(16, 64, 112, 112, 3, 3, 2, 2, 1, 1, 0).launch_info()["kernel"].startswith("merit_pool2d_stream")
