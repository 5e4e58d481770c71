"""The definition kernel (`merit_generic<...>`): descriptors no specialised kernel recognises.

Expected values come from the oracle's literal evaluator of Section III-C, Eq. 5
(`oracle.merit_literal.transform`: materialise M(A), M(B), reduce the rows) and, where the
operation has one, from a closed form that owes nothing to either (a matrix product against
numpy's, a true convolution against scipy's, the C oracle's correlation and depthwise loops).
"""
import ctypes

import numpy as np
import pytest

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

from oracle import merit_literal as lit   # noqa: E402
import oracle                              # noqa: E402

U = lit.UNUSED
PADS = {"zero": 0, "ninf": 1, "exclude": 2, "clamp": 3}


@pytest.fixture(scope="module")
def mb():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_1911_03458_amd import binding
    return binding


def make_desc(mb, op, dtype, pad, ranges, n_par, ta, shape_a, tb=None, shape_b=None):
    d = mb.merit_plan_desc()
    d.op, d.dtype, d.pad = op, dtype, PADS[pad]
    d.n_par, d.n_acc = n_par, len(ranges) - n_par
    for j, r in enumerate(ranges):
        d.range[j] = r
    for opnd, t, shape in ((d.a, ta, shape_a), (d.b, tb, shape_b)):
        if t is None:
            opnd.ndim = 0
            continue
        opnd.ndim = len(shape)
        for i, s in enumerate(shape):
            opnd.shape[i] = s
        for j in range(len(ranges)):
            opnd.axis[j], opnd.stride[j], opnd.offset[j] = t.axis[j], t.stride[j], t.offset[j]
    return d


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0")


def literal_dot(A, B, ranges, n_par, ta, tb, pad, relu=False):
    MA, _ = lit.transform(A.astype(np.float64), ranges, ta, n_par, pad)
    MB, _ = lit.transform(B.astype(np.float64), ranges, tb, n_par, pad)
    rows = np.einsum("pa,pa->p", MA, MB)
    if relu:
        rows = np.maximum(rows, 0.0)
    return rows.reshape(ranges[:n_par])


def check_dot(got, ref):
    got = got.astype(np.float64)
    assert got.shape == ref.shape
    assert np.all(np.abs(got - ref) <= 2e-2 * np.abs(ref) + 1e-3), np.max(np.abs(got - ref))


def test_matrix_product_as_a_transform(mb):
    """C[i,j] = sum_k A[i,k] B[k,j]: k = (i, j | k); A moves along (i, k), B along (k, j)."""
    rng = np.random.default_rng(1)
    M, N, K = 37, 50, 129
    A = rng.standard_normal((M, K)).astype(np.float16)
    B = rng.standard_normal((K, N)).astype(np.float16)
    ta = lit.Transform((0, U, 1), (1, 0, 1), (0, 0, 0))
    tb = lit.Transform((U, 1, 0), (0, 1, 1), (0, 0, 0))
    d = make_desc(mb, mb.MERIT_OP_CONV_DOT, mb.MERIT_F16, "zero", (M, N, K), 2, ta, A.shape, tb, B.shape)
    plan = mb.merit_plan_create(d)
    assert plan.launch_info()["kernel"] == "merit_generic<dot>" and plan.out_shape() == (M, N)
    y = mb.merit_conv2d(plan, dev(A), dev(B)).cpu().numpy()
    check_dot(y, A.astype(np.float64) @ B.astype(np.float64))                       # the closed form
    check_dot(y, literal_dot(A, B, (M, N, K), 2, ta, tb, "zero"))                   # and Eq. 5 literally


def test_true_convolution_flips_the_kernel(mb):
    """A stride of -1 on the window indices of the weights: convolution in the textbook sense
    (scipy.signal.convolve2d), which the specialised kernels (correlation-style, Eq. 6) are not."""
    scipy_signal = pytest.importorskip("scipy.signal")
    rng = np.random.default_rng(2)
    H, W, k = 19, 23, 5
    x = rng.standard_normal((H, W)).astype(np.float16)
    w = rng.standard_normal((k, k)).astype(np.float16)
    c = k // 2
    # k = (oy, ox | ky, kx): x[oy + ky - c, ox + kx - c] * w[k-1-ky, k-1-kx]
    ta = lit.Transform((0, 1, 0, 1), (1, 1, 1, 1), (0, 0, -c, -c))
    tb = lit.Transform((U, U, 0, 1), (0, 0, -1, -1), (0, 0, k - 1, k - 1))
    ranges = (H, W, k, k)
    d = make_desc(mb, mb.MERIT_OP_CONV_DOT, mb.MERIT_F16, "zero", ranges, 2, ta, x.shape, tb, w.shape)
    plan = mb.merit_plan_create(d)
    assert plan.launch_info()["kernel"] == "merit_generic<dot>"
    y = mb.merit_conv2d(plan, dev(x), dev(w)).cpu().numpy()
    check_dot(y, scipy_signal.convolve2d(x.astype(np.float64), w.astype(np.float64), mode="same"))
    check_dot(y, literal_dot(x, w, ranges, 2, ta, tb, "zero"))


@pytest.mark.parametrize("pad", ["zero", "clamp"])
def test_3d_convolution_with_clipping(mb, pad):
    """k = (n, co, oz, oy, ox | ci, kz, ky, kx): five parallel and four accumulation indices, a
    window over three axes, strides 2/1/2, the clipped product function; both padding rules."""
    rng = np.random.default_rng(3)
    N, Ci, D, H, W, Co, kz, ky, kx = 2, 3, 6, 7, 9, 4, 3, 2, 3
    sz, sy, sx, pz, py, px = 2, 1, 2, 1, 0, 1
    OD, OH, OW = (D + 2 * pz - kz) // sz + 1, (H + 2 * py - ky) // sy + 1, (W + 2 * px - kx) // sx + 1
    x = rng.standard_normal((N, Ci, D, H, W)).astype(np.float16)
    w = (rng.standard_normal((Co, Ci, kz, ky, kx)) / 7).astype(np.float16)
    ranges = (N, Co, OD, OH, OW, Ci, kz, ky, kx)
    ta = lit.Transform((0, U, 2, 3, 4, 1, 2, 3, 4), (1, 0, sz, sy, sx, 1, 1, 1, 1), (0, 0, -pz, -py, -px, 0, 0, 0, 0))
    tb = lit.Transform((U, 0, U, U, U, 1, 2, 3, 4), (0, 1, 0, 0, 0, 1, 1, 1, 1), (0,) * 9)
    d = make_desc(mb, mb.MERIT_OP_CONV_DOT_RELU, mb.MERIT_F16, pad, ranges, 5, ta, x.shape, tb, w.shape)
    plan = mb.merit_plan_create(d)
    assert plan.launch_info()["kernel"] == "merit_generic<dot>" and plan.out_shape() == ranges[:5]
    y = mb.merit_conv2d(plan, dev(x), dev(w)).cpu().numpy()
    assert not np.signbit(y).any()
    check_dot(y, literal_dot(x, w, ranges, 5, ta, tb, pad, relu=True))


@pytest.mark.parametrize("mode,pad", [("max", "ninf"), ("max", "clamp"), ("avg", "exclude"), ("avg", "zero"), ("avg", "clamp")])
def test_dilated_pooling_window(mb, mode, pad):
    """3x3 window with stride 2 on the window indices (a dilated window), stride 2, padding 2."""
    rng = np.random.default_rng(4)
    N, C, H, W = 2, 3, 17, 22
    x = rng.standard_normal((N, C, H, W)).astype(np.float32)
    k, s, p, dil = 3, 2, 2, 2
    e = (k - 1) * dil + 1
    OH, OW = (H + 2 * p - e) // s + 1, (W + 2 * p - e) // s + 1
    ranges = (N, C, OH, OW, k, k)
    ta = lit.Transform((0, 1, 2, 3, 2, 3), (1, 1, s, s, dil, dil), (0, 0, -p, -p, 0, 0))
    op = mb.MERIT_OP_POOL_MAX if mode == "max" else mb.MERIT_OP_POOL_AVG
    d = make_desc(mb, op, mb.MERIT_F32, pad, ranges, 4, ta, x.shape)
    plan = mb.merit_plan_create(d)
    assert plan.launch_info()["kernel"] == ("merit_generic<max>" if mode == "max" else "merit_generic<mean>")
    y = mb.merit_pool2d(plan, dev(x)).cpu().numpy().astype(np.float64)
    M, inside = lit.transform(x.astype(np.float64), ranges, ta, 4, pad)
    if mode == "max":
        ref = M.max(axis=1)
    elif pad == "exclude":
        cnt = inside.sum(axis=1)
        ref = np.where(cnt > 0, M.sum(axis=1) / np.maximum(cnt, 1), 0.0)
    else:
        ref = M.mean(axis=1)
    ref = ref.reshape(ranges[:4])
    assert y.shape == ref.shape
    if mode == "max":
        assert np.array_equal(y, ref.astype(np.float32).astype(np.float64))
    else:
        assert np.all(np.abs(y - ref) <= 1e-5 * np.abs(ref) + 1e-6)


def test_undilated_window_matches_the_specialised_pooling(mb):
    """The same descriptor with stride 1 on the window indices is the pooling kernels' pattern:
    both paths give the same tensor (and the C oracle's)."""
    rng = np.random.default_rng(5)
    x = rng.standard_normal((1, 2, 12, 16)).astype(np.float32)
    plan = mb.merit_plan_pool2d(1, 2, 12, 16, 3, 3, 2, 2, 1, 1, 0)
    assert not plan.launch_info()["kernel"].startswith("merit_generic")
    d = plan.desc()
    d.pad = PADS["clamp"]                          # a rule the pooling kernels do not have
    g = mb.merit_plan_create(d)
    assert g.launch_info()["kernel"] == "merit_generic<max>"
    y_fast = mb.merit_pool2d(plan, dev(x)).cpu().numpy()
    assert np.array_equal(y_fast, oracle.pool2d(x, (3, 3), (2, 2), (1, 1), "max"))
    # with border replication the padded elements repeat values of the window's own rows and
    # columns here (padding 1, window 3: the replicated pixel is inside the window): same maxima
    assert np.array_equal(mb.merit_pool2d(g, dev(x)).cpu().numpy(), y_fast)


@pytest.mark.parametrize("shape", [(1, 8, 16, 20, 2, 1), (2, 5, 9, 13, 3, 2), (1, 24, 10, 12, 20, 1)])
def test_correlation_shapes_the_mfma_kernel_does_not_take(mb, shape):
    """Widths that are not a multiple of 8, a search range above 15: Eq. 8 on the definition kernel,
    against the C oracle's loops."""
    N, C, H, W, R, sd = shape
    rng = np.random.default_rng(6)
    x1 = rng.standard_normal((N, C, H, W)).astype(np.float16)
    x2 = rng.standard_normal((N, C, H, W)).astype(np.float16)
    plan = mb.merit_plan_correlation(N, C, H, W, R, sd)
    assert plan.launch_info()["kernel"] == "merit_generic<dot>"
    y = mb.merit_correlation(plan, dev(x1), dev(x2)).cpu().numpy()
    check_dot(y, oracle.correlation(x1, x2, R, sd).astype(np.float64))


def test_depthwise_and_plain_convolution_on_request_shapes(mb):
    """A depthwise layer and a convolution with border replication, against the C oracle where it
    has the operation and the literal evaluator where it has not."""
    rng = np.random.default_rng(7)
    x = rng.standard_normal((2, 6, 11, 14)).astype(np.float16)
    w = (rng.standard_normal((8, 6, 3, 3)) / 7).astype(np.float16)
    d = mb.merit_plan_conv2d(2, 6, 11, 14, 8, 3, 3, 1, 1, 1, 1).desc()
    d.pad = PADS["clamp"]
    plan = mb.merit_plan_create(d)
    assert plan.launch_info()["kernel"] == "merit_generic<dot>"
    y = mb.merit_conv2d(plan, dev(x), dev(w)).cpu().numpy()
    ranges, n_par, tx, tw = lit.conv2d_desc(2, 6, 11, 14, 8, 3, 3, 1, 1, 1, 1)
    check_dot(y, literal_dot(x, w, ranges, n_par, tx, tw, "clamp"))
    # interior outputs do not see the border: there both rules agree with the C oracle
    ref = oracle.conv2d(x, w, (1, 1), (1, 1)).astype(np.float64)
    check_dot(y[:, :, 1:-1, 1:-1], ref[:, :, 1:-1, 1:-1])


def test_empty_and_misuse(mb):
    ta = lit.Transform((0, U, 1), (1, 0, 1), (0, 0, 0))
    tb = lit.Transform((U, 1, 0), (0, 1, 1), (0, 0, 0))
    d = make_desc(mb, mb.MERIT_OP_CONV_DOT, mb.MERIT_F16, "zero", (0, 5, 7), 2, ta, (1, 7), tb, (7, 5))
    plan = mb.merit_plan_create(d)                  # an empty parallel range: a no-op, whatever the pointers
    assert plan.out_shape() == (0, 5)
    L = mb.lib()
    assert L.merit_conv2d(plan.handle, None, None, None, None) == mb.MERIT_OK
    d.range[0] = 3
    d.a.shape[0] = 3
    plan = mb.merit_plan_create(d)
    assert L.merit_conv2d(plan.handle, None, 16, 16, None) == mb.MERIT_ERR_NULL
    assert L.merit_conv2d(plan.handle, 16, 24, 16, None) == mb.MERIT_ERR_ALIGNMENT
    assert L.merit_pool2d(plan.handle, 16, 16, None) == mb.MERIT_ERR_INVALID_ARG      # a dot product, not a pooling plan
    d.range[2] = 0                                  # an empty reduction has no value
    with pytest.raises(mb.MeritError) as e:
        mb.merit_plan_create(d)
    assert e.value.status == mb.MERIT_ERR_INVALID_ARG


@pytest.mark.parametrize("seed", [35, 81])
def test_random_descriptors(mb, seed):
    """Descriptors nobody designed: 1-4 parallel and 1-3 accumulation indices, each moving along
    any axis of a 1- to 4-axis operand (or none) with a stride in -2..3 and an offset in -3..3,
    several indices on one axis, every padding rule each product function has.  Expected values
    are Eq. 5 taken literally (M(A), M(B) materialised, rows reduced); whichever kernel the plan
    chose must agree with it."""
    rng = np.random.default_rng(seed)

    def ri(a, b):
        return int(rng.integers(a, b + 1))

    def operand(J):
        shape = tuple(ri(1, 7) for _ in range(ri(1, 4)))
        axis = tuple(ri(-1, len(shape) - 1) for _ in range(J))
        return shape, lit.Transform(axis, tuple(ri(-2, 3) for _ in range(J)), tuple(ri(-3, 3) for _ in range(J)))

    kernels = set()
    for it in range(60):
        n_par, n_acc = ri(1, 4), ri(1, 3)
        J = n_par + n_acc
        ranges = tuple(ri(1, 5) for _ in range(J))
        mode = str(rng.choice(["dot", "dot_relu", "max", "avg"]))
        sa, ta = operand(J)
        if mode in ("dot", "dot_relu"):
            pad = str(rng.choice(["zero", "clamp"]))
            sb, tb = operand(J)
            A = rng.standard_normal(sa).astype(np.float16)
            B = (rng.standard_normal(sb) / 4).astype(np.float16)
            op = mb.MERIT_OP_CONV_DOT_RELU if mode == "dot_relu" else mb.MERIT_OP_CONV_DOT
            d = make_desc(mb, op, mb.MERIT_F16, pad, ranges, n_par, ta, sa, tb, sb)
            print(it, mode, pad, ranges, n_par, sa, ta, sb, tb, flush=True)
            plan = mb.merit_plan_create(d)
            kernels.add(plan.launch_info()["kernel"])
            assert plan.out_shape() == ranges[:n_par]
            y = mb.merit_conv2d(plan, dev(A), dev(B)).cpu().numpy()
            check_dot(y, literal_dot(A, B, ranges, n_par, ta, tb, pad, relu=(mode == "dot_relu")))
        else:
            pad = str(rng.choice(["ninf", "clamp", "zero"] if mode == "max" else ["exclude", "zero", "clamp"]))
            A = rng.standard_normal(sa).astype(np.float32)
            op = mb.MERIT_OP_POOL_MAX if mode == "max" else mb.MERIT_OP_POOL_AVG
            d = make_desc(mb, op, mb.MERIT_F32, pad, ranges, n_par, ta, sa)
            print(it, mode, pad, ranges, n_par, sa, ta, flush=True)
            plan = mb.merit_plan_create(d)
            kernels.add(plan.launch_info()["kernel"])
            y = mb.merit_pool2d(plan, dev(A)).cpu().numpy().astype(np.float64)
            M, inside = lit.transform(A.astype(np.float64), ranges, ta, n_par, pad)
            if mode == "max":
                ref = M.max(axis=1).reshape(ranges[:n_par])
                assert np.array_equal(y, ref)
            else:
                if pad == "exclude":
                    cnt = inside.sum(axis=1)
                    ref = np.where(cnt > 0, M.sum(axis=1) / np.maximum(cnt, 1), 0.0)
                else:
                    ref = M.mean(axis=1)
                ref = ref.reshape(ranges[:n_par])
                assert y.shape == ref.shape and np.all(np.abs(y - ref) <= 1e-5 * np.abs(ref) + 1e-6)
    assert {"merit_generic<dot>", "merit_generic<max>", "merit_generic<mean>"} <= kernels, kernels
