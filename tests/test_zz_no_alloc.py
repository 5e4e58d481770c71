"""The entry point that allocates nothing (merit_conv2d_packed_noalloc) against the existing
pair merit_conv2d_pack_weights + merit_conv2d_packed, through the C ABI: same bits, on two calls
in a row, the second with a smaller input (the library's one scratch buffer keeps the first
call's contents).  Needs a real MI355X."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def mb():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_1911_03458_amd import binding
    binding.lib()
    return binding


def _one(mb, shape, seed):
    N, Cin, H, W, Cout = shape
    g = torch.Generator(device="cpu").manual_seed(seed)
    x = torch.randn((N, Cin, H, W), generator=g).to(torch.float16).to("cuda:0")
    w = (torch.randn((Cout, Cin, 3, 3), generator=g) / (Cin * 9) ** 0.5).to(torch.float16).to("cuda:0")
    plan = mb.merit_plan_conv2d(N, Cin, H, W, Cout, 3, 3, 1, 1, 1, 1)
    if plan.launch_info()["kernel"] != "merit_conv2d_chws":
        plan.set_tile((0, 0, 8, 64))
    assert plan.launch_info()["kernel"] == "merit_conv2d_chws"
    # the existing entry points: the caller brings the packed buffer
    packed = mb.merit_conv2d_pack_weights(plan, w)
    ref = mb.merit_conv2d_packed(plan, x, packed)
    # the new one: outputs preallocated here, nothing allocated inside
    y = torch.full(plan.out_shape(), 7.0, dtype=torch.float16, device="cuda:0")
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    mb.merit_conv2d_packed_noalloc(plan, x, w, y)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    assert torch.equal(y, ref), shape
    # and against the caller's-weights entry point as well
    assert torch.equal(mb.merit_conv2d(plan, x, w), y)
    return plan


def test_two_calls_in_a_row_the_second_smaller(mb):
    _one(mb, (2, 256, 28, 56, 256), 1)       # 1.18 MB of packed weights
    _one(mb, (1, 64, 20, 24, 64), 2)         # 74 KB: the rest of the buffer still holds the first call's
    _one(mb, (2, 256, 28, 56, 256), 3)       # and back, with other weights


def test_a_plan_beyond_the_scratch_limit_is_refused(mb):
    plan = mb.merit_plan_conv2d(1, 1024, 16, 16, 1024, 3, 3, 1, 1, 1, 1)     # 18.9 MB of packed weights
    assert plan.launch_info()["kernel"] == "merit_conv2d_chws"
    assert mb.merit_plan_packed_weights_bytes(plan) > mb.MERIT_NOALLOC_SCRATCH_BYTES
    x = torch.zeros((1, 1024, 16, 16), dtype=torch.float16, device="cuda:0")
    w = torch.zeros((1024, 1024, 3, 3), dtype=torch.float16, device="cuda:0")
    y = torch.full(plan.out_shape(), 3.0, dtype=torch.float16, device="cuda:0")
    with pytest.raises(mb.MeritError) as e:
        mb.merit_conv2d_packed_noalloc(plan, x, w, y)
    assert e.value.status == mb.MERIT_ERR_SCRATCH_LIMIT
    torch.cuda.synchronize()
    assert bool((y == 3.0).all())             # nothing was launched
    other = mb.merit_plan_conv2d(1, 3, 32, 32, 16, 7, 7, 2, 2, 3, 3)          # a kernel without packed weights
    with pytest.raises(mb.MeritError) as e:
        mb.merit_conv2d_packed_noalloc(other, torch.zeros((1, 3, 32, 32), dtype=torch.float16, device="cuda:0"),
                                       torch.zeros((16, 3, 7, 7), dtype=torch.float16, device="cuda:0"),
                                       torch.zeros(other.out_shape(), dtype=torch.float16, device="cuda:0"))
    assert e.value.status == mb.MERIT_ERR_UNSUPPORTED
