"""Random valid shapes for every entry point, the HIP path against the oracle (seeded).

The hand-picked cases of test_gpu_parity.py name the paths they cover; this sweep draws
shapes the authors did not think of: any window, stride, padding, dilation, channel count and
ragged extent within the documented limits, every operation, the oracle's bar for each
(bit-exact for block matching and max pooling, the stated tolerances otherwise).  A plan the
library refuses is reported and skipped (none is expected for convolution and pooling)."""
import numpy as np
import pytest
import torch

import oracle
from paper_1911_03458_amd import binding as mb

pytestmark = pytest.mark.gpu


def _guard(shape, dtype):
    n = int(np.prod(shape)); pad = 64
    buf = torch.full((n + 2 * pad,), 777, dtype=dtype, device="cuda:0")
    return buf, buf[pad:pad + n].view(shape), pad


def _canary(buf, pad):
    b = buf.cpu()
    return bool((b[:pad] == 777).all() and (b[-pad:] == 777).all())


@pytest.mark.parametrize("seed", [1911, 3458])
def test_random_shapes(seed):
    ncase = 40
    rng = np.random.default_rng(seed)
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0")
    guard, canary = _guard, _canary
    failures = []

    def report(name, case, ok, extra=""):
        if not ok:
            failures.append((name, case, extra))

    def ri(a, b):
        return int(rng.integers(a, b + 1))

    for it in range(ncase):
        # ---- conv2d family
        N, Cin, H, W, Cout = ri(1, 3), ri(1, 40), ri(5, 40), ri(5, 40), ri(1, 70)
        if rng.random() < 0.35: Cin = ri(41, 300); N = 1
        if rng.random() < 0.15: W = ri(41, 200)
        kh, kw, sh, sw = ri(1, 7), ri(1, 7), ri(1, 3), ri(1, 3)
        if rng.random() < 0.15: kh, kw, sh, sw = ri(8, 12), ri(8, 12), ri(1, 4), ri(1, 4); H = max(H, kh); W = max(W, kw)
        ph, pw = ri(0, min(3, kh - 1) if kh > 1 else 0), ri(0, min(3, kw - 1) if kw > 1 else 0)
        dh, dw = (ri(1, 3), ri(1, 3)) if rng.random() < 0.3 else (1, 1)
        relu = int(rng.random() < 0.5); resid = rng.random() < 0.3 and dh == 1 and dw == 1
        if (H + 2 * ph - ((kh - 1) * dh + 1)) < 0 or (W + 2 * pw - ((kw - 1) * dw + 1)) < 0: continue
        case = ("conv", N, Cin, H, W, Cout, kh, kw, sh, sw, ph, pw, dh, dw, relu, resid)
        print(it, case, flush=True)
        x = rng.standard_normal((N, Cin, H, W)).astype(np.float16)
        w = (rng.standard_normal((Cout, Cin, kh, kw)) / np.sqrt(Cin * kh * kw)).astype(np.float16)
        try:
            if resid: plan = mb.merit_plan_conv2d_residual(N, Cin, H, W, Cout, kh, kw, sh, sw, ph, pw, relu)
            else: plan = mb.merit_plan_conv2d_dilated(N, Cin, H, W, Cout, kh, kw, sh, sw, ph, pw, dh, dw, relu)
        except Exception as e:
            print("   plan refused:", e, flush=True); plan = None
        if plan is not None:
            buf, y, pad = guard(plan.out_shape(), torch.float16)
            if resid:
                r = rng.standard_normal(plan.out_shape()).astype(np.float16)
                mb.merit_conv2d_residual(plan, dev(x), dev(w), dev(r), y)
                ref = oracle.conv2d_residual(x, w, r, (sh, sw), (ph, pw), bool(relu))
            else:
                mb.merit_conv2d(plan, dev(x), dev(w), y)
                ref = oracle.conv2d(x, w, (sh, sw), (ph, pw), bool(relu), (dh, dw))
            torch.cuda.synchronize()
            got = y.cpu().numpy().astype(np.float64); ref = ref.astype(np.float64)
            report("conv", case, canary(buf, pad) and np.all(np.abs(got - ref) <= 2e-2 * np.abs(ref) + 1e-3), plan.launch_info()["kernel"])
        # ---- pool2d
        N, C, H, W = ri(1, 3), ri(1, 9), ri(3, 50), ri(3, 50)
        kh, kw, sh, sw = ri(1, 5), ri(1, 5), ri(1, 3), ri(1, 3)
        ph, pw = ri(0, kh // 2), ri(0, kw // 2); avg = int(rng.random() < 0.5)
        if H + 2 * ph >= kh and W + 2 * pw >= kw:
            case = ("pool", N, C, H, W, kh, kw, sh, sw, ph, pw, avg); print(it, case, flush=True)
            x = rng.standard_normal((N, C, H, W)).astype(np.float32)
            try: plan = mb.merit_plan_pool2d(N, C, H, W, kh, kw, sh, sw, ph, pw, avg)
            except Exception as e: print("   plan refused:", e, flush=True); plan = None
            if plan is not None:
                buf, y, pad = guard(plan.out_shape(), torch.float32)
                mb.merit_pool2d(plan, dev(x), y); torch.cuda.synchronize()
                ref = oracle.pool2d(x, (kh, kw), (sh, sw), (ph, pw), "avg" if avg else "max")
                got = y.cpu().numpy()
                ok = np.all(np.abs(got - ref) <= 1e-5 * np.abs(ref) + 1e-6) if avg else np.array_equal(got, ref.astype(np.float32))
                report("pool", case, canary(buf, pad) and ok, plan.launch_info()["kernel"])
        # ---- sad
        B = int(rng.choice([4, 8, 16, 32])); R = ri(1, 20) if rng.random() < 0.7 else int(rng.choice([8, 16, 32]))
        H, W = ri(B, 130), ri(B, 160)
        if rng.random() < 0.6: W = (W + 3) // 4 * 4
        case = ("sad", H, W, B, R); print(it, case, flush=True)
        ref_f = rng.integers(0, 256, (H, W), dtype=np.uint8); cur_f = np.roll(ref_f, (ri(-3, 3), ri(-3, 3)), (0, 1)).copy()
        cur_f[rng.random((H, W)) < 0.05] = 7
        try: plan = mb.merit_plan_sad(H, W, B, R)
        except Exception as e: print("   plan refused:", e, flush=True); plan = None
        if plan is not None:
            sad, mv = mb.merit_sad_search(plan, dev(cur_f), dev(ref_f)); torch.cuda.synchronize()
            rs, rm = oracle.sad_search(cur_f, ref_f, B, R)
            report("sad", case, np.array_equal(sad.cpu().numpy(), rs) and np.array_equal(mv.cpu().numpy(), rm), plan.launch_info()["kernel"])
        # ---- correlation
        N, C, H, W, R, sd = ri(1, 2), ri(1, 80), ri(3, 20), 8 * ri(1, 17), ri(0, 15), ri(1, 8)
        case = ("corr", N, C, H, W, R, sd); print(it, case, flush=True)
        x1 = (rng.standard_normal((N, C, H, W)) / np.sqrt(C)).astype(np.float16); x2 = rng.standard_normal((N, C, H, W)).astype(np.float16)
        try: plan = mb.merit_plan_correlation(N, C, H, W, R, sd)
        except Exception as e: print("   plan refused:", e, flush=True); plan = None
        if plan is not None:
            buf, y, pad = guard(plan.out_shape(), torch.float16)
            mb.merit_correlation(plan, dev(x1), dev(x2), y); torch.cuda.synchronize()
            got = y.cpu().numpy().astype(np.float64); ref = oracle.correlation(x1, x2, R, sd).astype(np.float64)
            report("corr", case, canary(buf, pad) and np.all(np.abs(got - ref) <= 2e-2 * np.abs(ref) + 1e-3), str(plan.launch_info()))
        # ---- depthwise
        N, C, H, W = ri(1, 3), ri(1, 20), ri(3, 40), ri(3, 72)
        kh, kw, sh, sw = ri(1, 5), ri(1, 5), ri(1, 2), ri(1, 2); ph, pw = ri(0, kh // 2), ri(0, kw // 2)
        if rng.random() < 0.4: kh = kw = 3; sh = sw = 1; ph = pw = 1; W = 8 * ri(1, 9)
        if H + 2 * ph >= kh and W + 2 * pw >= kw:
            case = ("dw", N, C, H, W, kh, kw, sh, sw, ph, pw); print(it, case, flush=True)
            x = rng.standard_normal((N, C, H, W)).astype(np.float16); w = (rng.standard_normal((C, kh, kw)) / 3).astype(np.float16)
            try: plan = mb.merit_plan_conv2d_depthwise(N, C, H, W, kh, kw, sh, sw, ph, pw)
            except Exception as e: print("   plan refused:", e, flush=True); plan = None
            if plan is not None:
                buf, y, pad = guard(plan.out_shape(), torch.float16)
                mb.merit_conv2d_depthwise(plan, dev(x), dev(w), y); torch.cuda.synchronize()
                got = y.cpu().numpy().astype(np.float64); ref = oracle.conv2d_depthwise(x, w, (sh, sw), (ph, pw)).astype(np.float64)
                report("dw", case, canary(buf, pad) and np.all(np.abs(got - ref) <= 2e-2 * np.abs(ref) + 1e-3), plan.launch_info()["kernel"])
        # ---- separable filter
        N, H, W, k = ri(1, 2), ri(1, 150), ri(1, 200), ri(1, 32)
        if rng.random() < 0.6: W = (W + 3) // 4 * 4
        case = ("sep", N, H, W, k); print(it, case, flush=True)
        x = rng.uniform(0, 255, (N, H, W)).astype(np.float32); kx = rng.standard_normal(k).astype(np.float32); ky = rng.standard_normal(k).astype(np.float32)
        try: plan = mb.merit_plan_sepfilter(N, H, W, k)
        except Exception as e: print("   plan refused:", e, flush=True); plan = None
        if plan is not None:
            buf, y, pad = guard((N, H, W), torch.float32)
            mb.merit_sepfilter(plan, dev(x), dev(kx), dev(ky), y); torch.cuda.synchronize()
            tol = 1e-5 * float(np.abs(kx).sum() * np.abs(ky).sum() * np.abs(x).max())
            err = np.abs(y.cpu().numpy().astype(np.float64) - oracle.sepfilter(x, kx, ky)).max()
            report("sep", case, canary(buf, pad) and err <= tol, "err %.2e tol %.2e" % (err, tol))
        # ---- bilateral
        N, H, W, k = 1, ri(1, 60), ri(1, 150), ri(1, 20)
        case = ("bil", N, H, W, k); print(it, case, flush=True)
        x = (rng.integers(0, 3, size=(N, H, W)) * 80.0 + rng.normal(0, 6.0, size=(N, H, W))).astype(np.float32)
        gx = np.exp(-0.5 * ((np.arange(k) - k // 2) / max(k / 4.0, 0.5)) ** 2).astype(np.float32); gy = rng.uniform(0.3, 1.0, k).astype(np.float32)
        norm = -1.0 / (2 * 25.0 * 25.0)
        try: plan = mb.merit_plan_bilateral(N, H, W, k)
        except Exception as e: print("   plan refused:", e, flush=True); plan = None
        if plan is not None:
            buf, y, pad = guard((N, H, W), torch.float32)
            mb.merit_bilateral(plan, dev(x), dev(gx), dev(gy), norm, y); torch.cuda.synchronize()
            err = np.abs(y.cpu().numpy().astype(np.float64) - oracle.bilateral(x, gx, gy, norm)).max()
            tol = (2e-5 + 1.2e-7 * k * k) * float(x.max() - x.min()) + 1e-30
            report("bil", case, canary(buf, pad) and err <= tol, "err %.2e tol %.2e" % (err, tol))
    assert not failures, failures


@pytest.mark.parametrize("seed", [1103, 458])
def test_random_layer_shapes(seed):
    """Layers with many channels (the shapes the wave-specialised convolution kernels take):
    3x3, 1x1 and 5x5 windows on 32..256 input channels, any output-channel count and ragged image
    extents, through every way a convolution can be called: plain, clipped, with an added
    tensor, with the fused 3x3 / stride 2 / padding 1 max pooling, with weights packed once,
    and through the entry point that allocates nothing."""
    rng = np.random.default_rng(seed)
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0")
    failures, kernels = [], set()

    def ri(a, b):
        return int(rng.integers(a, b + 1))

    for it in range(26):
        N, Cin, Cout = ri(1, 3), 8 * ri(4, 32), ri(33, 256)
        if rng.random() < 0.5: Cout = 32 * ri(2, 8)
        H, W = ri(4, 36), ri(4, 36)
        if rng.random() < 0.3: H = W = int(rng.choice([7, 14, 28, 56])); N = 1
        k = int(rng.choice([3, 3, 3, 3, 3, 3, 1, 1, 5, 5]))
        s = 1 if rng.random() < 0.8 else 2
        pd = ri(0, k // 2)
        if H + 2 * pd < k or W + 2 * pd < k: continue
        mode = str(rng.choice(["plain", "relu", "residual", "pool", "packed", "noalloc"]))
        relu = int(mode in ("relu", "pool") or (mode == "residual" and rng.random() < 0.5))
        case = (mode, N, Cin, H, W, Cout, k, s, pd, relu)
        print(it, case, flush=True)
        x = rng.standard_normal((N, Cin, H, W)).astype(np.float16)
        w = (rng.standard_normal((Cout, Cin, k, k)) / np.sqrt(Cin * k * k)).astype(np.float16)
        try:
            if mode == "residual": plan = mb.merit_plan_conv2d_residual(N, Cin, H, W, Cout, k, k, s, s, pd, pd, relu)
            elif mode == "pool": plan = mb.merit_plan_conv2d_pool(N, Cin, H, W, Cout, k, k, s, s, pd, pd, relu)
            else: plan = mb.merit_plan_conv2d_dilated(N, Cin, H, W, Cout, k, k, s, s, pd, pd, 1, 1, relu)
        except mb.MeritError as e:
            print("   plan refused:", e, flush=True)
            assert mode == "pool", case                     # only the fused pooling has shape conditions
            continue
        buf, y, pad = _guard(plan.out_shape(), torch.float16)
        try:
            if mode == "residual":
                r = rng.standard_normal(plan.out_shape()).astype(np.float16)
                mb.merit_conv2d_residual(plan, dev(x), dev(w), dev(r), y)
                ref = oracle.conv2d_residual(x, w, r, (s, s), (pd, pd), bool(relu))
            elif mode == "pool":
                mb.merit_conv2d(plan, dev(x), dev(w), y)
                ref = oracle.conv2d_pool(x, w, (s, s), (pd, pd), bool(relu))
            elif mode == "packed":
                packed = mb.merit_conv2d_pack_weights(plan, dev(w))
                mb.merit_conv2d_packed(plan, dev(x), packed, y)
                ref = oracle.conv2d(x, w, (s, s), (pd, pd), bool(relu))
            elif mode == "noalloc":
                mb.merit_conv2d_packed_noalloc(plan, dev(x), dev(w), y)
                ref = oracle.conv2d(x, w, (s, s), (pd, pd), bool(relu))
            else:
                mb.merit_conv2d(plan, dev(x), dev(w), y)
                ref = oracle.conv2d(x, w, (s, s), (pd, pd), bool(relu))
        except mb.MeritError as e:
            print("   call refused:", e, flush=True)
            assert mode in ("packed", "noalloc"), case      # packing is for the multi-pass kernels only
            continue
        torch.cuda.synchronize()
        kernels.add(plan.launch_info()["kernel"])
        got = y.cpu().numpy().astype(np.float64); ref = ref.astype(np.float64)
        if not (_canary(buf, pad) and got.shape == ref.shape and np.all(np.abs(got - ref) <= 2e-2 * np.abs(ref) + 1e-3)):
            failures.append((case, plan.launch_info()["kernel"]))
    assert not failures, failures
    assert any("chws" in k for k in kernels), kernels


@pytest.mark.parametrize("seed", [3, 227])
def test_random_few_channel_layers(seed):
    """First layers: 1..7 input channels on images of 20..130 pixels a side with any width (odd,
    even, a multiple of 8 or not), window rows of up to 16 taps, strides up to 4 -- several tiles per
    image, so the few-channel MFMA kernels' staging of rows that start on any element and their
    stores into output planes off the 16-byte grid are met in every alignment; plain, clipped, with
    an added tensor and (where the shape allows) with the fused pooling."""
    rng = np.random.default_rng(seed)
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0")
    failures, kernels = [], set()

    def ri(a, b):
        return int(rng.integers(a, b + 1))

    for it in range(30):
        N, Cin, Cout = ri(1, 6), ri(1, 7), ri(1, 100)
        H, W = ri(20, 130), ri(20, 130)
        kh, kw = ri(1, 7), ri(1, 7)
        if rng.random() < 0.25: kh, kw = ri(7, 11), ri(9, 16)
        sh, sw = ri(1, 4), ri(1, 4)
        if rng.random() < 0.5: sh = sw = ri(1, 2)
        ph, pw = ri(0, kh // 2), ri(0, min(kw // 2, 8))
        OH, OW = (H + 2 * ph - kh) // sh + 1, (W + 2 * pw - kw) // sw + 1
        while N > 1 and N * Cout * OH * OW * Cin * kh * kw > 4e8: N -= 1
        mode = str(rng.choice(["plain", "relu", "residual", "pool"], p=[0.4, 0.3, 0.15, 0.15]))
        relu = int(mode in ("relu", "pool") or (mode == "residual" and rng.random() < 0.5))
        case = (mode, N, Cin, H, W, Cout, kh, kw, sh, sw, ph, pw, relu)
        print(it, case, flush=True)
        x = rng.standard_normal((N, Cin, H, W)).astype(np.float16)
        w = (rng.standard_normal((Cout, Cin, kh, kw)) / np.sqrt(Cin * kh * kw)).astype(np.float16)
        try:
            if mode == "residual": plan = mb.merit_plan_conv2d_residual(N, Cin, H, W, Cout, kh, kw, sh, sw, ph, pw, relu)
            elif mode == "pool": plan = mb.merit_plan_conv2d_pool(N, Cin, H, W, Cout, kh, kw, sh, sw, ph, pw, relu)
            else: plan = mb.merit_plan_conv2d_dilated(N, Cin, H, W, Cout, kh, kw, sh, sw, ph, pw, 1, 1, relu)
        except mb.MeritError as e:
            print("   plan refused:", e, flush=True)
            assert mode == "pool", case                     # only the fused pooling has shape conditions
            continue
        if mode in ("plain", "relu") and rng.random() < 0.6:
            # the wave-specialised kernel, which the planner itself takes on grids of 512 tiles and more
            try:
                plan.set_tile((0, 0, 8, 64))
            except mb.MeritError:
                pass
        buf, y, pad = _guard(plan.out_shape(), torch.float16)
        if mode == "residual":
            r = rng.standard_normal(plan.out_shape()).astype(np.float16)
            mb.merit_conv2d_residual(plan, dev(x), dev(w), dev(r), y)
            ref = oracle.conv2d_residual(x, w, r, (sh, sw), (ph, pw), bool(relu))
        elif mode == "pool":
            mb.merit_conv2d(plan, dev(x), dev(w), y)
            ref = oracle.conv2d_pool(x, w, (sh, sw), (ph, pw), bool(relu))
        else:
            mb.merit_conv2d(plan, dev(x), dev(w), y)
            ref = oracle.conv2d(x, w, (sh, sw), (ph, pw), bool(relu))
        torch.cuda.synchronize()
        li = plan.launch_info()
        kernels.add(li["kernel"])
        print("   ", li["kernel"], li["grid"], flush=True)
        got = y.cpu().numpy().astype(np.float64); ref = ref.astype(np.float64)
        if not (_canary(buf, pad) and got.shape == ref.shape and np.all(np.abs(got - ref) <= 2e-2 * np.abs(ref) + 1e-3)):
            failures.append((case, li["kernel"]))
    assert not failures, failures
    assert "merit_conv2d_planar_ws" in kernels and "merit_conv2d_planar" in kernels, kernels
