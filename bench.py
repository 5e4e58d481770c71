#!/usr/bin/env python3
"""Benchmark of the MERIT hot path on one MI355X.

    python bench.py --gpus 1 --steps K --warmup W

A *step* is one pass of the pooling workload (fp32 NCHW 16x64x112x112, 3x3
stride 2 pad 1): one max-pool launch and one avg-pool launch, each reading a
cache-cold input (the launches rotate through buffer sets larger than the
256 MB Infinity Cache).  The JSON line carries

  value        pooled output elements per second (both launches)
  roofline     the pooling kernel against peak HBM bandwidth, algorithmic bytes
               (input read once + output written once) / average launch duration
  cpu_baseline the CPU oracle on the same workload, timed on the host cores
  extra        the other four workloads (block matching, both convolutions),
               each with its own roofline -- informational

Inputs are seeded synthetic tensors already resident in HBM when timing starts.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0            # MI355X HBM3E
MFMA_F16_PEAK_TFLOPS = 2500.0    # dense fp16 MFMA
VALU_PEAK_TOPS = 39.3216         # 256 CU x 64 lanes x 2.4 GHz, one lane-op per lane per clock
FP32_FMA_PEAK_TOPS = 78.6432     # fp32 vector: 157.3 TFLOP/s = 256 CU x 128 fused multiply-adds x 2.4 GHz


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--sets", type=int, default=8, help="rotating buffer sets for cache-cold timing")
    ap.add_argument("--no-extra", action="store_true", help="skip the other workloads")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline")
    ap.add_argument("--extra-warm-ms", type=float, default=100.0,
                    help="the other workloads launch untimed at least this long before their timed region")
    ap.add_argument("--extra-only", default=None, help="run only the other workloads whose name contains this")
    ap.add_argument("--extra-skip", default=None, help="skip the other workloads whose name contains this")
    ap.add_argument("--peaks", action="store_true",
                    help="only run the peak probes (streaming copy, MFMA / FMA / SAD / exp2 instruction "
                         "loops) and print the measured-achievable peaks beside the data-sheet ones")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="only run a plain 256 MiB device copy 10 times (known traffic, for scaling "
                         "rocprofv3 FETCH_SIZE / WRITE_SIZE readings) and exit")
    return ap.parse_args()


WARM_MS = 0.0         # extra workloads: keep launching (untimed) at least this long before the timed region


def timed_region(torch, fn, steps, warmup):
    """Run fn(i) warmup + steps times; return (wall seconds, event milliseconds) for the steps.

    With WARM_MS > 0 the warm-up is repeated until that much time has passed: after an idle spell
    (tensor set-up, the CPU baseline of the workload before) the chip needs some 10-20 ms of work
    to reach the clocks it then holds -- the 256 -> 256 convolution ran 37.0, 33.0, 31.8, 31.3,
    30.6, 30.3 us per launch in six regions of 200 launches back to back, the 7x7 layer 18.5 ->
    16.1 us, the HBM-bound pooling 12.25 -> 12.15 us."""
    t_start = time.perf_counter()
    n = 0
    while True:
        batch = warmup if WARM_MS <= 0 else max(warmup, steps)   # long batches: no idle gaps at the synchronisations
        for i in range(batch):
            fn(n + i)
        n += batch
        torch.cuda.synchronize()
        if batch == 0 or (time.perf_counter() - t_start) * 1e3 >= WARM_MS:
            break
    warmup = n
    e0 = torch.cuda.Event(enable_timing=True)
    e1 = torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    for i in range(steps):
        fn(warmup + i)
    e1.record()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    return t1 - t0, e0.elapsed_time(e1)


def measure_peaks(torch, mb):
    """What the chip sustains with kernels that do nothing else (include/merit_probe.h)."""
    out = {}
    # memory stream: 1 GiB copied (read + written = 2 GiB of traffic), rotating over two buffer pairs
    n = 256 << 20
    bufs = [(torch.empty(n, dtype=torch.float32, device="cuda:0").normal_(),
             torch.empty(n, dtype=torch.float32, device="cuda:0")) for _ in range(2)]
    wall, ms = timed_region(torch, lambda i: mb.merit_probe_copy(*bufs[i % 2]), 20, 4)
    assert torch.equal(bufs[0][0], bufs[0][1])
    out["hbm_copy"] = {"measured": 2 * n * 4 / (ms * 1e-3 / 20) / 1e9, "datasheet": HBM_PEAK_GBS, "unit": "GB/s",
                       "what": "16-byte streaming loads + stores, 1 GiB in, 1 GiB out"}
    del bufs
    wgs, iters = 256 * 8, 4096                       # 8 workgroups of 4 wavefronts per CU: 8 wavefronts per SIMD
    sink = torch.empty(wgs * 256, dtype=torch.int32, device="cuda:0")
    kinds = [("mfma_f16", mb.MERIT_PROBE_MFMA_F16, 32768.0 / 1e12, MFMA_F16_PEAK_TFLOPS, "TFLOP/s",
              "v_mfma_f32_32x32x16_f16, 8 independent accumulators per wavefront"),
             ("mfma_f16_random_operands", mb.MERIT_PROBE_MFMA_F16_RANDOM, 32768.0 / 1e12, MFMA_F16_PEAK_TFLOPS, "TFLOP/s",
              "the same loop on hashed binary16 operands (random sign and mantissa), four operand pairs in turn"),
             ("fma_f32", mb.MERIT_PROBE_FMA_F32, 64.0 / 1e12, FP32_FMA_PEAK_TOPS, "T lane-ops/s",
              "v_fma_f32 (not packed), 8 independent chains per lane; data sheet = 157.3 TFLOP/s fp32 vector"),
             ("sad_u8", mb.MERIT_PROBE_SAD_U8, 64.0 / 1e12, VALU_PEAK_TOPS, "T lane-ops/s",
              "v_sad_u8, 8 independent accumulators per lane"),
             ("exp2_f32", mb.MERIT_PROBE_EXP2_F32, 64.0 / 1e12, FP32_FMA_PEAK_TOPS / 4, "T lane-ops/s",
              "v_exp_f32, 8 independent chains per lane; data-sheet figure = a quarter of the fp32 rate")]
    for name, which, per_instr, sheet, unit, what in kinds:
        it = iters // 4 if which in (mb.MERIT_PROBE_MFMA_F16, mb.MERIT_PROBE_MFMA_F16_RANDOM) else iters
        wall, ms = timed_region(torch, lambda i: mb.merit_probe_alu(which, wgs, it, sink), 10, 2)
        instrs = wgs * 4 * it * 8
        out[name] = {"measured": instrs * per_instr / (ms * 1e-3 / 10), "datasheet": sheet, "unit": unit, "what": what}
    return out


CPU_EXTRA = True      # time the oracle beside every extra workload (off with --no-cpu)


def oracle_rate(fn, out_elems, sample):
    """The oracle as it stands on a bounded sample of the workload: output elements per second on
    all host threads (best of the passes that fit ~0.3 s, at least one) and on one thread (one pass)."""
    if not CPU_EXTRA:
        return None
    import oracle
    n = oracle.num_threads()
    fn()                                            # first touch
    best, reps, t_all = None, 0, time.perf_counter()
    while reps < 1 or (time.perf_counter() - t_all < 0.3 and reps < 20):
        t0 = time.perf_counter(); fn(); dt = time.perf_counter() - t0
        best = dt if best is None else min(best, dt)
        reps += 1
    oracle.set_num_threads(1)
    try:
        t0 = time.perf_counter(); fn(); one = time.perf_counter() - t0
    finally:
        oracle.set_num_threads(n)
    return {"kind": "oracle", "unit": "output elems/s", "value": out_elems / best, "cores": n,
            "value_1_thread": out_elems / one, "sample": sample}


def bench_pool(torch, mb, wl, steps, warmup, nsets):
    c = wl.CFG1_POOL
    x_host = torch.from_numpy(wl.make_pool_input(c))
    x0 = x_host.to("cuda:0")
    xs = [x0] + [x0.roll(i, dims=0).contiguous() for i in range(1, nsets)]   # distinct buffers
    ys = [torch.empty((c.N, c.C, c.OH, c.OW), dtype=torch.float32, device="cuda:0") for _ in range(nsets)]
    pmax = mb.merit_plan_pool2d(c.N, c.C, c.H, c.W, c.kh, c.kw, c.sh, c.sw, c.ph, c.pw, 0)
    pavg = mb.merit_plan_pool2d(c.N, c.C, c.H, c.W, c.kh, c.kw, c.sh, c.sw, c.ph, c.pw, 1)

    # arguments marshalled once per buffer set; a call is then one C entry-point invocation
    cmax = [mb.bind_pool2d(pmax, xs[i], ys[i]) for i in range(nsets)]
    cavg = [mb.bind_pool2d(pavg, xs[i], ys[i]) for i in range(nsets)]

    def step(i):
        cmax[(2 * i) % nsets]()
        cavg[(2 * i + 1) % nsets]()

    wall, ev_ms = timed_region(torch, step, steps, warmup)
    out_elems = c.N * c.C * c.OH * c.OW
    alg_bytes = c.N * c.C * (c.H * c.W + c.OH * c.OW) * 4
    launches = 2 * steps
    avg_launch_s = ev_ms * 1e-3 / launches
    # cache-warm figure for context: same buffers every launch
    wmax, wavg = mb.bind_pool2d(pmax, xs[0], ys[0]), mb.bind_pool2d(pavg, xs[0], ys[1])
    wall_w, ev_w = timed_region(torch, lambda i: (wmax(), wavg()), steps, warmup)
    return {
        "wall_s": wall, "event_ms": ev_ms, "out_elems_per_step": 2 * out_elems,
        "alg_bytes_per_launch": alg_bytes, "avg_launch_us": avg_launch_s * 1e6,
        "achieved_gbs": alg_bytes / avg_launch_s / 1e9,
        "warm_avg_launch_us": ev_w * 1e3 / launches,
        "kernel": pmax.launch_info()["kernel"], "launch": pmax.launch_info(),
    }


def bench_pool_extra(torch, mb, wl, c, steps, warmup, nsets):
    """One more pooling shape as an extra line: max pooling only, rotating buffers."""
    x = wl.make_pool_input(c)
    x0 = torch.from_numpy(x).to("cuda:0")
    plan = mb.merit_plan_pool2d(c.N, c.C, c.H, c.W, c.kh, c.kw, c.sh, c.sw, c.ph, c.pw, 0)
    out_shape = plan.out_shape()
    n_out = 1
    for e in out_shape:
        n_out *= int(e)
    alg_bytes = x.nbytes + n_out * 4
    xs = [x0] + [x0.roll(i, dims=0).contiguous() for i in range(1, nsets)]
    ys = [torch.empty(out_shape, dtype=torch.float32, device="cuda:0") for _ in range(nsets)]
    calls = [mb.bind_pool2d(plan, xs[i], ys[i]) for i in range(nsets)]
    wall, ev_ms = timed_region(torch, lambda i: calls[i % nsets](), steps, warmup)
    t = ev_ms * 1e-3 / steps
    import oracle
    cpu = oracle_rate(lambda: oracle.pool2d(x, (c.kh, c.kw), (c.sh, c.sw), (c.ph, c.pw), "max"), n_out, "full batch, max")
    return {
        "workload": c.name + " (max)", "kernel": plan.launch_info()["kernel"], "avg_launch_us": t * 1e6, "launches": steps,
        "cpu_baseline": cpu,
        "out_elems_per_s": n_out / t,
        "achieved_hbm_gbs": alg_bytes / t / 1e9, "hbm_frac": alg_bytes / t / 1e9 / HBM_PEAK_GBS,
        "rotating_sets": nsets,
        "roofline": {"bound": "hbm", "achieved": alg_bytes / t / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": alg_bytes / t / 1e9 / HBM_PEAK_GBS},
    }


def bench_sad(torch, mb, wl, cfg, steps, warmup):
    cur, ref, _ = wl.make_sad_frames(cfg)
    dcur, dref = torch.from_numpy(cur).to("cuda:0"), torch.from_numpy(ref).to("cuda:0")
    plan = mb.merit_plan_sad(cfg.H, cfg.W, cfg.block, cfg.search)
    nby, nbx = plan.out_shape()
    sad = torch.empty((nby, nbx), dtype=torch.int32, device="cuda:0")
    mv = torch.empty((nby, nbx, 2), dtype=torch.int32, device="cuda:0")
    call = mb.bind_sad_search(plan, dcur, dref, sad, mv)
    wall, ev_ms = timed_region(torch, lambda i: call(), steps, warmup)
    t = ev_ms * 1e-3 / steps
    alg_bytes = 2 * cfg.H * cfg.W + nby * nbx * 12
    absdiffs = nby * nbx * cfg.n_candidates * cfg.block * cfg.block
    sad_lane_ops = absdiffs / 4                       # v_sad_u8: four pixels per lane-op
    # oracle sample: the top two block rows (plus the search margin below them) of the frame pair
    import oracle
    rows = min(cfg.H, 2 * cfg.block + cfg.search)
    rows -= rows % cfg.block
    rows = max(rows, cfg.block)
    sub_c, sub_r = cur[:rows].copy(), ref[:rows].copy()
    cpu = oracle_rate(lambda: oracle.sad_search(sub_c, sub_r, cfg.block, cfg.search),
                      (rows // cfg.block) * nbx, f"blocks of the top {rows} rows of the frame pair (unit: blocks)")
    return {
        "workload": cfg.name, "kernel": plan.launch_info()["kernel"], "avg_launch_us": t * 1e6, "launches": steps,
        "cpu_baseline": cpu,
        "blocks_per_s": nby * nbx / t, "candidate_sads_per_s": nby * nbx * cfg.n_candidates / t,
        "achieved_hbm_gbs": alg_bytes / t / 1e9, "hbm_frac": alg_bytes / t / 1e9 / HBM_PEAK_GBS,
        "roofline": {"bound": "alu", "achieved": sad_lane_ops / t / 1e12, "peak": VALU_PEAK_TOPS,
                     "unit": "T lane-ops/s (4-pixel SAD)", "frac": sad_lane_ops / t / 1e12 / VALU_PEAK_TOPS},
    }


def bench_conv(torch, mb, wl, cfg, steps, warmup, nsets, relu=False, pool=False, residual=False, packed=False):
    import numpy as np
    x, w = wl.make_conv_inputs(cfg)
    x0 = torch.from_numpy(x).to("cuda:0")
    dw = torch.from_numpy(w).to("cuda:0")
    in_bytes = x.nbytes + w.nbytes
    # fused 3x3/s2/p1 max pooling: only the pooled tensor is written
    oh, ow = (cfg.OH // 2, cfg.OW // 2) if pool else (cfg.OH, cfg.OW)
    out_bytes = cfg.N * cfg.Cout * oh * ow * 2
    if residual:                                   # the added tensor is read once
        in_bytes += out_bytes
    # rotate only when a set would otherwise stay resident in the Infinity Cache
    ns = nsets if (in_bytes + out_bytes) > (8 << 20) else 1
    xs = [x0] + [x0.roll(i, dims=0).contiguous() for i in range(1, ns)]
    ys = [torch.empty((cfg.N, cfg.Cout, oh, ow), dtype=torch.float16, device="cuda:0") for _ in range(ns)]
    rs = None
    if residual:
        plan = mb.merit_plan_conv2d_residual(cfg.N, cfg.Cin, cfg.H, cfg.W, cfg.Cout, cfg.kh, cfg.kw, cfg.sh, cfg.sw,
                                             cfg.ph, cfg.pw, int(relu))
        r0 = torch.from_numpy(np.random.default_rng(wl.BASE_SEED + 77).standard_normal(
            (cfg.N, cfg.Cout, oh, ow)).astype(np.float16)).to("cuda:0")
        rs = [r0] + [r0.roll(i, dims=0).contiguous() for i in range(1, ns)]
    elif pool:
        plan = mb.merit_plan_conv2d_pool(cfg.N, cfg.Cin, cfg.H, cfg.W, cfg.Cout, cfg.kh, cfg.kw, cfg.sh, cfg.sw,
                                         cfg.ph, cfg.pw, int(relu))
    elif (cfg.dh, cfg.dw) != (1, 1):
        plan = mb.merit_plan_conv2d_dilated(cfg.N, cfg.Cin, cfg.H, cfg.W, cfg.Cout, cfg.kh, cfg.kw, cfg.sh, cfg.sw,
                                            cfg.ph, cfg.pw, cfg.dh, cfg.dw, int(relu))
    else:
        make = mb.merit_plan_conv2d_relu if relu else mb.merit_plan_conv2d
        plan = make(cfg.N, cfg.Cin, cfg.H, cfg.W, cfg.Cout, cfg.kh, cfg.kw, cfg.sh, cfg.sw, cfg.ph, cfg.pw)
    if residual:
        calls = [mb.bind_conv2d_residual(plan, xs[i], dw, rs[i], ys[i]) for i in range(ns)]
    elif packed:
        # the weights regrouped once, outside the timed region (they do not change between calls)
        pk = mb.merit_conv2d_pack_weights(plan, dw)
        calls = [mb.bind_conv2d_packed(plan, xs[i], pk, ys[i]) for i in range(ns)]
    else:
        calls = [mb.bind_conv2d(plan, xs[i], dw, ys[i]) for i in range(ns)]
    wall, ev_ms = timed_region(torch, lambda i: calls[i % ns](), steps, warmup)
    t = ev_ms * 1e-3 / steps
    flops = 2.0 * cfg.N * cfg.Cout * cfg.OH * cfg.OW * cfg.Cin * cfg.kh * cfg.kw
    # oracle sample: one image, one output channel per host thread (the oracle's parallel loop is over
    # (image, output channel)), at least 8
    import oracle
    nco = min(cfg.Cout, max(8, oracle.num_threads()))
    xs1, ws8 = x[:1].copy(), w[:nco].copy()
    if pool:
        ofn = lambda: oracle.conv2d_pool(xs1, ws8, (cfg.sh, cfg.sw), (cfg.ph, cfg.pw), relu=relu)
    elif residual:
        r1 = np.zeros((1, nco, cfg.OH, cfg.OW), np.float16)
        ofn = lambda: oracle.conv2d_residual(xs1, ws8, r1, (cfg.sh, cfg.sw), (cfg.ph, cfg.pw), relu=relu)
    else:
        ofn = lambda: oracle.conv2d(xs1, ws8, (cfg.sh, cfg.sw), (cfg.ph, cfg.pw), relu=relu, dilation=(cfg.dh, cfg.dw))
    cpu = oracle_rate(ofn, nco * oh * ow, "one image, the first %d output channels" % nco)
    return {
        "workload": cfg.name + (" + residual tensor" if residual else "") + (" + fused ReLU" if relu else "")
        + (" + fused 3x3/s2/p1 max pooling" if pool else "") + (" (weights packed once)" if packed else ""),
        "kernel": plan.launch_info()["kernel"],
        "avg_launch_us": t * 1e6, "launches": steps, "cpu_baseline": cpu,
        "out_elems_per_s": cfg.N * cfg.Cout * oh * ow / t,
        "achieved_tflops": flops / t / 1e12, "mfma_frac": flops / t / 1e12 / MFMA_F16_PEAK_TFLOPS,
        "achieved_hbm_gbs": (in_bytes + out_bytes) / t / 1e9,
        "hbm_frac": (in_bytes + out_bytes) / t / 1e9 / HBM_PEAK_GBS,
        "rotating_sets": ns,
        # the roof that binds this layer: whichever of its MFMA time and its HBM time at peak is longer
        "roofline": ({"bound": "mfma", "achieved": flops / t / 1e12, "peak": MFMA_F16_PEAK_TFLOPS, "unit": "TFLOP/s",
                      "frac": flops / t / 1e12 / MFMA_F16_PEAK_TFLOPS}
                     if flops / (MFMA_F16_PEAK_TFLOPS * 1e12) >= (in_bytes + out_bytes) / (HBM_PEAK_GBS * 1e9) else
                     {"bound": "hbm", "achieved": (in_bytes + out_bytes) / t / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                      "frac": (in_bytes + out_bytes) / t / 1e9 / HBM_PEAK_GBS}),
    }


def bench_depthwise(torch, mb, wl, cfg, steps, warmup, nsets):
    x, w = wl.make_depthwise_inputs(cfg)
    x0 = torch.from_numpy(x).to("cuda:0")
    dw = torch.from_numpy(w).to("cuda:0")
    plan = mb.merit_plan_conv2d_depthwise(cfg.N, cfg.C, cfg.H, cfg.W, cfg.kh, cfg.kw, cfg.sh, cfg.sw, cfg.ph, cfg.pw)
    out_shape = plan.out_shape()
    n_out = 1
    for e in out_shape:
        n_out *= int(e)
    alg_bytes = x.nbytes + w.nbytes + n_out * 2
    ns = nsets if alg_bytes > (8 << 20) else 1
    xs = [x0] + [x0.roll(i, dims=0).contiguous() for i in range(1, ns)]
    ys = [torch.empty(out_shape, dtype=torch.float16, device="cuda:0") for _ in range(ns)]
    calls = [mb.bind_conv2d_depthwise(plan, xs[i], dw, ys[i]) for i in range(ns)]
    wall, ev_ms = timed_region(torch, lambda i: calls[i % ns](), steps, warmup)
    t = ev_ms * 1e-3 / steps
    import oracle
    x1 = x[:1].copy()
    cpu = oracle_rate(lambda: oracle.conv2d_depthwise(x1, w, (cfg.sh, cfg.sw), (cfg.ph, cfg.pw)),
                      n_out // cfg.N, "one image")
    return {
        "workload": cfg.name, "kernel": plan.launch_info()["kernel"], "avg_launch_us": t * 1e6, "launches": steps,
        "cpu_baseline": cpu,
        "out_elems_per_s": n_out / t,
        "achieved_hbm_gbs": alg_bytes / t / 1e9, "hbm_frac": alg_bytes / t / 1e9 / HBM_PEAK_GBS,
        "rotating_sets": ns,
        "roofline": {"bound": "hbm", "achieved": alg_bytes / t / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": alg_bytes / t / 1e9 / HBM_PEAK_GBS},
    }


def bench_sepfilter(torch, mb, wl, cfg, steps, warmup, nsets):
    x, kx, ky = wl.make_sepfilter_inputs(cfg)
    x0 = torch.from_numpy(x).to("cuda:0")
    dkx, dky = torch.from_numpy(kx).to("cuda:0"), torch.from_numpy(ky).to("cuda:0")
    plan = mb.merit_plan_sepfilter(cfg.N, cfg.H, cfg.W, cfg.k)
    alg_bytes = 2 * x.nbytes + 2 * kx.nbytes
    ns = nsets if alg_bytes > (8 << 20) else 1
    xs = [x0] + [x0.roll(i, dims=0).contiguous() for i in range(1, ns)]
    ys = [torch.empty_like(x0) for _ in range(ns)]
    calls = [mb.bind_sepfilter(plan, xs[i], dkx, dky, ys[i]) for i in range(ns)]
    wall, ev_ms = timed_region(torch, lambda i: calls[i % ns](), steps, warmup)
    t = ev_ms * 1e-3 / steps
    fmas = 2.0 * cfg.k * cfg.N * cfg.H * cfg.W          # k per pass and pixel
    # whichever published peak the workload needs longer at binds: memory up to k = 39 here
    if fmas / (FP32_FMA_PEAK_TOPS * 1e12) > alg_bytes / (HBM_PEAK_GBS * 1e9):
        roof = {"bound": "alu", "achieved": 2 * fmas / t / 1e12, "peak": 2 * FP32_FMA_PEAK_TOPS,
                "unit": "TFLOP/s (fp32 vector)", "frac": fmas / t / 1e12 / FP32_FMA_PEAK_TOPS}
    else:
        roof = {"bound": "hbm", "achieved": alg_bytes / t / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": alg_bytes / t / 1e9 / HBM_PEAK_GBS}
    import oracle
    band = x[:1, :256].copy()
    cpu = oracle_rate(lambda: oracle.sepfilter(band, kx, ky), band.size, "the top 256 rows of one image")
    return {
        "workload": cfg.name, "kernel": plan.launch_info()["kernel"], "avg_launch_us": t * 1e6, "launches": steps,
        "cpu_baseline": cpu,
        "out_elems_per_s": cfg.N * cfg.H * cfg.W / t,
        "achieved_hbm_gbs": alg_bytes / t / 1e9, "hbm_frac": alg_bytes / t / 1e9 / HBM_PEAK_GBS,
        "achieved_fp32_tflops": 2 * fmas / t / 1e12,
        "rotating_sets": ns,
        "roofline": roof,
    }


def bench_bilateral(torch, mb, wl, cfg, steps, warmup):
    x, g = wl.make_bilateral_inputs(cfg)
    dx, dg = torch.from_numpy(x).to("cuda:0"), torch.from_numpy(g).to("cuda:0")
    y = torch.empty_like(dx)
    plan = mb.merit_plan_bilateral(cfg.N, cfg.H, cfg.W, cfg.k)
    call = mb.bind_bilateral(plan, dx, dg, dg, cfg.norm, y)
    wall, ev_ms = timed_region(torch, lambda i: call(), steps, warmup)
    t = ev_ms * 1e-3 / steps
    taps = float(cfg.N * cfg.H * cfg.W * cfg.k * cfg.k)
    # Algorithmic work is taps (one weight and two accumulations per window element); the ceiling
    # is what the chip's vector ALU could do per tap at the published rates whatever the
    # instruction recipe: the definition needs one exponential (a transcendental: a quarter of
    # the fp32 vector rate) and at least 3 plain fp32 operations (the squared difference times
    # the constant, sum w, sum w*v, as fused multiply-adds), i.e. 4 + 3 = 7 issue slots of the
    # 78.6 T slots/s (157.3 TFLOP/s fp32 vector = 256 CU x 128 lanes x 2.4 GHz): 11.2 T taps/s.
    peak_taps = FP32_FMA_PEAK_TOPS / 7.0
    alg_bytes = 2 * x.nbytes
    import oracle
    band = x[:, :64].copy()
    cpu = oracle_rate(lambda: oracle.bilateral(band, g, g, cfg.norm), band.size, "the top 64 rows of the image")
    return {
        "workload": cfg.name, "kernel": plan.launch_info()["kernel"], "avg_launch_us": t * 1e6, "launches": steps,
        "cpu_baseline": cpu,
        "out_elems_per_s": cfg.N * cfg.H * cfg.W / t, "taps_per_s": taps / t,
        "achieved_hbm_gbs": alg_bytes / t / 1e9, "hbm_frac": alg_bytes / t / 1e9 / HBM_PEAK_GBS,
        "roofline": {"bound": "alu", "achieved": taps / t / 1e12, "peak": peak_taps,
                     "unit": "T taps/s (ceiling: 1 exponential at a quarter rate + 3 fp32 operations per tap "
                             "at 78.6 T vector operations/s)", "frac": taps / t / 1e12 / peak_taps},
    }


def bench_corr(torch, mb, wl, cfg, steps, warmup):
    x1, x2 = wl.make_correlation_inputs(cfg)
    d1, d2 = torch.from_numpy(x1).to("cuda:0"), torch.from_numpy(x2).to("cuda:0")
    plan = mb.merit_plan_correlation(cfg.N, cfg.C, cfg.H, cfg.W, cfg.search, cfg.stride)
    y = torch.empty(plan.out_shape(), dtype=torch.float16, device="cuda:0")
    call = mb.bind_correlation(plan, d1, d2, y)
    wall, ev_ms = timed_region(torch, lambda i: call(), steps, warmup)
    t = ev_ms * 1e-3 / steps
    n = 2 * cfg.search + 1
    alg_bytes = x1.nbytes + x2.nbytes + y.numel() * 2
    flops = 2.0 * cfg.N * cfg.H * cfg.W * n * n * cfg.C          # zero-padded positions included
    import oracle
    nr = min(cfg.H, max(8, oracle.num_threads()))  # the oracle's parallel loop is over (image, row)
    r1, r2 = x1[:, :, :nr].copy(), x2[:, :, :nr].copy()
    cpu = oracle_rate(lambda: oracle.correlation(r1, r2, cfg.search, cfg.stride), cfg.N * nr * cfg.W * n * n,
                      "the top %d rows of the feature maps (as a map of their own)" % nr)
    return {
        "workload": cfg.name, "kernel": plan.launch_info()["kernel"], "avg_launch_us": t * 1e6, "launches": steps,
        "cpu_baseline": cpu,
        "out_elems_per_s": y.numel() / t, "achieved_tflops": flops / t / 1e12,
        "achieved_hbm_gbs": alg_bytes / t / 1e9, "hbm_frac": alg_bytes / t / 1e9 / HBM_PEAK_GBS,
        "mfma_frac": flops / t / 1e12 / MFMA_F16_PEAK_TFLOPS,
        # both ideal times are far below a launch (bytes: 0.65 us, flops: 0.1 us); the larger one is quoted
        "roofline": {"bound": "hbm", "achieved": alg_bytes / t / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": alg_bytes / t / 1e9 / HBM_PEAK_GBS},
    }


def cpu_baseline(wl):
    """The oracle as it stands, timed on the host cores: max + avg pool of the full batch."""
    import oracle
    c = wl.CFG1_POOL
    x = wl.make_pool_input(c)
    oracle.pool2d(x[:1], (c.kh, c.kw), (c.sh, c.sw), (c.ph, c.pw), "max")      # load + first touch
    best = None
    reps = 0
    t_all = time.perf_counter()
    while reps < 3 or (time.perf_counter() - t_all < 10.0 and reps < 40):
        t0 = time.perf_counter()
        oracle.pool2d(x, (c.kh, c.kw), (c.sh, c.sw), (c.ph, c.pw), "max")
        oracle.pool2d(x, (c.kh, c.kw), (c.sh, c.sw), (c.ph, c.pw), "avg")
        dt = time.perf_counter() - t0
        best = dt if best is None else min(best, dt)
        reps += 1
    elems = 2 * c.N * c.C * c.OH * c.OW
    return {"value": elems / best, "unit": "elems/s", "cores": oracle.num_threads(), "kind": "oracle",
            "sample": f"full pooling batch (max + avg, {elems} outputs), best of {reps} passes, "
                      f"gcc -O2 + OpenMP over (n,c) planes"}


def pool_traffic_from_profiles():
    """HBM-side bytes per pooling launch: counters cannot be read from inside this process, so the
    figure is the one the committed rocprofv3 summaries hold (two --pmc runs of this file,
    FETCH_SIZE then WRITE_SIZE, each scaled by what the same counter reads for a plain 256 MiB
    device copy).  Read from the files, mean of the max and the avg kernel; None if a summary
    is missing or has no counter section (then `traffic` is null rather than stale)."""
    import re
    vals, names = [], []
    for mode in ("max", "avg"):
        name = f"pool2d_stream_k3s2p1_{mode}__pool_16x64x112x112_k3s2p1.txt"
        path = os.path.join(ROOT, "profiles", name)
        try:
            text = open(path).read()
        except OSError:
            return None, None
        m = re.search(r"scaled: read ([0-9.]+) MB \+ written ([0-9.]+) MB = ([0-9.]+) MB per launch", text)
        if not m:
            return None, None
        vals.append(float(m.group(3)) * 1e6)
        names.append("profiles/" + name)
    stamp = time.strftime("%Y-%m-%d", time.gmtime(min(os.path.getmtime(os.path.join(ROOT, n)) for n in names)))
    return sum(vals) / len(vals), {"files": names, "file_date": stamp}


def main():
    global CPU_EXTRA, WARM_MS
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)
    import torch
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    from paper_1911_03458_amd import binding as mb
    from paper_1911_03458_amd import workloads as wl
    mb.lib()
    torch.cuda.set_device(0)

    if args.peaks:
        WARM_MS = args.extra_warm_ms             # the probes too are timed at settled clocks
        print(json.dumps({"peaks": measure_peaks(torch, mb)}))
        return

    if args.copy_calibration:
        # one elementwise copy kernel per iteration: reads 256 MiB and writes 256 MiB
        src = torch.empty(64 << 20, dtype=torch.float32, device="cuda:0").normal_()
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        for _ in range(10):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration_bytes_read": src.numel() * 4, "bytes_written": src.numel() * 4,
                          "launches": 10}))
        return

    pool = bench_pool(torch, mb, wl, args.steps, args.warmup, args.sets)
    value = pool["out_elems_per_step"] * args.steps / pool["wall_s"]
    traffic, traffic_src = pool_traffic_from_profiles()
    result = {
        "metric": "pool2d output elems/s (max + avg, cache-cold)",
        "value": value,
        "unit": "elems/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": pool["wall_s"] * 1e3 / args.steps,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": wl.CFG1_POOL.name + " (max-pool launch + avg-pool launch per step)",
                   "rotating_buffer_sets": args.sets, "kernel": pool["kernel"],
                   "grid": pool["launch"]["grid"][0], "lds_bytes": pool["launch"]["lds_bytes"]},
        "roofline": {"bound": "hbm", "achieved": pool["achieved_gbs"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": pool["achieved_gbs"] / HBM_PEAK_GBS, "traffic": traffic,
                     "traffic_unit": "bytes per launch", "traffic_source": traffic_src,
                     "time_base": "HIP events over the timed region / launches (includes the dispatch gap "
                                  "between back-to-back launches; rocprofv3's per-kernel duration in profiles/ "
                                  "is a few percent shorter, the wall-clock ms_per_step a few percent longer)",
                     "avg_launch_us": pool["avg_launch_us"], "alg_bytes_per_launch": pool["alg_bytes_per_launch"],
                     "cache_warm_avg_launch_us": pool["warm_avg_launch_us"]},
    }
    CPU_EXTRA = not args.no_cpu
    WARM_MS = args.extra_warm_ms                 # the headline above keeps exactly --warmup launches
    if not args.no_extra:
        k = max(200, args.steps)             # launches per extra workload, whatever --steps says
        w = max(20, args.warmup)
        kl = k
        extras = [
            (wl.CFG0_ME_SMALL.name, lambda: bench_sad(torch, mb, wl, wl.CFG0_ME_SMALL, k, w)),
            (wl.CFG_POOL_ODD.name, lambda: bench_pool_extra(torch, mb, wl, wl.CFG_POOL_ODD, k, w, args.sets)),
            (wl.CFG2_CONV3.name, lambda: bench_conv(torch, mb, wl, wl.CFG2_CONV3, k, w, args.sets)),
            (wl.CFG3_ME_FHD.name, lambda: bench_sad(torch, mb, wl, wl.CFG3_ME_FHD, kl, w)),
            (wl.CFG_ME_720P.name, lambda: bench_sad(torch, mb, wl, wl.CFG_ME_720P, k, w)),
            (wl.CFG_ME_1080P.name, lambda: bench_sad(torch, mb, wl, wl.CFG_ME_1080P, kl, w)),
            (wl.CFG4_CONV7.name, lambda: bench_conv(torch, mb, wl, wl.CFG4_CONV7, k, w, args.sets)),
            (wl.CFG4_CONV7.name, lambda: bench_conv(torch, mb, wl, wl.CFG4_CONV7, k, w, args.sets, relu=True)),
            (wl.CFG4_CONV7.name, lambda: bench_conv(torch, mb, wl, wl.CFG4_CONV7, k, w, args.sets, relu=True, pool=True)),
            (wl.CFG2_CONV3.name, lambda: bench_conv(torch, mb, wl, wl.CFG2_CONV3, k, w, args.sets, relu=True, residual=True)),
            (wl.CFG2_CONV3.name, lambda: bench_conv(torch, mb, wl, wl.CFG2_CONV3, k, w, args.sets, relu=True, pool=True)),
            (wl.CFG_DILATED.name, lambda: bench_conv(torch, mb, wl, wl.CFG_DILATED, k, w, args.sets)),
            (wl.CFG_CONV256.name, lambda: bench_conv(torch, mb, wl, wl.CFG_CONV256, kl, w, args.sets)),
            (wl.CFG_CONV256.name, lambda: bench_conv(torch, mb, wl, wl.CFG_CONV256, kl, w, args.sets, packed=True)),
            (wl.CFG_CONV256.name, lambda: bench_conv(torch, mb, wl, wl.CFG_CONV256, kl, w, args.sets, relu=True, pool=True)),
            (wl.CFG_CONV256_B64.name, lambda: bench_conv(torch, mb, wl, wl.CFG_CONV256_B64, kl, w, 3)),
            (wl.CFG_CONV5X5.name, lambda: bench_conv(torch, mb, wl, wl.CFG_CONV5X5, kl, w, args.sets)),
            (wl.CFG_CONV14.name, lambda: bench_conv(torch, mb, wl, wl.CFG_CONV14, kl, w, args.sets)),
            (wl.CFG_CONV11.name, lambda: bench_conv(torch, mb, wl, wl.CFG_CONV11, kl, w, args.sets)),
            (wl.CFG_CORRELATION.name, lambda: bench_corr(torch, mb, wl, wl.CFG_CORRELATION, k, w)),
            (wl.CFG_DEPTHWISE.name, lambda: bench_depthwise(torch, mb, wl, wl.CFG_DEPTHWISE, k, w, args.sets)),
            (wl.CFG_SEP_K3.name, lambda: bench_sepfilter(torch, mb, wl, wl.CFG_SEP_K3, k, w, args.sets)),
            (wl.CFG_SEP_K30.name, lambda: bench_sepfilter(torch, mb, wl, wl.CFG_SEP_K30, kl, w, args.sets)),
            (wl.CFG_BILATERAL.name, lambda: bench_bilateral(torch, mb, wl, wl.CFG_BILATERAL, kl, w)),
        ]
        # --extra-only / --extra-skip: substrings of a workload's name (for profiling one launch shape alone)
        result["extra_timing"] = ("each workload below: at least %g ms of untimed launches (settled clocks), then %d timed "
                                  "launches between two HIP events" % (args.extra_warm_ms, k))
        result["extra"] = [run() for name, run in extras
                           if (args.extra_only is None or args.extra_only in name)
                           and (args.extra_skip is None or args.extra_skip not in name)]
    if not args.no_cpu:
        result["cpu_baseline"] = cpu_baseline(wl)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
