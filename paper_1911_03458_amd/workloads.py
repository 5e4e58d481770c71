"""Seeded synthetic input generators for the five MERIT hot-path workloads.

This module holds *no* arithmetic of the method itself (no window gather, no
reduction): it only draws the random tensors and frames that both the CPU
oracle and the HIP path consume.  It imports neither of them.

The paper's GPU experiments (Section VI-B, Table "Speedup on GPUs") ran on
Parboil / Caffe inputs whose sizes are not stated; these generators stand in
for them with the shapes and value distributions fixed by the build's
configuration list:

  cfg 0  block-matching ME, 64x64 u8, 8x8 blocks, search +-4
  cfg 1  max / average pool, fp32 NCHW 16x64x112x112, 3x3 stride 2 pad 1
  cfg 2  conv fp16 NCHW 8x64x56x56, 64 output channels, 3x3 stride 1 pad 1
  cfg 3  block-matching ME, 1920x1088 u8, 16x16 blocks, search +-32
  cfg 4  conv fp16 NCHW 32x3x224x224, 64 output channels, 7x7 stride 2 pad 3

Every generator takes a seed; the default seed is 1911 + config index.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np

BASE_SEED = 1911


# --------------------------------------------------------------------------
# descriptors
# --------------------------------------------------------------------------
@dataclass(frozen=True)
class SadWorkload:
    name: str
    H: int
    W: int
    block: int
    search: int          # R: candidates dy,dx in [-R, R]
    noise: int           # uniform integer noise amplitude added to the displaced copy
    texture: str         # "uniform" or "sinusoid"

    @property
    def n_blocks(self):
        return (self.H // self.block) * (self.W // self.block)

    @property
    def n_candidates(self):
        return (2 * self.search + 1) ** 2


@dataclass(frozen=True)
class PoolWorkload:
    name: str
    N: int
    C: int
    H: int
    W: int
    kh: int
    kw: int
    sh: int
    sw: int
    ph: int
    pw: int

    @property
    def OH(self):
        return (self.H + 2 * self.ph - self.kh) // self.sh + 1

    @property
    def OW(self):
        return (self.W + 2 * self.pw - self.kw) // self.sw + 1


@dataclass(frozen=True)
class ConvWorkload:
    name: str
    N: int
    Cin: int
    H: int
    W: int
    Cout: int
    kh: int
    kw: int
    sh: int
    sw: int
    ph: int
    pw: int
    x_dist: str          # "normal" or "uniform"
    dh: int = 1          # dilation: input rows / columns per window step
    dw: int = 1

    @property
    def OH(self):
        return (self.H + 2 * self.ph - ((self.kh - 1) * self.dh + 1)) // self.sh + 1

    @property
    def OW(self):
        return (self.W + 2 * self.pw - ((self.kw - 1) * self.dw + 1)) // self.sw + 1


CFG0_ME_SMALL = SadWorkload("me_64x64_b8_r4", 64, 64, 8, 4, 3, "uniform")
CFG1_POOL = PoolWorkload("pool_16x64x112x112_k3s2p1", 16, 64, 112, 112, 3, 3, 2, 2, 1, 1)
# an odd width and no padding: the first pooling layer of AlexNet (55 x 55 -> 27 x 27), which the 16-byte
# row kernels do not take
CFG_POOL_ODD = PoolWorkload("pool_32x96x55x55_k3s2p0", 32, 96, 55, 55, 3, 3, 2, 2, 0, 0)
CFG2_CONV3 = ConvWorkload("conv_8x64x56x56_co64_k3s1p1", 8, 64, 56, 56, 64, 3, 3, 1, 1, 1, 1, "normal")
CFG3_ME_FHD = SadWorkload("me_1920x1088_b16_r32", 1088, 1920, 16, 32, 0, "sinusoid")
CFG4_CONV7 = ConvWorkload("conv_32x3x224x224_co64_k7s2p3", 32, 3, 224, 224, 64, 7, 7, 2, 2, 3, 3, "uniform")

CONFIGS = [CFG0_ME_SMALL, CFG1_POOL, CFG2_CONV3, CFG3_ME_FHD, CFG4_CONV7]

# Beyond the five configurations: the motion-estimation row of the paper's table of further
# workloads (720p, 8x8 blocks; the search range is not given there: +-16 here), and the dilated layer of the paper's table of further workloads
# (output 64 x 64 x 32; channel count and batch are not given there: 32 in, batch 8 here).
CFG_CORRELATION = None   # defined below (needs its dataclass)
CFG_ME_720P = SadWorkload("me_1280x720_b8_r16", 720, 1280, 8, 16, 0, "sinusoid")
# full HD at its real height: 1080 = 67.5 blocks of 16, the last block row reaches past the frame
CFG_ME_1080P = SadWorkload("me_1920x1080_b16_r32", 1080, 1920, 16, 32, 0, "uniform")
CFG_DILATED = ConvWorkload("conv_8x32x64x64_co32_k3s1p2_d2", 8, 32, 64, 64, 32, 3, 3, 1, 1, 2, 2, "normal", 2, 2)
# The paper's strided example (Section III-C, Eq. 6): 48 output channels of 55 x 55 from 3 input
# channels under an 11 x 11 window, x = 4p + a - 5 (stride 4, padding 5 => a 220 x 220 input);
# the batch is not given there: 8 here.  Its window is wider than the small-channel MFMA
# kernel's fragments: the one-element-per-thread kernel takes it.
CFG_CONV11 = ConvWorkload("conv_8x3x220x220_co48_k11s4p5", 8, 3, 220, 220, 48, 11, 11, 4, 4, 5, 5, "uniform")
# A layer whose weights and input rows do not fit LDS at once (256 -> 256 channels, 3 x 3 on
# 56 x 56, the shape class of the deeper layers of the paper's per-layer table): channels in passes.
CFG_CONV256 = ConvWorkload("conv_8x256x56x56_co256_k3s1p1", 8, 256, 56, 56, 256, 3, 3, 1, 1, 1, 1, "normal")
# The same layer on a batch of 64: 200 704 pixels = 784 tiles of 256, three rounds of the 256 CUs,
# so that the launch and the pipeline fill of the first tile weigh a third as much.
# The 5x5 layer of the paper's per-layer table (Section VI-C; 96 -> 256 channels on 27x27) and one of its
# 3x3 layers on small images (512 -> 512 on 14x14): few pixels, many channels.
CFG_CONV5X5 = ConvWorkload("conv_8x96x27x27_co256_k5s1p2", 8, 96, 27, 27, 256, 5, 5, 1, 1, 2, 2, "normal")
CFG_CONV14 = ConvWorkload("conv_8x512x14x14_co512_k3s1p1", 8, 512, 14, 14, 512, 3, 3, 1, 1, 1, 1, "normal")
CFG_CONV256_B64 = ConvWorkload("conv_64x256x56x56_co256_k3s1p1", 64, 256, 56, 56, 256, 3, 3, 1, 1, 1, 1, "normal")


@dataclass(frozen=True)
class DepthwiseWorkload:
    name: str
    N: int
    C: int
    H: int
    W: int
    kh: int
    kw: int
    sh: int
    sw: int
    ph: int
    pw: int


# The depthwise row of the paper's table of further workloads: output 64 x 64 x 32 per image
# (window and batch are not given there: the 3x3 / stride 1 / pad 1 MobileNet layer, batch 32).
CFG_DEPTHWISE = DepthwiseWorkload("dwconv_32x32x64x64_k3s1p1", 32, 32, 64, 64, 3, 3, 1, 1, 1, 1)


@dataclass(frozen=True)
class CorrWorkload:
    name: str
    N: int
    C: int
    H: int
    W: int
    search: int          # R: displacement indices p3, p4 in [0, 2R]
    stride: int          # displacement stride


# The correlation row of the paper's table of further workloads: output 64 x 64 x 11 x 11
# (channel count and displacement stride are not given there: 256 channels, stride 2 here).
CFG_CORRELATION = CorrWorkload("corr_1x256x64x64_r5_s2", 1, 256, 64, 64, 5, 2)


# --------------------------------------------------------------------------
# generators
# --------------------------------------------------------------------------
def _texture_uniform(rng, H, W):
    return rng.integers(0, 256, size=(H, W), dtype=np.int64)


def _texture_sinusoid(rng, H, W):
    """Smooth random texture: 128 + eight sinusoids of amplitude 14 + noise +-8."""
    fx = rng.uniform(0.004, 0.06, size=8)
    fy = rng.uniform(0.004, 0.06, size=8)
    ph = rng.uniform(0.0, 2.0 * np.pi, size=8)
    yy, xx = np.meshgrid(np.arange(H, dtype=np.float64),
                         np.arange(W, dtype=np.float64), indexing="ij")
    acc = np.full((H, W), 128.0)
    for k in range(8):
        acc += 14.0 * np.sin(2.0 * np.pi * (fx[k] * xx + fy[k] * yy) + ph[k])
    tex = np.rint(acc).astype(np.int64)
    tex += rng.integers(-8, 9, size=(H, W), dtype=np.int64)
    return tex


def make_sad_frames(wl: SadWorkload, seed: int | None = None):
    """Return (cur, ref, planted) for a block-matching workload.

    ref  = "frame1", the texture.
    cur  = "frame0": every block of cur is the block of ref displaced by that
           block's planted vector (coordinates clamped to the frame), plus
           uniform integer noise in [-noise, noise], clipped to [0, 255].
    planted[by, bx] = (vy, vx), drawn uniformly from [-R, R]^2.
    """
    if seed is None:
        seed = BASE_SEED + (CONFIGS.index(wl) if wl in CONFIGS else 6)
    rng = np.random.default_rng(seed)
    H, W, B, R = wl.H, wl.W, wl.block, wl.search
    if wl.texture == "uniform":
        tex = _texture_uniform(rng, H, W)
    elif wl.texture == "sinusoid":
        tex = _texture_sinusoid(rng, H, W)
    else:
        raise ValueError(wl.texture)
    ref = np.clip(tex, 0, 255).astype(np.uint8)
    nby, nbx = -(-H // B), -(-W // B)               # blocks past the edge are cropped below
    planted = rng.integers(-R, R + 1, size=(nby, nbx, 2), dtype=np.int64)
    vy = np.repeat(np.repeat(planted[:, :, 0], B, axis=0), B, axis=1)
    vx = np.repeat(np.repeat(planted[:, :, 1], B, axis=0), B, axis=1)
    yy, xx = np.meshgrid(np.arange(nby * B), np.arange(nbx * B), indexing="ij")
    sy = np.clip(yy + vy, 0, H - 1)
    sx = np.clip(xx + vx, 0, W - 1)
    cur = ref[sy, sx].astype(np.int64)[:H, :W]
    if wl.noise > 0:
        cur += rng.integers(-wl.noise, wl.noise + 1, size=(H, W), dtype=np.int64)
    cur = np.clip(cur, 0, 255).astype(np.uint8)
    return cur, ref, planted.astype(np.int32)


def make_pool_input(wl: PoolWorkload, seed: int | None = None, N: int | None = None):
    """fp32 NCHW tensor of N(0,1) values.  `N` overrides the batch (for samples)."""
    if seed is None:
        seed = BASE_SEED + 1
    rng = np.random.default_rng(seed)
    n = wl.N if N is None else N
    return rng.standard_normal(size=(n, wl.C, wl.H, wl.W), dtype=np.float32)


def make_conv_inputs(wl: ConvWorkload, seed: int | None = None, N: int | None = None):
    """Return (x fp16 NCHW, w fp16 OIHW).  Weights are N(0, 1/(Cin*kh*kw))."""
    if seed is None:
        seed = BASE_SEED + (CONFIGS.index(wl) if wl in CONFIGS else 5)
    rng = np.random.default_rng(seed)
    n = wl.N if N is None else N
    shape = (n, wl.Cin, wl.H, wl.W)
    if wl.x_dist == "normal":
        x = rng.standard_normal(size=shape, dtype=np.float32)
    elif wl.x_dist == "uniform":
        x = rng.uniform(-1.0, 1.0, size=shape).astype(np.float32)
    else:
        raise ValueError(wl.x_dist)
    fan_in = wl.Cin * wl.kh * wl.kw
    w = rng.standard_normal(size=(wl.Cout, wl.Cin, wl.kh, wl.kw), dtype=np.float32)
    w *= np.float32(1.0 / np.sqrt(fan_in))
    return x.astype(np.float16), w.astype(np.float16)


def make_correlation_inputs(wl: CorrWorkload, seed: int | None = None):
    """Two fp16 feature maps [N,C,H,W]: the second is the first shifted by a few pixels plus
    noise (so that the correlation has structure), both scaled to keep sums O(1)."""
    rng = np.random.default_rng(BASE_SEED + 7 if seed is None else seed)
    a = rng.standard_normal(size=(wl.N, wl.C, wl.H, wl.W)).astype(np.float32)
    b = np.roll(a, shift=(2, -4), axis=(2, 3)) + 0.5 * rng.standard_normal(size=a.shape).astype(np.float32)
    s = np.float32(1.0 / np.sqrt(wl.C))
    return (a * s).astype(np.float16), b.astype(np.float16)


def make_depthwise_inputs(wl: DepthwiseWorkload, seed: int | None = None):
    """x fp16 [N,C,H,W] ~ N(0,1); w fp16 [C,kh,kw] ~ N(0, 1/(kh*kw))."""
    rng = np.random.default_rng(BASE_SEED + 8 if seed is None else seed)
    x = rng.standard_normal(size=(wl.N, wl.C, wl.H, wl.W), dtype=np.float32)
    w = rng.standard_normal(size=(wl.C, wl.kh, wl.kw), dtype=np.float32) / np.float32(np.sqrt(wl.kh * wl.kw))
    return x.astype(np.float16), w.astype(np.float16)


# --------------------------------------------------------------------------
# separable filter (a row of the paper's GPU speed-up table: k = 3 and k = 30; the image
# size is not given there: four full-HD fp32 planes here, normalised Gaussian taps)
# --------------------------------------------------------------------------
@dataclass(frozen=True)
class SepWorkload:
    name: str
    N: int
    H: int
    W: int
    k: int


CFG_SEP_K3 = SepWorkload("sepfilter_4x1080x1920_k3", 4, 1080, 1920, 3)
CFG_SEP_K30 = SepWorkload("sepfilter_4x1080x1920_k30", 4, 1080, 1920, 30)


def make_sepfilter_inputs(wl: SepWorkload, seed: int | None = None, N: int | None = None):
    """(x fp32 [N,H,W] uniform in [0,255], kx, ky fp32 [k]: Gaussians of sigma k/6 and k/4, sum 1)."""
    rng = np.random.default_rng(BASE_SEED + 9 if seed is None else seed)
    n = wl.N if N is None else N
    x = rng.uniform(0.0, 255.0, size=(n, wl.H, wl.W)).astype(np.float32)
    a = np.arange(wl.k, dtype=np.float64) - wl.k // 2
    taps = []
    for sigma in (max(wl.k / 6.0, 0.5), max(wl.k / 4.0, 0.5)):
        g = np.exp(-0.5 * (a / sigma) ** 2)
        taps.append((g / g.sum()).astype(np.float32))
    return x, taps[0], taps[1]


# --------------------------------------------------------------------------
# bilateral filter (Section VI-A, Listings 2 and 3; the image size and the constants are not
# given there: one full-HD fp32 plane, a 9 x 9 window, sigma_s = 3, sigma_r = 25 on a 0..255
# range here).  The image is smooth regions with steps plus noise, so that both regimes of
# the range term (weights near 1 and weights near 0) occur.
# --------------------------------------------------------------------------
@dataclass(frozen=True)
class BilateralWorkload:
    name: str
    N: int
    H: int
    W: int
    k: int
    sigma_s: float
    sigma_r: float

    @property
    def norm(self) -> float:
        return -1.0 / (2.0 * self.sigma_r * self.sigma_r)


CFG_BILATERAL = BilateralWorkload("bilateral_1x1080x1920_k9", 1, 1080, 1920, 9, 3.0, 25.0)


def make_bilateral_inputs(wl: BilateralWorkload, seed: int | None = None, N: int | None = None):
    """(x fp32 [N,H,W] in [0,255], g fp32 [k]: the spatial lookup table, used for both axes)."""
    rng = np.random.default_rng(BASE_SEED + 10 if seed is None else seed)
    n = wl.N if N is None else N
    coarse = rng.integers(0, 4, size=(n, -(-wl.H // 40), -(-wl.W // 40))) * 60.0 + 30.0    # piecewise constant
    x = np.repeat(np.repeat(coarse, 40, axis=1), 40, axis=2)[:, :wl.H, :wl.W]
    x = np.clip(x + rng.normal(0.0, 8.0, size=x.shape), 0.0, 255.0).astype(np.float32)
    a = np.arange(wl.k, dtype=np.float64) - wl.k // 2
    g = np.exp(-0.5 * (a / wl.sigma_s) ** 2).astype(np.float32)
    return x, g
