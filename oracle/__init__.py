"""CPU oracle for the MERIT hot path -- TEST INFRASTRUCTURE ONLY.

`merit_oracle.c` holds the plain nested-loop definitions (conv2d, pool2d,
sad_search); this module compiles it with gcc into `libmerit_oracle.so` and
wraps it with ctypes over numpy arrays.  `merit_literal.py` is a second,
separately written evaluator that materialises the transformed tensors of
Section III-C, Eq. 5 literally and reduces their rows (tiny inputs only).

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import
this package.  It never imports the HIP package, and the HIP package never
imports it.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "merit_oracle.c")
_LIB = os.path.join(_HERE, "libmerit_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain C, -O2, OpenMP over the outer loop)."""
    if (not force and os.path.exists(_LIB)
            and os.path.getmtime(_LIB) >= os.path.getmtime(_SRC)):
        return _LIB
    cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp",
           "-ffp-contract=off", "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
    subprocess.run(cmd, check=True)
    return _LIB


def build_sanitized_check() -> str:
    """merit_oracle.c + oracle_check.c under AddressSanitizer and UBSan, as an executable."""
    exe = os.path.join(_HERE, "oracle_check_asan")
    chk = os.path.join(_HERE, "oracle_check.c")
    if os.path.exists(exe) and os.path.getmtime(exe) >= max(os.path.getmtime(_SRC), os.path.getmtime(chk)):
        return exe
    cmd = ["gcc", "-O1", "-g", "-std=c11", "-fopenmp", "-ffp-contract=off", "-fsanitize=address,undefined",
           "-fno-sanitize-recover=all", "-static-libasan", "-Wall", "-Wextra", "-o", exe, _SRC, chk, "-lm"]
    subprocess.run(cmd, check=True)
    return exe


def _load():
    global _lib
    if _lib is not None:
        return _lib
    build()
    lib = ctypes.CDLL(_LIB)
    c_int = ctypes.c_int
    vp = ctypes.c_void_p
    lib.ref_half_to_double.restype = ctypes.c_double
    lib.ref_half_to_double.argtypes = [ctypes.c_uint16]
    lib.ref_double_to_half.restype = ctypes.c_uint16
    lib.ref_double_to_half.argtypes = [ctypes.c_double]
    lib.ref_conv2d.restype = c_int
    lib.ref_conv2d.argtypes = [vp, vp, vp] + [c_int] * 11
    lib.ref_conv2d_relu.restype = c_int
    lib.ref_conv2d_relu.argtypes = [vp, vp, vp] + [c_int] * 11
    lib.ref_conv2d_depthwise.restype = c_int
    lib.ref_conv2d_depthwise.argtypes = [vp, vp, vp] + [c_int] * 10
    lib.ref_correlation.restype = c_int
    lib.ref_correlation.argtypes = [vp, vp, vp] + [c_int] * 6
    lib.ref_conv2d_dilated.restype = c_int
    lib.ref_conv2d_dilated.argtypes = [vp, vp, vp] + [c_int] * 14
    lib.ref_bilateral.restype = c_int
    lib.ref_bilateral.argtypes = [vp, vp, vp, vp] + [c_int] * 4 + [ctypes.c_double]
    lib.ref_sepfilter.restype = c_int
    lib.ref_sepfilter.argtypes = [vp, vp, vp, vp] + [c_int] * 4
    lib.ref_conv2d_residual.restype = c_int
    lib.ref_conv2d_residual.argtypes = [vp, vp, vp, vp] + [c_int] * 12
    lib.ref_pool2d.restype = c_int
    lib.ref_pool2d.argtypes = [vp, vp] + [c_int] * 11
    lib.ref_sad_search.restype = c_int
    lib.ref_sad_search.argtypes = [vp, vp, vp, vp] + [c_int] * 4
    lib.ref_sad_surface.restype = c_int
    lib.ref_sad_surface.argtypes = [vp, vp, vp] + [c_int] * 6
    lib.ref_sad_candidate.restype = ctypes.c_int32
    lib.ref_sad_candidate.argtypes = [vp, vp] + [c_int] * 7
    lib.ref_num_threads.restype = c_int
    lib.ref_set_num_threads.argtypes = [c_int]
    _lib = lib
    return lib


def _ptr(a: np.ndarray):
    return ctypes.c_void_p(a.ctypes.data)


def _c(a, dtype):
    a = np.ascontiguousarray(a)
    if a.dtype != dtype:
        raise TypeError(f"expected {dtype}, got {a.dtype}")
    return a


def num_threads() -> int:
    return int(_load().ref_num_threads())


def set_num_threads(n: int) -> None:
    _load().ref_set_num_threads(int(n))


def half_to_double(bits: int) -> float:
    return float(_load().ref_half_to_double(int(bits)))


def double_to_half(v: float) -> int:
    return int(_load().ref_double_to_half(float(v)))


def out_extent(I: int, k: int, s: int, p: int) -> int:
    """floor((I + 2p - k) / s) + 1 -- number of window positions along one axis."""
    return (I + 2 * p - k) // s + 1


def conv2d(x: np.ndarray, w: np.ndarray, stride=(1, 1), pad=(0, 0), relu=False, dilation=(1, 1)) -> np.ndarray:
    """x fp16 [N,Cin,H,W], w fp16 [Cout,Cin,kh,kw] -> fp16 [N,Cout,OH,OW]; relu: the
    product function max(v1.v2, 0) of Section III-B instead of the plain dot product;
    dilation: input rows / columns per step of the window indices (Section III-C)."""
    x = _c(x, np.float16)
    w = _c(w, np.float16)
    N, Cin, H, W = x.shape
    Cout, Cin2, kh, kw = w.shape
    if Cin2 != Cin:
        raise ValueError("channel mismatch")
    sh, sw = stride
    ph, pw = pad
    dh, dw = dilation
    y = np.empty((N, Cout, out_extent(H, (kh - 1) * dh + 1, sh, ph), out_extent(W, (kw - 1) * dw + 1, sw, pw)),
                 np.float16)
    if (dh, dw) == (1, 1):
        fn = _load().ref_conv2d_relu if relu else _load().ref_conv2d
        rc = fn(_ptr(x), _ptr(w), _ptr(y), N, Cin, H, W, Cout, kh, kw, sh, sw, ph, pw)
    else:
        rc = _load().ref_conv2d_dilated(_ptr(x), _ptr(w), _ptr(y), N, Cin, H, W, Cout, kh, kw, sh, sw, ph, pw,
                                        dh, dw, 1 if relu else 0)
    if rc != 0:
        raise ValueError("ref_conv2d: bad shape")
    return y


def conv2d_residual(x: np.ndarray, w: np.ndarray, r: np.ndarray, stride=(1, 1), pad=(0, 0), relu=False) -> np.ndarray:
    """Residual layer (Section III-B, remark after Listing 1): r fp16 [N,Cout,OH,OW] is added to
    the exact sum in PostLoop, before the optional clip and the one rounding to fp16."""
    x = _c(x, np.float16)
    w = _c(w, np.float16)
    r = _c(r, np.float16)
    N, Cin, H, W = x.shape
    Cout, Cin2, kh, kw = w.shape
    if Cin2 != Cin:
        raise ValueError("channel mismatch")
    sh, sw = stride
    ph, pw = pad
    shape = (N, Cout, out_extent(H, kh, sh, ph), out_extent(W, kw, sw, pw))
    if r.shape != shape:
        raise ValueError("residual tensor must have the output's shape")
    y = np.empty(shape, np.float16)
    if _load().ref_conv2d_residual(_ptr(x), _ptr(w), _ptr(r), _ptr(y), N, Cin, H, W, Cout, kh, kw, sh, sw, ph, pw,
                                   1 if relu else 0) != 0:
        raise ValueError("ref_conv2d_residual: bad shape")
    return y


def conv2d_pool(x: np.ndarray, w: np.ndarray, stride=(1, 1), pad=(0, 0), relu=True) -> np.ndarray:
    """Convolution (optionally with the clipped product function) followed by 3x3 / stride 2 /
    pad 1 max pooling of its binary16 results: two ranged inner products in a row, each as
    defined above (the maximum of binary16 values is exact, so nothing else is rounded)."""
    y = conv2d(x, w, stride, pad, relu=relu)
    return pool2d(y.astype(np.float32), (3, 3), (2, 2), (1, 1), "max").astype(np.float16)


def conv2d_depthwise(x: np.ndarray, w: np.ndarray, stride=(1, 1), pad=(0, 0)) -> np.ndarray:
    """x fp16 [N,C,H,W], w fp16 [C,kh,kw] (one kernel per channel) -> fp16 [N,C,OH,OW]."""
    x = _c(x, np.float16)
    w = _c(w, np.float16)
    N, C, H, W = x.shape
    if w.ndim != 3 or w.shape[0] != C:
        raise ValueError("channel mismatch")
    _, kh, kw = w.shape
    sh, sw = stride
    ph, pw = pad
    y = np.empty((N, C, out_extent(H, kh, sh, ph), out_extent(W, kw, sw, pw)), np.float16)
    if _load().ref_conv2d_depthwise(_ptr(x), _ptr(w), _ptr(y), N, C, H, W, kh, kw, sh, sw, ph, pw) != 0:
        raise ValueError("ref_conv2d_depthwise: bad shape")
    return y


def correlation(x1: np.ndarray, x2: np.ndarray, search: int, stride: int = 1) -> np.ndarray:
    """Correlation layer (Section III-C, Eq. 8): x1, x2 fp16 [N,C,H,W] -> fp16 [N,H,W,n,n],
    n = 2*search + 1, displacement (p3 - search)*stride rows, (p4 - search)*stride columns."""
    x1 = _c(x1, np.float16)
    x2 = _c(x2, np.float16)
    if x1.shape != x2.shape or x1.ndim != 4:
        raise ValueError("shape mismatch")
    N, C, H, W = x1.shape
    n = 2 * search + 1
    y = np.empty((N, H, W, n, n), np.float16)
    if _load().ref_correlation(_ptr(x1), _ptr(x2), _ptr(y), N, C, H, W, search, stride) != 0:
        raise ValueError("ref_correlation: bad shape")
    return y


def pool2d(x: np.ndarray, kernel=(3, 3), stride=(2, 2), pad=(1, 1), mode="max") -> np.ndarray:
    """x fp32 [N,C,H,W] -> fp32 [N,C,OH,OW]; mode 'max' or 'avg' (padding excluded)."""
    x = _c(x, np.float32)
    N, C, H, W = x.shape
    kh, kw = kernel
    sh, sw = stride
    ph, pw = pad
    y = np.empty((N, C, out_extent(H, kh, sh, ph), out_extent(W, kw, sw, pw)), np.float32)
    rc = _load().ref_pool2d(_ptr(x), _ptr(y), N, C, H, W, kh, kw, sh, sw, ph, pw,
                            {"max": 0, "avg": 1}[mode])
    if rc != 0:
        raise ValueError("ref_pool2d: bad shape")
    return y


def sepfilter(x: np.ndarray, kx: np.ndarray, ky: np.ndarray) -> np.ndarray:
    """Separable filter: x fp32 [N,H,W], kx (along W) and ky (along H) fp32 [k] -> fp32 [N,H,W];
    window offset -k//2, no flip, coordinates clamped to the image."""
    x = _c(x, np.float32)
    kx = _c(kx, np.float32)
    ky = _c(ky, np.float32)
    if x.ndim != 3 or kx.ndim != 1 or ky.shape != kx.shape:
        raise ValueError("sepfilter: x must be [N,H,W], kx and ky vectors of one length")
    N, H, W = x.shape
    y = np.empty_like(x)
    if _load().ref_sepfilter(_ptr(x), _ptr(kx), _ptr(ky), _ptr(y), N, H, W, kx.shape[0]) != 0:
        raise ValueError("ref_sepfilter: bad shape")
    return y


def bilateral(x: np.ndarray, gx: np.ndarray, gy: np.ndarray, norm: float) -> np.ndarray:
    """Bilateral filter (Section VI-A, Listings 2 and 3): x fp32 [N,H,W]; gx, gy: spatial lookup
    tables fp32 [k]; norm: the range constant (weight exp(d*d*norm) for a pixel difference d).
    Window offset -k//2, coordinates clamped to the image."""
    x = _c(x, np.float32)
    gx = _c(gx, np.float32)
    gy = _c(gy, np.float32)
    if x.ndim != 3 or gx.ndim != 1 or gy.shape != gx.shape:
        raise ValueError("bilateral: x must be [N,H,W], gx and gy vectors of one length")
    N, H, W = x.shape
    y = np.empty_like(x)
    if _load().ref_bilateral(_ptr(x), _ptr(gx), _ptr(gy), _ptr(y), N, H, W, gx.shape[0], float(norm)) != 0:
        raise ValueError("ref_bilateral: bad shape")
    return y


def sad_search(cur: np.ndarray, ref: np.ndarray, block: int, search: int):
    """cur, ref u8 [H,W] -> (sad int32 [nby,nbx], mv int32 [nby,nbx,2] = (dy,dx));
    nby = ceil(H / block), nbx = ceil(W / block): blocks that reach past the edge read both
    frames with clamped coordinates."""
    cur = _c(cur, np.uint8)
    ref = _c(ref, np.uint8)
    H, W = cur.shape
    if ref.shape != (H, W):
        raise ValueError("frame shape mismatch")
    nby, nbx = -(-H // block), -(-W // block)
    sad = np.empty((nby, nbx), np.int32)
    mv = np.empty((nby, nbx, 2), np.int32)
    rc = _load().ref_sad_search(_ptr(cur), _ptr(ref), _ptr(sad), _ptr(mv), H, W, block, search)
    if rc != 0:
        raise ValueError("ref_sad_search: bad shape")
    return sad, mv


def sad_surface(cur: np.ndarray, ref: np.ndarray, block: int, search: int, by: int, bx: int):
    """All candidate SADs of one block as int32 [(2R+1),(2R+1)] indexed [dy+R, dx+R]."""
    cur = _c(cur, np.uint8)
    ref = _c(ref, np.uint8)
    H, W = cur.shape
    n = 2 * search + 1
    out = np.empty((n, n), np.int32)
    rc = _load().ref_sad_surface(_ptr(cur), _ptr(ref), _ptr(out), H, W, block, search, by, bx)
    if rc != 0:
        raise ValueError("ref_sad_surface: bad arguments")
    return out
