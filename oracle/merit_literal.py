"""Literal evaluator of the MERIT transform -- TEST INFRASTRUCTURE ONLY.

A second opinion on `merit_oracle.c`, written separately from it: instead of
nested loops per operation, it *materialises* the transformed tensors

    M(A)[p, a] = A[x],   x_i = sum_j delta(i, d_j) * (k_j * s_j + o_j),  k = (p, a)
                                                     (Section III-C, Eq. 5)

for both operands as 2-D arrays (rows p = parallelism, columns a = accumulation,
Section III-C) and then applies the product function to every row pair
(Section III, Eq. 1).  Memory grows as |p|*|a|, so this is for tiny inputs.

Also here: the minimal covering sub-tensor of a tile (Section IV-A, Eq. 9).
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Sequence

import numpy as np

UNUSED = -1   # an index k_j that does not move along any axis of this tensor


@dataclass
class Transform:
    """Per-index (axis d_j, stride s_j, offset o_j) triples for one tensor."""
    axis: Sequence[int]
    stride: Sequence[int]
    offset: Sequence[int]


def coordinates(ranges: Sequence[int], t: Transform, ndim: int) -> np.ndarray:
    """x[i][k] for every k in NDRange(ranges): int64 array [ndim, *ranges]."""
    J = len(ranges)
    assert len(t.axis) == len(t.stride) == len(t.offset) == J
    k = np.indices(tuple(ranges), dtype=np.int64)            # [J, *ranges]
    x = np.zeros((ndim,) + tuple(ranges), dtype=np.int64)
    for i in range(ndim):
        for j in range(J):
            if t.axis[j] == i:                               # Kronecker delta(i, d_j)
                x[i] += k[j] * t.stride[j] + t.offset[j]
    return x


def transform(A: np.ndarray, ranges: Sequence[int], t: Transform, n_par: int, pad: str):
    """Materialise M(A) as [prod(p-ranges), prod(a-ranges)] plus an in-range mask.

    pad: what an out-of-range coordinate yields --
      'zero'   the value 0            (convolution)
      'ninf'   -infinity              (max pooling)
      'exclude' value 0, mask False   (average pooling: not counted)
      'clamp'  the nearest in-range element (border replication; block matching)
    """
    x = coordinates(ranges, t, A.ndim)
    inside = np.ones(tuple(ranges), dtype=bool)
    for i in range(A.ndim):
        inside &= (x[i] >= 0) & (x[i] < A.shape[i])
    xc = [np.clip(x[i], 0, A.shape[i] - 1) for i in range(A.ndim)]
    vals = A[tuple(xc)]
    if pad == "clamp":
        inside[...] = True
    elif pad in ("zero", "exclude"):
        vals = np.where(inside, vals, np.zeros((), dtype=vals.dtype))
    elif pad == "ninf":
        vals = np.where(inside, vals, -np.inf)
    else:
        raise ValueError(pad)
    P = int(np.prod(ranges[:n_par], dtype=np.int64))
    Acc = int(np.prod(ranges[n_par:], dtype=np.int64))
    return vals.reshape(P, Acc), inside.reshape(P, Acc)


def footprint(tile: Sequence[int], t: Transform, ndim: int):
    """Size of the minimal sub-tensor of A containing a (t_p, t_a) tile of M(A):
    1 + sum_j (t_j - 1) * s_j * delta(d_j, i) along axis i   (Section IV-A, Eq. 9)."""
    out = []
    for i in range(ndim):
        n = 1
        for j, tj in enumerate(tile):
            if t.axis[j] == i:
                n += (tj - 1) * t.stride[j]
        out.append(n)
    return tuple(out)


# --------------------------------------------------------------------------
# the three operations as (ranges, transforms)
# --------------------------------------------------------------------------
def conv2d_desc(N, Cin, H, W, Cout, kh, kw, sh, sw, ph, pw, dh=1, dw=1):
    """k = (n, co, oy, ox | ci, ky, kx), after the strided example of Eq. 6; the window
    indices step dh rows / dw columns (the dilated example that follows it)."""
    OH = (H + 2 * ph - ((kh - 1) * dh + 1)) // sh + 1
    OW = (W + 2 * pw - ((kw - 1) * dw + 1)) // sw + 1
    ranges = (N, Cout, OH, OW, Cin, kh, kw)
    tx = Transform(axis=(0, UNUSED, 2, 3, 1, 2, 3),
                   stride=(1, 0, sh, sw, 1, dh, dw),
                   offset=(0, 0, 0, 0, 0, -ph, -pw))
    tw = Transform(axis=(UNUSED, 0, UNUSED, UNUSED, 1, 2, 3),
                   stride=(0, 1, 0, 0, 1, 1, 1),
                   offset=(0,) * 7)
    return ranges, 4, tx, tw


def pool2d_desc(N, C, H, W, kh, kw, sh, sw, ph, pw):
    """k = (n, c, oy, ox | ky, kx); one operand."""
    OH = (H + 2 * ph - kh) // sh + 1
    OW = (W + 2 * pw - kw) // sw + 1
    ranges = (N, C, OH, OW, kh, kw)
    tx = Transform(axis=(0, 1, 2, 3, 2, 3),
                   stride=(1, 1, sh, sw, 1, 1),
                   offset=(0, 0, 0, 0, -ph, -pw))
    return ranges, 4, tx


def sad_desc(H, W, B, R):
    """k = (by, bx | dy, dx, i, j): the reference frame is displaced by the
    search indices (the index pattern of the correlation layer, Eq. 8)."""
    n = 2 * R + 1
    ranges = (-(-H // B), -(-W // B), n, n, B, B)           # blocks past the edge read clamped
    tref = Transform(axis=(0, 1, 0, 1, 0, 1),
                     stride=(B, B, 1, 1, 1, 1),
                     offset=(0, 0, -R, -R, 0, 0))
    tcur = Transform(axis=(0, 1, UNUSED, UNUSED, 0, 1),
                     stride=(B, B, 0, 0, 1, 1),
                     offset=(0,) * 6)
    return ranges, 2, tref, tcur


# --------------------------------------------------------------------------
# row-wise reductions R(M(A), M(B), (.))
# --------------------------------------------------------------------------
def conv2d(x: np.ndarray, w: np.ndarray, stride=(1, 1), pad=(0, 0), relu=False, dilation=(1, 1),
           residual=None) -> np.ndarray:
    N, Cin, H, W = x.shape
    Cout, _, kh, kw = w.shape
    ranges, n_par, tx, tw = conv2d_desc(N, Cin, H, W, Cout, kh, kw, *stride, *pad, *dilation)
    MA, _ = transform(x.astype(np.float64), ranges, tx, n_par, "zero")
    MB, _ = transform(w.astype(np.float64), ranges, tw, n_par, "zero")
    rows = np.einsum("pa,pa->p", MA, MB)                    # v1^T v2 per row
    if residual is not None:                                # a loaded tensor added in PostLoop: row p gets r[p]
        rows = rows + residual.astype(np.float64).reshape(-1)
    if relu:
        rows = np.maximum(rows, 0.0)                        # max(v1^T v2, 0), Section III-B
    return rows.reshape(ranges[:4]).astype(np.float16)


def pool2d(x: np.ndarray, kernel=(3, 3), stride=(2, 2), pad=(1, 1), mode="max") -> np.ndarray:
    N, C, H, W = x.shape
    ranges, n_par, tx = pool2d_desc(N, C, H, W, *kernel, *stride, *pad)
    if mode == "max":
        MA, _ = transform(x.astype(np.float64), ranges, tx, n_par, "ninf")
        rows = MA.max(axis=1)
    elif mode == "avg":
        MA, inside = transform(x.astype(np.float64), ranges, tx, n_par, "exclude")
        cnt = inside.sum(axis=1)
        rows = np.where(cnt > 0, MA.sum(axis=1) / np.maximum(cnt, 1), 0.0)
    else:
        raise ValueError(mode)
    return rows.reshape(ranges[:4]).astype(np.float32)


def depthwise_desc(N, C, H, W, kh, kw, sh, sw, ph, pw):
    """k = (n, c, oy, ox | ky, kx): the input as in pooling, the weights w[c, ky, kx]."""
    OH = (H + 2 * ph - kh) // sh + 1
    OW = (W + 2 * pw - kw) // sw + 1
    ranges = (N, C, OH, OW, kh, kw)
    tx = Transform(axis=(0, 1, 2, 3, 2, 3), stride=(1, 1, sh, sw, 1, 1), offset=(0, 0, 0, 0, -ph, -pw))
    tw = Transform(axis=(UNUSED, 0, UNUSED, UNUSED, 1, 2), stride=(0, 1, 0, 0, 1, 1), offset=(0,) * 6)
    return ranges, 4, tx, tw


def conv2d_depthwise(x: np.ndarray, w: np.ndarray, stride=(1, 1), pad=(0, 0)) -> np.ndarray:
    N, C, H, W = x.shape
    _, kh, kw = w.shape
    ranges, n_par, tx, tw = depthwise_desc(N, C, H, W, kh, kw, *stride, *pad)
    MA, _ = transform(x.astype(np.float64), ranges, tx, n_par, "zero")
    MB, _ = transform(w.astype(np.float64), ranges, tw, n_par, "zero")
    return np.einsum("pa,pa->p", MA, MB).reshape(ranges[:4]).astype(np.float16)


def correlation_desc(N, C, H, W, R, sd):
    """k = (b, p1, p2, p3, p4 | a1), Eq. 8: the second tensor moves with p1 + p3 and p2 + p4
    (two indices on one axis); displacements centred: offset -R*sd, stride sd."""
    n = 2 * R + 1
    ranges = (N, H, W, n, n, C)
    t1 = Transform(axis=(0, 2, 3, UNUSED, UNUSED, 1), stride=(1, 1, 1, 0, 0, 1), offset=(0,) * 6)
    t2 = Transform(axis=(0, 2, 3, 2, 3, 1), stride=(1, 1, 1, sd, sd, 1), offset=(0, 0, 0, -R * sd, -R * sd, 0))
    return ranges, 5, t1, t2


def correlation(x1: np.ndarray, x2: np.ndarray, search: int, stride: int = 1) -> np.ndarray:
    N, C, H, W = x1.shape
    ranges, n_par, t1, t2 = correlation_desc(N, C, H, W, search, stride)
    M1, _ = transform(x1.astype(np.float64), ranges, t1, n_par, "zero")
    M2, _ = transform(x2.astype(np.float64), ranges, t2, n_par, "zero")
    rows = np.einsum("pa,pa->p", M1, M2)
    return rows.reshape(ranges[:5]).astype(np.float16)


def sad_search(cur: np.ndarray, ref: np.ndarray, block: int, search: int):
    H, W = cur.shape
    ranges, n_par, tref, tcur = sad_desc(H, W, block, search)
    Mref, _ = transform(ref.astype(np.int64), ranges, tref, n_par, "clamp")
    Mcur, _ = transform(cur.astype(np.int64), ranges, tcur, n_par, "clamp")
    nby, nbx, n, _, B, _ = ranges
    # inner level: L1 distance over the block pixels (i, j)
    l1 = np.abs(Mcur - Mref).reshape(nby * nbx, n * n, B * B).sum(axis=2)
    # outer level: min over the candidates; argmin returns the first (lowest
    # raster index) minimiser
    idx = np.argmin(l1, axis=1)
    sad = l1[np.arange(nby * nbx), idx].astype(np.int32).reshape(nby, nbx)
    mv = np.stack([idx // n - search, idx % n - search], axis=1).astype(np.int32)
    return sad, mv.reshape(nby, nbx, 2)


# --------------------------------------------------------------------------
# separable filter: two 1-D ranged inner products in a row
# --------------------------------------------------------------------------
def sepfilter_desc(N, H, W, k):
    """Row pass k = (n, p1, p2 | a2) on the image, column pass k = (n, p1, p2 | a1) on its
    result; window offset -k//2 as in the bilateral-filter call of Section VI-A."""
    ranges = (N, H, W, k)
    t_row = Transform(axis=(0, 1, 2, 2), stride=(1, 1, 1, 1), offset=(0, 0, 0, -(k // 2)))
    t_col = Transform(axis=(0, 1, 2, 1), stride=(1, 1, 1, 1), offset=(0, 0, 0, -(k // 2)))
    t_ker = Transform(axis=(UNUSED, UNUSED, UNUSED, 0), stride=(0, 0, 0, 1), offset=(0, 0, 0, 0))
    return ranges, 3, t_row, t_col, t_ker


def sepfilter(x: np.ndarray, kx: np.ndarray, ky: np.ndarray) -> np.ndarray:
    N, H, W = x.shape
    ranges, n_par, t_row, t_col, t_ker = sepfilter_desc(N, H, W, len(kx))
    MA, _ = transform(x.astype(np.float64), ranges, t_row, n_par, "clamp")
    MB, _ = transform(kx.astype(np.float64), ranges, t_ker, n_par, "clamp")
    t = np.einsum("pa,pa->p", MA, MB).reshape(N, H, W)
    MA, _ = transform(t, ranges, t_col, n_par, "clamp")
    MB, _ = transform(ky.astype(np.float64), ranges, t_ker, n_par, "clamp")
    return np.einsum("pa,pa->p", MA, MB).reshape(N, H, W).astype(np.float32)
