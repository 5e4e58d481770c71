"""ctypes binding of libmerit.so -- argument marshalling only.

Function names mirror include/merit.h.  Tensors are torch CUDA (ROCm) tensors:
PyTorch provides device memory and the current HIP stream, nothing else; every
step of the computation runs in the library's kernels.  There is no fallback:
if the library is missing or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes
import os

from . import build as _build

MERIT_MAX_INDEX = 12
MERIT_MAX_DIMS = 6
MERIT_AXIS_UNUSED = -1

MERIT_OK = 0
(MERIT_ERR_NULL, MERIT_ERR_INVALID_ARG, MERIT_ERR_SHAPE, MERIT_ERR_UNSUPPORTED,
 MERIT_ERR_ALIGNMENT, MERIT_ERR_HIP, MERIT_ERR_SCRATCH_LIMIT) = range(1, 8)
MERIT_NOALLOC_SCRATCH_BYTES = 8 << 20
(MERIT_OP_CONV_DOT, MERIT_OP_POOL_MAX, MERIT_OP_POOL_AVG, MERIT_OP_SAD_ARGMIN, MERIT_OP_CONV_DOT_RELU,
 MERIT_OP_CORR_DOT, MERIT_OP_DWCONV_DOT, MERIT_OP_CONV_DOT_POOLMAX, MERIT_OP_CONV_DOT_RELU_POOLMAX,
 MERIT_OP_CONV_DOT_ADD, MERIT_OP_CONV_DOT_ADD_RELU, MERIT_OP_SEPFILTER_DOT,
 MERIT_OP_BILATERAL) = range(13)
MERIT_U8, MERIT_F16, MERIT_F32 = range(3)
MERIT_PAD_ZERO, MERIT_PAD_NEG_INF, MERIT_PAD_EXCLUDE, MERIT_PAD_CLAMP = range(4)


class MeritError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = lib().merit_status_string(status).decode() if _lib is not None else str(status)
        super().__init__(f"{where}: {msg} (merit_status {status})")


class merit_operand(ctypes.Structure):
    _fields_ = [("ndim", ctypes.c_int32),
                ("shape", ctypes.c_int64 * MERIT_MAX_DIMS),
                ("axis", ctypes.c_int32 * MERIT_MAX_INDEX),
                ("stride", ctypes.c_int64 * MERIT_MAX_INDEX),
                ("offset", ctypes.c_int64 * MERIT_MAX_INDEX)]


class merit_plan_desc(ctypes.Structure):
    _fields_ = [("op", ctypes.c_int), ("dtype", ctypes.c_int), ("pad", ctypes.c_int),
                ("n_par", ctypes.c_int32), ("n_acc", ctypes.c_int32),
                ("range", ctypes.c_int64 * MERIT_MAX_INDEX),
                ("a", merit_operand), ("b", merit_operand)]


class merit_launch_info(ctypes.Structure):
    _fields_ = [("kernel", ctypes.c_char_p),
                ("grid", ctypes.c_int64 * 3),
                ("block", ctypes.c_int32 * 3),
                ("lds_bytes", ctypes.c_int64),
                ("tile", ctypes.c_int64 * MERIT_MAX_INDEX)]


_lib = None


def lib_path() -> str:
    return _build.LIB_PATH


def lib():
    """Load libmerit.so (building it only if no built library exists)."""
    global _lib
    if _lib is not None:
        return _lib
    path = lib_path()
    if not os.path.exists(path):
        _build.build_library(force=True)
    L = ctypes.CDLL(path)
    P = ctypes.c_void_p
    c_int = ctypes.c_int
    PP = ctypes.POINTER(P)
    L.merit_plan_create.argtypes = [ctypes.POINTER(merit_plan_desc), PP]
    L.merit_plan_destroy.argtypes = [P]
    L.merit_plan_conv2d.argtypes = [c_int] * 11 + [PP]
    L.merit_plan_conv2d_relu.argtypes = [c_int] * 11 + [PP]
    L.merit_plan_conv2d_dilated.argtypes = [c_int] * 14 + [PP]
    L.merit_plan_conv2d_pool.argtypes = [c_int] * 12 + [PP]
    L.merit_plan_conv2d_residual.argtypes = [c_int] * 12 + [PP]
    L.merit_plan_sepfilter.argtypes = [c_int] * 4 + [PP]
    L.merit_sepfilter.argtypes = [P, P, P, P, P, P]
    L.merit_probe_copy.argtypes = [P, P, ctypes.c_size_t, P]
    L.merit_probe_alu.argtypes = [c_int, c_int, c_int, P, P]
    L.merit_plan_bilateral.argtypes = [c_int] * 4 + [PP]
    L.merit_bilateral.argtypes = [P, P, P, P, ctypes.c_double, P, P]
    L.merit_conv2d_residual.argtypes = [P, P, P, P, P, P]
    L.merit_plan_pool2d.argtypes = [c_int] * 11 + [PP]
    L.merit_plan_sad.argtypes = [c_int] * 4 + [PP]
    L.merit_plan_correlation.argtypes = [c_int] * 6 + [PP]
    L.merit_plan_conv2d_depthwise.argtypes = [c_int] * 10 + [PP]
    L.merit_conv2d_depthwise.argtypes = [P, P, P, P, P]
    L.merit_correlation.argtypes = [P, P, P, P, P]
    L.merit_plan_get_desc.argtypes = [P, ctypes.POINTER(merit_plan_desc)]
    L.merit_plan_out_shape.argtypes = [P, ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(ctypes.c_int64)]
    L.merit_plan_footprint.argtypes = [P, c_int, ctypes.POINTER(ctypes.c_int64), ctypes.POINTER(ctypes.c_int64)]
    L.merit_plan_launch_info.argtypes = [P, ctypes.POINTER(merit_launch_info)]
    L.merit_plan_set_tile.argtypes = [P, ctypes.POINTER(ctypes.c_int64)]
    L.merit_conv2d.argtypes = [P, P, P, P, P]
    L.merit_plan_packed_weights_bytes.argtypes = [P, ctypes.POINTER(ctypes.c_int64)]
    L.merit_conv2d_pack_weights.argtypes = [P, P, P, P]
    L.merit_conv2d_packed.argtypes = [P, P, P, P, P]
    L.merit_conv2d_packed_noalloc.argtypes = [P, P, P, P, P]
    L.merit_pool2d.argtypes = [P, P, P, P]
    L.merit_sad_search.argtypes = [P, P, P, P, P, P]
    for name in ("merit_plan_create", "merit_plan_destroy", "merit_plan_conv2d", "merit_plan_conv2d_relu",
                 "merit_plan_conv2d_dilated", "merit_plan_conv2d_pool", "merit_plan_conv2d_residual",
                 "merit_conv2d_residual", "merit_plan_sepfilter", "merit_sepfilter",
                 "merit_plan_bilateral", "merit_bilateral", "merit_probe_copy", "merit_probe_alu",
                 "merit_plan_pool2d",
                 "merit_plan_sad", "merit_plan_correlation", "merit_correlation", "merit_plan_conv2d_depthwise",
                 "merit_conv2d_depthwise", "merit_plan_get_desc", "merit_plan_out_shape", "merit_plan_footprint",
                 "merit_plan_launch_info", "merit_plan_set_tile", "merit_conv2d", "merit_pool2d",
                 "merit_sad_search", "merit_plan_packed_weights_bytes", "merit_conv2d_pack_weights",
                 "merit_conv2d_packed", "merit_conv2d_packed_noalloc"):
        getattr(L, name).restype = c_int
    L.merit_status_string.argtypes = [c_int]
    L.merit_status_string.restype = ctypes.c_char_p
    _lib = L
    return L


def _check(status: int, where: str):
    if status != MERIT_OK:
        raise MeritError(status, where)


class Plan:
    """Owner of one merit_plan handle."""

    def __init__(self, handle: ctypes.c_void_p):
        self._h = handle
        self._shapes = None

    def shapes(self):
        """(out_shape, a_shape, b_shape), computed once (a plan's shapes never change)."""
        if self._shapes is None:
            d = self.desc()
            self._shapes = (self.out_shape(), tuple(d.a.shape[:d.a.ndim]), tuple(d.b.shape[:d.b.ndim]))
        return self._shapes

    @property
    def handle(self):
        if not self._h:
            raise ValueError("plan already destroyed")
        return self._h

    def destroy(self):
        if self._h:
            lib().merit_plan_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass

    def desc(self) -> merit_plan_desc:
        d = merit_plan_desc()
        _check(lib().merit_plan_get_desc(self.handle, ctypes.byref(d)), "merit_plan_get_desc")
        return d

    def out_shape(self):
        nd = ctypes.c_int32()
        shp = (ctypes.c_int64 * MERIT_MAX_DIMS)()
        _check(lib().merit_plan_out_shape(self.handle, ctypes.byref(nd), shp), "merit_plan_out_shape")
        return tuple(shp[i] for i in range(nd.value))

    def footprint(self, which: int, tile):
        t = (ctypes.c_int64 * MERIT_MAX_INDEX)(*list(tile) + [0] * (MERIT_MAX_INDEX - len(tile)))
        out = (ctypes.c_int64 * MERIT_MAX_DIMS)()
        _check(lib().merit_plan_footprint(self.handle, which, t, out), "merit_plan_footprint")
        d = self.desc()
        nd = d.a.ndim if which == 0 else d.b.ndim
        return tuple(out[i] for i in range(nd))

    def launch_info(self) -> dict:
        li = merit_launch_info()
        _check(lib().merit_plan_launch_info(self.handle, ctypes.byref(li)), "merit_plan_launch_info")
        return {"kernel": li.kernel.decode(), "grid": tuple(li.grid), "block": tuple(li.block),
                "lds_bytes": li.lds_bytes, "tile": tuple(li.tile)}

    def set_tile(self, tile):
        t = (ctypes.c_int64 * MERIT_MAX_INDEX)(*list(tile) + [0] * (MERIT_MAX_INDEX - len(tile)))
        _check(lib().merit_plan_set_tile(self.handle, t), "merit_plan_set_tile")
        return self


def merit_plan_create(desc: merit_plan_desc) -> Plan:
    h = ctypes.c_void_p()
    _check(lib().merit_plan_create(ctypes.byref(desc), ctypes.byref(h)), "merit_plan_create")
    return Plan(h)


def merit_plan_conv2d(N, Cin, H, W, Cout, kh, kw, sh, sw, ph, pw) -> Plan:
    h = ctypes.c_void_p()
    _check(lib().merit_plan_conv2d(N, Cin, H, W, Cout, kh, kw, sh, sw, ph, pw, ctypes.byref(h)),
           "merit_plan_conv2d")
    return Plan(h)


def merit_plan_conv2d_relu(N, Cin, H, W, Cout, kh, kw, sh, sw, ph, pw) -> Plan:
    h = ctypes.c_void_p()
    _check(lib().merit_plan_conv2d_relu(N, Cin, H, W, Cout, kh, kw, sh, sw, ph, pw, ctypes.byref(h)),
           "merit_plan_conv2d_relu")
    return Plan(h)


def merit_plan_conv2d_dilated(N, Cin, H, W, Cout, kh, kw, sh, sw, ph, pw, dh, dw, relu=0) -> Plan:
    h = ctypes.c_void_p()
    _check(lib().merit_plan_conv2d_dilated(N, Cin, H, W, Cout, kh, kw, sh, sw, ph, pw, dh, dw, int(relu),
                                           ctypes.byref(h)), "merit_plan_conv2d_dilated")
    return Plan(h)


def merit_plan_conv2d_pool(N, Cin, H, W, Cout, kh, kw, sh, sw, ph, pw, relu=1) -> Plan:
    h = ctypes.c_void_p()
    _check(lib().merit_plan_conv2d_pool(N, Cin, H, W, Cout, kh, kw, sh, sw, ph, pw, int(relu), ctypes.byref(h)),
           "merit_plan_conv2d_pool")
    return Plan(h)


def merit_plan_conv2d_residual(N, Cin, H, W, Cout, kh, kw, sh, sw, ph, pw, relu=0) -> Plan:
    h = ctypes.c_void_p()
    _check(lib().merit_plan_conv2d_residual(N, Cin, H, W, Cout, kh, kw, sh, sw, ph, pw, int(relu), ctypes.byref(h)),
           "merit_plan_conv2d_residual")
    return Plan(h)


def merit_plan_pool2d(N, C, H, W, kh, kw, sh, sw, ph, pw, is_avg) -> Plan:
    h = ctypes.c_void_p()
    _check(lib().merit_plan_pool2d(N, C, H, W, kh, kw, sh, sw, ph, pw, int(bool(is_avg)), ctypes.byref(h)),
           "merit_plan_pool2d")
    return Plan(h)


def merit_plan_sad(H, W, block, search) -> Plan:
    h = ctypes.c_void_p()
    _check(lib().merit_plan_sad(H, W, block, search, ctypes.byref(h)), "merit_plan_sad")
    return Plan(h)


# --------------------------------------------------------------------------
# operations on torch device tensors
# --------------------------------------------------------------------------
def _dev_ptr(t, dtype, name):
    import torch
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise TypeError(f"{name}: expected a device tensor")
    if t.dtype != dtype:
        raise TypeError(f"{name}: expected {dtype}, got {t.dtype}")
    if not t.is_contiguous():
        raise ValueError(f"{name}: tensor must be contiguous")
    return ctypes.c_void_p(t.data_ptr())


def _stream(stream):
    import torch
    if stream is None:
        return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    if isinstance(stream, int):
        return ctypes.c_void_p(stream)
    return ctypes.c_void_p(stream.cuda_stream)


def merit_conv2d(plan: Plan, x, w, y=None, stream=None):
    import torch
    out_shape, a_shape, b_shape = plan.shapes()
    if y is None:
        y = torch.empty(out_shape, dtype=torch.float16, device=x.device)
    if tuple(y.shape) != out_shape:
        raise ValueError("y has the wrong shape")
    if tuple(x.shape) != a_shape or tuple(w.shape) != b_shape:
        raise ValueError("x / w do not match the plan")
    _check(lib().merit_conv2d(plan.handle, _dev_ptr(x, torch.float16, "x"), _dev_ptr(w, torch.float16, "w"),
                              _dev_ptr(y, torch.float16, "y"), _stream(stream)), "merit_conv2d")
    return y


def merit_plan_packed_weights_bytes(plan: Plan) -> int:
    n = ctypes.c_int64(0)
    _check(lib().merit_plan_packed_weights_bytes(plan.handle, ctypes.byref(n)), "merit_plan_packed_weights_bytes")
    return int(n.value)


def merit_conv2d_pack_weights(plan: Plan, w, packed=None, stream=None):
    import torch
    nbytes = merit_plan_packed_weights_bytes(plan)
    if tuple(w.shape) != plan.shapes()[2]:
        raise ValueError("w does not match the plan")
    if packed is None:
        packed = torch.empty(nbytes // 2, dtype=torch.float16, device=w.device)
    if packed.numel() * packed.element_size() != nbytes:
        raise ValueError("packed has the wrong size")
    _check(lib().merit_conv2d_pack_weights(plan.handle, _dev_ptr(w, torch.float16, "w"),
                                           _dev_ptr(packed, torch.float16, "packed"), _stream(stream)),
           "merit_conv2d_pack_weights")
    return packed


def merit_conv2d_packed(plan: Plan, x, packed, y=None, stream=None):
    import torch
    out_shape, a_shape, _ = plan.shapes()
    if y is None:
        y = torch.empty(out_shape, dtype=torch.float16, device=x.device)
    if tuple(y.shape) != out_shape or tuple(x.shape) != a_shape:
        raise ValueError("x / y do not match the plan")
    if packed.numel() * packed.element_size() != merit_plan_packed_weights_bytes(plan):
        raise ValueError("packed has the wrong size")
    _check(lib().merit_conv2d_packed(plan.handle, _dev_ptr(x, torch.float16, "x"),
                                     _dev_ptr(packed, torch.float16, "packed"), _dev_ptr(y, torch.float16, "y"),
                                     _stream(stream)), "merit_conv2d_packed")
    return y


def merit_conv2d_packed_noalloc(plan: Plan, x, w, y, stream=None):
    """No allocation anywhere: the caller passes every tensor, the packed weights live in the library."""
    import torch
    out_shape, a_shape, b_shape = plan.shapes()
    if tuple(y.shape) != out_shape or tuple(x.shape) != a_shape or tuple(w.shape) != b_shape:
        raise ValueError("tensors do not match the plan")
    _check(lib().merit_conv2d_packed_noalloc(plan.handle, _dev_ptr(x, torch.float16, "x"),
                                             _dev_ptr(w, torch.float16, "w"), _dev_ptr(y, torch.float16, "y"),
                                             _stream(stream)), "merit_conv2d_packed_noalloc")
    return y


def merit_conv2d_residual(plan: Plan, x, w, r, y=None, stream=None):
    import torch
    out_shape, a_shape, b_shape = plan.shapes()
    if y is None:
        y = torch.empty(out_shape, dtype=torch.float16, device=x.device)
    if tuple(y.shape) != out_shape or tuple(r.shape) != out_shape:
        raise ValueError("y / r have the wrong shape")
    if tuple(x.shape) != a_shape or tuple(w.shape) != b_shape:
        raise ValueError("x / w do not match the plan")
    _check(lib().merit_conv2d_residual(plan.handle, _dev_ptr(x, torch.float16, "x"), _dev_ptr(w, torch.float16, "w"),
                                       _dev_ptr(r, torch.float16, "r"), _dev_ptr(y, torch.float16, "y"),
                                       _stream(stream)), "merit_conv2d_residual")
    return y


def merit_pool2d(plan: Plan, x, y=None, stream=None):
    import torch
    out_shape, a_shape, _ = plan.shapes()
    if y is None:
        y = torch.empty(out_shape, dtype=torch.float32, device=x.device)
    if tuple(y.shape) != out_shape:
        raise ValueError("y has the wrong shape")
    if tuple(x.shape) != a_shape:
        raise ValueError("x does not match the plan")
    _check(lib().merit_pool2d(plan.handle, _dev_ptr(x, torch.float32, "x"), _dev_ptr(y, torch.float32, "y"),
                              _stream(stream)), "merit_pool2d")
    return y


def merit_sad_search(plan: Plan, cur, ref, sad=None, mv=None, stream=None):
    import torch
    (nby, nbx), a_shape, b_shape = plan.shapes()
    if sad is None:
        sad = torch.empty((nby, nbx), dtype=torch.int32, device=cur.device)
    if mv is None:
        mv = torch.empty((nby, nbx, 2), dtype=torch.int32, device=cur.device)
    if tuple(cur.shape) != b_shape or tuple(ref.shape) != a_shape:
        raise ValueError("frames do not match the plan")
    if tuple(sad.shape) != (nby, nbx) or tuple(mv.shape) != (nby, nbx, 2):
        raise ValueError("outputs have the wrong shape")
    _check(lib().merit_sad_search(plan.handle, _dev_ptr(cur, torch.uint8, "cur"), _dev_ptr(ref, torch.uint8, "ref"),
                                  _dev_ptr(sad, torch.int32, "sad"), _dev_ptr(mv, torch.int32, "mv"),
                                  _stream(stream)), "merit_sad_search")
    return sad, mv


def merit_plan_conv2d_depthwise(N, C, H, W, kh, kw, sh, sw, ph, pw) -> Plan:
    h = ctypes.c_void_p()
    _check(lib().merit_plan_conv2d_depthwise(N, C, H, W, kh, kw, sh, sw, ph, pw, ctypes.byref(h)),
           "merit_plan_conv2d_depthwise")
    return Plan(h)


def merit_conv2d_depthwise(plan: Plan, x, w, y=None, stream=None):
    import torch
    out_shape, a_shape, b_shape = plan.shapes()
    if y is None:
        y = torch.empty(out_shape, dtype=torch.float16, device=x.device)
    if tuple(x.shape) != a_shape or tuple(w.shape) != b_shape or tuple(y.shape) != out_shape:
        raise ValueError("tensors do not match the plan")
    _check(lib().merit_conv2d_depthwise(plan.handle, _dev_ptr(x, torch.float16, "x"), _dev_ptr(w, torch.float16, "w"),
                                        _dev_ptr(y, torch.float16, "y"), _stream(stream)), "merit_conv2d_depthwise")
    return y


def merit_plan_sepfilter(N, H, W, k) -> Plan:
    h = ctypes.c_void_p()
    _check(lib().merit_plan_sepfilter(N, H, W, k, ctypes.byref(h)), "merit_plan_sepfilter")
    return Plan(h)


def _sep_args(plan, x, kx, ky, y, stream):
    import torch
    out_shape, a_shape, b_shape = plan.shapes()
    if tuple(x.shape) != a_shape or tuple(y.shape) != out_shape or tuple(kx.shape) != b_shape \
            or tuple(ky.shape) != b_shape:
        raise ValueError("tensors do not match the plan")
    return (plan.handle, _dev_ptr(x, torch.float32, "x"), _dev_ptr(kx, torch.float32, "kx"),
            _dev_ptr(ky, torch.float32, "ky"), _dev_ptr(y, torch.float32, "y"), _stream(stream))


def merit_sepfilter(plan: Plan, x, kx, ky, y=None, stream=None):
    import torch
    if y is None:
        y = torch.empty(plan.out_shape(), dtype=torch.float32, device=x.device)
    _check(lib().merit_sepfilter(*_sep_args(plan, x, kx, ky, y, stream)), "merit_sepfilter")
    return y


def bind_sepfilter(plan: Plan, x, kx, ky, y, stream=None) -> BoundCall:
    return BoundCall(lib().merit_sepfilter, "merit_sepfilter", _sep_args(plan, x, kx, ky, y, stream),
                     (plan, x, kx, ky, y))


def merit_plan_bilateral(N, H, W, k) -> Plan:
    h = ctypes.c_void_p()
    _check(lib().merit_plan_bilateral(N, H, W, k, ctypes.byref(h)), "merit_plan_bilateral")
    return Plan(h)


def _bilateral_args(plan, x, gx, gy, norm, y, stream):
    import torch
    out_shape, a_shape, b_shape = plan.shapes()
    if tuple(x.shape) != a_shape or tuple(y.shape) != out_shape or tuple(gx.shape) != b_shape \
            or tuple(gy.shape) != b_shape:
        raise ValueError("tensors do not match the plan")
    return (plan.handle, _dev_ptr(x, torch.float32, "x"), _dev_ptr(gx, torch.float32, "gx"),
            _dev_ptr(gy, torch.float32, "gy"), ctypes.c_double(float(norm)), _dev_ptr(y, torch.float32, "y"),
            _stream(stream))


def merit_bilateral(plan: Plan, x, gx, gy, norm, y=None, stream=None):
    import torch
    if y is None:
        y = torch.empty(plan.out_shape(), dtype=torch.float32, device=x.device)
    _check(lib().merit_bilateral(*_bilateral_args(plan, x, gx, gy, norm, y, stream)), "merit_bilateral")
    return y


def bind_bilateral(plan: Plan, x, gx, gy, norm, y, stream=None) -> BoundCall:
    return BoundCall(lib().merit_bilateral, "merit_bilateral", _bilateral_args(plan, x, gx, gy, norm, y, stream),
                     (plan, x, gx, gy, y))


(MERIT_PROBE_MFMA_F16, MERIT_PROBE_FMA_F32, MERIT_PROBE_SAD_U8, MERIT_PROBE_EXP2_F32, MERIT_PROBE_MFMA_F16_RANDOM) = range(5)


def merit_probe_copy(src, dst, stream=None):
    """Streaming copy of one device tensor into another of the same size (peak probe)."""
    if src.numel() * src.element_size() != dst.numel() * dst.element_size():
        raise ValueError("sizes differ")
    _check(lib().merit_probe_copy(_dev_ptr(src, src.dtype, "src"), _dev_ptr(dst, dst.dtype, "dst"),
                                  src.numel() * src.element_size(), _stream(stream)), "merit_probe_copy")


def merit_probe_alu(which, workgroups, iters, sink, stream=None):
    """Instruction-rate probe: workgroups x 4 wavefronts x iters x 8 instructions of one kind."""
    import torch
    if sink.numel() < workgroups * 256:
        raise ValueError("sink too small")
    _check(lib().merit_probe_alu(which, workgroups, iters, _dev_ptr(sink, torch.int32, "sink"), _stream(stream)),
           "merit_probe_alu")


def merit_plan_correlation(N, C, H, W, R, sd=1) -> Plan:
    h = ctypes.c_void_p()
    _check(lib().merit_plan_correlation(N, C, H, W, R, sd, ctypes.byref(h)), "merit_plan_correlation")
    return Plan(h)


def merit_correlation(plan: Plan, x1, x2, y=None, stream=None):
    import torch
    out_shape, a_shape, b_shape = plan.shapes()
    if y is None:
        y = torch.empty(out_shape, dtype=torch.float16, device=x1.device)
    if tuple(x1.shape) != a_shape or tuple(x2.shape) != b_shape or tuple(y.shape) != out_shape:
        raise ValueError("tensors do not match the plan")
    _check(lib().merit_correlation(plan.handle, _dev_ptr(x1, torch.float16, "x1"), _dev_ptr(x2, torch.float16, "x2"),
                                   _dev_ptr(y, torch.float16, "y"), _stream(stream)), "merit_correlation")
    return y


# --------------------------------------------------------------------------
# pre-marshalled calls: validate tensors once, then re-issue the same C call
# with raw pointers (for tight loops where ~10 us of Python checks per call
# would exceed the kernel's own duration)
# --------------------------------------------------------------------------
class BoundCall:
    """The C entry point plus its marshalled arguments; calling it enqueues one launch."""

    def __init__(self, fn, name, args, keep):
        self._fn, self._name, self._args, self._keep = fn, name, args, keep

    def __call__(self):
        st = self._fn(*self._args)
        if st != MERIT_OK:
            raise MeritError(st, self._name)


def bind_conv2d(plan: Plan, x, w, y, stream=None) -> BoundCall:
    import torch
    out_shape, a_shape, b_shape = plan.shapes()
    if tuple(y.shape) != out_shape or tuple(x.shape) != a_shape or tuple(w.shape) != b_shape:
        raise ValueError("tensors do not match the plan")
    args = (plan.handle, _dev_ptr(x, torch.float16, "x"), _dev_ptr(w, torch.float16, "w"),
            _dev_ptr(y, torch.float16, "y"), _stream(stream))
    return BoundCall(lib().merit_conv2d, "merit_conv2d", args, (plan, x, w, y))


def bind_conv2d_packed(plan: Plan, x, packed, y, stream=None) -> BoundCall:
    import torch
    out_shape, a_shape, _ = plan.shapes()
    if tuple(y.shape) != out_shape or tuple(x.shape) != a_shape:
        raise ValueError("tensors do not match the plan")
    if packed.numel() * packed.element_size() != merit_plan_packed_weights_bytes(plan):
        raise ValueError("packed has the wrong size")
    args = (plan.handle, _dev_ptr(x, torch.float16, "x"), _dev_ptr(packed, torch.float16, "packed"),
            _dev_ptr(y, torch.float16, "y"), _stream(stream))
    return BoundCall(lib().merit_conv2d_packed, "merit_conv2d_packed", args, (plan, x, packed, y))


def bind_conv2d_residual(plan: Plan, x, w, r, y, stream=None) -> BoundCall:
    import torch
    out_shape, a_shape, b_shape = plan.shapes()
    if (tuple(y.shape) != out_shape or tuple(r.shape) != out_shape or tuple(x.shape) != a_shape
            or tuple(w.shape) != b_shape):
        raise ValueError("tensors do not match the plan")
    args = (plan.handle, _dev_ptr(x, torch.float16, "x"), _dev_ptr(w, torch.float16, "w"),
            _dev_ptr(r, torch.float16, "r"), _dev_ptr(y, torch.float16, "y"), _stream(stream))
    return BoundCall(lib().merit_conv2d_residual, "merit_conv2d_residual", args, (plan, x, w, r, y))


def bind_pool2d(plan: Plan, x, y, stream=None) -> BoundCall:
    import torch
    out_shape, a_shape, _ = plan.shapes()
    if tuple(y.shape) != out_shape or tuple(x.shape) != a_shape:
        raise ValueError("tensors do not match the plan")
    args = (plan.handle, _dev_ptr(x, torch.float32, "x"), _dev_ptr(y, torch.float32, "y"), _stream(stream))
    return BoundCall(lib().merit_pool2d, "merit_pool2d", args, (plan, x, y))


def bind_sad_search(plan: Plan, cur, ref, sad, mv, stream=None) -> BoundCall:
    import torch
    (nby, nbx), a_shape, b_shape = plan.shapes()
    if (tuple(cur.shape) != b_shape or tuple(ref.shape) != a_shape or tuple(sad.shape) != (nby, nbx)
            or tuple(mv.shape) != (nby, nbx, 2)):
        raise ValueError("tensors do not match the plan")
    args = (plan.handle, _dev_ptr(cur, torch.uint8, "cur"), _dev_ptr(ref, torch.uint8, "ref"),
            _dev_ptr(sad, torch.int32, "sad"), _dev_ptr(mv, torch.int32, "mv"), _stream(stream))
    return BoundCall(lib().merit_sad_search, "merit_sad_search", args, (plan, cur, ref, sad, mv))


def bind_correlation(plan: Plan, x1, x2, y, stream=None) -> BoundCall:
    import torch
    out_shape, a_shape, b_shape = plan.shapes()
    if tuple(x1.shape) != a_shape or tuple(x2.shape) != b_shape or tuple(y.shape) != out_shape:
        raise ValueError("tensors do not match the plan")
    args = (plan.handle, _dev_ptr(x1, torch.float16, "x1"), _dev_ptr(x2, torch.float16, "x2"),
            _dev_ptr(y, torch.float16, "y"), _stream(stream))
    return BoundCall(lib().merit_correlation, "merit_correlation", args, (plan, x1, x2, y))


def bind_conv2d_depthwise(plan: Plan, x, w, y, stream=None) -> BoundCall:
    import torch
    out_shape, a_shape, b_shape = plan.shapes()
    if tuple(x.shape) != a_shape or tuple(w.shape) != b_shape or tuple(y.shape) != out_shape:
        raise ValueError("tensors do not match the plan")
    args = (plan.handle, _dev_ptr(x, torch.float16, "x"), _dev_ptr(w, torch.float16, "w"),
            _dev_ptr(y, torch.float16, "y"), _stream(stream))
    return BoundCall(lib().merit_conv2d_depthwise, "merit_conv2d_depthwise", args, (plan, x, w, y))
