"""Thin Python binding of the C-ABI library (include/psb.h).

Argument marshalling only: every step of the layer runs in the HIP kernels of
libpsb_hip.so.  PyTorch supplies device memory (tensor.data_ptr()) and the stream.
There is no fallback: if the library is missing or a call fails, PsbError is raised.
"""
import ctypes as C
import os

import torch

from . import build as _build

OK = 0
ERR_NULL, ERR_SHAPE, ERR_VALUE, ERR_OVERFLOW_UNSAFE, ERR_TOO_LARGE, ERR_DEVICE, ERR_ALLOC = -1, -2, -3, -4, -5, -6, -7
_NAMES = {0: "PSB_OK", -1: "PSB_ERR_NULL", -2: "PSB_ERR_SHAPE", -3: "PSB_ERR_VALUE",
          -4: "PSB_ERR_OVERFLOW_UNSAFE", -5: "PSB_ERR_TOO_LARGE", -6: "PSB_ERR_DEVICE", -7: "PSB_ERR_ALLOC"}

MAPPING_AUTO, MAPPING_PIXEL_LANE, MAPPING_CHANNEL_LANE, MAPPING_PRODUCT_LIST = 0, 1, 2, 3

SYMBOLS = ["psb_quantize_weights", "psb_weights_info", "psb_weights_export", "psb_weights_destroy",
           "psb_conv2d_out_dims", "psb_linear", "psb_conv2d", "psb_conv2d_progressive",
           "psb_sample_filter", "psb_linear_shared", "psb_conv2d_shared", "psb_conv2d_progressive_shared",
           "psb_conv2d_requant", "psb_conv2d_requant_static", "psb_conv2d_shared_requant_blocked", "psb_shared_prepare_filters", "psb_shared_prepare_filters_levels", "psb_conv2d_shared_budget_requant_blocked", "psb_shared_budget_levels", "psb_requantize", "psb_maxpool2d_i8", "psb_maxpool2d_i8_blocked", "psb_global_avgpool_requantize", "psb_budget_resample",
           "psb_attention_budget", "psb_last_device_error", "psb_build_id", "psb_set_mapping", "psb_query_mapping", "psb_shared_window_slots", "psb_profile_enable",
           "psb_profile_read"]


class PsbError(RuntimeError):
    def __init__(self, code, where=""):
        self.code = code
        dev = ""
        if code == ERR_DEVICE and _lib is not None:
            dev = f" (hipError {_lib.psb_last_device_error()})"
        super().__init__(f"{where}: {_NAMES.get(code, code)}{dev}")


class WShape(C.Structure):
    _fields_ = [("oc", C.c_int32), ("cin", C.c_int32), ("kh", C.c_int32), ("kw", C.c_int32), ("groups", C.c_int32)]


class ConvGeom(C.Structure):
    _fields_ = [("n", C.c_int32), ("h", C.c_int32), ("w", C.c_int32), ("stride_h", C.c_int32),
                ("stride_w", C.c_int32), ("pad_h", C.c_int32), ("pad_w", C.c_int32)]


class Requant(C.Structure):
    _fields_ = [("relu", C.c_int32), ("inv_step", C.c_float), ("lo", C.c_int32), ("hi", C.c_int32),
                ("res_f32_dev", C.c_void_p), ("res_i8_dev", C.c_void_p), ("res_step", C.c_float)]


class WInfo(C.Structure):
    _fields_ = [("e_top", C.c_int32), ("e_min", C.c_int32), ("n_zero", C.c_int64), ("n_flushed", C.c_int64),
                ("n_live", C.c_int64)]


_lib = None


def library_path():
    return _build.LIB


def lib():
    """Load libpsb_hip.so (built in-tree; built here only if it does not exist; refused if it was built from
    other sources than the ones in the tree)."""
    global _lib
    if _lib is None:
        path = _build.ensure_built()
        if not os.path.exists(path):
            raise PsbError(ERR_DEVICE, f"HIP library {path} is missing")
        L = C.CDLL(path)
        vp, i32, u32, u64 = C.c_void_p, C.c_int32, C.c_uint32, C.c_uint64
        L.psb_quantize_weights.argtypes = [vp, C.POINTER(WShape), i32, i32, i32, i32, vp, C.POINTER(vp)]
        L.psb_weights_info.argtypes = [vp, C.POINTER(WInfo)]
        L.psb_weights_export.argtypes = [vp, vp]
        L.psb_weights_destroy.argtypes = [vp]
        L.psb_weights_destroy.restype = None
        L.psb_conv2d_out_dims.argtypes = [C.POINTER(WShape), C.POINTER(ConvGeom), C.POINTER(i32), C.POINTER(i32)]
        L.psb_linear.argtypes = [vp, vp, i32, i32, u64, u32, vp, vp, vp, vp, vp]
        L.psb_conv2d.argtypes = [vp, vp, C.POINTER(ConvGeom), i32, u64, u32, vp, vp, vp, vp, vp]
        L.psb_conv2d_progressive.argtypes = [vp, vp, C.POINTER(ConvGeom), vp, vp, u64, u32, vp, vp, vp, vp, vp]
        L.psb_sample_filter.argtypes = [vp, i32, i32, u64, u32, vp, vp]
        L.psb_linear_shared.argtypes = L.psb_linear.argtypes
        L.psb_conv2d_shared.argtypes = L.psb_conv2d.argtypes
        L.psb_conv2d_progressive_shared.argtypes = L.psb_conv2d_progressive.argtypes
        f32 = C.c_float
        L.psb_conv2d_shared_requant_blocked.argtypes = [vp, vp, C.POINTER(ConvGeom), i32, u64, u32, vp, vp, vp,
                                                        C.POINTER(Requant), vp, i32, vp]
        L.psb_shared_prepare_filters.argtypes = [vp, i32, i32, vp, vp, vp]
        L.psb_shared_budget_levels.argtypes = [vp, i32]
        L.psb_shared_prepare_filters_levels.argtypes = [vp, i32, vp, i32, vp, vp, vp]
        L.psb_conv2d_shared_budget_requant_blocked.argtypes = [vp, vp, C.POINTER(ConvGeom), vp, vp, i32, u64, u32, vp, vp,
                                                               vp, C.POINTER(Requant), vp, i32, vp]
        L.psb_conv2d_requant.argtypes = [vp, vp, C.POINTER(ConvGeom), i32, vp, u64, u32, vp, vp, vp, vp,
                                         C.POINTER(Requant), vp, i32, vp]
        L.psb_conv2d_requant_static.argtypes = [vp, vp, C.POINTER(ConvGeom), i32, vp, u64, u32, vp, vp, vp,
                                                C.POINTER(Requant), vp, vp]
        L.psb_requantize.argtypes = [vp, vp, vp, f32, i32, f32, i32, i32, C.c_int64, vp, vp]
        L.psb_maxpool2d_i8.argtypes = [vp] + [i32] * 10 + [vp, vp]
        L.psb_maxpool2d_i8_blocked.argtypes = [vp] + [i32] * 10 + [vp, vp]
        L.psb_global_avgpool_requantize.argtypes = [vp, i32, i32, i32, i32, f32, i32, i32, vp, vp]
        L.psb_budget_resample.argtypes = [vp, i32, i32, i32, i32, i32, vp, vp]
        L.psb_attention_budget.argtypes = [vp, f32, i32, i32, i32, i32, C.c_uint8, C.c_uint8, vp, vp, vp, vp]
        L.psb_last_device_error.argtypes = []
        L.psb_set_mapping.argtypes = [C.c_int]
        L.psb_query_mapping.argtypes = [vp, C.POINTER(ConvGeom)]
        L.psb_shared_window_slots.argtypes = [i32, i32, C.POINTER(ConvGeom), i32]
        L.psb_profile_enable.argtypes = [C.c_int]
        L.psb_profile_read.argtypes = [C.POINTER(C.c_double), C.POINTER(C.c_int64)]
        for name in SYMBOLS:
            if name not in ("psb_weights_destroy", "psb_build_id"):
                getattr(L, name).restype = C.c_int
        L.psb_build_id.argtypes = []
        L.psb_build_id.restype = C.c_char_p
        built_from, sources = L.psb_build_id().decode(), _build.source_id()
        if built_from != sources:        # a kernel was edited and the library not rebuilt: never run the old code
            raise PsbError(ERR_DEVICE, f"{path} was built from other sources ({built_from[:12]}) than the ones beside "
                                       f"it ({sources[:12]}): run python -m paper_1904_02205_amd.build")
        _lib = L
    return _lib


def _check(rc, where):
    if rc != OK:
        raise PsbError(rc, where)


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _ptr(t, dtype, name):
    if t is None:
        return None
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.is_contiguous() and t.dtype == dtype):
        raise TypeError(f"{name}: expected a contiguous CUDA tensor of dtype {dtype}")
    return C.c_void_p(t.data_ptr())


def _expect(t, shape, name):
    """The library cannot see tensor shapes behind the raw pointers it is given: a wrong one is refused here."""
    if t is not None and tuple(t.shape) != tuple(shape):
        raise ValueError(f"{name}: shape {tuple(t.shape)}, expected {tuple(shape)}")


def _expect_layer_io(q, out_shape, acc=None, y=None, mult=None, bias=None, budget_to=None, budget_from=None,
                     x_out=None, x_out_shape=None, res_f32=None, res_i8=None, res_i8_shape=None):
    """Shapes of everything a layer call reads or writes besides x, for output shape (N, OC, OH, OW) or (B, OC)."""
    oc = q.wshape[0]
    _expect(acc, out_shape, "acc")
    _expect(y, out_shape, "y")
    _expect(mult, (oc,), "mult")
    _expect(bias, (oc,), "bias")
    if len(out_shape) == 4:
        pix = (out_shape[0], out_shape[2], out_shape[3])
        _expect(budget_to, pix, "budget_to")
        _expect(budget_from, pix, "budget_from")
    _expect(x_out, x_out_shape or out_shape, "x_out")
    _expect(res_f32, out_shape, "res_f32")
    _expect(res_i8, res_i8_shape or out_shape, "res_i8")


def set_mapping(mapping):
    return lib().psb_set_mapping(int(mapping))


def query_mapping(q, geom):
    """Mapping (1, 2, 3) a layer call on handle q with geom = (n, h, w, stride_h, stride_w, pad_h, pad_w) would use."""
    rc = lib().psb_query_mapping(q._h, C.byref(ConvGeom(*geom)))
    if rc < 0:
        raise PsbError(rc, "psb_query_mapping")
    return rc


def shared_window_slots(kernel, geom, half_tiles):
    """LDS window slots of the 3 x 3 shared-filter kernel for kernel = (kh, kw) and geom = (n, h, w, stride_h, stride_w,
    pad_h, pad_w) with pixel tiles of 128 * half_tiles outputs; 0 when that kernel does not take the layer.  Host only."""
    rc = lib().psb_shared_window_slots(int(kernel[0]), int(kernel[1]), C.byref(ConvGeom(*geom)), int(half_tiles))
    if rc < 0:
        raise PsbError(rc, "psb_shared_window_slots")
    return rc


def profile_enable(on=True):
    _check(lib().psb_profile_enable(1 if on else 0), "psb_profile_enable")


def profile_read():
    """(sum of sampling-kernel milliseconds, number of launches) since the last read."""
    ms, n = C.c_double(0.0), C.c_int64(0)
    _check(lib().psb_profile_read(C.byref(ms), C.byref(n)), "psb_profile_read")
    return ms.value, n.value


def conv2d_out_dims(wshape, geom):
    """wshape = (oc, cin, kh, kw, groups); geom = (n, h, w, stride_h, stride_w, pad_h, pad_w)."""
    oh, ow = C.c_int32(0), C.c_int32(0)
    rc = lib().psb_conv2d_out_dims(C.byref(WShape(*wshape)), C.byref(ConvGeom(*geom)), C.byref(oh), C.byref(ow))
    _check(rc, "psb_conv2d_out_dims")
    return oh.value, ow.value


class Weights:
    """Handle returned by psb_quantize_weights."""

    def __init__(self, w, groups=1, exp_bits=0, x_absmax=127, s_max=16, prob_bits=23):
        """w: CUDA float32 [oc, cin/groups, kh, kw] (a 2-D [oc, k] tensor is a linear layer)."""
        if w.dim() == 2:
            w = w.reshape(w.shape[0], w.shape[1], 1, 1)
        oc, cg, kh, kw = w.shape
        self.wshape = (oc, cg * groups, kh, kw, groups)
        self.K = cg * kh * kw
        self.s_max = s_max
        self.prob_bits = prob_bits
        self._h = C.c_void_p(None)
        shape = WShape(*self.wshape)
        rc = lib().psb_quantize_weights(_ptr(w, torch.float32, "w"), C.byref(shape), prob_bits, exp_bits, x_absmax,
                                        s_max, _stream(), C.byref(self._h))
        _check(rc, "psb_quantize_weights")
        info = WInfo()
        _check(lib().psb_weights_info(self._h, C.byref(info)), "psb_weights_info")
        self.e_top, self.e_min = info.e_top, info.e_min
        self.n_zero, self.n_flushed, self.n_live = info.n_zero, info.n_flushed, info.n_live

    def export(self):
        """numpy uint32 [oc, K]: sign<<31 | shift<<23 | mantissa; shift 0xFF = not live."""
        import numpy as np
        out = np.empty((self.wshape[0], self.K), dtype=np.uint32)
        _check(lib().psb_weights_export(self._h, out.ctypes.data_as(C.c_void_p)), "psb_weights_export")
        return out

    def close(self):
        if getattr(self, "_h", None) is not None and self._h.value:
            lib().psb_weights_destroy(self._h)
            self._h = C.c_void_p(None)

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def sample_filter(q, sample_to, sample_from=0, seed=0, layer_id=0, out=None):
    """The shared-filter mode's integer filter for samples [sample_from, sample_to): int32 [OC, K] on the device."""
    if out is None:
        out = torch.empty((q.wshape[0], q.K), dtype=torch.int32, device="cuda")
    _expect(out, (q.wshape[0], q.K), "out")
    rc = lib().psb_sample_filter(q._h, sample_from, sample_to, seed, layer_id, _ptr(out, torch.int32, "out"), _stream())
    _check(rc, "psb_sample_filter")
    return out


def linear(q, x, S, seed=0, layer_id=0, acc=None, y=None, mult=None, bias=None, shared=False):
    """x int8 [B, K] -> acc int32 [B, OC] (and y float32 if given).  shared: one sampled filter per pass."""
    if x.dim() != 2 or x.shape[1] != q.K or q.wshape[2:] != (1, 1, 1):
        raise ValueError(f"x: shape {tuple(x.shape)}, expected (B, {q.K}) and a handle of a linear layer")
    B = x.shape[0]
    oc = q.wshape[0]
    if acc is None:
        acc = torch.empty((B, oc), dtype=torch.int32, device=x.device)
    _expect_layer_io(q, (B, oc), acc=acc, y=y, mult=mult, bias=bias)
    fn = lib().psb_linear_shared if shared else lib().psb_linear
    rc = fn(q._h, _ptr(x, torch.int8, "x"), B, S, seed, layer_id, _ptr(acc, torch.int32, "acc"),
            _ptr(y, torch.float32, "y"), _ptr(mult, torch.float32, "mult"), _ptr(bias, torch.float32, "bias"), _stream())
    _check(rc, "psb_linear_shared" if shared else "psb_linear")
    return acc


def _geom(q, x, stride, pad):
    """Geometry of a convolution call and its output shape; the input must have the handle's channel count."""
    if x.dim() != 4 or x.shape[1] != q.wshape[1]:
        raise ValueError(f"x: shape {tuple(x.shape)}, expected (N, {q.wshape[1]}, H, W)")
    n, _, h, w = x.shape
    g = ConvGeom(n, h, w, stride[0], stride[1], pad[0], pad[1])
    oh, ow = conv2d_out_dims(q.wshape, (g.n, g.h, g.w, g.stride_h, g.stride_w, g.pad_h, g.pad_w))
    return g, (n, q.wshape[0], oh, ow)


def conv2d(q, x, S, stride=(1, 1), pad=(0, 0), seed=0, layer_id=0, acc=None, y=None, mult=None, bias=None,
           shared=False):
    """x int8 [N, C, H, W] -> acc int32 [N, OC, OH, OW]."""
    g, shape = _geom(q, x, stride, pad)
    if acc is None:
        acc = torch.empty(shape, dtype=torch.int32, device=x.device)
    _expect_layer_io(q, shape, acc=acc, y=y, mult=mult, bias=bias)
    fn = lib().psb_conv2d_shared if shared else lib().psb_conv2d
    rc = fn(q._h, _ptr(x, torch.int8, "x"), C.byref(g), S, seed, layer_id, _ptr(acc, torch.int32, "acc"),
            _ptr(y, torch.float32, "y"), _ptr(mult, torch.float32, "mult"), _ptr(bias, torch.float32, "bias"), _stream())
    _check(rc, "psb_conv2d_shared" if shared else "psb_conv2d")
    return acc


def conv2d_progressive(q, x, budget_to, budget_from=None, stride=(1, 1), pad=(0, 0), seed=0, layer_id=0, acc=None,
                       y=None, mult=None, bias=None, shared=False):
    """budget_to / budget_from uint8 [N, OH, OW]; with budget_from, acc is updated in place."""
    g, shape = _geom(q, x, stride, pad)
    if acc is None:
        if budget_from is not None:
            raise ValueError("a refinement call needs the accumulators of the first pass")
        acc = torch.empty(shape, dtype=torch.int32, device=x.device)
    _expect_layer_io(q, shape, acc=acc, y=y, mult=mult, bias=bias, budget_to=budget_to, budget_from=budget_from)
    fn = lib().psb_conv2d_progressive_shared if shared else lib().psb_conv2d_progressive
    rc = fn(q._h, _ptr(x, torch.int8, "x"), C.byref(g), _ptr(budget_to, torch.uint8, "budget_to"),
            _ptr(budget_from, torch.uint8, "budget_from"), seed, layer_id, _ptr(acc, torch.int32, "acc"),
            _ptr(y, torch.float32, "y"), _ptr(mult, torch.float32, "mult"), _ptr(bias, torch.float32, "bias"), _stream())
    _check(rc, "psb_conv2d_progressive_shared" if shared else "psb_conv2d_progressive")
    return acc


def conv2d_requant(q, x, inv_step, S=None, budget_to=None, stride=(1, 1), pad=(0, 0), seed=0, layer_id=0, relu=True,
                   lo=0, hi=127, res_f32=None, res_i8=None, res_step=0.0, mult=None, bias=None, acc=None, y=None,
                   x_out=None, shared=False, want_acc=True):
    """Layer call with the requantisation fused in: returns the int8 activations [N, OC, OH, OW].  want_acc=False
    (and acc None): no accumulators are handed out."""
    g, shape = _geom(q, x, stride, pad)
    if acc is None and want_acc:
        acc = torch.empty(shape, dtype=torch.int32, device=x.device)
    if x_out is None:
        x_out = torch.empty(shape, dtype=torch.int8, device=x.device)
    _expect_layer_io(q, shape, acc=acc, y=y, mult=mult, bias=bias, budget_to=budget_to, x_out=x_out, res_f32=res_f32,
                     res_i8=res_i8)
    rq = Requant(1 if relu else 0, inv_step, lo, hi,
                 None if res_f32 is None else _ptr(res_f32, torch.float32, "res_f32").value,
                 None if res_i8 is None else _ptr(res_i8, torch.int8, "res_i8").value, res_step)
    rc = lib().psb_conv2d_requant(q._h, _ptr(x, torch.int8, "x"), C.byref(g), 0 if S is None else S,
                                  _ptr(budget_to, torch.uint8, "budget_to"), seed, layer_id,
                                  _ptr(acc, torch.int32, "acc"), _ptr(y, torch.float32, "y"),
                                  _ptr(mult, torch.float32, "mult"), _ptr(bias, torch.float32, "bias"), C.byref(rq),
                                  _ptr(x_out, torch.int8, "x_out"), 1 if shared else 0, _stream())
    _check(rc, "psb_conv2d_requant")
    return x_out


STATIC_MAX_OUTPUTS = 8 * 1024 * 1024


def conv2d_requant_static(q, x, inv_step, x_out, S=None, budget_to=None, stride=(1, 1), pad=(0, 0), seed=0, layer_id=0,
                          relu=True, lo=0, hi=127, res_f32=None, res_i8=None, res_step=0.0, mult=None, bias=None, y=None):
    """psb_conv2d_requant_static: conv2d_requant without accumulators out (per-product mode) that allocates nothing;
    the caller passes every tensor, x_out [N, OC, OH, OW] included.  At most STATIC_MAX_OUTPUTS output elements,
    counted with OC rounded up to a multiple of 64."""
    g, shape = _geom(q, x, stride, pad)
    _expect_layer_io(q, shape, y=y, mult=mult, bias=bias, budget_to=budget_to, x_out=x_out, res_f32=res_f32,
                     res_i8=res_i8)
    rq = Requant(1 if relu else 0, inv_step, lo, hi,
                 None if res_f32 is None else _ptr(res_f32, torch.float32, "res_f32").value,
                 None if res_i8 is None else _ptr(res_i8, torch.int8, "res_i8").value, res_step)
    rc = lib().psb_conv2d_requant_static(q._h, _ptr(x, torch.int8, "x"), C.byref(g), 0 if S is None else S,
                                         _ptr(budget_to, torch.uint8, "budget_to"), seed, layer_id,
                                         _ptr(y, torch.float32, "y"), _ptr(mult, torch.float32, "mult"),
                                         _ptr(bias, torch.float32, "bias"), C.byref(rq),
                                         _ptr(x_out, torch.int8, "x_out"), _stream())
    _check(rc, "psb_conv2d_requant_static")
    return x_out


BLOCKED_IN, BLOCKED_OUT, BLOCKED_RES = 1, 2, 4


def blocked_shape(n, c, h, w):
    """Shape of the blocked channels-last form of an [n, c, h, w] int8 tensor: [n, h, ceil(c/32), w, 32]."""
    return (n, h, (c + 31) // 32, w, 32)


def conv2d_shared_requant_blocked(q, x, x_shape, inv_step, S, stride=(1, 1), pad=(0, 0), seed=0, layer_id=0, relu=True,
                                  lo=0, hi=127, res_f32=None, res_i8=None, res_step=0.0, mult=None, bias=None,
                                  x_out=None, y=None, layout=0, want_x=True):
    """Shared-filter layer with fused requantisation whose int8 tensors may be in the blocked channels-last layout
    (layout: BLOCKED_IN | BLOCKED_OUT | BLOCKED_RES).  x_shape = (N, C, H, W) of the input whatever its layout.
    Returns x_out: [N, OC, OH, OW], or its blocked form with BLOCKED_OUT.  want_x=False: only the rescaled fp32
    values are computed, into y [N, OC, OH, OW] (allocated if None), which is returned."""
    n, c, h, w = x_shape
    g = ConvGeom(n, h, w, stride[0], stride[1], pad[0], pad[1])
    oh, ow = conv2d_out_dims(q.wshape, (g.n, g.h, g.w, g.stride_h, g.stride_w, g.pad_h, g.pad_w))
    oc = q.wshape[0]
    if want_x and x_out is None:
        shape = blocked_shape(n, oc, oh, ow) if layout & BLOCKED_OUT else (n, oc, oh, ow)
        x_out = torch.empty(shape, dtype=torch.int8, device=x.device)
    if not want_x and y is None:
        y = torch.empty((n, oc, oh, ow), dtype=torch.float32, device=x.device)
    if c != q.wshape[1]:
        raise ValueError(f"x_shape: {c} channels, the handle has {q.wshape[1]}")
    _expect(x, blocked_shape(n, c, h, w) if layout & BLOCKED_IN else (n, c, h, w), "x")
    _expect_layer_io(q, (n, oc, oh, ow), y=y, mult=mult, bias=bias, x_out=x_out if want_x else None,
                     x_out_shape=blocked_shape(n, oc, oh, ow) if layout & BLOCKED_OUT else None, res_f32=res_f32,
                     res_i8=res_i8, res_i8_shape=blocked_shape(n, oc, oh, ow) if layout & BLOCKED_RES else None)
    rq = Requant(1 if relu else 0, inv_step, lo, hi,
                 None if res_f32 is None else _ptr(res_f32, torch.float32, "res_f32").value,
                 None if res_i8 is None else _ptr(res_i8, torch.int8, "res_i8").value, res_step)
    rc = lib().psb_conv2d_shared_requant_blocked(q._h, _ptr(x, torch.int8, "x"), C.byref(g), S, seed, layer_id,
                                                 _ptr(y, torch.float32, "y"), _ptr(mult, torch.float32, "mult"),
                                                 _ptr(bias, torch.float32, "bias"), C.byref(rq),
                                                 _ptr(x_out if want_x else None, torch.int8, "x_out"), layout, _stream())
    _check(rc, "psb_conv2d_shared_requant_blocked")
    return x_out if want_x else y


def _levels_array(levels):
    vals = sorted({int(v) for v in levels})
    if not vals or min(vals) < 0 or max(vals) > 255:
        raise ValueError("levels: one or more budget values in 0..255")
    return (C.c_uint8 * len(vals))(*vals), len(vals)


def conv2d_shared_budget_requant_blocked(q, x, x_shape, inv_step, budget_to, levels, stride=(1, 1), pad=(0, 0), seed=0,
                                         layer_id=0, relu=True, lo=0, hi=127, res_f32=None, res_i8=None, res_step=0.0,
                                         mult=None, bias=None, x_out=None, y=None, layout=0, want_x=True):
    """conv2d_shared_requant_blocked with a per-pixel budget map [N, OH, OW] whose values are rounded down to
    `levels` (at most four distinct values): all sample segments in one launch, epilogue fused."""
    n, c, h, w = x_shape
    g = ConvGeom(n, h, w, stride[0], stride[1], pad[0], pad[1])
    oh, ow = conv2d_out_dims(q.wshape, (g.n, g.h, g.w, g.stride_h, g.stride_w, g.pad_h, g.pad_w))
    oc = q.wshape[0]
    if want_x and x_out is None:
        shape = blocked_shape(n, oc, oh, ow) if layout & BLOCKED_OUT else (n, oc, oh, ow)
        x_out = torch.empty(shape, dtype=torch.int8, device=x.device)
    if not want_x and y is None:
        y = torch.empty((n, oc, oh, ow), dtype=torch.float32, device=x.device)
    if c != q.wshape[1]:
        raise ValueError(f"x_shape: {c} channels, the handle has {q.wshape[1]}")
    _expect(x, blocked_shape(n, c, h, w) if layout & BLOCKED_IN else (n, c, h, w), "x")
    _expect_layer_io(q, (n, oc, oh, ow), y=y, mult=mult, bias=bias, budget_to=budget_to,
                     x_out=x_out if want_x else None,
                     x_out_shape=blocked_shape(n, oc, oh, ow) if layout & BLOCKED_OUT else None, res_f32=res_f32,
                     res_i8=res_i8, res_i8_shape=blocked_shape(n, oc, oh, ow) if layout & BLOCKED_RES else None)
    if budget_to is None:
        raise ValueError("budget_to: a budget map is required")
    lv, n_lv = _levels_array(levels)
    rq = Requant(1 if relu else 0, inv_step, lo, hi,
                 None if res_f32 is None else _ptr(res_f32, torch.float32, "res_f32").value,
                 None if res_i8 is None else _ptr(res_i8, torch.int8, "res_i8").value, res_step)
    rc = lib().psb_conv2d_shared_budget_requant_blocked(
        q._h, _ptr(x, torch.int8, "x"), C.byref(g), _ptr(budget_to, torch.uint8, "budget_to"), lv, n_lv, seed, layer_id,
        _ptr(y, torch.float32, "y"), _ptr(mult, torch.float32, "mult"), _ptr(bias, torch.float32, "bias"), C.byref(rq),
        _ptr(x_out if want_x else None, torch.int8, "x_out"), layout, _stream())
    _check(rc, "psb_conv2d_shared_budget_requant_blocked")
    return x_out if want_x else y


def shared_prepare_filters_levels(handles, levels, seeds, layer_ids):
    """Sample the filters of every segment of the sample axis cut at `levels`, for several layers in one launch; the
    next conv2d_shared_budget_requant_blocked call of each with the same levels uses them."""
    n = len(handles)
    hs = (C.c_void_p * n)(*[q._h for q in handles])
    sd = (C.c_uint64 * n)(*[int(v) for v in seeds])
    li = (C.c_uint32 * n)(*[int(v) for v in layer_ids])
    lv, n_lv = _levels_array(levels)
    _check(lib().psb_shared_prepare_filters_levels(hs, n, lv, n_lv, sd, li, _stream()), "psb_shared_prepare_filters_levels")


def shared_prepare_filters(handles, S, seeds, layer_ids):
    """Sample the digit planes of several layers in one launch; the next matching shared-filter call of each uses them."""
    n = len(handles)
    hs = (C.c_void_p * n)(*[q._h for q in handles])
    sd = (C.c_uint64 * n)(*[int(v) for v in seeds])
    li = (C.c_uint32 * n)(*[int(v) for v in layer_ids])
    _check(lib().psb_shared_prepare_filters(hs, n, S, sd, li, _stream()), "psb_shared_prepare_filters")


def shared_budget_levels(levels=None):
    """Announce the budget values of the NEXT shared-filter call with a budget map (an iterable of ints; every value
    that occurs in its maps must be listed), so that it need not read them back; None or () withdraws an
    announcement."""
    vals = sorted({int(v) for v in levels}) if levels is not None else []
    arr = (C.c_uint8 * max(1, len(vals)))(*vals)
    _check(lib().psb_shared_budget_levels(arr if vals else None, len(vals)), "psb_shared_budget_levels")


# ---- glue between layers ---------------------------------------------------------------------------------

def requantize(y, inv_step, relu=True, lo=0, hi=127, res_f32=None, res_i8=None, res_step=0.0, out=None):
    """int8 tensor of y's shape: clamp(rint(g(y [+ r]) * inv_step), lo, hi)."""
    if out is None:
        out = torch.empty(y.shape, dtype=torch.int8, device=y.device)
    _expect(out, y.shape, "out")
    _expect(res_f32, y.shape, "res_f32")
    _expect(res_i8, y.shape, "res_i8")
    rc = lib().psb_requantize(_ptr(y, torch.float32, "y"), _ptr(res_f32, torch.float32, "res_f32"),
                              _ptr(res_i8, torch.int8, "res_i8"), res_step, 1 if relu else 0, inv_step, lo, hi,
                              y.numel(), _ptr(out, torch.int8, "out"), _stream())
    _check(rc, "psb_requantize")
    return out


def maxpool2d_i8(x, kernel, stride, pad, out=None):
    n, c, h, w = x.shape
    oh, ow = (h + 2 * pad[0] - kernel[0]) // stride[0] + 1, (w + 2 * pad[1] - kernel[1]) // stride[1] + 1
    if out is None:
        out = torch.empty((n, c, max(oh, 0), max(ow, 0)), dtype=torch.int8, device=x.device)
    _expect(out, (n, c, max(oh, 0), max(ow, 0)), "out")
    rc = lib().psb_maxpool2d_i8(_ptr(x, torch.int8, "x"), n, c, h, w, kernel[0], kernel[1], stride[0], stride[1],
                                pad[0], pad[1], _ptr(out, torch.int8, "out"), _stream())
    _check(rc, "psb_maxpool2d_i8")
    return out


def maxpool2d_i8_blocked(x, x_shape, kernel, stride, pad, out=None):
    """maxpool2d_i8 on the blocked channels-last layout: x is blocked_shape(*x_shape), x_shape = (N, C, H, W); returns
    the blocked form of [N, C, OH, OW]."""
    n, c, h, w = x_shape
    oh, ow = (h + 2 * pad[0] - kernel[0]) // stride[0] + 1, (w + 2 * pad[1] - kernel[1]) // stride[1] + 1
    _expect(x, blocked_shape(n, c, h, w), "x")
    if out is None:
        out = torch.empty(blocked_shape(n, c, max(oh, 0), max(ow, 0)), dtype=torch.int8, device=x.device)
    _expect(out, blocked_shape(n, c, max(oh, 0), max(ow, 0)), "out")
    rc = lib().psb_maxpool2d_i8_blocked(_ptr(x, torch.int8, "x"), n, c, h, w, kernel[0], kernel[1], stride[0], stride[1],
                                        pad[0], pad[1], _ptr(out, torch.int8, "out"), _stream())
    _check(rc, "psb_maxpool2d_i8_blocked")
    return out


def global_avgpool_requantize(x, scale, lo=0, hi=127, out=None):
    n, c, h, w = x.shape
    if out is None:
        out = torch.empty((n, c), dtype=torch.int8, device=x.device)
    _expect(out, (n, c), "out")
    rc = lib().psb_global_avgpool_requantize(_ptr(x, torch.int8, "x"), n, c, h, w, scale, lo, hi,
                                             _ptr(out, torch.int8, "out"), _stream())
    _check(rc, "psb_global_avgpool_requantize")
    return out


def budget_resample(b, oh, ow, out=None):
    n, h, w = b.shape
    if out is None:
        out = torch.empty((n, oh, ow), dtype=torch.uint8, device=b.device)
    _expect(out, (n, oh, ow), "out")
    rc = lib().psb_budget_resample(_ptr(b, torch.uint8, "budget"), n, h, w, oh, ow, _ptr(out, torch.uint8, "out"),
                                   _stream())
    _check(rc, "psb_budget_resample")
    return out


def attention_budget(act, step, lo, hi):
    """(entropy float32 [n,h,w], mean float32 [n], budget uint8 [n,h,w]) from int8 activations [n,c,h,w]."""
    n, c, h, w = act.shape
    ent = torch.empty((n, h, w), dtype=torch.float32, device=act.device)
    mean = torch.empty((n,), dtype=torch.float32, device=act.device)
    bud = torch.empty((n, h, w), dtype=torch.uint8, device=act.device)
    rc = lib().psb_attention_budget(_ptr(act, torch.int8, "act"), step, n, c, h, w, lo, hi,
                                    _ptr(ent, torch.float32, "entropy"), _ptr(mean, torch.float32, "mean"),
                                    _ptr(bud, torch.uint8, "budget"), _stream())
    _check(rc, "psb_attention_budget")
    return ent, mean, bud
