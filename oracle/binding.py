"""ctypes view of libpsb_oracle.so (TEST INFRASTRUCTURE ONLY).

numpy in, numpy out; no arithmetic of the method happens here.
"""
import ctypes as C
import os

import numpy as np

from . import build_oracle

ZERO, NORMAL, SUBNORMAL, NONFINITE = 0, 1, 2, 3
OK, ERR_ARG, ERR_VALUE, ERR_OVERFLOW_UNSAFE = 0, -1, -3, -4


class WInfo(C.Structure):
    _fields_ = [("e_top", C.c_int32), ("e_min", C.c_int32),
                ("n_zero", C.c_int64), ("n_flushed", C.c_int64), ("n_live", C.c_int64)]


class Weights(C.Structure):
    _fields_ = [("oc", C.c_int32), ("K", C.c_int32),
                ("sign", C.POINTER(C.c_int8)), ("shift", C.POINTER(C.c_int32)),
                ("p", C.POINTER(C.c_double)), ("prob_bits", C.c_int32), ("info", WInfo)]


class WShape(C.Structure):
    _fields_ = [("oc", C.c_int32), ("cin", C.c_int32), ("kh", C.c_int32),
                ("kw", C.c_int32), ("groups", C.c_int32)]


class Geom(C.Structure):
    _fields_ = [("n", C.c_int32), ("h", C.c_int32), ("w", C.c_int32),
                ("stride_h", C.c_int32), ("stride_w", C.c_int32),
                ("pad_h", C.c_int32), ("pad_w", C.c_int32)]


_lib = None


def lib():
    global _lib
    if _lib is None:
        path = build_oracle.ensure_built()
        L = C.CDLL(path)
        L.psbo_decode.argtypes = [C.c_float, C.POINTER(C.c_int32), C.POINTER(C.c_int32), C.POINTER(C.c_double)]
        L.psbo_decode.restype = C.c_int
        L.psbo_philox4x32_10.argtypes = [C.POINTER(C.c_uint32)] * 3
        L.psbo_philox4x32_10.restype = None
        L.psbo_uniform.argtypes = [C.c_uint64, C.c_uint32, C.c_uint32, C.c_uint32, C.c_uint32]
        L.psbo_uniform.restype = C.c_uint32
        L.psbo_quantize.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_int32,
                                    C.POINTER(Weights)]
        L.psbo_uniform7.argtypes = [C.c_uint64, C.c_uint32, C.c_uint32, C.c_uint32, C.c_uint32]
        L.psbo_uniform7.restype = C.c_uint32
        L.psbo_quantize.restype = C.c_int
        L.psbo_weights_free.argtypes = [C.POINTER(Weights)]
        L.psbo_weights_free.restype = None
        L.psbo_linear.argtypes = [C.POINTER(Weights), C.c_void_p, C.c_int32, C.c_int32, C.c_uint64, C.c_uint32,
                                  C.c_void_p, C.c_void_p, C.POINTER(C.c_int64)]
        L.psbo_linear.restype = C.c_int
        L.psbo_conv2d.argtypes = [C.POINTER(Weights), C.POINTER(WShape), C.c_void_p, C.POINTER(Geom),
                                  C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_uint64, C.c_uint32,
                                  C.c_void_p, C.c_int64, C.c_void_p, C.POINTER(C.c_int64), C.POINTER(C.c_int64)]
        L.psbo_conv2d.restype = C.c_int
        L.psbo_sample_filter.argtypes = [C.POINTER(Weights), C.c_int32, C.c_int32, C.c_uint64, C.c_uint32,
                                         C.c_void_p, C.c_int32, C.c_void_p]
        L.psbo_sample_filter.restype = C.c_int
        L.psbo_conv2d_shared.argtypes = [C.POINTER(Weights), C.POINTER(WShape), C.c_void_p, C.POINTER(Geom),
                                         C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_uint64, C.c_uint32,
                                         C.c_void_p, C.c_int64, C.c_void_p, C.POINTER(C.c_int64)]
        L.psbo_conv2d_shared.restype = C.c_int
        L.psbo_rescale.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_int32,
                                   C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p]
        L.psbo_rescale.restype = C.c_int
        L.psbo_requantize.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_float, C.c_int, C.c_float, C.c_int32,
                                      C.c_int32, C.c_int64, C.c_void_p]
        L.psbo_requantize.restype = C.c_int
        L.psbo_maxpool_i8.argtypes = [C.c_void_p] + [C.c_int32] * 10 + [C.c_void_p]
        L.psbo_maxpool_i8.restype = C.c_int
        L.psbo_avgpool_requantize.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_float,
                                              C.c_int32, C.c_int32, C.c_void_p]
        L.psbo_avgpool_requantize.restype = C.c_int
        L.psbo_budget_resample.argtypes = [C.c_void_p] + [C.c_int32] * 5 + [C.c_void_p]
        L.psbo_budget_resample.restype = C.c_int
        L.psbo_attention_budget.argtypes = [C.c_void_p, C.c_float, C.c_int32, C.c_int32, C.c_int32, C.c_int32,
                                            C.c_uint8, C.c_uint8, C.c_void_p, C.c_void_p, C.c_void_p]
        L.psbo_attention_budget.restype = C.c_int
        L.psbo_num_threads.argtypes = []
        L.psbo_num_threads.restype = C.c_int
        _lib = L
    return _lib


class OracleError(RuntimeError):
    def __init__(self, code):
        super().__init__(f"oracle status {code}")
        self.code = code


def _ptr(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def num_threads():
    return int(lib().psbo_num_threads())


def decode(w):
    """(class, s, e, p) of one binary32 weight."""
    s, e, p = C.c_int32(0), C.c_int32(0), C.c_double(0.0)
    cls = lib().psbo_decode(C.c_float(float(np.float32(w))), C.byref(s), C.byref(e), C.byref(p))
    return cls, s.value, e.value, p.value


def philox(ctr, key):
    c = (C.c_uint32 * 4)(*[int(v) & 0xFFFFFFFF for v in ctr])
    k = (C.c_uint32 * 2)(*[int(v) & 0xFFFFFFFF for v in key])
    out = (C.c_uint32 * 4)()
    lib().psbo_philox4x32_10(c, k, out)
    return [int(v) for v in out]


def uniform(seed, layer_id, o, k, s):
    return int(lib().psbo_uniform(int(seed), int(layer_id), int(o), int(k), int(s)))


def uniform7(seed, layer_id, o, k, s):
    return int(lib().psbo_uniform7(int(seed), int(layer_id), int(o), int(k), int(s)))


class QWeights:
    """Quantised layer held by the oracle; arrays are numpy views, [oc, K]."""

    def __init__(self, w, exp_bits=0, x_absmax=127, s_max=16, prob_bits=23):
        w = np.ascontiguousarray(w, dtype=np.float32)
        oc = w.shape[0]
        K = int(np.prod(w.shape[1:]))
        self._q = Weights()
        rc = lib().psbo_quantize(_ptr(w), oc, K, prob_bits, exp_bits, x_absmax, s_max, C.byref(self._q))
        self.prob_bits = prob_bits
        if rc != OK:
            self._q = None
            raise OracleError(rc)
        n = oc * K
        self.oc, self.K = oc, K
        self.sign = np.ctypeslib.as_array(self._q.sign, shape=(n,)).reshape(oc, K)
        self.shift = np.ctypeslib.as_array(self._q.shift, shape=(n,)).reshape(oc, K)
        self.p = np.ctypeslib.as_array(self._q.p, shape=(n,)).reshape(oc, K)
        i = self._q.info
        self.e_top, self.e_min = i.e_top, i.e_min
        self.n_zero, self.n_flushed, self.n_live = i.n_zero, i.n_flushed, i.n_live
        self.s_max = s_max
        self.shape = w.shape

    def __del__(self):
        # at interpreter shutdown the module globals may already be gone: then the process frees the memory
        if getattr(self, "_q", None) is not None and lib is not None and C is not None:
            self.sign = self.shift = self.p = None
            lib().psbo_weights_free(C.byref(self._q))
            self._q = None

    def represented(self):
        """The real numbers the encoding stands for: s 2^e (1+p); 0 when not live."""
        return self.sign.astype(np.float64) * np.ldexp(1.0 + self.p, self.shift + self.e_min)


def linear(q, x, S, seed=0, layer_id=0, u_table=None):
    """acc[B, OC] (int32), number of outputs whose exact sum leaves int32."""
    x = np.ascontiguousarray(x, dtype=np.int8)
    B = x.shape[0]
    assert x.shape[1] == q.K
    acc = np.zeros((B, q.oc), dtype=np.int32)
    over = C.c_int64(0)
    if u_table is not None:
        u_table = np.ascontiguousarray(u_table, dtype=np.uint32)
        assert u_table.size == B * q.oc * q.K * S
    rc = lib().psbo_linear(C.byref(q._q), _ptr(x), B, S, int(seed), int(layer_id), _ptr(u_table), _ptr(acc),
                           C.byref(over))
    if rc != OK:
        raise OracleError(rc)
    return acc, over.value


def out_hw(h, w, kh, kw, stride, pad):
    sh, sw = stride
    ph, pw = pad
    return (h + 2 * ph - kh) // sh + 1, (w + 2 * pw - kw) // sw + 1


def conv2d(q, wshape, x, stride=(1, 1), pad=(0, 0), S=None, s_max=None, budget_to=None, budget_from=None,
           seed=0, layer_id=0, points=None, acc_in=None):
    """wshape = (oc, cin, kh, kw, groups); x int8 [n, cin, h, w].

    Returns (acc, overflow_count, n_smac).  acc is [n, oc, oh, ow], or [len(points)] when points is given.
    """
    oc, cin, kh, kw, groups = wshape
    x = np.ascontiguousarray(x, dtype=np.int8)
    n, c, h, w = x.shape
    assert c == cin
    ws = WShape(oc, cin, kh, kw, groups)
    g = Geom(n, h, w, stride[0], stride[1], pad[0], pad[1])
    oh, ow = out_hw(h, w, kh, kw, stride, pad)
    if s_max is None:
        s_max = q.s_max
    if budget_to is not None:
        budget_to = np.ascontiguousarray(budget_to, dtype=np.uint8)
        assert budget_to.shape == (n, oh, ow)
    if budget_from is not None:
        budget_from = np.ascontiguousarray(budget_from, dtype=np.uint8)
        assert budget_from.shape == (n, oh, ow)
    if points is not None:
        points = np.ascontiguousarray(points, dtype=np.int64)
        shape = (points.size,)
    else:
        shape = (n, oc, oh, ow)
    if budget_from is not None:
        assert acc_in is not None
        acc = np.ascontiguousarray(acc_in, dtype=np.int32).copy().reshape(shape)
    else:
        acc = np.zeros(shape, dtype=np.int32)
    over, smac = C.c_int64(0), C.c_int64(0)
    rc = lib().psbo_conv2d(C.byref(q._q), C.byref(ws), _ptr(x), C.byref(g), 0 if S is None else int(S),
                           int(s_max), _ptr(budget_to), _ptr(budget_from), int(seed), int(layer_id),
                           _ptr(points), 0 if points is None else points.size, _ptr(acc),
                           C.byref(over), C.byref(smac))
    if rc != OK:
        raise OracleError(rc)
    return acc, over.value, smac.value


def sample_filter(q, S=None, seed=0, layer_id=0, sample_from=0, sample_to=None, u_table=None):
    """W int64 [oc, K] = sigma 2^shift ((to-from) + count) for samples [from, to) of every weight."""
    if sample_to is None:
        sample_to = S
    W = np.zeros((q.oc, q.K), dtype=np.int64)
    table_S = 0
    if u_table is not None:
        u_table = np.ascontiguousarray(u_table, dtype=np.uint32)
        table_S = u_table.size // (q.oc * q.K)
        assert u_table.size == q.oc * q.K * table_S
    rc = lib().psbo_sample_filter(C.byref(q._q), int(sample_from), int(sample_to), int(seed), int(layer_id),
                                  _ptr(u_table), table_S, _ptr(W))
    if rc != OK:
        raise OracleError(rc)
    return W


def conv2d_shared(q, wshape, x, stride=(1, 1), pad=(0, 0), S=None, s_max=None, budget_to=None, budget_from=None,
                  seed=0, layer_id=0, acc_in=None, points=None):
    """Shared-filter layer: (acc int32 [n, oc, oh, ow] or [len(points)], overflow count)."""
    oc, cin, kh, kw, groups = wshape
    x = np.ascontiguousarray(x, dtype=np.int8)
    n, c, h, w = x.shape
    assert c == cin
    ws = WShape(oc, cin, kh, kw, groups)
    g = Geom(n, h, w, stride[0], stride[1], pad[0], pad[1])
    oh, ow = out_hw(h, w, kh, kw, stride, pad)
    if s_max is None:
        s_max = q.s_max
    if budget_to is not None:
        budget_to = np.ascontiguousarray(budget_to, dtype=np.uint8)
        assert budget_to.shape == (n, oh, ow)
    if budget_from is not None:
        budget_from = np.ascontiguousarray(budget_from, dtype=np.uint8)
        assert budget_from.shape == (n, oh, ow) and acc_in is not None
    if points is not None:
        points = np.ascontiguousarray(points, dtype=np.int64)
        shape = (points.size,)
    else:
        shape = (n, oc, oh, ow)
    if budget_from is not None:
        acc = np.ascontiguousarray(acc_in, dtype=np.int32).copy().reshape(shape)
    else:
        acc = np.zeros(shape, dtype=np.int32)
    over = C.c_int64(0)
    rc = lib().psbo_conv2d_shared(C.byref(q._q), C.byref(ws), _ptr(x), C.byref(g), 0 if S is None else int(S),
                                  int(s_max), _ptr(budget_to), _ptr(budget_from), int(seed), int(layer_id),
                                  _ptr(points), 0 if points is None else points.size, _ptr(acc), C.byref(over))
    if rc != OK:
        raise OracleError(rc)
    return acc, over.value


def rescale(acc, e_min, S=None, s_max=255, budget_to=None, mult=None, bias=None):
    """acc [n, oc, ...] int32 -> y float32 of the same shape."""
    acc = np.ascontiguousarray(acc, dtype=np.int32)
    n, oc = acc.shape[0], acc.shape[1]
    spatial = int(np.prod(acc.shape[2:])) if acc.ndim > 2 else 1
    y = np.zeros(acc.shape, dtype=np.float32)
    if budget_to is not None:
        budget_to = np.ascontiguousarray(budget_to, dtype=np.uint8)
        assert budget_to.size == n * spatial
    if mult is not None:
        mult = np.ascontiguousarray(mult, dtype=np.float32)
    if bias is not None:
        bias = np.ascontiguousarray(bias, dtype=np.float32)
    rc = lib().psbo_rescale(_ptr(acc), n, oc, spatial, 0 if S is None else int(S), int(s_max), _ptr(budget_to),
                            int(e_min), _ptr(mult), _ptr(bias), _ptr(y))
    if rc != OK:
        raise OracleError(rc)
    return y


def requantize(y, inv_step, relu=True, lo=0, hi=127, res_f32=None, res_i8=None, res_step=0.0):
    """int8 array of y's shape: clamp(rint(g(y [+ r]) * inv_step), lo, hi)."""
    y = np.ascontiguousarray(y, dtype=np.float32)
    out = np.zeros(y.shape, dtype=np.int8)
    if res_f32 is not None:
        res_f32 = np.ascontiguousarray(res_f32, dtype=np.float32)
        assert res_f32.shape == y.shape
    if res_i8 is not None:
        res_i8 = np.ascontiguousarray(res_i8, dtype=np.int8)
        assert res_i8.shape == y.shape
    rc = lib().psbo_requantize(_ptr(y), _ptr(res_f32), _ptr(res_i8), float(np.float32(res_step)), 1 if relu else 0,
                               float(np.float32(inv_step)), int(lo), int(hi), y.size, _ptr(out))
    if rc != OK:
        raise OracleError(rc)
    return out


def maxpool_i8(x, kernel, stride, pad):
    x = np.ascontiguousarray(x, dtype=np.int8)
    n, c, h, w = x.shape
    oh, ow = out_hw(h, w, kernel[0], kernel[1], stride, pad)
    out = np.zeros((n, c, oh, ow), dtype=np.int8)
    rc = lib().psbo_maxpool_i8(_ptr(x), n, c, h, w, kernel[0], kernel[1], stride[0], stride[1], pad[0], pad[1],
                               _ptr(out))
    if rc != OK:
        raise OracleError(rc)
    return out


def avgpool_requantize(x, scale, lo=0, hi=127):
    x = np.ascontiguousarray(x, dtype=np.int8)
    n, c, h, w = x.shape
    out = np.zeros((n, c), dtype=np.int8)
    rc = lib().psbo_avgpool_requantize(_ptr(x), n, c, h, w, float(np.float32(scale)), int(lo), int(hi), _ptr(out))
    if rc != OK:
        raise OracleError(rc)
    return out


def budget_resample(b, oh, ow):
    b = np.ascontiguousarray(b, dtype=np.uint8)
    n, h, w = b.shape
    out = np.zeros((n, oh, ow), dtype=np.uint8)
    rc = lib().psbo_budget_resample(_ptr(b), n, h, w, oh, ow, _ptr(out))
    if rc != OK:
        raise OracleError(rc)
    return out


def attention_budget(act, step, lo, hi):
    """(entropy float32 [n,h,w], mean float32 [n], budget uint8 [n,h,w]) from int8 activations [n,c,h,w]."""
    act = np.ascontiguousarray(act, dtype=np.int8)
    n, c, h, w = act.shape
    ent = np.zeros((n, h, w), dtype=np.float32)
    mean = np.zeros(n, dtype=np.float32)
    bud = np.zeros((n, h, w), dtype=np.uint8)
    rc = lib().psbo_attention_budget(_ptr(act), float(np.float32(step)), n, c, h, w, int(lo), int(hi), _ptr(ent),
                                     _ptr(mean), _ptr(bud))
    if rc != OK:
        raise OracleError(rc)
    return ent, mean, bud
