"""The C-ABI library loads without a GPU, exports what include/psb.h declares, and rejects bad
arguments on the host before any device work."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def psb():
    from paper_1904_02205_amd import psb as m
    m.lib()
    return m


def _declared():
    text = open(os.path.join(ROOT, "include", "psb.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(psb_[a-z0-9_]+)\s*\(", text)))


def test_header_and_library_agree(psb):
    names = _declared()
    assert set(names) == set(psb.SYMBOLS)
    L = C.CDLL(psb.library_path())
    for n in names:
        assert getattr(L, n) is not None


def test_out_dims_and_shape_errors(psb):
    assert psb.conv2d_out_dims((64, 64, 3, 3, 1), (1, 56, 56, 1, 1, 1, 1)) == (56, 56)
    assert psb.conv2d_out_dims((64, 3, 7, 7, 1), (32, 224, 224, 2, 2, 3, 3)) == (112, 112)
    assert psb.conv2d_out_dims((128, 64, 1, 1, 1), (2, 56, 56, 2, 2, 0, 0)) == (28, 28)
    assert psb.conv2d_out_dims((8, 8, 2, 3, 2), (1, 6, 8, 1, 2, 0, 2)) == (5, 5)
    bad = [((0, 64, 3, 3, 1), (1, 8, 8, 1, 1, 1, 1), psb.ERR_SHAPE),
           ((64, 64, 3, 3, 3), (1, 8, 8, 1, 1, 1, 1), psb.ERR_SHAPE),       # groups do not divide
           ((64, 64, 3, 3, 1), (1, 8, 8, 0, 1, 1, 1), psb.ERR_SHAPE),       # stride 0
           ((64, 64, 3, 3, 1), (1, 8, 8, 1, 1, -1, 1), psb.ERR_SHAPE),
           ((64, 64, 9, 9, 1), (1, 4, 4, 1, 1, 1, 1), psb.ERR_SHAPE),       # kernel larger than padded input
           ((64, 64, 3, 3, 1), (0, 8, 8, 1, 1, 1, 1), psb.ERR_SHAPE),
           ((1024, 64, 1, 1, 1), (4096, 64, 64, 1, 1, 0, 0), psb.ERR_TOO_LARGE),   # 2^34 outputs
           ((64, 1 << 22, 3, 3, 1), (1, 8, 8, 1, 1, 1, 1), psb.ERR_TOO_LARGE),     # K >= 2^24
           ((4, 1, 1 << 15, 1, 1), (1, 1 << 16, 1, 1, 1, 0, 0), psb.ERR_TOO_LARGE)]  # a kernel side of 2^15
    for ws, g, code in bad:
        with pytest.raises(psb.PsbError) as ei:
            psb.conv2d_out_dims(ws, g)
        assert ei.value.code == code
    L = psb.lib()
    assert L.psb_conv2d_out_dims(None, None, None, None) == psb.ERR_NULL


def test_null_arguments_are_rejected_before_any_device_work(psb):
    L = psb.lib()
    g = psb.ConvGeom(1, 8, 8, 1, 1, 1, 1)
    ws = psb.WShape(4, 4, 3, 3, 1)
    h = C.c_void_p(None)
    assert L.psb_quantize_weights(None, C.byref(ws), 23, 0, 127, 8, None, C.byref(h)) == psb.ERR_NULL
    assert L.psb_quantize_weights(C.c_void_p(16), None, 23, 0, 127, 8, None, C.byref(h)) == psb.ERR_NULL
    assert L.psb_quantize_weights(C.c_void_p(16), C.byref(ws), 23, 0, 127, 8, None, None) == psb.ERR_NULL
    # value errors are found before the pointer is ever dereferenced
    for prob_bits, exp_bits, xmax, smax in ((24, 0, 127, 8), (0, 0, 127, 8), (32, 0, 127, 8), (-3, 0, 127, 8),
                                            (23, 6, 127, 8), (23, 0, 0, 8), (23, 0, 129, 8),
                                            (23, 0, 127, 0), (23, 0, 127, 256)):
        assert L.psb_quantize_weights(C.c_void_p(16), C.byref(ws), prob_bits, exp_bits, xmax, smax, None,
                                      C.byref(h)) == psb.ERR_VALUE
    bad_ws = psb.WShape(4, 4, 0, 3, 1)
    assert L.psb_quantize_weights(C.c_void_p(16), C.byref(bad_ws), 23, 0, 127, 8, None, C.byref(h)) == psb.ERR_SHAPE
    assert L.psb_weights_info(None, None) == psb.ERR_NULL
    assert L.psb_weights_export(None, None) == psb.ERR_NULL
    L.psb_weights_destroy(None)
    assert L.psb_linear(None, None, 1, 1, 0, 0, None, None, None, None, None) == psb.ERR_NULL
    assert L.psb_conv2d(None, None, C.byref(g), 1, 0, 0, None, None, None, None, None) == psb.ERR_NULL
    assert L.psb_conv2d_progressive(None, None, C.byref(g), None, None, 0, 0, None, None, None, None, None) == psb.ERR_NULL
    assert L.psb_last_device_error() == 0


def test_later_entry_points_validate_on_the_host(psb):
    """Shared-filter, glue and attention entry points: every argument error is found before any device work."""
    L = psb.lib()
    g = psb.ConvGeom(1, 8, 8, 1, 1, 1, 1)
    P = C.c_void_p(16)                       # a non-NULL pointer that is never dereferenced
    assert L.psb_sample_filter(None, 0, 4, 0, 0, P, None) == psb.ERR_NULL
    assert L.psb_linear_shared(None, P, 1, 1, 0, 0, P, None, None, None, None) == psb.ERR_NULL
    assert L.psb_conv2d_shared(None, P, C.byref(g), 1, 0, 0, P, None, None, None, None) == psb.ERR_NULL
    assert L.psb_conv2d_progressive_shared(None, P, C.byref(g), P, None, 0, 0, P, None, None, None, None) == psb.ERR_NULL
    assert L.psb_conv2d_requant(None, P, C.byref(g), 4, None, 0, 0, P, None, None, None, None, P, 0, None) == psb.ERR_NULL
    # the chained shared-filter pass
    bl = L.psb_conv2d_shared_requant_blocked
    assert bl(None, P, C.byref(g), 4, 0, 0, None, None, None, None, P, 0, None) == psb.ERR_NULL
    pf = L.psb_shared_prepare_filters
    assert pf(None, 1, 4, P, P, None) == psb.ERR_NULL
    assert pf(P, 1, 4, None, P, None) == psb.ERR_NULL
    assert pf(P, 0, 4, P, P, None) == psb.ERR_SHAPE
    handles = (C.c_void_p * 1)(None)
    assert pf(handles, 1, 4, P, P, None) == psb.ERR_NULL                             # a NULL handle in the list
    # announced budget values (host-only state of the calling thread)
    lv = L.psb_shared_budget_levels
    assert lv(None, 1) == psb.ERR_NULL
    assert lv(None, -1) == psb.ERR_SHAPE and lv(None, 257) == psb.ERR_SHAPE
    two = (C.c_uint8 * 2)(8, 16)
    assert lv(two, 2) == psb.OK
    assert lv(None, 0) == psb.OK                                                      # back to the default
    # requantize
    rq = L.psb_requantize
    for inv in (-1.0, float("nan")):
        assert rq(P, None, None, 0.0, 1, inv, 0, 127, 8, P, None) == psb.ERR_VALUE   # the step cannot be negative
    assert rq(None, None, None, 0.0, 1, 1.0, 0, 127, 8, P, None) == psb.ERR_NULL
    assert rq(P, None, None, 0.0, 1, 1.0, 0, 127, 8, None, None) == psb.ERR_NULL
    assert rq(P, None, None, 0.0, 1, 1.0, 0, 127, 0, P, None) == psb.ERR_SHAPE
    assert rq(P, P, P, 0.0, 1, 1.0, 0, 127, 8, P, None) == psb.ERR_VALUE             # two residual operands
    for lo, hi in ((-129, 0), (0, 128), (5, 4)):
        assert rq(P, None, None, 0.0, 1, 1.0, lo, hi, 8, P, None) == psb.ERR_VALUE
    # pooling
    mp = L.psb_maxpool2d_i8
    assert mp(None, 1, 1, 8, 8, 3, 3, 2, 2, 1, 1, P, None) == psb.ERR_NULL
    assert mp(P, 1, 1, 8, 8, 3, 3, 0, 2, 1, 1, P, None) == psb.ERR_SHAPE              # stride 0
    assert mp(P, 1, 1, 8, 8, 2, 2, 2, 2, 2, 2, P, None) == psb.ERR_SHAPE              # a window inside the padding
    assert mp(P, 1, 1, 2, 2, 5, 5, 1, 1, 1, 1, P, None) == psb.ERR_SHAPE              # kernel larger than padded image
    mb = L.psb_maxpool2d_i8_blocked
    assert mb(None, 1, 1, 8, 8, 3, 3, 2, 2, 1, 1, P, None) == psb.ERR_NULL
    assert mb(P, 1, 1, 8, 8, 3, 3, 2, 0, 1, 1, P, None) == psb.ERR_SHAPE
    assert mb(P, 1, 1, 8, 8, 2, 2, 2, 2, 2, 2, P, None) == psb.ERR_SHAPE
    ap = L.psb_global_avgpool_requantize
    assert ap(None, 1, 1, 7, 7, 1.0, 0, 127, P, None) == psb.ERR_NULL
    assert ap(P, 0, 1, 7, 7, 1.0, 0, 127, P, None) == psb.ERR_SHAPE
    assert ap(P, 1, 1, 4096, 4096, 1.0, 0, 127, P, None) == psb.ERR_TOO_LARGE         # 2^24 positions per image
    assert ap(P, 1, 1, 7, 7, 1.0, 3, 2, P, None) == psb.ERR_VALUE
    rs = L.psb_budget_resample
    assert rs(None, 1, 7, 7, 14, 14, P, None) == psb.ERR_NULL
    assert rs(P, 1, 7, 7, 0, 14, P, None) == psb.ERR_SHAPE
    # attention
    at = L.psb_attention_budget
    assert at(None, 0.1, 1, 8, 7, 7, 8, 16, P, None, P, None) == psb.ERR_NULL
    assert at(P, 0.1, 1, 8, 7, 7, 8, 16, None, None, P, None) == psb.ERR_NULL
    assert at(P, 0.1, 1, 0, 7, 7, 8, 16, P, None, P, None) == psb.ERR_SHAPE
    for step in (0.0, -1.0, float("nan"), float("inf")):
        assert at(P, step, 1, 8, 7, 7, 8, 16, P, None, P, None) == psb.ERR_VALUE
    assert L.psb_last_device_error() == 0


def test_query_mapping_null_arguments(psb):
    L = psb.lib()
    g = psb.ConvGeom(1, 8, 8, 1, 1, 1, 1)
    assert L.psb_query_mapping(None, C.byref(g)) == psb.ERR_NULL
    assert L.psb_query_mapping(C.c_void_p(16), None) == psb.ERR_NULL


def test_mapping_switch(psb):
    prev = psb.set_mapping(psb.MAPPING_PIXEL_LANE)
    assert psb.set_mapping(99) == psb.MAPPING_PIXEL_LANE      # out of range: ignored
    assert psb.set_mapping(prev) == psb.MAPPING_PIXEL_LANE


def test_binding_refuses_cpu_tensors(psb):
    import torch
    with pytest.raises(TypeError):
        psb.Weights(torch.zeros(4, 4, 3, 3))


def _fake_handle(psb, wshape):
    """A handle object without a library handle behind it: the binding must refuse wrong shapes before it would
    dereference anything."""
    q = object.__new__(psb.Weights)
    q.wshape = wshape
    q.K = wshape[1] // wshape[4] * wshape[2] * wshape[3]
    q.s_max, q.prob_bits, q._h = 16, 23, C.c_void_p(None)
    return q


def test_binding_refuses_wrong_tensor_shapes(psb):
    """The C-ABI takes raw pointers and cannot check sizes: every tensor's shape is compared with what the handle
    and the geometry imply, and a mismatch is a ValueError before any pointer is handed over."""
    import torch
    q = _fake_handle(psb, (6, 4, 3, 3, 1))
    x = torch.zeros((2, 4, 8, 8), dtype=torch.int8)
    ok_acc = torch.zeros((2, 6, 8, 8), dtype=torch.int32)
    with pytest.raises(ValueError, match="x: shape"):
        psb.conv2d(q, torch.zeros((2, 5, 8, 8), dtype=torch.int8), 8, pad=(1, 1), acc=ok_acc)     # wrong channel count
    with pytest.raises(ValueError, match="x: shape"):
        psb.conv2d(q, torch.zeros((2, 4, 8), dtype=torch.int8), 8, pad=(1, 1), acc=ok_acc)
    with pytest.raises(ValueError, match="acc"):
        psb.conv2d(q, x, 8, pad=(1, 1), acc=torch.zeros((2, 6, 8, 7), dtype=torch.int32))
    with pytest.raises(ValueError, match="y"):
        psb.conv2d(q, x, 8, pad=(1, 1), acc=ok_acc, y=torch.zeros((2, 6, 6, 6)))
    with pytest.raises(ValueError, match="mult"):
        psb.conv2d(q, x, 8, pad=(1, 1), acc=ok_acc, mult=torch.zeros(5))
    with pytest.raises(ValueError, match="bias"):
        psb.conv2d(q, x, 8, pad=(1, 1), acc=ok_acc, bias=torch.zeros(7))
    bt = torch.zeros((2, 8, 8), dtype=torch.uint8)
    with pytest.raises(ValueError, match="budget_to"):
        psb.conv2d_progressive(q, x, torch.zeros((2, 8, 9), dtype=torch.uint8), pad=(1, 1), acc=ok_acc)
    with pytest.raises(ValueError, match="budget_from"):
        psb.conv2d_progressive(q, x, bt, torch.zeros((1, 8, 8), dtype=torch.uint8), pad=(1, 1), acc=ok_acc)
    xo = torch.zeros((2, 6, 8, 8), dtype=torch.int8)
    with pytest.raises(ValueError, match="x_out"):
        psb.conv2d_requant(q, x, 1.0, S=8, pad=(1, 1), acc=ok_acc, x_out=torch.zeros((2, 6, 8), dtype=torch.int8))
    with pytest.raises(ValueError, match="res_i8"):
        psb.conv2d_requant(q, x, 1.0, S=8, pad=(1, 1), acc=ok_acc, x_out=xo, res_i8=torch.zeros((2, 4, 8, 8), dtype=torch.int8))
    with pytest.raises(ValueError, match="res_f32"):
        psb.conv2d_requant(q, x, 1.0, S=8, pad=(1, 1), acc=ok_acc, x_out=xo, res_f32=torch.zeros((2, 6, 8, 9)))
    with pytest.raises(ValueError, match="x_out"):
        psb.conv2d_requant_static(q, x, 1.0, torch.zeros((2, 6, 7, 8), dtype=torch.int8), S=8, pad=(1, 1))
    # blocked layouts
    xb = torch.zeros(psb.blocked_shape(2, 4, 8, 8), dtype=torch.int8)
    with pytest.raises(ValueError, match="x: shape"):
        psb.conv2d_shared_requant_blocked(q, x, (2, 4, 8, 8), 1.0, 8, pad=(1, 1), layout=psb.BLOCKED_IN)
    with pytest.raises(ValueError, match="x_shape"):
        psb.conv2d_shared_requant_blocked(q, xb, (2, 5, 8, 8), 1.0, 8, pad=(1, 1), layout=psb.BLOCKED_IN)
    with pytest.raises(ValueError, match="x_out"):
        psb.conv2d_shared_requant_blocked(q, xb, (2, 4, 8, 8), 1.0, 8, pad=(1, 1), layout=psb.BLOCKED_IN | psb.BLOCKED_OUT,
                                          x_out=xo)
    with pytest.raises(ValueError, match="res_i8"):
        psb.conv2d_shared_requant_blocked(q, xb, (2, 4, 8, 8), 1.0, 8, pad=(1, 1), layout=psb.BLOCKED_IN | psb.BLOCKED_RES,
                                          x_out=xo, res_i8=xo)
    # linear layers
    ql = _fake_handle(psb, (6, 20, 1, 1, 1))
    with pytest.raises(ValueError, match="x: shape"):
        psb.linear(ql, torch.zeros((3, 21), dtype=torch.int8), 8)
    with pytest.raises(ValueError, match="x: shape"):
        psb.linear(q, torch.zeros((3, 36), dtype=torch.int8), 8)                # a convolution's handle
    with pytest.raises(ValueError, match="acc"):
        psb.linear(ql, torch.zeros((3, 20), dtype=torch.int8), 8, acc=torch.zeros((3, 5), dtype=torch.int32))
    # glue
    y = torch.zeros((2, 3, 4, 4))
    with pytest.raises(ValueError, match="out"):
        psb.requantize(y, 1.0, out=torch.zeros((2, 3, 4, 5), dtype=torch.int8))
    with pytest.raises(ValueError, match="res_i8"):
        psb.requantize(y, 1.0, res_i8=torch.zeros((2, 3, 4), dtype=torch.int8), out=torch.zeros((2, 3, 4, 4), dtype=torch.int8))
    xi = torch.zeros((2, 3, 8, 8), dtype=torch.int8)
    with pytest.raises(ValueError, match="out"):
        psb.maxpool2d_i8(xi, (3, 3), (2, 2), (1, 1), out=torch.zeros((2, 3, 4, 5), dtype=torch.int8))
    with pytest.raises(ValueError, match="out"):
        psb.global_avgpool_requantize(xi, 1.0, out=torch.zeros((2, 4), dtype=torch.int8))
    with pytest.raises(ValueError, match="x"):
        psb.maxpool2d_i8_blocked(xi, (2, 3, 8, 8), (3, 3), (2, 2), (1, 1))           # not the blocked form
    with pytest.raises(ValueError, match="out"):
        psb.maxpool2d_i8_blocked(torch.zeros((2, 8, 1, 8, 32), dtype=torch.int8), (2, 3, 8, 8), (3, 3), (2, 2), (1, 1),
                                 out=torch.zeros((2, 4, 1, 5, 32), dtype=torch.int8))
    with pytest.raises(ValueError, match="out"):
        psb.budget_resample(torch.zeros((2, 4, 4), dtype=torch.uint8), 8, 8, out=torch.zeros((2, 8, 7), dtype=torch.uint8))
    with pytest.raises(ValueError, match="out"):
        psb.sample_filter(q, 8, out=torch.zeros((6, 35), dtype=torch.int32))


def test_static_entry_point_rejects_on_the_host(psb):
    L = psb.lib()
    g = psb.ConvGeom(1, 8, 8, 1, 1, 1, 1)
    rq = psb.Requant(1, 1.0, 0, 127, None, None, 0.0)
    dummy = C.c_void_p(16)
    assert L.psb_conv2d_requant_static(None, dummy, C.byref(g), 8, None, 0, 0, None, None, None, C.byref(rq), dummy,
                                       None) == psb.ERR_NULL
    assert psb.STATIC_MAX_OUTPUTS == 8 * 1024 * 1024
    text = open(os.path.join(ROOT, "include", "psb.h")).read()
    assert "#define PSB_STATIC_MAX_OUTPUTS (8 * 1024 * 1024)" in text


def test_window_of_the_3x3_shared_filter_kernel_covers_every_tile(psb):
    """Host logic: the slot count that the launcher reserves per pixel tile is an upper bound of what any tile of
    any batch needs - brute force over every tile start of small geometries - and geometries the kernel does not
    take answer 0."""
    def vpos(pix, h, w):
        n, r = divmod(pix, h * w)
        oy, ox = divmod(r, w)
        return (n * (h + 1) + oy) * (w + 1) + ox
    for h, w in ((1, 1), (1, 9), (9, 1), (2, 3), (4, 4), (7, 7), (14, 14), (5, 28), (28, 28), (13, 56), (56, 56), (3, 100)):
        for ht in (1, 2):
            T = 128 * ht
            slots = psb.shared_window_slots((3, 3), (1, h, w, 1, 1, 1, 1), ht)
            need = 0
            period = h * w                               # tile starts repeat with the image
            for start in range(0, period * T, T):        # every residue of a tile start modulo the image size
                need = max(need, vpos(start + T - 1, h, w) - vpos(start, h, w) + 2 * (w + 1) + 3)
                if start // T > 4 * period:
                    break
            if slots:
                assert need <= slots <= 512, (h, w, ht, need, slots)
            else:
                assert need > 0                          # refused: more than 512 slots by the launcher's bound
                rows, images = (T + w - 2) // w, (T + h * w - 2) // (h * w)
                assert T - 1 + rows + images * (w + 1) + 2 * (w + 1) + 3 > 512
    g = (2, 14, 14, 1, 1, 1, 1)
    assert psb.shared_window_slots((3, 3), g, 1) > 0
    for kernel, geom in (((1, 1), g), ((3, 1), g), ((5, 5), g), ((3, 3), (2, 14, 14, 2, 1, 1, 1)), ((3, 3), (2, 14, 14, 1, 1, 0, 1)),
                         ((3, 3), (2, 14, 14, 1, 1, 1, 2)), ((3, 3), (1, 8, 300, 1, 1, 1, 1))):
        assert psb.shared_window_slots(kernel, geom, 1) == 0, (kernel, geom)
    L = psb.lib()
    assert L.psb_shared_window_slots(3, 3, None, 1) == psb.ERR_NULL
    gg = psb.ConvGeom(*g)
    import ctypes
    assert L.psb_shared_window_slots(3, 3, ctypes.byref(gg), 3) == psb.ERR_SHAPE
    assert L.psb_shared_window_slots(0, 3, ctypes.byref(gg), 1) == psb.ERR_SHAPE


def test_micro_benchmarks_compile(tmp_path):
    """The two stand-alone micro-benchmarks beside bench.py build with the line build() uses."""
    import subprocess
    import __graft_entry__ as entry
    for name in entry.MICRO_BENCHMARKS:
        out = tmp_path / name
        r = subprocess.run(entry.micro_benchmark_command(name, str(out)), capture_output=True, text=True)
        assert r.returncode == 0, r.stderr[-2000:]
        assert out.exists()
