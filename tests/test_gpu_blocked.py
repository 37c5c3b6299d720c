"""The chained shared-filter pass: blocked channels-last int8 tensors on any side of a layer call, and filters
sampled ahead of the calls in one launch.  Expected values come from the oracle's plain chain
(shared-filter layer -> rescale -> requantize) on [N][C][H][W] tensors; the layout conversions of this file are
plain numpy."""
import ctypes

import numpy as np
import pytest

import helpers
from test_gpu_parity import _layer

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def psb():
    from paper_1904_02205_amd import psb as m
    m.lib()
    m.set_mapping(m.MAPPING_AUTO)
    return m


def to_blocked(t, fill):
    """[n, c, h, w] int8 -> [n, h, ceil(c/32), w, 32]; the padding channels hold `fill` (they must be ignored)."""
    n, c, h, w = t.shape
    cb = (c + 31) // 32
    full = np.full((n, cb * 32, h, w), fill, dtype=np.int8)
    full[:, :c] = t
    return np.ascontiguousarray(full.reshape(n, cb, 32, h, w).transpose(0, 3, 1, 4, 2))


def from_blocked(tb, c):
    n, h, cb, w, _ = tb.shape
    return np.ascontiguousarray(tb.transpose(0, 2, 4, 1, 3).reshape(n, cb * 32, h, w)[:, :c])


CASES = [
    dict(n=2, c=40, oc=70, hw=(9, 11), k=3, pad=1, S=8),            # padding channels on both sides, OH*OW odd
    dict(n=2, c=64, oc=64, hw=8, k=3, stride=2, pad=1, S=4),        # whole blocks, OH*OW a multiple of 4
    dict(n=1, c=256, oc=64, hw=6, k=3, pad=1, S=8),                 # split reduction: separate rescale pass
    dict(n=3, c=33, oc=32, hw=(5, 8), k=1, S=16),                   # 1x1, one channel in the second block
    dict(n=1, c=32, oc=40, hw=(260, 264), k=3, pad=1, S=4),         # many pixel tiles: the persistent kernel variant
    dict(n=2, c=128, oc=64, hw=14, k=3, pad=1, S=8),                # 3x3 with both operands in LDS, two teams
    dict(n=2, c=32, oc=480, hw=50, k=3, pad=1, S=4),                # ... two half tiles per wave
]


@pytest.mark.parametrize("case", CASES)
def test_blocked_tensors_on_every_side(psb, orc, case):
    import torch
    rng = np.random.default_rng(9)
    L = _layer(rng, **case)
    oc = L.w.shape[0]
    n, c, h, w = L.x.shape
    oh, ow = L.out_hw
    shape = (n, oc, oh, ow)
    mult = (rng.uniform(0.5, 2.0, size=oc) * 2.0 ** -6).astype(np.float32)
    bias = rng.standard_normal(oc).astype(np.float32)
    qo, qg = helpers.oracle_quantize(orc, L), helpers.gpu_quantize(psb, L)
    acc, _, _ = helpers.oracle_layer(orc, L, qo, shared=True)
    y = orc.rescale(acc, qo.e_min, S=L.S, s_max=L.s_max, mult=mult, bias=bias)
    res = (rng.standard_normal(shape) * 2).astype(np.float32)
    res.reshape(-1)[:6] = np.array([np.nan, np.inf, -np.inf, -0.0, 1e30, -1e30], np.float32)   # special values
    res8 = rng.integers(-128, 128, size=shape).astype(np.int8)
    inv = float(np.float32(127.0 / 6.0))
    x_plain = torch.from_numpy(L.x).cuda()
    x_blocked = torch.from_numpy(to_blocked(L.x, 77)).cuda()
    kw = dict(stride=L.stride, pad=L.pad, seed=L.seed, layer_id=L.layer_id, mult=torch.from_numpy(mult).cuda(),
              bias=torch.from_numpy(bias).cuda())
    # the rescaled values alone, from either input layout
    for layout in (0, psb.BLOCKED_IN):
        got = psb.conv2d_shared_requant_blocked(qg, x_blocked if layout else x_plain, L.x.shape, 0.0, L.S,
                                                layout=layout, want_x=False, **kw)
        assert np.array_equal(got.cpu().numpy(), y), layout
    variants = [(dict(), dict(), False),
                (dict(res_f32=res), dict(res_f32=torch.from_numpy(res).cuda()), False),
                (dict(res_i8=res8, res_step=np.float32(0.05)), dict(res_step=float(np.float32(0.05))), True),
                (dict(relu=False, lo=-128, hi=127), dict(relu=False, lo=-128, hi=127), False),
                (dict(res_f32=res, relu=False, lo=-100, hi=50),
                 dict(res_f32=torch.from_numpy(res).cuda(), relu=False, lo=-100, hi=50), False)]
    for kw_o, kw_g, with_res8 in variants:
        ref = orc.requantize(y, inv, **kw_o)
        for layout in range(8):
            if (layout & psb.BLOCKED_RES) and not with_res8:
                continue
            kw_l = dict(kw_g)
            if with_res8:
                r8 = to_blocked(res8, -5) if layout & psb.BLOCKED_RES else res8
                kw_l["res_i8"] = torch.from_numpy(r8).cuda()
            got = psb.conv2d_shared_requant_blocked(qg, x_blocked if layout & psb.BLOCKED_IN else x_plain, L.x.shape,
                                                    inv, L.S, layout=layout, **kw, **kw_l).cpu().numpy()
            if layout & psb.BLOCKED_OUT:
                assert got.shape == psb.blocked_shape(*shape)
                got = from_blocked(got, oc)
            assert np.array_equal(got, ref), (case, layout, list(kw_o))


def test_filters_sampled_ahead_give_the_same_results(psb, orc):
    import torch
    rng = np.random.default_rng(10)
    layers = [_layer(rng, 2, 40, 70, (9, 11), 3, pad=1, S=8, seed=21, layer_id=0),
              _layer(rng, 2, 3, 16, 20, 7, stride=2, pad=3, S=8, seed=22, layer_id=1),         # row-packed first layer
              _layer(rng, 2, 70, 70, 9, 3, pad=1, groups=70, S=8, seed=23, layer_id=2),        # not on the matrix cores
              _layer(rng, 1, 256, 64, 6, 3, pad=1, S=8, seed=24, layer_id=3)]                  # split reduction
    qs = [helpers.gpu_quantize(psb, L) for L in layers]
    xs = [torch.from_numpy(L.x).cuda() for L in layers]
    refs = [helpers.oracle_layer(orc, L, shared=True)[0] for L in layers]

    def run(i, S=None):
        L = layers[i]
        return psb.conv2d(qs[i], xs[i], L.S if S is None else S, stride=L.stride, pad=L.pad, seed=L.seed,
                          layer_id=L.layer_id, shared=True).cpu().numpy()

    psb.shared_prepare_filters(qs, 8, [L.seed for L in layers], [L.layer_id for L in layers])
    for i in range(len(layers)):
        assert np.array_equal(run(i), refs[i]), i          # uses the prepared planes
        assert np.array_equal(run(i), refs[i]), i          # samples for itself again
    # prepared for other parameters than the call's: the call samples its own filter
    psb.shared_prepare_filters(qs, 8, [L.seed + 1 for L in layers], [L.layer_id for L in layers])
    for i in range(len(layers)):
        assert np.array_equal(run(i), refs[i]), i
    psb.shared_prepare_filters(qs, 4, [L.seed for L in layers], [L.layer_id for L in layers])
    for i in range(len(layers)):
        assert np.array_equal(run(i), refs[i]), i
    # more handles than one launch takes
    many = [qs[0]] * 40
    psb.shared_prepare_filters(many, 8, [layers[0].seed] * 40, [layers[0].layer_id] * 40)
    assert np.array_equal(run(0), refs[0])
    with pytest.raises(psb.PsbError) as ei:
        psb.shared_prepare_filters(qs, 9, [0] * 4, [0] * 4)      # s_max is 8
    assert ei.value.code == psb.ERR_VALUE


def test_blocked_call_errors(psb):
    import torch
    rng = np.random.default_rng(12)
    first = _layer(rng, 1, 3, 16, 12, 7, stride=2, pad=3, S=8)                   # row-packed: takes [N][C][H][W] only
    dw = _layer(rng, 1, 64, 64, 6, 3, pad=1, groups=64, S=8)
    plain = _layer(rng, 1, 64, 32, 6, 3, pad=1, S=8)
    for L, code in ((first, psb.ERR_SHAPE), (dw, psb.ERR_SHAPE)):
        q = helpers.gpu_quantize(psb, L)
        xb = torch.from_numpy(to_blocked(L.x, 0)).cuda()
        with pytest.raises(psb.PsbError) as ei:
            psb.conv2d_shared_requant_blocked(q, xb, L.x.shape, 1.0, 8, stride=L.stride, pad=L.pad, layout=psb.BLOCKED_IN)
        assert ei.value.code == code
    q = helpers.gpu_quantize(psb, plain)
    xb = torch.from_numpy(to_blocked(plain.x, 0)).cuda()
    xn = torch.from_numpy(plain.x).cuda()
    shifted = torch.zeros(xb.numel() + 16, dtype=torch.int8, device="cuda")[1:1 + xb.numel()].view(xb.shape)
    for kw, code in ((dict(layout=8), psb.ERR_VALUE), (dict(layout=psb.BLOCKED_IN, S=9), psb.ERR_VALUE),
                     (dict(layout=psb.BLOCKED_IN, x=shifted), psb.ERR_VALUE)):
        args = dict(S=8, layout=0)
        args.update(kw)
        args.setdefault("x", xb if args["layout"] & psb.BLOCKED_IN else xn)      # the binding checks the shape
        with pytest.raises(psb.PsbError) as ei:
            psb.conv2d_shared_requant_blocked(q, args["x"], plain.x.shape, 1.0, args["S"], stride=plain.stride,
                                              pad=plain.pad, layout=args["layout"])
        assert ei.value.code == code
    lib = psb.lib()
    g = psb.ConvGeom(1, 6, 6, 1, 1, 1, 1)
    rc = lib.psb_conv2d_shared_requant_blocked(q._h, ctypes.c_void_p(xb.data_ptr()), ctypes.byref(g), 8, 0, 0, None,
                                               None, None, None, None, 0, None)
    assert rc == psb.ERR_NULL


def _random_blocked_case(i):
    rng = np.random.default_rng(9100 + i)
    kh, kw = int(rng.integers(1, 5)), int(rng.integers(1, 5))
    c = int(rng.integers(max(1, 32 // kw + 1), 100))          # more than 32 / kw channels: the layer can take blocked input
    oc = int(rng.integers(1, 100))
    sh, sw = int(rng.integers(1, 3)), int(rng.integers(1, 3))
    ph, pw = int(rng.integers(0, kh)), int(rng.integers(0, kw))
    h = max(int(rng.integers(1, 14)), kh - 2 * ph)
    w = max(int(rng.integers(1, 14)), kw - 2 * pw)
    n = int(rng.integers(1, 4))
    S = int(rng.integers(1, 17))
    return dict(n=n, c=c, oc=oc, hw=(h, w), k=(kh, kw), stride=(sh, sw), pad=(ph, pw), S=S, s_max=16,
                xkind=str(rng.choice(["relu", "signed"])), seed=int(rng.integers(0, 2 ** 40)),
                layer_id=int(rng.integers(0, 2 ** 31)))


@pytest.mark.parametrize("i", range(24))
def test_random_blocked_layer(psb, orc, i):
    """Seeded random shapes, every combination of blocked and plain tensors, int8 residual."""
    import torch
    case = _random_blocked_case(i)
    print(f"[blocked {i}] {case}", flush=True)
    rng = np.random.default_rng(9500 + i)
    L = _layer(rng, **case)
    oc = L.w.shape[0]
    oh, ow = L.out_hw
    shape = (L.x.shape[0], oc, oh, ow)
    mult = (rng.uniform(0.5, 2.0, size=oc) * 2.0 ** -6).astype(np.float32)
    bias = rng.standard_normal(oc).astype(np.float32)
    qo, qg = helpers.oracle_quantize(orc, L), helpers.gpu_quantize(psb, L)
    acc, _, _ = helpers.oracle_layer(orc, L, qo, shared=True)
    y = orc.rescale(acc, qo.e_min, S=L.S, s_max=L.s_max, mult=mult, bias=bias)
    res8 = rng.integers(-128, 128, size=shape).astype(np.int8)
    inv, step = float(np.float32(127.0 / 6.0)), np.float32(0.05)
    relu = bool(i % 2)
    lo, hi = (0, 127) if relu else (-128, 127)
    ref = orc.requantize(y, inv, res_i8=res8, res_step=step, relu=relu, lo=lo, hi=hi)
    x_plain = torch.from_numpy(L.x).cuda()
    x_blocked = torch.from_numpy(to_blocked(L.x, -3)).cuda()
    for layout in range(8):
        r8 = to_blocked(res8, 9) if layout & psb.BLOCKED_RES else res8
        got = psb.conv2d_shared_requant_blocked(
            qg, x_blocked if layout & psb.BLOCKED_IN else x_plain, L.x.shape, inv, L.S, stride=L.stride, pad=L.pad,
            seed=L.seed, layer_id=L.layer_id, mult=torch.from_numpy(mult).cuda(), bias=torch.from_numpy(bias).cuda(),
            res_i8=torch.from_numpy(r8).cuda(), res_step=float(step), relu=relu, lo=lo, hi=hi, layout=layout).cpu().numpy()
        if layout & psb.BLOCKED_OUT:
            got = from_blocked(got, oc)
        assert np.array_equal(got, ref), (case, layout)
