"""Glue kernels between layers vs the CPU oracle (bit-exact integers), and the ResNet-18-shaped network
chained end to end through the C-ABI vs the same chain on the oracle."""
import numpy as np
import pytest

import oracle_network
from paper_1904_02205_amd import resnet_synth as rs

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def psb():
    import torch
    assert torch.cuda.is_available()
    from paper_1904_02205_amd import psb as m
    m.lib()
    m.set_mapping(m.MAPPING_AUTO)
    return m


@pytest.mark.parametrize("n", [1, 3, 4, 1023, 4096, 100003])
def test_requantize(psb, orc, n):
    import torch
    rng = np.random.default_rng(n)
    y = (rng.standard_normal(n) * 2).astype(np.float32)
    y[: min(n, 8)] = np.array([0.5, 1.5, 2.5, -0.5, np.nan, np.inf, -np.inf, 1e30], np.float32)[: min(n, 8)]
    r = (rng.standard_normal(n) * 2).astype(np.float32)
    ri = rng.integers(-128, 128, size=n).astype(np.int8)
    inv, step = np.float32(127.0 / 6.0), np.float32(4.0 / 127.0)
    yd, rd, rid = (torch.from_numpy(a).cuda() for a in (y, r, ri))
    for kw_o, kw_g in ((dict(), dict()),
                       (dict(res_f32=r), dict(res_f32=rd)),
                       (dict(res_i8=ri, res_step=step), dict(res_i8=rid, res_step=float(step))),
                       (dict(relu=False, lo=-127, hi=127), dict(relu=False, lo=-127, hi=127)),
                       (dict(relu=False, lo=-128, hi=5, res_f32=r), dict(relu=False, lo=-128, hi=5, res_f32=rd))):
        ref = orc.requantize(y, inv, **kw_o)
        got = psb.requantize(yd, float(inv), **kw_g).cpu().numpy()
        assert np.array_equal(got, ref), kw_o.keys()
    if n > 8:       # pointers that are not 16-byte aligned take the one-element-per-thread kernel
        ref = orc.requantize(y[1:], inv, res_f32=r[1:])
        out = torch.empty(n, dtype=torch.int8, device="cuda")
        got = psb.requantize(yd[1:], float(inv), res_f32=rd[1:], out=out[1:]).cpu().numpy()
        assert np.array_equal(got, ref)


def test_requantize_errors(psb):
    import torch
    y = torch.zeros(8, device="cuda")
    r8 = torch.zeros(8, dtype=torch.int8, device="cuda")
    for kw in (dict(lo=-129), dict(hi=128), dict(lo=5, hi=4), dict(res_f32=y, res_i8=r8)):
        with pytest.raises(psb.PsbError) as ei:
            psb.requantize(y, 1.0, **kw)
        assert ei.value.code == psb.ERR_VALUE


@pytest.mark.parametrize("geom", [((3, 3), (2, 2), (1, 1), 112, 112), ((2, 2), (2, 2), (0, 0), 8, 8),
                                  ((3, 2), (1, 2), (1, 0), 5, 7), ((1, 1), (1, 1), (0, 0), 4, 4),
                                  ((3, 3), (2, 2), (1, 1), 9, 11), ((3, 3), (2, 2), (1, 1), 4, 20000),   # rows too long for LDS
                                  ((3, 3), (1, 1), (1, 1), 300, 12), ((2, 2), (2, 2), (1, 1), 64, 64),
                                  ((3, 3), (2, 2), (1, 1), 9, 16), ((3, 3), (2, 2), (1, 1), 1, 8)])   # the stem-pooling kernel
def test_maxpool(psb, orc, geom):
    import torch
    kernel, stride, pad, h, w = geom
    x = np.random.default_rng(h * w).integers(-128, 128, size=(3, 5, h, w)).astype(np.int8)
    got = psb.maxpool2d_i8(torch.from_numpy(x).cuda(), kernel, stride, pad).cpu().numpy()
    assert np.array_equal(got, orc.maxpool_i8(x, kernel, stride, pad))


@pytest.mark.parametrize("geom", [((3, 3), (2, 2), (1, 1), 3, 64, 112, 112), ((2, 2), (2, 2), (0, 0), 2, 40, 8, 8),
                                  ((3, 2), (1, 2), (1, 0), 3, 5, 5, 7), ((1, 1), (1, 1), (0, 0), 1, 33, 4, 4),
                                  ((3, 3), (2, 2), (1, 1), 2, 96, 9, 11), ((2, 2), (2, 2), (1, 1), 1, 32, 64, 64)])
def test_maxpool_on_the_blocked_layout(psb, orc, geom):
    """Same maxima as the oracle's [N][C][H][W] pooling; the layout conversions here are plain numpy."""
    import torch
    from test_gpu_blocked import to_blocked, from_blocked
    kernel, stride, pad, n, c, h, w = geom
    x = np.random.default_rng(h * w + c).integers(-128, 128, size=(n, c, h, w)).astype(np.int8)
    got = psb.maxpool2d_i8_blocked(torch.from_numpy(to_blocked(x, -77)).cuda(), x.shape, kernel, stride, pad).cpu().numpy()
    ref = orc.maxpool_i8(x, kernel, stride, pad)
    assert got.shape == psb.blocked_shape(*ref.shape)
    assert np.array_equal(from_blocked(got, c), ref)
    with pytest.raises(psb.PsbError) as ei:        # the blocked tensors move as 16-byte words
        flat = torch.zeros(int(np.prod(psb.blocked_shape(*x.shape))) + 16, dtype=torch.int8, device="cuda")
        psb.maxpool2d_i8_blocked(flat[4:-12].view(psb.blocked_shape(*x.shape)), x.shape, kernel, stride, pad)
    assert ei.value.code == psb.ERR_VALUE


def test_maxpool_refuses_windows_that_can_lie_in_the_padding(psb):
    import torch
    with pytest.raises(psb.PsbError) as ei:
        psb.maxpool2d_i8(torch.zeros((1, 1, 8, 8), dtype=torch.int8, device="cuda"), (2, 2), (2, 2), (2, 2))
    assert ei.value.code == psb.ERR_SHAPE


@pytest.mark.parametrize("shape", [(4, 16, 7, 7), (1, 3, 1, 1), (2, 70, 9, 13), (3, 1, 64, 64)])
def test_global_avgpool(psb, orc, shape):
    import torch
    rng = np.random.default_rng(shape[1])
    x = rng.integers(-128, 128, size=shape).astype(np.int8)
    for scale, lo, hi in ((1.0, 0, 127), (0.731, -128, 127), (3.5, -20, 20)):
        got = psb.global_avgpool_requantize(torch.from_numpy(x).cuda(), scale, lo, hi).cpu().numpy()
        assert np.array_equal(got, orc.avgpool_requantize(x, scale, lo, hi))


def test_budget_resample(psb, orc):
    import torch
    b = np.random.default_rng(7).integers(0, 33, size=(3, 7, 9)).astype(np.uint8)
    for oh, ow in ((7, 9), (14, 18), (3, 5), (56, 56), (1, 1)):
        got = psb.budget_resample(torch.from_numpy(b).cuda(), oh, ow).cpu().numpy()
        assert np.array_equal(got, orc.budget_resample(b, oh, ow))


@pytest.mark.parametrize("shared", [False, True])
def test_fused_requantisation_equals_layer_then_requantize(psb, orc, shared):
    """psb_conv2d_requant on every kernel vs the oracle's layer -> rescale -> requantize chain."""
    import torch
    import helpers
    from test_gpu_parity import _layer
    rng = np.random.default_rng(77)
    cases = [(_layer(rng, 2, 20, 70, (9, 11), 3, pad=1, S=8), (1, 2, 3, 0)),            # several tap chunks
             (_layer(rng, 2, 24, 40, 9, 1, stride=2, S=4), (1, 2, 3, 0)),               # one chunk: fused in the sampling kernel
             (_layer(rng, 1, 256, 64, 6, 3, pad=1, S=8), (0,)),                         # shared: split reduction
             (_layer(rng, 2, 70, 70, 9, 3, pad=1, groups=70, S=16), (1, 3, 0))]         # depthwise
    inv = float(np.float32(127.0 / 6.0))
    for L, mappings in cases:
        oc = L.w.shape[0]
        mult = (rng.uniform(0.5, 2.0, size=oc) * 2.0 ** -6).astype(np.float32)
        bias = rng.standard_normal(oc).astype(np.float32)
        qo, qg = helpers.oracle_quantize(orc, L), helpers.gpu_quantize(psb, L)
        x = torch.from_numpy(L.x).cuda()
        oh, ow = L.out_hw
        shape = (L.x.shape[0], oc, oh, ow)
        res = (rng.standard_normal(shape) * 2).astype(np.float32)
        res8 = rng.integers(0, 128, size=shape).astype(np.int8)
        budget = rng.choice([0, 2, L.S], size=(shape[0], oh, ow)).astype(np.uint8)
        for bt in (None, budget):
            acc, _, _ = helpers.oracle_layer(orc, L, qo, budget_to=bt, shared=shared)
            y = orc.rescale(acc, qo.e_min, S=None if bt is not None else L.S, s_max=L.s_max, budget_to=bt, mult=mult,
                            bias=bias)
            for kw_o, kw_g in ((dict(), dict()),
                               (dict(res_f32=res), dict(res_f32=torch.from_numpy(res).cuda())),
                               (dict(res_i8=res8, res_step=np.float32(0.05)),
                                dict(res_i8=torch.from_numpy(res8).cuda(), res_step=float(np.float32(0.05)))),
                               (dict(relu=False, lo=-128, hi=127), dict(relu=False, lo=-128, hi=127))):
                ref = orc.requantize(y, inv, **kw_o)
                for m in mappings:
                    psb.set_mapping(m)
                    accg = torch.empty(shape, dtype=torch.int32, device="cuda")
                    got = psb.conv2d_requant(qg, x, inv, S=None if bt is not None else L.S,
                                             budget_to=None if bt is None else torch.from_numpy(bt).cuda(),
                                             stride=L.stride, pad=L.pad, seed=L.seed, layer_id=L.layer_id,
                                             mult=torch.from_numpy(mult).cuda(), bias=torch.from_numpy(bias).cuda(),
                                             acc=accg, shared=shared, **kw_g)
                    assert np.array_equal(accg.cpu().numpy(), acc), (L.w.shape, m)
                    assert np.array_equal(got.cpu().numpy(), ref), (L.w.shape, m, list(kw_o))
                    # without an accumulator output: same activations
                    got2 = psb.conv2d_requant(qg, x, inv, S=None if bt is not None else L.S,
                                              budget_to=None if bt is None else torch.from_numpy(bt).cuda(),
                                              stride=L.stride, pad=L.pad, seed=L.seed, layer_id=L.layer_id,
                                              mult=torch.from_numpy(mult).cuda(), bias=torch.from_numpy(bias).cuda(),
                                              shared=shared, want_acc=False, **kw_g)
                    assert np.array_equal(got2.cpu().numpy(), ref), (L.w.shape, m, "no acc")
    psb.set_mapping(psb.MAPPING_AUTO)
    q = psb.Weights(torch.ones((4, 4, 1, 1), device="cuda"))
    xx = torch.zeros((1, 4, 2, 2), dtype=torch.int8, device="cuda")
    for kw in (dict(lo=-129), dict(hi=128), dict(lo=3, hi=2), dict(S=0), dict(S=17)):
        with pytest.raises(psb.PsbError) as ei:
            psb.conv2d_requant(q, xx, 1.0, **{**dict(S=4), **kw})
        assert ei.value.code == psb.ERR_VALUE
    for bad in (-1.0, float("nan")):
        with pytest.raises(psb.PsbError) as ei:
            psb.conv2d_requant(q, xx, bad, S=4)
        assert ei.value.code == psb.ERR_VALUE


# ------------------------------------------------------------------ the chained network

def test_fused_requantisation_on_a_large_ragged_layer(psb, orc):
    """The channel-lane kernel with a split tap reduction and more than 2^20 outputs: the tiled pass that turns the
    channels-last partial sums into outputs also requantises (residual in either form, no ReLU, with and without an
    accumulator output, with a budget map).  100 channels, 2 x 75 x 77 pixels: ragged in both directions."""
    import torch
    import helpers
    from test_gpu_parity import _layer
    rng = np.random.default_rng(78)
    L = _layer(rng, 2, 8, 100, (75, 77), 3, pad=1, S=4, s_max=8)
    oc = 100
    oh, ow = L.out_hw
    shape = (2, oc, oh, ow)
    assert int(np.prod(shape)) > (1 << 20)
    inv = float(np.float32(127.0 / 6.0))
    mult = (rng.uniform(0.5, 2.0, size=oc) * 2.0 ** -6).astype(np.float32)
    bias = rng.standard_normal(oc).astype(np.float32)
    qo, qg = helpers.oracle_quantize(orc, L), helpers.gpu_quantize(psb, L)
    x = torch.from_numpy(L.x).cuda()
    res = (rng.standard_normal(shape) * 2).astype(np.float32)
    res8 = rng.integers(0, 128, size=shape).astype(np.int8)
    budget = rng.choice([0, 2, 4, 8], size=(2, oh, ow)).astype(np.uint8)
    psb.set_mapping(2)
    try:
        for bt in (None, budget):
            acc, _, _ = helpers.oracle_layer(orc, L, qo, budget_to=bt)
            y = orc.rescale(acc, qo.e_min, S=None if bt is not None else L.S, s_max=L.s_max, budget_to=bt, mult=mult,
                            bias=bias)
            for kw_o, kw_g in ((dict(res_f32=res), dict(res_f32=torch.from_numpy(res).cuda())),
                               (dict(res_i8=res8, res_step=np.float32(0.05)),
                                dict(res_i8=torch.from_numpy(res8).cuda(), res_step=float(np.float32(0.05)))),
                               (dict(relu=False, lo=-128, hi=127), dict(relu=False, lo=-128, hi=127))):
                ref = orc.requantize(y, inv, **kw_o)
                common = dict(S=None if bt is not None else L.S, budget_to=None if bt is None else torch.from_numpy(bt).cuda(),
                              stride=L.stride, pad=L.pad, seed=L.seed, layer_id=L.layer_id,
                              mult=torch.from_numpy(mult).cuda(), bias=torch.from_numpy(bias).cuda())
                accg = torch.empty(shape, dtype=torch.int32, device="cuda")
                got = psb.conv2d_requant(qg, x, inv, acc=accg, **common, **kw_g)
                assert np.array_equal(accg.cpu().numpy(), acc)
                assert np.array_equal(got.cpu().numpy(), ref), list(kw_o)
                got2 = psb.conv2d_requant(qg, x, inv, want_acc=False, **common, **kw_g)
                assert np.array_equal(got2.cpu().numpy(), ref), (list(kw_o), "no acc")
    finally:
        psb.set_mapping(psb.MAPPING_AUTO)


def _compare(psb, orc, net, prob_bits=23, **kw):
    from paper_1904_02205_amd import network
    ref_acts, got_acts = [], []
    kw_ref = {k: v for k, v in kw.items() if k not in ("fused", "chain")}
    ref = oracle_network.OracleResNet18(orc, net, prob_bits=prob_bits).forward(collect=ref_acts, **kw_ref)
    model = network.ResNet18(net, prob_bits=prob_bits)
    kw_g = dict(kw)
    if kw_g.get("budget") is not None:
        import torch
        kw_g["budget"] = torch.from_numpy(kw_g["budget"]).cuda()
    got = model.forward(collect=got_acts, **kw_g).cpu().numpy()
    assert len(ref_acts) == len(got_acts)
    for i, (r, g) in enumerate(zip(ref_acts, got_acts)):        # the first differing activation names the layer
        assert np.array_equal(g.cpu().numpy(), r), f"activation {i} of {len(ref_acts)} differs"
    assert np.array_equal(got, ref)                               # fp32 logits, bit for bit
    return got


def test_network_end_to_end(psb, orc):
    net = rs.resnet18(batch=2, hw=64, width=32, classes=10)
    a = _compare(psb, orc, net, S=8)
    _compare(psb, orc, net, S=8, fused=False)
    _compare(psb, orc, net, S=8, shared=True, fused=False)
    b = _compare(psb, orc, net, S=8, shared=True)                  # as one chain: blocked activations, filters up front
    assert not np.array_equal(a, b)
    _compare(psb, orc, net, S=8, shared=True, chain=False)         # layer by layer
    _compare(psb, orc, net, prob_bits=4, S=16)
    _compare(psb, orc, net, prob_bits=4, S=16, shared=True)


def test_network_with_a_budget_map_on_all_layers(psb, orc):
    net = rs.resnet18(batch=2, hw=64, width=32, classes=10)
    budget = np.random.default_rng(5).choice([8, 16], size=(2, 2, 2), p=[0.65, 0.35]).astype(np.uint8)
    _compare(psb, orc, net, budget=budget, s_fc=16)
    _compare(psb, orc, net, budget=budget, s_fc=16, shared=True)


@pytest.mark.parametrize("shared", [False, True])
def test_network_as_a_hip_graph(psb, orc, shared):
    """A captured pass replays to the bits of the eager pass, every time, with eager work in between."""
    import torch
    from paper_1904_02205_amd import network
    net = rs.resnet18(batch=2, hw=64, width=32, classes=10)
    model = network.ResNet18(net)
    eager = model.forward(S=8, shared=shared).cpu().numpy()
    graph, logits = model.capture(S=8, shared=shared)
    for i in range(4):
        logits.zero_()
        graph.replay()
        torch.cuda.synchronize()
        assert np.array_equal(logits.cpu().numpy(), eager), f"replay {i}"
        other = model.forward(S=4, shared=not shared)          # eager work between the replays
        torch.cuda.synchronize()
        assert other.shape == logits.shape
