"""psb_conv2d_shared_budget_requant_blocked: a shared-filter layer with a per-pixel budget map whose values are rounded
down to the levels given with the call (Sect. 4.5: two kinds of regions, the first samples reused), all sample
segments in one launch.  Expected values: the oracle's shared-filter layer on the map rounded down in numpy, then its
rescale and requantize."""
import numpy as np
import pytest

import helpers
from test_gpu_blocked import from_blocked, to_blocked
from test_gpu_parity import _layer

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def psb():
    from paper_1904_02205_amd import psb as m
    m.lib()
    m.set_mapping(m.MAPPING_AUTO)
    return m


def round_down(budget, levels, s_max):
    lv = sorted({min(int(v), s_max) for v in levels if v > 0})
    b = np.minimum(budget.astype(np.int64), s_max)
    out = np.zeros_like(b)
    for v in lv:
        out[b >= v] = v
    return out.astype(np.uint8)


CASES = [
    # (layer arguments, levels, values the map is drawn from)
    (dict(n=2, c=40, oc=70, hw=(9, 11), k=3, pad=1, S=16), (8, 16), (0, 3, 8, 11, 16, 200)),        # the paper's two levels
    (dict(n=2, c=64, oc=64, hw=8, k=3, stride=2, pad=1, S=16), (16, 8), (8, 16)),
    (dict(n=3, c=33, oc=32, hw=(5, 8), k=1, S=32), (2, 4, 8, 32), (0, 1, 2, 3, 4, 7, 8, 31, 32, 255)),   # four levels
    (dict(n=1, c=32, oc=40, hw=(70, 66), k=3, pad=1, S=8), (4, 8, 0, 4), (4, 8)),                    # many pixel tiles; duplicates, a zero
    (dict(n=2, c=3, oc=16, hw=20, k=7, stride=2, pad=3, S=16), (8, 16), (8, 16, 5)),                 # row-packed first layer
    (dict(n=1, c=256, oc=64, hw=6, k=3, pad=1, S=16), (8, 16), (0, 8, 16)),                          # split reduction: segment by segment
    (dict(n=2, c=24, oc=24, hw=9, k=3, pad=1, groups=24, S=16), (8, 16), (3, 8, 16)),                # depthwise: direct kernel
    (dict(n=2, c=40, oc=70, hw=(9, 11), k=3, pad=1, S=16), (12,), (0, 11, 12, 13)),                  # one level
    (dict(n=2, c=40, oc=70, hw=(9, 11), k=3, pad=1, S=8), (8, 16, 200), (5, 8, 16, 100)),            # levels beyond s_max = 8
    (dict(n=2, c=128, oc=64, hw=14, k=3, pad=1, S=16), (8, 16), (0, 8, 16)),                         # 3x3 from LDS, two teams
    (dict(n=2, c=32, oc=480, hw=50, k=3, pad=1, S=8), (2, 4, 8), (0, 2, 4, 8)),                      # ... two half tiles
    (dict(n=2, c=64, oc=256, hw=9, k=3, pad=1, S=16), (4, 16), (4, 16)),                             # ... XCDs by channels
]


@pytest.mark.parametrize("case", CASES, ids=[str(i) for i in range(len(CASES))])
def test_levels_in_one_launch(psb, orc, case):
    import torch
    kw_layer, levels, values = case
    rng = np.random.default_rng(31)
    L = _layer(rng, **kw_layer)
    oc = L.w.shape[0]
    n, c, h, w = L.x.shape
    oh, ow = L.out_hw
    shape = (n, oc, oh, ow)
    budget = rng.choice(values, size=(n, oh, ow)).astype(np.uint8)
    budget[0, :2, :] = values[-1]                     # a coherent region, so that whole tiles skip segments
    rounded = round_down(budget, levels, L.s_max)
    mult = (rng.uniform(0.5, 2.0, size=oc) * 2.0 ** -6).astype(np.float32)
    bias = rng.standard_normal(oc).astype(np.float32)
    qo, qg = helpers.oracle_quantize(orc, L), helpers.gpu_quantize(psb, L)
    acc, over, _ = helpers.oracle_layer(orc, L, qo, budget_to=rounded, shared=True)
    assert over == 0
    y = orc.rescale(acc, qo.e_min, s_max=L.s_max, budget_to=rounded, mult=mult, bias=bias)
    res8 = rng.integers(-128, 128, size=shape).astype(np.int8)
    inv = float(np.float32(127.0 / 6.0))
    mfma = L.groups == 1
    rowpack = mfma and L.w.shape[3] > 1 and L.w.shape[3] * c <= 32
    can_block_in = mfma and not rowpack
    x_plain, x_blocked = torch.from_numpy(L.x).cuda(), torch.from_numpy(to_blocked(L.x, 77)).cuda()
    bt = torch.from_numpy(budget).cuda()
    kw = dict(stride=L.stride, pad=L.pad, seed=L.seed, layer_id=L.layer_id, mult=torch.from_numpy(mult).cuda(),
              bias=torch.from_numpy(bias).cuda())
    for layout in ((0, psb.BLOCKED_IN) if can_block_in else (0,)):
        got = psb.conv2d_shared_budget_requant_blocked(qg, x_blocked if layout else x_plain, L.x.shape, 0.0, bt, levels,
                                                       layout=layout, want_x=False, **kw)
        assert np.array_equal(got.cpu().numpy(), y), layout
    for prepared in (False, True):
        for layout in range(8):
            if (layout & psb.BLOCKED_IN) and not can_block_in:
                continue
            if prepared:
                psb.shared_prepare_filters_levels([qg], levels, [L.seed], [L.layer_id])
            r8 = to_blocked(res8, -5) if layout & psb.BLOCKED_RES else res8
            got = psb.conv2d_shared_budget_requant_blocked(
                qg, x_blocked if layout & psb.BLOCKED_IN else x_plain, L.x.shape, inv, bt, levels, layout=layout,
                res_i8=torch.from_numpy(r8).cuda(), res_step=float(np.float32(0.05)), **kw).cpu().numpy()
            if layout & psb.BLOCKED_OUT:
                got = from_blocked(got, oc)
            ref = orc.requantize(y, inv, res_i8=res8, res_step=np.float32(0.05))
            assert np.array_equal(got, ref), (layout, prepared)
    # the same map through the existing entry point, given the rounded map: same integers
    ref2 = psb.conv2d_requant(qg, x_plain, inv, budget_to=torch.from_numpy(rounded).cuda(), shared=True, want_acc=False,
                              **kw).cpu().numpy()
    assert np.array_equal(ref2, orc.requantize(y, inv))


def test_levels_errors_and_one_shot_announcement(psb, orc):
    import torch
    rng = np.random.default_rng(32)
    L = _layer(rng, 2, 40, 70, (9, 11), 3, pad=1, S=16)
    q = helpers.gpu_quantize(psb, L)
    x = torch.from_numpy(L.x).cuda()
    bt = torch.full((2, 9, 11), 8, dtype=torch.uint8, device="cuda")
    with pytest.raises(psb.PsbError) as ei:
        psb.conv2d_shared_budget_requant_blocked(q, x, L.x.shape, 1.0, bt, (1, 2, 3, 4, 5), pad=L.pad)
    assert ei.value.code == psb.ERR_VALUE
    with pytest.raises(psb.PsbError) as ei:
        psb.shared_prepare_filters_levels([q], (0,), [0], [0])
    assert ei.value.code == psb.ERR_VALUE
    with pytest.raises(ValueError):
        psb.conv2d_shared_budget_requant_blocked(q, x, L.x.shape, 1.0, bt[:, :8], (8,), pad=L.pad)
    # an announcement serves exactly one call: the second call reads the values back by itself and is still right
    budget = rng.choice([4, 16], size=(2, 9, 11)).astype(np.uint8)
    ref, _, _ = helpers.oracle_layer(orc, L, budget_to=budget, shared=True)
    psb.shared_budget_levels((4,))                      # would be wrong for the second call if it were still in force
    first, _ = helpers.gpu_layer(psb, L, q, budget_to=np.full_like(budget, 4), shared=True)
    second, _ = helpers.gpu_layer(psb, L, q, budget_to=budget, shared=True)
    assert np.array_equal(second, ref)
    only4, _, _ = helpers.oracle_layer(orc, L, budget_to=np.full_like(budget, 4), shared=True)
    assert np.array_equal(first, only4)
