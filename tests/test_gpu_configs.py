"""The five benchmark configurations at full size, in the launch configuration bench.py times (needs an MI355X).

Configs 1, 2, 3 and 5 are compared with the oracle on every output element; the ResNet-18-shaped layers of
config 4 on every output element at batch 2, and at batch 32 on 100,000 randomly chosen output elements per
layer, which the oracle computes one by one (possible because the random bits are keyed by output coordinate).
"""
import numpy as np
import pytest

import helpers
from paper_1904_02205_amd import synth

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def psb():
    from paper_1904_02205_amd import psb as m
    m.lib()
    m.set_mapping(m.MAPPING_AUTO)
    return m


def _full(psb, orc, L, **kw):
    print(f"[config] {L.name} x{L.x.shape} w{L.w.shape} S={L.S} seed={L.seed}", flush=True)
    qo = helpers.oracle_quantize(orc, L)
    ref, over, smac = helpers.oracle_layer(orc, L, qo, **kw)
    acc, y = helpers.gpu_layer(psb, L, want_y=True, **kw)
    assert over == 0
    assert np.array_equal(acc, ref)
    ref_y = orc.rescale(ref, qo.e_min, S=None if L.budget_to is not None else L.S, s_max=L.s_max,
                        budget_to=L.budget_to)
    np.testing.assert_allclose(y, ref_y, rtol=1e-6, atol=0)
    return smac


def test_config1_linear(psb, orc):
    assert _full(psb, orc, synth.config1()) == 64 * 8 * (256 * 512 - 6)


def test_config2_conv3x3(psb, orc):
    _full(psb, orc, synth.config2())


def test_config3_progressive(psb, orc):
    L = synth.config3()
    _full(psb, orc, L)
    # the incremental pair: 8 samples first (where the budget allows), then up to the budget
    qo = helpers.oracle_quantize(orc, L)
    qg = helpers.gpu_quantize(psb, L)
    first = np.minimum(L.budget_to, 8).astype(np.uint8)
    a1, _ = helpers.gpu_layer(psb, L, qg, budget_to=first)
    a2, _ = helpers.gpu_layer(psb, L, qg, budget_to=L.budget_to, budget_from=first, acc_in=a1)
    ref, _, _ = helpers.oracle_layer(orc, L, qo)
    assert np.array_equal(a2, ref)


def test_config5_mobilenet_block(psb, orc):
    for L in synth.config5():
        _full(psb, orc, L)


def test_config4_resnet18_layers_sampled(psb, orc):
    rng = np.random.default_rng(4040)
    for L in synth.config4_layers():
        print(f"[config4] {L.name} x{L.x.shape} w{L.w.shape}", flush=True)
        qo = helpers.oracle_quantize(orc, L)
        acc, y = helpers.gpu_layer(psb, L, want_y=True)
        pts = rng.choice(acc.size, size=min(100000, acc.size), replace=False).astype(np.int64)
        ref, over, _ = helpers.oracle_layer(orc, L, qo, points=pts)
        assert over == 0
        assert np.array_equal(acc.ravel()[pts], ref), L.name
        ref_y = orc.rescale(ref.reshape(1, 1, -1), qo.e_min, S=L.S).ravel()
        np.testing.assert_allclose(y.ravel()[pts], ref_y, rtol=1e-6, atol=0)
        # the call is repeatable
        acc2, _ = helpers.gpu_layer(psb, L)
        assert np.array_equal(acc, acc2)


def test_config4_resnet18_layers_full_at_batch_2(psb, orc):
    for L in synth.config4_layers(batch=2):
        _full(psb, orc, L)


# ------------------------------------------------------------------ shared-filter mode at the same sizes

def _full_shared(psb, orc, L):
    print(f"[config, shared filter] {L.name} x{L.x.shape} w{L.w.shape} S={L.S}", flush=True)
    qo = helpers.oracle_quantize(orc, L)
    ref, over, _ = helpers.oracle_layer(orc, L, qo, shared=True)
    acc, y = helpers.gpu_layer(psb, L, want_y=True, shared=True)
    assert over == 0
    assert np.array_equal(acc, ref)
    ref_y = orc.rescale(ref, qo.e_min, S=None if L.budget_to is not None else L.S, s_max=L.s_max,
                        budget_to=L.budget_to)
    np.testing.assert_allclose(y, ref_y, rtol=1e-6, atol=0)


def test_shared_filter_configs_1_2_3_5(psb, orc):
    for L in [synth.config1(), synth.config2(), synth.config3()] + synth.config5():
        _full_shared(psb, orc, L)


def test_shared_filter_config4_layers_sampled(psb, orc):
    rng = np.random.default_rng(4041)
    for L in synth.config4_layers():
        print(f"[config4, shared filter] {L.name} x{L.x.shape} w{L.w.shape}", flush=True)
        qo = helpers.oracle_quantize(orc, L)
        qg = helpers.gpu_quantize(psb, L)
        # the whole sampled filter, then 20,000 outputs
        W = psb.sample_filter(qg, L.S, seed=L.seed, layer_id=L.layer_id).cpu().numpy()
        assert np.array_equal(W.astype(np.int64), orc.sample_filter(qo, L.S, seed=L.seed, layer_id=L.layer_id))
        acc, y = helpers.gpu_layer(psb, L, qg, want_y=True, shared=True)
        pts = rng.choice(acc.size, size=min(20000, acc.size), replace=False).astype(np.int64)
        ref, over, _ = helpers.oracle_layer(orc, L, qo, points=pts, shared=True)
        assert over == 0
        assert np.array_equal(acc.ravel()[pts], ref), L.name
        ref_y = orc.rescale(ref.reshape(1, 1, -1), qo.e_min, S=L.S).ravel()
        np.testing.assert_allclose(y.ravel()[pts], ref_y, rtol=1e-6, atol=0)


# ------------------------------------------------------------------ properties that hold at any size

def test_config2_mean_over_seeds_approaches_the_float_convolution(psb, orc):
    """Unbiasedness (Sect. 3.1) at full size, in both modes: the mean of the rescaled output over 48 seeds lies
    within five standard errors of the exact convolution with the represented weights, element by element (a
    handful of the 200,704 elements may exceed it by chance: at most 10 are tolerated, none by more than 7)."""
    import torch
    L = synth.config2()
    qo = helpers.oracle_quantize(orc, L)
    ref = torch.nn.functional.conv2d(torch.from_numpy(L.x.astype(np.float64)),
                                     torch.from_numpy(qo.represented().reshape(L.w.shape)), padding=L.pad).numpy()
    qg = helpers.gpu_quantize(psb, L)
    x = torch.from_numpy(L.x).cuda()
    for shared in (False, True):
        ys = []
        for seed in range(48):
            y = torch.empty((1, 64, 56, 56), dtype=torch.float32, device="cuda")
            psb.conv2d(qg, x, L.S, pad=L.pad, seed=1000 + seed, layer_id=L.layer_id, y=y, shared=shared)
            ys.append(y.double())
        ys = torch.stack(ys)
        mean, sd = ys.mean(dim=0).cpu().numpy(), ys.std(dim=0).cpu().numpy()
        z = np.abs(mean - ref) / (sd / np.sqrt(48) + 1e-9)
        assert (z > 5).sum() <= 10 and z.max() < 7, (shared, float(z.max()), int((z > 5).sum()))
        assert 0.5 < np.median(z) < 0.9          # |N(0,1)| has median 0.67: the spread is the predicted one
