"""Attention mask on the GPU vs the oracle (Sect. 4.5), and the two-pass psb8/16 driver.

The entropy is floating point.  Both sides evaluate it in binary64 (different exp/log implementations and a
different but equivalent formula, so they agree to about 1e-14) and round once to binary32: the results are
equal except when the exact value lies next to a rounding boundary, so they are compared within one unit in
the last place of binary32 (1.2e-7 relative, 1e-37 absolute for values that round to zero).  The mask is an
integer decided by comparing two such numbers: it must equal the oracle's wherever the oracle's entropy is
further than 1e-6 from its mean; closer pixels may fall either way."""
import numpy as np
import pytest

import oracle_network
from paper_1904_02205_amd import resnet_synth as rs

pytestmark = pytest.mark.gpu
TOL_ABS, TOL_REL, TIE_BAND = 1e-37, 1.2e-7, 1e-6


@pytest.fixture(scope="module")
def psb():
    import torch
    assert torch.cuda.is_available()
    from paper_1904_02205_amd import psb as m
    m.lib()
    m.set_mapping(m.MAPPING_AUTO)
    return m


def _check(psb, orc, act, step, lo, hi):
    import torch
    ent_r, mean_r, bud_r = orc.attention_budget(act, step, lo, hi)
    ent_g, mean_g, bud_g = (t.cpu().numpy() for t in psb.attention_budget(torch.from_numpy(act).cuda(), float(step), lo, hi))
    assert np.all(np.abs(ent_g - ent_r) <= TOL_ABS + TOL_REL * np.abs(ent_r))
    assert np.all(np.abs(mean_g - mean_r) <= TOL_ABS + TOL_REL * np.abs(mean_r))
    clear = np.abs(ent_r - mean_r[:, None, None]) > TIE_BAND
    assert np.array_equal(bud_g[clear], bud_r[clear])
    assert set(np.unique(bud_g)) <= {lo, hi}
    # the GPU's own decision is the stated rule applied to the GPU's own numbers
    assert np.array_equal(bud_g == hi, ent_g > mean_g[:, None, None]) or lo == hi
    return clear.mean()


@pytest.mark.parametrize("shape", [(32, 512, 7, 7), (3, 40, 5, 6), (1, 2, 1, 1), (2, 70, 56, 56), (5, 1, 3, 3)])
def test_attention_budget(psb, orc, shape):
    rng = np.random.default_rng(shape[1])
    act = np.clip(np.rint(rng.exponential(20.0, size=shape)), 0, 127).astype(np.int8)
    act[rng.random(size=shape) < 0.4] = 0
    clear = _check(psb, orc, act, np.float32(6.0 / 127.0), 8, 16)
    assert clear > 0.99 or shape[1] == 1 or shape[2] * shape[3] < 25      # the test is not vacuous
    signed = rng.integers(-128, 128, size=shape).astype(np.int8)
    _check(psb, orc, signed, np.float32(0.3), 2, 32)


def test_attention_closed_forms(psb, orc):
    import torch
    act = np.full((2, 512, 4, 4), 9, np.int8)                # uniform distribution: h = log 512, no pixel above the mean
    ent, mean, bud = (t.cpu().numpy() for t in psb.attention_budget(torch.from_numpy(act).cuda(), 0.05, 8, 16))
    assert np.allclose(ent, np.log(512.0), rtol=1e-6) and np.all(bud == 8)
    act = np.zeros((1, 64, 1, 1), np.int8)
    act[0, 5] = 127
    ent, _, _ = psb.attention_budget(torch.from_numpy(act).cuda(), 1.0, 8, 16)
    assert 0 <= float(ent[0, 0, 0]) < 1e-30
    for bad in (0.0, -1.0, float("nan"), float("inf")):
        with pytest.raises(psb.PsbError) as ei:
            psb.attention_budget(torch.from_numpy(act).cuda(), bad, 8, 16)
        assert ei.value.code == psb.ERR_VALUE


@pytest.mark.parametrize("shared", [False, True])
def test_two_pass_network(psb, orc, shared):
    """psb8/16: low-precision pass, mask, mixed-precision pass.  Up to the mask both sides agree bit for bit;
    where no pixel lies in the tie band the masks agree and so do the final logits.  (shared: the first pass runs
    as one chain on the GPU, and so does the second, with the two budget values given to every layer call.)"""
    from paper_1904_02205_amd import network
    net = rs.resnet18(batch=2, hw=96, width=32, classes=10)
    ref_logits, ref_budget, ent, mean = oracle_network.OracleResNet18(orc, net).forward_attention(8, 16, shared=shared)
    logits, budget = network.ResNet18(net).forward_attention(8, 16, shared=shared)
    clear = np.abs(ent - mean[:, None, None]) > TIE_BAND
    assert np.array_equal(budget.cpu().numpy()[clear], ref_budget[clear])
    assert set(np.unique(ref_budget)) == {8, 16}
    if clear.all():
        assert np.array_equal(logits.cpu().numpy(), ref_logits)


def test_masked_chain_as_a_hip_graph(psb, orc):
    """The second pass of psb8/16 in shared-filter mode is a chain like the first (levels given with every call, all
    segments in one launch): it can be captured, and replays give the eager pass's bits; a replay reads the map
    tensor as it is then."""
    import torch
    from paper_1904_02205_amd import network
    net = rs.resnet18(batch=2, hw=96, width=32, classes=10)
    model = network.ResNet18(net)
    rng = np.random.default_rng(3)
    b1 = rng.choice([8, 16], size=(2, 3, 3), p=[0.6, 0.4]).astype(np.uint8)
    b2 = rng.choice([8, 16], size=(2, 3, 3), p=[0.3, 0.7]).astype(np.uint8)
    budget = torch.from_numpy(b1).cuda()
    ref1 = oracle_network.OracleResNet18(orc, net).forward(budget=b1, s_fc=16, shared=True)
    ref2 = oracle_network.OracleResNet18(orc, net).forward(budget=b2, s_fc=16, shared=True)
    eager = model.forward(budget=budget, s_fc=16, shared=True, levels=(8, 16)).cpu().numpy()
    assert np.array_equal(eager, ref1)
    layerwise = model.forward(budget=budget, s_fc=16, shared=True, levels=(8, 16), chain=False).cpu().numpy()
    assert np.array_equal(layerwise, ref1)
    graph, logits = model.capture(shared=True, budget=budget, s_fc=16, levels=(8, 16))
    for i in range(3):
        logits.zero_()
        graph.replay()
        torch.cuda.synchronize()
        assert np.array_equal(logits.cpu().numpy(), ref1), f"replay {i}"
        model.forward(S=8, shared=True)                       # eager work between the replays
    budget.copy_(torch.from_numpy(b2).cuda())
    graph.replay()
    torch.cuda.synchronize()
    assert np.array_equal(logits.cpu().numpy(), ref2)
