"""Seeded random layer shapes through every kernel mapping and both sampling modes vs the oracle.

Shapes, strides, paddings, groups, sample counts, budgets and probability widths are drawn from a fixed seed,
so the cases are the same on every run; they are meant to reach index arithmetic the hand-picked cases miss
(ragged channel blocks, kernels wider than the image interior, strides that skip the last columns, ...)."""
import numpy as np
import pytest

import helpers
from paper_1904_02205_amd import synth

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def psb():
    import torch
    assert torch.cuda.is_available()
    from paper_1904_02205_amd import psb as m
    m.lib()
    yield m
    m.set_mapping(m.MAPPING_AUTO)


def _random_case(i):
    rng = np.random.default_rng(7000 + i)
    groups = int(rng.choice([1, 1, 1, 2, 4, 0]))            # 0: depthwise
    kh, kw = int(rng.integers(1, 6)), int(rng.integers(1, 6))
    if groups == 0:
        c = int(rng.integers(1, 40))
        oc, groups = c * int(rng.choice([1, 2])), c
    else:
        c = groups * int(rng.integers(1, 50 if groups == 1 else 12))
        oc = groups * int(rng.integers(1, 40 if groups == 1 else 10))
    sh, sw = int(rng.integers(1, 4)), int(rng.integers(1, 4))
    ph, pw = int(rng.integers(0, kh)), int(rng.integers(0, kw))
    h = int(rng.integers(max(1, kh - 2 * ph), 14)) + (kh - 1) // 2
    w = int(rng.integers(max(1, kw - 2 * pw), 14)) + (kw - 1) // 2
    h, w = max(h, kh - 2 * ph), max(w, kw - 2 * pw)
    n = int(rng.integers(1, 4))
    s_max = int(rng.choice([1, 3, 8, 16, 33, 64]))
    S = int(rng.integers(1, s_max + 1))
    xkind = rng.choice(["relu", "signed", "u4"])
    wt = (rng.standard_normal((oc, c // groups, kh, kw)) * 10.0 ** rng.uniform(-3, 0)).astype(np.float32)
    if rng.random() < 0.3:
        wt = synth.prune_by_magnitude(wt, float(rng.uniform(0.3, 0.95)))
    shape = (n, c, h, w)
    if xkind == "relu":
        x = synth.sparse_relu_int8(shape, rng)
    elif xkind == "signed":
        x = rng.integers(-128, 128, size=shape).astype(np.int8)
    else:
        x = synth.uniform_uint4(shape, rng)
    L = synth.Layer(f"r{i}", wt, x, groups=groups, stride=(sh, sw), pad=(ph, pw), S=S, s_max=s_max,
                    x_absmax=128 if xkind == "signed" else 127, seed=int(rng.integers(0, 2 ** 62)),
                    layer_id=int(rng.integers(0, 2 ** 32)))
    prob_bits = int(rng.choice([23, 23, 4, 7, 1]))
    oh, ow = L.out_hw
    budget = None
    if rng.random() < 0.4:
        budget = rng.integers(0, s_max + 3, size=(n, oh, ow)).astype(np.uint8)
    return L, prob_bits, budget


@pytest.mark.parametrize("i", range(48))
def test_random_layer(psb, orc, i):
    L, prob_bits, budget = _random_case(i)
    print(f"[random {i}] x{L.x.shape} w{L.w.shape} groups={L.groups} stride={L.stride} pad={L.pad} S={L.S}/{L.s_max} "
          f"prob_bits={prob_bits} budget={'map' if budget is not None else 'none'}", flush=True)
    qo = helpers.oracle_quantize(orc, L, prob_bits=prob_bits)
    qg = helpers.gpu_quantize(psb, L, prob_bits=prob_bits)
    assert np.array_equal(qg.export(), helpers.pack_from_oracle(qo))
    ref, over, _ = helpers.oracle_layer(orc, L, qo, budget_to=budget)
    assert over == 0
    for m in ((1, 2, 3, 0) if L.groups == 1 else (1, 3, 0)):
        psb.set_mapping(m)
        acc, _ = helpers.gpu_layer(psb, L, qg, budget_to=budget)
        assert np.array_equal(acc, ref), f"per-product, mapping {m}"
    ref_s, over_s, _ = helpers.oracle_layer(orc, L, qo, budget_to=budget, shared=True)
    assert over_s == 0
    for m in (0, 1):
        psb.set_mapping(m)
        acc, y = helpers.gpu_layer(psb, L, qg, budget_to=budget, shared=True, want_y=True)
        assert np.array_equal(acc, ref_s), f"shared filter, mapping {m}"
        ref_y = orc.rescale(ref_s, qo.e_min, S=None if budget is not None else L.S, s_max=L.s_max, budget_to=budget)
        assert np.array_equal(y, ref_y)
    psb.set_mapping(psb.MAPPING_AUTO)
