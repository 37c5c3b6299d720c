"""Pins of the oracle's attention mask (Sect. 4.5: pixelwise entropy of the softmax over channels, hard
threshold at the image's mean entropy).  CPU only."""
import numpy as np
import scipy.special
import scipy.stats


def test_entropy_closed_forms(orc):
    # equal activations in all channels: the uniform distribution, h = log C (the paper's "highest entropy" case)
    for c in (2, 10, 512):
        act = np.full((1, c, 2, 3), 17, np.int8)
        ent, mean, _ = orc.attention_budget(act, 0.05, 8, 16)
        assert np.allclose(ent, np.log(c), rtol=1e-6)
        assert np.isclose(mean[0], np.log(c), rtol=1e-6)
    # one channel far above the rest: h -> 0 (the "lowest entropy" case)
    act = np.zeros((1, 64, 1, 1), np.int8)
    act[0, 5] = 127
    ent, _, _ = orc.attention_budget(act, 1.0, 8, 16)
    assert 0 <= ent[0, 0, 0] < 1e-40 or ent[0, 0, 0] == 0
    # two channels, logits 0 and log 3: p = (1/4, 3/4)
    act = np.zeros((1, 2, 1, 1), np.int8)
    act[0, 1] = 100
    ent, _, _ = orc.attention_budget(act, np.log(3.0) / 100.0, 8, 16)
    assert np.isclose(ent[0, 0, 0], -(0.25 * np.log(0.25) + 0.75 * np.log(0.75)), rtol=1e-6)


def test_entropy_matches_scipy_and_is_shift_invariant(orc):
    rng = np.random.default_rng(1)
    act = rng.integers(0, 100, size=(3, 40, 5, 6)).astype(np.int8)
    step = np.float32(6.0 / 127.0)
    ent, mean, _ = orc.attention_budget(act, step, 8, 16)
    p = scipy.special.softmax(act.astype(np.float64) * float(step), axis=1)
    ref = scipy.stats.entropy(p, axis=1)
    assert np.allclose(ent, ref, rtol=2e-7, atol=1e-7)
    assert np.allclose(mean, ref.mean(axis=(1, 2)), rtol=1e-6)
    ent2, _, _ = orc.attention_budget((act + 27).astype(np.int8), step, 8, 16)      # softmax ignores a common offset
    assert np.allclose(ent, ent2, rtol=1e-6, atol=1e-7)
    # channel axis is axis 1 of NCHW: permuting channels changes nothing, permuting pixels permutes the map
    perm = rng.permutation(40)
    ent3, _, _ = orc.attention_budget(act[:, perm], step, 8, 16)
    assert np.allclose(ent, ent3, rtol=1e-6, atol=1e-7)
    ent4, _, _ = orc.attention_budget(act[:, :, ::-1, :], step, 8, 16)
    assert np.array_equal(ent4, ent[:, ::-1, :])


def test_mask_is_a_threshold_at_the_image_mean(orc):
    rng = np.random.default_rng(2)
    act = rng.integers(0, 128, size=(4, 16, 7, 7)).astype(np.int8)
    act[1] = 0                                       # an image with constant entropy: nothing is above the mean
    ent, mean, bud = orc.attention_budget(act, 0.1, 8, 16)
    assert set(np.unique(bud)) <= {8, 16}
    for b in range(4):
        assert np.array_equal(bud[b] == 16, ent[b] > mean[b])           # strictly above, per image
    assert np.all(bud[1] == 8)
    assert 0.2 < (bud[[0, 2, 3]] == 16).mean() < 0.8
    # images are independent: changing one leaves the others' masks alone
    act2 = act.copy()
    act2[0] = rng.integers(0, 128, size=(16, 7, 7))
    _, _, bud2 = orc.attention_budget(act2, 0.1, 8, 16)
    assert np.array_equal(bud2[1:], bud[1:])
    _, _, bud3 = orc.attention_budget(act, 0.1, 2, 32)
    assert np.array_equal(bud3 == 32, bud == 16)
