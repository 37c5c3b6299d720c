"""Pins of the oracle's shared-filter mode (Eq. numbersystem:simulation; Sect. 4.1 "Setup"; suppl.
"Efficient simulation of the forward pass", Eq. binomial) against what the paper and the mathematics fix.
CPU only."""
import math

import numpy as np
import pytest
import torch


def _conv_f64(x, W, stride, pad, groups):
    """Integer convolution by an independent implementation (float64 is exact below 2^53)."""
    y = torch.nn.functional.conv2d(torch.from_numpy(x.astype(np.float64)), torch.from_numpy(W.astype(np.float64)),
                                   stride=stride, padding=pad, groups=groups)
    return y.numpy()


def test_counts_follow_the_binomial_distribution(orc):
    """Eq. (binomial): the count of one weight over n samples is Bin(n, p).  Chi-square over 6000 equal weights."""
    n = 8
    for w, p in ((1.25, 0.25), (-1.5, 0.5), (1.875, 0.875)):
        q = orc.QWeights(np.full((60, 100), w, np.float32), x_absmax=1, s_max=n)
        W = orc.sample_filter(q, n, seed=77, layer_id=5)
        shift = int(q.shift[0, 0])
        B = np.abs(W) // (1 << shift) - n
        assert B.min() >= 0 and B.max() <= n and np.all(np.sign(W) == np.sign(w))
        obs = np.bincount(B.ravel(), minlength=n + 1).astype(np.float64)
        exp = np.array([math.comb(n, k) * p ** k * (1 - p) ** (n - k) for k in range(n + 1)]) * B.size
        keep = exp > 5
        chi2 = float(((obs[keep] - exp[keep]) ** 2 / exp[keep]).sum())
        assert chi2 < 33.0, (w, chi2)          # 99.99 % quantile of chi-square with 8 degrees of freedom: 31.8


def test_mean_and_variance_of_the_sampled_weight(orc):
    """E[w_bar_n] = w and Var[w_bar_n] = 2^(2e) p (1-p) / n (Sect. 3.2 with the binomial of Eq. numbersystem:simulation)."""
    rng = np.random.default_rng(5)
    w = rng.uniform(0.26, 0.49, size=8).astype(np.float32) * rng.choice([-1, 1], size=8)   # one exponent: e = -2
    q = orc.QWeights(np.tile(w, (1, 1)), x_absmax=1, s_max=16)
    for n in (4, 16):
        runs = np.stack([orc.sample_filter(q, n, seed=s, layer_id=1)[0] for s in range(4000)]).astype(np.float64)
        wbar = runs * 2.0 ** q.e_min / n
        p = np.abs(w.astype(np.float64)) / 0.25 - 1.0
        var = 0.25 ** 2 * p * (1 - p) / n
        assert np.all(np.abs(wbar.mean(axis=0) - w) < 5 * np.sqrt(var / 4000))
        assert np.allclose(wbar.var(axis=0), var, rtol=0.15)


def test_exact_mean_by_enumeration(orc):
    """All 4^2 outcomes of two samples on a four-point uniform grid, through the injected table."""
    w = np.array([[1.25, -1.75, 2.0]], np.float32)
    q = orc.QWeights(w, x_absmax=1, s_max=2)
    grid = [0, 1 << 30, 2 << 30, 3 << 30]
    tot = np.zeros(3, dtype=np.int64)
    for a in grid:
        for b in grid:
            tab = np.tile(np.array([a, b], np.uint32), (3, 1))
            tot += orc.sample_filter(q, 2, u_table=tab)[0]
    # E[W] * 16 = 16 * sigma 2^shift (n + n p) with p = 1/4, 3/4, 0 (exactly representable on the grid)
    unit = (1 << q.shift[0]).astype(np.int64)
    assert np.array_equal(tot, np.array([16 * unit[0] * 2 * 5 // 4, -16 * unit[1] * 2 * 7 // 4, 16 * unit[2] * 2]))


def test_counts_use_the_stream_of_the_output_channel(orc):
    """Keying: weight (oc, k), sample i draws uniform(seed, layer, o := oc, k, i), strict comparison with p."""
    rng = np.random.default_rng(9)
    w = rng.uniform(1.0, 2.0, size=(5, 7)).astype(np.float32)
    q = orc.QWeights(w, x_absmax=1, s_max=12)
    seed, layer = (123 << 32) | 456, 9
    W = orc.sample_filter(q, seed=seed, layer_id=layer, sample_from=3, sample_to=11)
    for oc in range(5):
        for k in range(7):
            B = sum(1 for i in range(3, 11) if orc.uniform(seed, layer, oc, k, i) / 2.0 ** 32 < q.p[oc, k])
            assert W[oc, k] == (1 << int(q.shift[oc, k])) * (8 + B)
    q7 = orc.QWeights(w, x_absmax=1, s_max=40, prob_bits=4)
    W7 = orc.sample_filter(q7, seed=seed, layer_id=layer, sample_from=5, sample_to=37)
    for oc in range(5):
        for k in range(7):
            B = sum(1 for i in range(5, 37) if orc.uniform7(seed, layer, oc, k, i) / 128.0 < q7.p[oc, k])
            assert W7[oc, k] == (1 << int(q7.shift[oc, k])) * (32 + B)


def test_prefix_property_of_the_filters(orc):
    rng = np.random.default_rng(10)
    q = orc.QWeights(rng.standard_normal((6, 20)).astype(np.float32), x_absmax=4, s_max=32)
    full = orc.sample_filter(q, seed=4, sample_from=0, sample_to=32)
    a = orc.sample_filter(q, seed=4, sample_from=0, sample_to=13)
    b = orc.sample_filter(q, seed=4, sample_from=13, sample_to=32)
    assert np.array_equal(full, a + b)
    assert np.array_equal(orc.sample_filter(q, seed=4, sample_from=7, sample_to=7), np.zeros_like(full))


@pytest.mark.parametrize("shape", [
    # n, c, oc, h, w, kh, kw, stride, pad, groups
    (2, 6, 8, 9, 7, 3, 3, (1, 1), (1, 1), 1),
    (1, 4, 6, 11, 10, 5, 3, (2, 1), (2, 0), 2),
    (2, 8, 8, 6, 6, 3, 3, (1, 2), (1, 1), 8),
    (3, 10, 5, 1, 1, 1, 1, (1, 1), (0, 0), 1),
])
def test_layer_is_a_convolution_with_the_sampled_filter(orc, shape):
    n, c, oc, h, w, kh, kw, stride, pad, groups = shape
    rng = np.random.default_rng(11)
    wt = (rng.standard_normal((oc, c // groups, kh, kw)) * 0.2).astype(np.float32)
    wt[0, 0, 0, 0] = 0.0
    x = rng.integers(-128, 128, size=(n, c, h, w)).astype(np.int8)
    q = orc.QWeights(wt.reshape(oc, -1), x_absmax=128, s_max=16)
    acc, over = orc.conv2d_shared(q, (oc, c, kh, kw, groups), x, stride, pad, S=16, seed=21, layer_id=2)
    W = orc.sample_filter(q, 16, seed=21, layer_id=2).reshape(oc, c // groups, kh, kw)
    assert over == 0
    assert np.array_equal(acc.astype(np.float64), _conv_f64(x, W, stride, pad, groups))


def test_all_pixels_of_a_channel_share_one_filter(orc):
    """A constant image: interior outputs of a channel are all equal in shared-filter mode, and are not in
    per-product mode, where every output element draws its own bits."""
    rng = np.random.default_rng(12)
    wt = rng.uniform(0.3, 0.45, size=(4, 3, 3, 3)).astype(np.float32)
    x = np.full((1, 3, 10, 10), 7, np.int8)
    q = orc.QWeights(wt.reshape(4, -1), x_absmax=7, s_max=8)
    acc, _ = orc.conv2d_shared(q, (4, 3, 3, 3, 1), x, S=8, seed=1)
    assert np.all(acc == acc[:, :, :1, :1])
    per_product, _, _ = orc.conv2d(q, (4, 3, 3, 3, 1), x, S=8, seed=1)
    assert not np.all(per_product == per_product[:, :, :1, :1])


def test_powers_of_two_make_both_modes_the_same_deterministic_convolution(orc):
    rng = np.random.default_rng(13)
    wt = (2.0 ** rng.integers(-4, 1, size=(5, 4, 3, 3)) * rng.choice([-1, 1], size=(5, 4, 3, 3))).astype(np.float32)
    x = rng.integers(-20, 21, size=(2, 4, 6, 6)).astype(np.int8)
    q = orc.QWeights(wt.reshape(5, -1), x_absmax=20, s_max=4)
    a, _ = orc.conv2d_shared(q, (5, 4, 3, 3, 1), x, pad=(1, 1), S=4, seed=1)
    b, _ = orc.conv2d_shared(q, (5, 4, 3, 3, 1), x, pad=(1, 1), S=4, seed=2)
    c, _, _ = orc.conv2d(q, (5, 4, 3, 3, 1), x, pad=(1, 1), S=4, seed=3)
    assert np.array_equal(a, b) and np.array_equal(a, c)
    ref = _conv_f64(x, wt.astype(np.float64) * 4 / 2.0 ** q.e_min, (1, 1), (1, 1), 1)
    assert np.array_equal(a.astype(np.float64), ref)


def test_progressive_budgets_nest(orc):
    rng = np.random.default_rng(14)
    wt = (rng.standard_normal((6, 5, 3, 3)) * 0.1).astype(np.float32)
    x = rng.integers(0, 50, size=(2, 5, 7, 8)).astype(np.int8)
    ws = (6, 5, 3, 3, 1)
    q = orc.QWeights(wt.reshape(6, -1), x_absmax=50, s_max=16)
    to = rng.choice([0, 1, 4, 8, 16, 40], size=(2, 7, 8)).astype(np.uint8)        # 40 is clamped to 16
    full, over = orc.conv2d_shared(q, ws, x, pad=(1, 1), budget_to=to, seed=6, layer_id=1)
    assert over == 0
    # a pixel with budget t sees the filter of samples [0, t): compare level by level with plain calls
    for level in (1, 4, 8, 16):
        plain, _ = orc.conv2d_shared(q, ws, x, pad=(1, 1), S=level, seed=6, layer_id=1)
        sel = np.broadcast_to((np.minimum(to, 16) == level)[:, None], full.shape)
        assert np.array_equal(full[sel], plain[sel])
    assert np.all(full[np.broadcast_to((to == 0)[:, None], full.shape)] == 0)
    # refinement in two calls equals one call
    first = np.minimum(to, 4).astype(np.uint8)
    a1, _ = orc.conv2d_shared(q, ws, x, pad=(1, 1), budget_to=first, seed=6, layer_id=1)
    a2, _ = orc.conv2d_shared(q, ws, x, pad=(1, 1), budget_to=to, budget_from=first, seed=6, layer_id=1, acc_in=a1)
    assert np.array_equal(a2, full)
    # constant map = plain call
    const, _ = orc.conv2d_shared(q, ws, x, pad=(1, 1), budget_to=np.full((2, 7, 8), 8, np.uint8), seed=6, layer_id=1)
    plain, _ = orc.conv2d_shared(q, ws, x, pad=(1, 1), S=8, seed=6, layer_id=1)
    assert np.array_equal(const, plain)


def test_points_variant_equals_the_full_one(orc):
    rng = np.random.default_rng(16)
    wt = (rng.standard_normal((6, 4, 3, 3)) * 0.1).astype(np.float32)
    x = rng.integers(-9, 10, size=(2, 4, 6, 5)).astype(np.int8)
    q = orc.QWeights(wt.reshape(6, -1), x_absmax=9, s_max=8)
    to = rng.choice([0, 3, 8], size=(2, 3, 5)).astype(np.uint8)
    full, _ = orc.conv2d_shared(q, (6, 4, 3, 3, 1), x, stride=(2, 1), pad=(1, 1), budget_to=to, seed=3)
    pts = rng.choice(full.size, 40, replace=False)
    some, _ = orc.conv2d_shared(q, (6, 4, 3, 3, 1), x, stride=(2, 1), pad=(1, 1), budget_to=to, seed=3, points=pts)
    assert np.array_equal(some, full.ravel()[pts])


def test_layer_output_is_unbiased(orc):
    """Mean over seeds of the rescaled shared-filter output approaches the float convolution (Sect. 3.1)."""
    rng = np.random.default_rng(15)
    wt = (rng.standard_normal((3, 4, 3, 3)) * 0.2).astype(np.float32)
    x = rng.integers(0, 16, size=(1, 4, 5, 5)).astype(np.int8)
    q = orc.QWeights(wt.reshape(3, -1), x_absmax=15, s_max=4, exp_bits=5)
    runs = np.stack([orc.conv2d_shared(q, (3, 4, 3, 3, 1), x, pad=(1, 1), S=4, seed=s)[0] for s in range(1500)])
    mean = runs.astype(np.float64).mean(axis=0) * 2.0 ** q.e_min / 4
    sd = runs.astype(np.float64).std(axis=0) * 2.0 ** q.e_min / 4
    ref = _conv_f64(x, q.represented().reshape(3, 4, 3, 3), (1, 1), (1, 1), 1)
    assert np.all(np.abs(mean - ref) < 5 * sd / np.sqrt(1500) + 1e-12)
