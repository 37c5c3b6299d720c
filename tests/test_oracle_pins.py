"""Pins of the CPU oracle against what the paper and the mathematics fix.

None of these tests touches the GPU library.  Each one is chosen so that a plausible mistake in the
oracle (dropped term, wrong sign, wrong index, `<` vs `<=`, wrong word of the generator, transposed
operand) makes it fail.
"""
import itertools
import os
import struct

import numpy as np
import pytest
from scipy import stats

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ------------------------------------------------------------------ number system (Sect. 3.1)

def _fields(w):
    bits = struct.unpack("<I", struct.pack("<f", w))[0]
    return bits >> 31, (bits >> 23) & 0xFF, bits & 0x7FFFFF


def test_decode_worked_example_w3(orc):
    # Sect. 3.2: "the representation for w = 3 is (e=1, p=0.5)"
    assert orc.decode(3.0) == (orc.NORMAL, 1, 1, 0.5)
    assert orc.decode(-3.0) == (orc.NORMAL, -1, 1, 0.5)


def test_decode_powers_of_two_have_p_zero(orc):
    # Fig. numbersystem (b): filled markers at (+-2^k, 0)
    for k in range(-126, 128):
        for sgn in (1.0, -1.0):
            cls, s, e, p = orc.decode(sgn * 2.0 ** k)
            assert (cls, s, e, p) == (orc.NORMAL, int(sgn), k, 0.0)


def test_decode_equals_ieee_fields(orc):
    # e = floor(log2|w|), p = |w|/2^e - 1 is, for a normal binary32, (exponent field - 127, mantissa / 2^23)
    rng = np.random.default_rng(7)
    bits = rng.integers(0, 2 ** 32, size=20000, dtype=np.uint64).astype(np.uint32)
    edge = np.array([0x00800000, 0x00800001, 0x7F7FFFFF, 0x3F800000, 0x3FFFFFFF, 0x40000000, 0x807FFFFF,
                     0x00000001, 0x007FFFFF, 0x80000000, 0x00000000], dtype=np.uint32)
    for b in np.concatenate([bits, edge]):
        w = struct.unpack("<f", struct.pack("<I", int(b)))[0]
        sign, ef, m = _fields(w)
        cls, s, e, p = orc.decode(w)
        if ef == 255:
            assert cls == orc.NONFINITE
        elif ef == 0 and m == 0:
            assert cls == orc.ZERO
        elif ef == 0:
            assert cls == orc.SUBNORMAL
            assert 0.0 <= p < 1.0 and abs(w) == (1.0 + p) * 2.0 ** e
        else:
            assert cls == orc.NORMAL
            assert s == (-1 if sign else 1)
            assert e == ef - 127
            assert p == m / 2.0 ** 23


def test_decode_is_unbiased_identity(orc):
    # E[w_bar] = s 2^e ((1-p) + 2p) = w   (Sect. 3.1, line after the definition of p)
    rng = np.random.default_rng(8)
    for w in rng.standard_normal(2000).astype(np.float32) * 0.1:
        cls, s, e, p = orc.decode(float(w))
        assert s * 2.0 ** e * (1.0 + p) == float(w)


# ------------------------------------------------------------------ generator

def _kat():
    rows = []
    with open(os.path.join(GOLDEN, "philox4x32_10_kat.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            v = [int(t, 16) for t in line.split()]
            rows.append((v[0:4], v[4:6], v[6:10]))
    return rows


def test_philox_known_answers(orc):
    rows = _kat()
    assert len(rows) == 3
    for ctr, key, out in rows:
        assert orc.philox(ctr, key) == out


def test_uniform_keying(orc):
    # u(o,k,s) = word (s mod 4) of the block with counter (o, k, s div 4, layer) and key (seed lo, seed hi).
    # The pi-digit vector pins every position: o, k, s div 4, layer, both key halves and the word order.
    ctr, key, out = _kat()[2]
    seed = key[0] | (key[1] << 32)
    for word in range(4):
        assert orc.uniform(seed, ctr[3], ctr[0], ctr[1], 4 * ctr[2] + word) == out[word]


def test_uniform_is_uniform_and_streams_differ(orc):
    u = np.array([orc.uniform(5, 1, o, k, s) for o in range(40) for k in range(25) for s in range(8)],
                 dtype=np.float64)
    hist, _ = np.histogram(u, bins=16, range=(0, 2.0 ** 32))
    assert stats.chisquare(hist).pvalue > 1e-4
    a = np.array([orc.uniform(5, 1, o, 0, 0) for o in range(2000)], dtype=np.float64)
    b = np.array([orc.uniform(5, 1, o, 1, 0) for o in range(2000)], dtype=np.float64)
    c = np.array([orc.uniform(5, 2, o, 0, 0) for o in range(2000)], dtype=np.float64)
    d = np.array([orc.uniform(6, 1, o, 0, 0) for o in range(2000)], dtype=np.float64)
    for other in (b, c, d):
        assert abs(np.corrcoef(a, other)[0, 1]) < 0.1
        assert not np.array_equal(a, other)


# ------------------------------------------------------------------ exact expectation by enumeration

@pytest.mark.parametrize("K,S", [(2, 3), (3, 2), (1, 4), (5, 1)])
def test_enumeration_gives_exact_expectation(orc, K, S):
    """All outcomes of the random bits of a tiny layer, each weighted equally.

    Mantissas have two significant bits (p in {0, 1/4, 1/2, 3/4}); the injected uniforms take the four
    values j*2^30 + 12345 (j = 0..3), so exactly 4p of them lie below p.  The mean of acc over all
    4^(K*S) tables must equal S * sum_k sigma_k x_k 2^shift_k (1+p_k) exactly, as integers.
    """
    w = np.array([[1.25, -0.75, 3.5, -2.0, 0.4375][:K]], dtype=np.float32)   # p = .25, .5, .75, 0, .75
    x = np.array([[3, -5, 7, -128, 127][:K]], dtype=np.int8)
    q = orc.QWeights(w, x_absmax=128, s_max=S)
    total = 0
    n = 0
    for combo in itertools.product(range(4), repeat=K * S):
        table = (np.array(combo, dtype=np.uint64) * (1 << 30) + 12345).astype(np.uint32)
        acc, over = orc.linear(q, x, S, u_table=table)
        assert over == 0
        total += int(acc[0, 0])
        n += 1
    expect = 0
    for k in range(K):
        cls, s, e, p = orc.decode(float(w[0, k]))
        expect += S * s * int(x[0, k]) * (2 ** (e - q.e_min)) * (1.0 + p)
    assert total == expect * n


def test_threshold_is_strict(orc):
    # p = 1/2: u = 2^31 - 1 is below, u = 2^31 is not.  p = 0: even u = 0 is not below.
    w = np.array([[1.5]], dtype=np.float32)
    x = np.array([[1]], dtype=np.int8)
    q = orc.QWeights(w, x_absmax=1, s_max=1, exp_bits=1)
    lo, _ = orc.linear(q, x, 1, u_table=np.array([2 ** 31 - 1], dtype=np.uint32))
    hi, _ = orc.linear(q, x, 1, u_table=np.array([2 ** 31], dtype=np.uint32))
    assert int(hi[0, 0]) * 2 == int(lo[0, 0])
    w1 = np.array([[1.0]], dtype=np.float32)
    q1 = orc.QWeights(w1, x_absmax=1, s_max=1, exp_bits=1)
    z, _ = orc.linear(q1, x, 1, u_table=np.array([0], dtype=np.uint32))
    assert int(z[0, 0]) == 2 ** (0 - q1.e_min)


# ------------------------------------------------------------------ deterministic special case

def test_power_of_two_weights_sample_deterministically(orc):
    rng = np.random.default_rng(11)
    e = rng.integers(-6, 1, size=(7, 33))
    sgn = rng.choice([-1.0, 1.0], size=e.shape)
    w = (sgn * 2.0 ** e).astype(np.float32)
    x = rng.integers(-128, 128, size=(5, 33)).astype(np.int8)
    q = orc.QWeights(w, x_absmax=128, s_max=8)
    ref = 8 * (x.astype(np.int64) @ (sgn * 2.0 ** (e - q.e_min)).astype(np.int64).T)
    for seed in (0, 1, 2 ** 40 + 3):
        acc, over = orc.linear(q, x, 8, seed=seed, layer_id=seed % 5)
        assert over == 0
        assert np.array_equal(acc.astype(np.int64), ref)


# ------------------------------------------------------------------ statistics (Sect. 3.2)

def _single_weight_samples(orc, w, n, S=1, seed=3):
    """n independent draws of the S-sample sum of one weight with x = 1 (one output row per draw)."""
    q = orc.QWeights(np.array([[w]], dtype=np.float32), x_absmax=1, s_max=S)
    x = np.ones((n, 1), dtype=np.int8)
    acc, over = orc.linear(q, x, S, seed=seed)
    assert over == 0
    return acc[:, 0].astype(np.float64) * 2.0 ** q.e_min / S


@pytest.mark.parametrize("w", [3.0, 0.75, -1.1, 4.0 / 3.0, 0.3, -0.0123])
def test_single_weight_mean_and_variance(orc, w):
    n = 200000
    v = _single_weight_samples(orc, w, n)
    w32 = float(np.float32(w))
    e = np.floor(np.log2(abs(w32)))
    var = (2.0 ** (e + 1) - abs(w32)) * (abs(w32) - 2.0 ** e)       # Fig. numbersystem (c)
    assert set(np.unique(np.abs(v))) <= {2.0 ** e, 2.0 ** (e + 1)}
    assert abs(v.mean() - w32) < 6 * np.sqrt(var / n)
    # variance of the sample variance of a two-point variable: (mu4 - var^2)/n
    p = abs(w32) / 2.0 ** e - 1
    mu4 = (2.0 ** e) ** 4 * p * (1 - p) * ((1 - p) ** 3 + p ** 3)
    # (+ the second-order term from centring at the sample mean, which is all that is left at p = 1/2)
    assert abs(v.var() - var) < 6 * np.sqrt((mu4 - var ** 2) / n) + 40 * var / n + 1e-12
    assert var <= w32 * w32 / 8 + 1e-12                               # Sect. 3.2 bound


def test_variance_closed_form_values():
    # values read off the plotted closed form: w=3 -> 1, w=0.75 -> 1/16; bound tight at p = 1/3
    f = lambda w: (2.0 ** (np.floor(np.log2(abs(w))) + 1) - abs(w)) * (abs(w) - 2.0 ** np.floor(np.log2(abs(w))))
    assert f(3.0) == 1.0 and f(0.75) == 0.0625
    assert abs(f(4.0 / 3.0) - (4.0 / 3.0) ** 2 / 8) < 1e-15


def test_n_sample_variance_scales_as_one_over_n(orc):
    w = 4.0 / 3.0
    n = 100000
    for S in (2, 8, 32):
        v = _single_weight_samples(orc, w, n, S=S, seed=9)
        var1 = float(np.float32(w)) ** 2 / 8
        assert abs(v.var() - var1 / S) < 0.03 * var1 / S
        assert v.std() / abs(v.mean()) <= 1.02 / np.sqrt(8 * S)     # relative error bound


def test_count_of_large_shifts_is_binomial(orc):
    # Eq. (numbersystem:simulation): the number of (e+1)-choices among n samples is Bin(n, p)
    w, S, n = 1.375, 8, 100000           # p = 0.375
    v = _single_weight_samples(orc, w, n, S=S, seed=12)
    cnt = np.rint(v * S - S).astype(int)                # sum = S + count  (2^e = 1)
    hist = np.bincount(cnt, minlength=S + 1)
    expect = stats.binom.pmf(np.arange(S + 1), S, 0.375) * n
    assert stats.chisquare(hist, expect).pvalue > 1e-4


def test_layer_mean_converges_to_dot_product(orc):
    """CLT: over T seeds the mean of acc*2^e_min/S is within 6 sigma/sqrt(T) of sum_k x_k w_k."""
    rng = np.random.default_rng(21)
    K, OC, B, S, T = 96, 6, 4, 8, 300
    w = (rng.standard_normal((OC, K)) * 0.05).astype(np.float32)
    x = rng.integers(0, 16, size=(B, K)).astype(np.int8)
    q = orc.QWeights(w, x_absmax=15, s_max=S)
    what = q.represented()                                       # flushed weights count as 0
    exact = x.astype(np.float64) @ what.T
    aw = np.abs(what)
    e = np.floor(np.log2(np.where(aw > 0, aw, 1.0)))
    var_w = np.where(aw > 0, (2.0 ** (e + 1) - aw) * (aw - 2.0 ** e), 0.0)
    sigma = np.sqrt((x.astype(np.float64) ** 2) @ var_w.T / S)
    mean = np.zeros((B, OC))
    sq = np.zeros((B, OC))
    for t in range(T):
        acc, over = orc.linear(q, x, S, seed=1000 + t)
        assert over == 0
        v = acc.astype(np.float64) * 2.0 ** q.e_min / S
        mean += v
        sq += v * v
    mean /= T
    var_emp = sq / T - mean ** 2
    assert np.all(np.abs(mean - exact) < 6 * sigma / np.sqrt(T))
    assert np.all(np.abs(var_emp / sigma ** 2 - 1) < 0.5)
    # and the represented weights are the true ones up to what was flushed
    assert np.all(np.abs(what - w)[q.sign != 0] == 0)


# ------------------------------------------------------------------ window / overflow rule

def test_e_min_closed_form_cases(orc):
    # all weights 1.0 (e=0): bound = x_absmax*s_max*K*2^(1-e_min) <= 2^31-1
    q = orc.QWeights(np.ones((1, 4), np.float32), x_absmax=128, s_max=16)     # 2^13*2^(1-e_min): window caps
    assert (q.e_top, q.e_min) == (0, -15)
    q = orc.QWeights(np.ones((1, 64), np.float32), x_absmax=128, s_max=16)    # 2^17*2^(1-e_min) <= 2^31-1
    assert (q.e_top, q.e_min) == (0, -12)
    q = orc.QWeights(np.ones((3, 64), np.float32), x_absmax=128, s_max=16, exp_bits=3)
    assert (q.e_top, q.e_min) == (0, -7)
    # the channel with the largest sum decides
    w = np.zeros((2, 64), np.float32)
    w[0, :] = 1.0
    w[1, :2] = 1.0
    assert orc.QWeights(w, x_absmax=128, s_max=16).e_min == -12
    assert orc.QWeights(w, x_absmax=128, s_max=16).n_zero == 62


def test_flush_zero_subnormal_and_errors(orc):
    w = np.array([[1.0, 2.0 ** -20, 0.0, -0.0, 1e-40, -1.5]], dtype=np.float32)
    q = orc.QWeights(w, x_absmax=1, s_max=1)
    assert q.e_min == -15
    assert list(q.sign[0]) == [1, 0, 0, 0, 0, -1]
    assert (q.n_zero, q.n_flushed, q.n_live) == (2, 2, 2)
    for bad in (np.nan, np.inf, -np.inf):
        with pytest.raises(orc.OracleError) as ei:
            orc.QWeights(np.array([[1.0, bad]], dtype=np.float32))
        assert ei.value.code == orc.ERR_VALUE
    with pytest.raises(orc.OracleError) as ei:            # cannot fit even with a one-exponent window
        orc.QWeights(np.ones((1, 2 ** 16), np.float32), x_absmax=128, s_max=255)
    assert ei.value.code == orc.ERR_OVERFLOW_UNSAFE
    sub = orc.QWeights(np.array([[1e-40, 0.0]], dtype=np.float32))
    assert sub.n_live == 0 and sub.n_flushed == 1


def test_adversarial_input_stays_inside_int32(orc):
    rng = np.random.default_rng(31)
    w = np.abs(rng.standard_normal((3, 1152)) * 0.04).astype(np.float32)
    q = orc.QWeights(w, x_absmax=128, s_max=32)
    x = np.full((1, 1152), -128, dtype=np.int8)
    # force every sample to take the larger shift
    table = np.zeros(3 * 1152 * 32, dtype=np.uint32)
    acc, over = orc.linear(q, x, 32, u_table=table)
    assert over == 0 and np.all(acc < 0)
    live = q.sign != 0
    worst = (128 * 32 * (2.0 ** (q.shift + 1) * live).sum(axis=1)).max()
    assert worst <= 2 ** 31 - 1
    worst_next = 128 * 32 * np.array([(2.0 ** (np.floor(np.log2(r)) - (q.e_min - 1) + 1) *
                                       (np.floor(np.log2(r)) >= q.e_min - 1)).sum() for r in w]).max()
    assert q.e_min - 1 < q.e_top - 15 or worst_next > 2 ** 31 - 1       # e_min is the smallest admissible


# ------------------------------------------------------------------ convolution indexing

@pytest.mark.parametrize("cin,oc,groups,kh,kw,stride,pad,h,w", [
    (4, 6, 1, 3, 3, (1, 1), (1, 1), 7, 9),
    (4, 6, 2, 3, 3, (2, 2), (1, 1), 8, 7),
    (6, 6, 6, 3, 3, (1, 1), (1, 1), 6, 6),
    (3, 5, 1, 7, 7, (2, 2), (3, 3), 15, 13),
    (8, 4, 1, 1, 1, (2, 2), (0, 0), 9, 9),
    (4, 4, 2, 2, 3, (1, 2), (0, 2), 6, 8),
])
def test_conv_reduces_to_textbook_convolution(orc, cin, oc, groups, kh, kw, stride, pad, h, w):
    """With power-of-two weights the layer is a deterministic integer convolution: compare with torch."""
    import torch
    rng = np.random.default_rng(41)
    e = rng.integers(-5, 1, size=(oc, cin // groups, kh, kw))
    sgn = rng.choice([-1.0, 1.0], size=e.shape)
    wt = (sgn * 2.0 ** e).astype(np.float32)
    wt[rng.random(wt.shape) < 0.2] = 0.0
    x = rng.integers(-128, 128, size=(2, cin, h, w)).astype(np.int8)
    S = 4
    q = orc.QWeights(wt, x_absmax=128, s_max=S)
    acc, over, smac = orc.conv2d(q, (oc, cin, kh, kw, groups), x, stride, pad, S=S, seed=77, layer_id=3)
    ref = torch.nn.functional.conv2d(torch.from_numpy(x.astype(np.float64)),
                                     torch.from_numpy(wt.astype(np.float64) * 2.0 ** (-q.e_min)),
                                     stride=stride, padding=pad, groups=groups).numpy() * S
    assert over == 0
    assert np.array_equal(acc.astype(np.float64), ref)
    # sampled-MAC count = S * (live taps inside the image), via a convolution of ones
    ones = torch.ones((2, cin, h, w), dtype=torch.float64)
    live = torch.from_numpy((wt != 0).astype(np.float64))
    cnt = torch.nn.functional.conv2d(ones, live, stride=stride, padding=pad, groups=groups).sum().item()
    assert smac == S * int(cnt)


def test_linear_is_a_1x1_convolution(orc):
    rng = np.random.default_rng(43)
    w = (rng.standard_normal((9, 37)) * 0.1).astype(np.float32)
    x = rng.integers(-128, 128, size=(5, 37)).astype(np.int8)
    q = orc.QWeights(w, x_absmax=128, s_max=6)
    a, _ = orc.linear(q, x, 6, seed=99, layer_id=4)
    b, _, smac = orc.conv2d(q, (9, 37, 1, 1, 1), x.reshape(5, 37, 1, 1), S=6, seed=99, layer_id=4)
    assert np.array_equal(a, b.reshape(5, 9))
    assert smac == 5 * 6 * q.n_live


def test_conv_mean_converges_to_float_convolution(orc):
    import torch
    rng = np.random.default_rng(45)
    w = (rng.standard_normal((4, 3, 3, 3)) * 0.2).astype(np.float32)
    x = rng.integers(-20, 60, size=(1, 3, 6, 6)).astype(np.int8)
    S, T = 4, 400
    q = orc.QWeights(w, x_absmax=128, s_max=S)
    what = q.represented().reshape(w.shape)
    exact = torch.nn.functional.conv2d(torch.from_numpy(x.astype(np.float64)), torch.from_numpy(what),
                                       padding=1).numpy()
    aw = np.abs(what)
    e = np.floor(np.log2(np.where(aw > 0, aw, 1.0)))
    var_w = np.where(aw > 0, (2.0 ** (e + 1) - aw) * (aw - 2.0 ** e), 0.0)
    sigma = np.sqrt(torch.nn.functional.conv2d(torch.from_numpy(x.astype(np.float64) ** 2),
                                               torch.from_numpy(var_w), padding=1).numpy() / S)
    mean = np.zeros(exact.shape)
    for t in range(T):
        acc, over, _ = orc.conv2d(q, (4, 3, 3, 3, 1), x, pad=(1, 1), S=S, seed=t, layer_id=1)
        mean += acc * 2.0 ** q.e_min / S
    mean /= T
    assert np.all(np.abs(mean - exact) <= 6 * sigma / np.sqrt(T) + 1e-12)


# ------------------------------------------------------------------ progressive budgets (Sect. 4.5)

def _small_conv(orc, s_max=16, seed=5):
    rng = np.random.default_rng(51)
    w = (rng.standard_normal((5, 4, 3, 3)) * 0.1).astype(np.float32)
    x = rng.integers(-30, 100, size=(2, 4, 6, 7)).astype(np.int8)
    x[rng.random(x.shape) < 0.4] = 0
    q = orc.QWeights(w, x_absmax=128, s_max=s_max)
    return q, (5, 4, 3, 3, 1), x


def test_progressive_constant_map_equals_plain_call(orc):
    q, ws, x = _small_conv(orc)
    plain, _, n1 = orc.conv2d(q, ws, x, pad=(1, 1), S=8, seed=5, layer_id=2)
    full = np.full((2, 6, 7), 8, np.uint8)
    prog, _, n2 = orc.conv2d(q, ws, x, pad=(1, 1), budget_to=full, seed=5, layer_id=2)
    assert np.array_equal(plain, prog) and n1 == n2


def test_progressive_refinement_reuses_first_samples(orc):
    q, ws, x = _small_conv(orc)
    rng = np.random.default_rng(52)
    to = rng.choice([0, 2, 4, 8, 16], size=(2, 6, 7)).astype(np.uint8)
    mid = np.minimum(to, 4).astype(np.uint8)
    one, o1, n_one = orc.conv2d(q, ws, x, pad=(1, 1), budget_to=to, seed=5, layer_id=2)
    a, o2, n_a = orc.conv2d(q, ws, x, pad=(1, 1), budget_to=mid, seed=5, layer_id=2)
    b, o3, n_b = orc.conv2d(q, ws, x, pad=(1, 1), budget_to=to, budget_from=mid, seed=5, layer_id=2, acc_in=a)
    assert np.array_equal(one, b)
    assert n_one == n_a + n_b and o1 == o2 == o3 == 0
    # a pixel with budget 0 stays 0; a pixel's result depends on its own budget only
    assert np.all(one[:, :, :, :][np.broadcast_to((to == 0)[:, None], one.shape)] == 0)
    for level in (2, 4, 8, 16):
        const, _, _ = orc.conv2d(q, ws, x, pad=(1, 1), S=level, seed=5, layer_id=2)
        m = np.broadcast_to((to == level)[:, None], one.shape)
        assert np.array_equal(one[m], const[m])


def test_budget_clamping(orc):
    q, ws, x = _small_conv(orc, s_max=8)
    to = np.full((2, 6, 7), 200, np.uint8)
    frm = np.full((2, 6, 7), 100, np.uint8)
    a, _, n = orc.conv2d(q, ws, x, pad=(1, 1), budget_to=to, seed=5)
    b, _, _ = orc.conv2d(q, ws, x, pad=(1, 1), S=8, seed=5)
    assert np.array_equal(a, b)
    c, _, n0 = orc.conv2d(q, ws, x, pad=(1, 1), budget_to=to, budget_from=frm, seed=5, acc_in=a)
    assert np.array_equal(c, a) and n0 == 0


def test_progressive_cost_accounting(orc):
    # Sect. 4.5: 35 % of the pixels at 16 samples, 65 % at 8 => 0.675 of the cost of 16 everywhere ("-33 %");
    # 16/32 => 1.35 ("+33 %").  Only true when refinement reuses the first samples.
    rng = np.random.default_rng(53)
    w = (rng.standard_normal((3, 2, 1, 1)) * 0.1).astype(np.float32)
    x = rng.integers(0, 100, size=(1, 2, 10, 10)).astype(np.int8)
    q = orc.QWeights(w, x_absmax=128, s_max=32)
    mask = np.zeros(100, bool)
    mask[:35] = True
    mask = mask.reshape(1, 10, 10)
    for lo, hi, ratio in ((8, 16, 0.675), (16, 32, 1.35)):
        to = np.where(mask, hi, lo).astype(np.uint8)
        first = np.full_like(to, lo)
        _, _, n_uniform = orc.conv2d(q, (3, 2, 1, 1, 1), x, S=16, seed=1)
        a, _, n1 = orc.conv2d(q, (3, 2, 1, 1, 1), x, budget_to=first, seed=1)
        _, _, n2 = orc.conv2d(q, (3, 2, 1, 1, 1), x, budget_to=to, budget_from=first, seed=1, acc_in=a)
        assert (n1 + n2) == pytest.approx(ratio * n_uniform)


def test_points_variant_matches_full(orc):
    q, ws, x = _small_conv(orc)
    rng = np.random.default_rng(54)
    to = rng.choice([2, 4, 8, 16], size=(2, 6, 7)).astype(np.uint8)
    full, _, _ = orc.conv2d(q, ws, x, pad=(1, 1), budget_to=to, seed=8, layer_id=1)
    pts = rng.choice(full.size, size=50, replace=False)
    part, _, _ = orc.conv2d(q, ws, x, pad=(1, 1), budget_to=to, seed=8, layer_id=1, points=pts)
    assert np.array_equal(part, full.ravel()[pts])


# ------------------------------------------------------------------ rescale

def test_rescale_is_four_separately_rounded_operations(orc):
    rng = np.random.default_rng(61)
    acc = rng.integers(-2 ** 31, 2 ** 31, size=(3, 5, 4, 4), dtype=np.int64).astype(np.int32)
    mult = (rng.standard_normal(5) * 1e-4).astype(np.float32)
    bias = rng.standard_normal(5).astype(np.float32)
    to = rng.choice([0, 2, 3, 7, 16, 32], size=(3, 4, 4)).astype(np.uint8)
    y = orc.rescale(acc, e_min=-12, budget_to=to, s_max=32, mult=mult, bias=bias)
    inv = np.where(to > 0, np.float32(1.0) / np.maximum(to, 1).astype(np.float32), np.float32(0)).astype(np.float32)
    ref = (acc.astype(np.float32) * mult[None, :, None, None]).astype(np.float32)
    ref = (ref * inv[:, None]).astype(np.float32)
    ref = (ref + bias[None, :, None, None]).astype(np.float32)
    assert np.array_equal(y, ref)
    # default multiplier 2^e_min, no bias: equals the exact quotient to binary32 accuracy
    y2 = orc.rescale(acc, e_min=-12, S=16)
    exact = acc.astype(np.float64) * 2.0 ** -12 / 16
    assert np.allclose(y2, exact, rtol=1e-6, atol=0)


# ------------------------------------------------------------------ discretised probabilities (Sect. 4.4)

def test_probability_grid_includes_zero_excludes_one(orc):
    # p = 0.99 with 2 bits rounds to 4/4: the weight moves to the next exponent with p = 0
    q = orc.QWeights(np.array([[1.99, 1.0]], np.float32), x_absmax=1, s_max=1, prob_bits=2)
    assert q.e_top == 1 and list(q.p[0]) == [0.0, 0.0] and list(q.shift[0] + q.e_min) == [1, 0]
    # ties go to the even grid point: 1.125 -> p = 1/8 -> P = 0.5 -> 0;  1.375 -> P = 1.5 -> 2
    q = orc.QWeights(np.array([[1.125, 1.375, 1.625, 1.875]], np.float32), x_absmax=1, s_max=1, prob_bits=2)
    assert list(q.p[0][:3]) == [0.0, 0.5, 0.5] and q.p[0][3] == 0.0 and q.shift[0][3] + q.e_min == 1
    rng = np.random.default_rng(71)
    w = (rng.standard_normal((6, 200)) * 0.1).astype(np.float32)
    for kp in (1, 2, 3, 4, 6, 7, 8, 12, 22):
        q = orc.QWeights(w, x_absmax=1, s_max=1, prob_bits=kp)
        live = q.sign != 0
        grid = q.p[live] * 2 ** kp
        assert np.all(grid == np.rint(grid)) and grid.min() >= 0 and grid.max() <= 2 ** kp - 1
        rep = q.represented()
        e = np.floor(np.log2(np.abs(w.astype(np.float64))))
        assert np.all(np.abs(rep - w)[live] <= 2.0 ** e[live] * 2.0 ** -(kp + 1) + 1e-18)
    full = orc.QWeights(w, x_absmax=1, s_max=1, prob_bits=23)
    assert np.all(full.represented()[full.sign != 0] == w[full.sign != 0])
    for bad in (0, -1, 24, 32):
        with pytest.raises(orc.OracleError) as ei:
            orc.QWeights(w, prob_bits=bad)
        assert ei.value.code == orc.ERR_VALUE


def test_uniform7_keying(orc):
    # byte b of a block = bits 8*(b mod 4)..+7 of word b div 4; the 7-bit uniform is its low 7 bits
    ctr, key, out = _kat()[0]                     # all-zero counter and key: block 0 of product (0,0), layer 0
    for b in range(16):
        assert orc.uniform7(0, 0, 0, 0, b) == (out[b // 4] >> (8 * (b % 4))) & 0x7F
    # counter positions, through the generator that the known answers pin
    seed, layer, o, k = 0xA4093822299F31D0, 0x03707344, 0x243F6A88, 0x85A308D3
    for j in (0, 1, 5):
        blk = orc.philox([o, k, j, layer], [seed & 0xFFFFFFFF, seed >> 32])
        for b in range(16):
            assert orc.uniform7(seed, layer, o, k, 16 * j + b) == (blk[b // 4] >> (8 * (b % 4))) & 0x7F
    u = np.array([orc.uniform7(9, 0, o, 1, s) for o in range(300) for s in range(40)])
    hist = np.bincount(u, minlength=128)
    assert len(hist) == 128 and stats.chisquare(hist).pvalue > 1e-4


def test_discretised_enumeration_gives_exact_expectation(orc):
    # 2-bit probabilities, all 128 values of the 7-bit uniform for each of K*S = 2 draws
    w = np.array([[1.25, -0.875]], dtype=np.float32)          # p = 1/4 ; -0.875 = -(1/2)(1 + 3/4): p = 3/4
    x = np.array([[5, -9]], dtype=np.int8)
    q = orc.QWeights(w, x_absmax=16, s_max=1, prob_bits=2)
    total = 0
    for a in range(128):
        for b in range(128):
            acc, over = orc.linear(q, x, 1, u_table=np.array([a, b], dtype=np.uint32))
            total += int(acc[0, 0])
    unit = 2.0 ** -q.e_min
    assert total == 128 * 128 * (5 * 1.25 * unit + (-9) * (-0.875) * unit)
    # threshold is strict: p = 1/4 means u7 in 0..31
    one = orc.QWeights(np.array([[1.25]], np.float32), x_absmax=1, s_max=1, prob_bits=2, exp_bits=1)
    lo, _ = orc.linear(one, np.array([[1]], np.int8), 1, u_table=np.array([31], dtype=np.uint32))
    hi, _ = orc.linear(one, np.array([[1]], np.int8), 1, u_table=np.array([32], dtype=np.uint32))
    assert int(lo[0, 0]) == 2 * int(hi[0, 0])


def test_discretised_mean_converges_to_quantised_weights(orc):
    rng = np.random.default_rng(72)
    K, OC, B, S, T = 64, 5, 3, 16, 300
    w = (rng.standard_normal((OC, K)) * 0.05).astype(np.float32)
    x = rng.integers(0, 16, size=(B, K)).astype(np.int8)
    q = orc.QWeights(w, x_absmax=15, s_max=S, prob_bits=4)
    what = q.represented()
    exact = x.astype(np.float64) @ what.T
    aw = np.abs(what)
    e = np.floor(np.log2(np.where(aw > 0, aw, 1.0)))
    var_w = np.where(aw > 0, (2.0 ** (e + 1) - aw) * (aw - 2.0 ** e), 0.0)
    sigma = np.sqrt((x.astype(np.float64) ** 2) @ var_w.T / S)
    mean = np.zeros((B, OC))
    for t in range(T):
        acc, over = orc.linear(q, x, S, seed=500 + t)
        assert over == 0
        mean += acc.astype(np.float64) * 2.0 ** q.e_min / S
    mean /= T
    assert np.all(np.abs(mean - exact) < 6 * sigma / np.sqrt(T) + 1e-12)
    # the convolution path uses the same draws as the linear path
    a, _ = orc.linear(q, x, S, seed=3, layer_id=2)
    b, _, _ = orc.conv2d(q, (OC, K, 1, 1, 1), x.reshape(B, K, 1, 1), S=S, seed=3, layer_id=2)
    assert np.array_equal(a, b.reshape(B, OC))


# ------------------------------------------------------------------ counter keying of the convolution

def _conv_by_hand(orc, q, wshape, x, stride, pad, seed, layer, outputs, ranges, key_o=None, key_k=None, p7=False):
    """Accumulators of selected outputs (n, oc, oy, ox), rebuilt in Python from the pinned uniforms: one
    independent bit per (output element, tap, sample) (Sect. 3.1, shift form after Eq. "numbersystem:simulation";
    Sect. 2: one random bit per shift), B = [u / 2^32 < p] (7-bit uniforms: u7 / 128), term sigma x 2^(shift + B).
    key_o / key_k replace the keying functions (used to show that a transposed index would be noticed)."""
    OC, C, KH, KW, G = wshape
    N, _, H, W = x.shape
    Cg, OCg = C // G, OC // G
    OH, OW = (H + 2 * pad[0] - KH) // stride[0] + 1, (W + 2 * pad[1] - KW) // stride[1] + 1
    if key_o is None:
        key_o = lambda n, oc, oy, ox: ((n * OC + oc) * OH + oy) * OW + ox            # flat NCHW output index
    if key_k is None:
        key_k = lambda ci, kh, kw: (ci * KH + kh) * KW + kw                          # flat tap index in the group
    draw, denom = (orc.uniform7, 128.0) if p7 else (orc.uniform, 4294967296.0)
    res = []
    for (n, oc, oy, ox), (lo, hi) in zip(outputs, ranges):
        total = 0
        for ci in range(Cg):
            for kh in range(KH):
                for kw in range(KW):
                    wi = (ci * KH + kh) * KW + kw                # position in the weight tensor [oc][ci][kh][kw]
                    if q.sign[oc, wi] == 0:
                        continue
                    iy, ix = oy * stride[0] - pad[0] + kh, ox * stride[1] - pad[1] + kw
                    if not (0 <= iy < H and 0 <= ix < W):
                        continue
                    xv = int(x[n, (oc // OCg) * Cg + ci, iy, ix])
                    for s in range(lo, hi):
                        B = 1 if draw(seed, layer, key_o(n, oc, oy, ox), key_k(ci, kh, kw), s) / denom < q.p[oc, wi] else 0
                        total += int(q.sign[oc, wi]) * xv * (1 << (int(q.shift[oc, wi]) + B))
        res.append(total)
    return np.array(res, dtype=np.int64)


@pytest.mark.parametrize("prob_bits", [23, 4])
def test_conv_counter_keying(orc, prob_bits):
    """The uniform of (output, tap, sample) is keyed o = ((n OC + oc) OH + oy) OW + ox, k = (ci KH + kh) KW + kw:
    a non-square, strided, padded, grouped layer with general weights, every size different from every other, so
    that no transposition of indices leaves the result unchanged."""
    rng = np.random.default_rng(81)
    OC, C, KH, KW, G = 6, 8, 3, 2, 2
    N, H, W = 2, 7, 9
    stride, pad = (2, 1), (1, 1)
    wshape = (OC, C, KH, KW, G)
    w = (rng.standard_normal((OC, C // G, KH, KW)) * 0.2).astype(np.float32)
    w[rng.random(w.shape) < 0.1] = 0.0
    x = rng.integers(-100, 101, size=(N, C, H, W)).astype(np.int8)
    x[rng.random(x.shape) < 0.2] = 0
    S, seed, layer = 5, 0x1234567890ABCDEF, 7
    q = orc.QWeights(w, x_absmax=128, s_max=16, prob_bits=prob_bits)
    OH, OW = (H + 2 * pad[0] - KH) // stride[0] + 1, (W + 2 * pad[1] - KW) // stride[1] + 1
    assert len({N, OC, OH, OW}) == 4 and KH != KW and OH != OW
    full, over, _ = orc.conv2d(q, wshape, x, stride, pad, S=S, seed=seed, layer_id=layer)
    assert over == 0 and full.shape == (N, OC, OH, OW)
    outs = [tuple(int(v) for v in rng.integers(0, (N, OC, OH, OW))) for _ in range(40)]
    outs += [(N - 1, OC - 1, OH - 1, OW - 1), (0, 0, 0, 0), (1, 2, 0, OW - 1), (0, OC - 1, OH - 1, 0)]
    want = np.array([full[o] for o in outs], dtype=np.int64)
    p7 = prob_bits != 23
    hand = _conv_by_hand(orc, q, wshape, x, stride, pad, seed, layer, outs, [(0, S)] * len(outs), p7=p7)
    assert np.array_equal(hand, want)
    # the comparison notices each of these mistakes (so the oracle makes none of them)
    wrong = {
        "kh/kw transposed": dict(key_k=lambda ci, kh, kw: (ci * KW + kw) * KH + kh),
        "channel innermost": dict(key_k=lambda ci, kh, kw: (kh * KW + kw) * (C // G) + ci),
        "oy/ox transposed": dict(key_o=lambda n, oc, oy, ox: ((n * OC + oc) * OW + ox) * OH + oy),
        "channels-last output index": dict(key_o=lambda n, oc, oy, ox: ((n * OH + oy) * OW + ox) * OC + oc),
        "channel counted over all groups": dict(key_k=lambda ci, kh, kw: ((ci + C // G) * KH + kh) * KW + kw),
    }
    for name, kw_ in wrong.items():
        assert not np.array_equal(_conv_by_hand(orc, q, wshape, x, stride, pad, seed, layer, outs,
                                                [(0, S)] * len(outs), p7=p7, **kw_), want), name
    # per-pixel ranges use the same keying and the sample index itself: refinement from a first pass
    to = rng.choice([0, 3, 5, 9, 16], size=(N, OH, OW)).astype(np.uint8)
    frm = np.minimum(to, rng.choice([0, 2, 5], size=(N, OH, OW))).astype(np.uint8)
    first, _, _ = orc.conv2d(q, wshape, x, stride, pad, budget_to=frm, seed=seed, layer_id=layer)
    both, _, _ = orc.conv2d(q, wshape, x, stride, pad, budget_to=to, budget_from=frm, seed=seed, layer_id=layer,
                            acc_in=first)
    ranges = [(int(frm[n, oy, ox]), int(to[n, oy, ox])) for n, oc, oy, ox in outs]
    added = _conv_by_hand(orc, q, wshape, x, stride, pad, seed, layer, outs, ranges, p7=p7)
    assert np.array_equal(np.array([both[o] for o in outs], dtype=np.int64),
                          np.array([first[o] for o in outs], dtype=np.int64) + added)


# ------------------------------------------------------------------ memory and arithmetic hygiene of the oracle

def test_oracle_under_address_and_undefined_behaviour_sanitizers():
    """Every oracle entry point on small, exactly sized buffers in a build with -fsanitize=address,undefined
    (oracle/sanitize_check.cpp): an access outside a buffer, a signed overflow or an invalid shift aborts the run."""
    import shutil
    if shutil.which("g++") is None:
        pytest.skip("no host compiler")
    from oracle import build_oracle
    assert build_oracle.sanitize() == 0


def test_wider_probability_grids_compare_the_top_bits_of_the_32_bit_uniform(orc):
    """prob_bits = 8..22 (Sect. 4.4; suppl. "Stochastic multiplier": a k_p-bit comparator): the rounded p is compared
    with the top k_p bits of the sample's 32-bit uniform, B = [u < P 2^(32 - k_p)]: only those bits decide, the
    threshold is strict, all 2^8 top bytes give the exact mean, and the stream is the 32-bit one (four samples per
    generator block), not the 7-bit one."""
    w = np.array([[1.25, -0.87890625]], dtype=np.float32)      # p = 64/256 ; 0.87890625 = (1/2)(1 + 194.5/256): tie -> 194
    x = np.array([[5, -9]], dtype=np.int8)
    q = orc.QWeights(w, x_absmax=16, s_max=1, prob_bits=8)
    assert list(q.p[0] * 256) == [64.0, 194.0]
    unit = 2.0 ** -q.e_min
    total = 0
    for a in range(256):
        row = []
        for b in range(256):
            lo_bits = (a * 7919 + b * 104729) & 0xFFFFFF          # the low 24 bits must not matter
            acc, _ = orc.linear(q, x, 1, u_table=np.array([(a << 24) | lo_bits, (b << 24) | (lo_bits ^ 0xABCDEF)], dtype=np.uint32))
            row.append(int(acc[0, 0]))
        total += sum(row)
        if a in (63, 64):                                         # strict: P = 64 means top byte 0..63
            first = 5 * unit * (2 if a < 64 else 1)
            assert row[255] == first + (-9) * (-0.5) * unit       # b = 255: never below
    assert total == 256 * 256 * (5 * 1.25 * unit + (-9) * -(0.5 * (1 + 194 / 256)) * unit)
    # the generator stream is the 32-bit one
    one = orc.QWeights(np.array([[1.5]], np.float32), x_absmax=1, s_max=16, prob_bits=8, exp_bits=1)
    xs = np.array([[1]], np.int8)
    for seed in range(5):
        acc, _ = orc.linear(one, xs, 16, seed=seed, layer_id=2)
        ones = sum(1 for s_ in range(16) if orc.uniform(seed, 2, 0, 0, s_) < (1 << 31))
        assert int(acc[0, 0]) == (16 + ones) << int(one.shift[0, 0])
    # exact p (23 bits) is the same rule with P = the mantissa
    full = orc.QWeights(np.array([[1.5]], np.float32), x_absmax=1, s_max=16, prob_bits=23, exp_bits=1)
    assert np.array_equal(orc.linear(full, xs, 16, seed=3, layer_id=2)[0], orc.linear(one, xs, 16, seed=3, layer_id=2)[0])
