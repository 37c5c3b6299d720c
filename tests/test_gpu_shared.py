"""Shared-filter mode (Eq. numbersystem:simulation) on the GPU vs the CPU oracle: the sampled integer filter
and the layers built on it (int8 matrix cores for groups = 1, direct kernel otherwise).  Bit-exact."""
import numpy as np
import pytest

import helpers
from paper_1904_02205_amd import synth
from test_gpu_parity import _layer

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def psb():
    import torch
    assert torch.cuda.is_available()
    from paper_1904_02205_amd import psb as m
    m.lib()
    yield m
    m.set_mapping(m.MAPPING_AUTO)


@pytest.mark.parametrize("prob_bits", [23, 4, 7])
def test_sampled_filter_matches_oracle(psb, orc, prob_bits):
    rng = np.random.default_rng(800 + prob_bits)
    L = _layer(rng, 1, 20, 70, 5, 3, pad=1, S=32, s_max=48, prune=0.3)
    qo = helpers.oracle_quantize(orc, L, prob_bits=prob_bits)
    qg = helpers.gpu_quantize(psb, L, prob_bits=prob_bits)
    for a, b in ((0, 16), (0, 1), (0, 48), (3, 4), (5, 37), (16, 32)):
        ref = orc.sample_filter(qo, seed=L.seed, layer_id=L.layer_id, sample_from=a, sample_to=b)
        got = psb.sample_filter(qg, b, a, seed=L.seed, layer_id=L.layer_id).cpu().numpy()
        assert np.array_equal(got.astype(np.int64), ref), (a, b)
    for a, b in ((-1, 4), (4, 4), (5, 3), (0, 49)):
        with pytest.raises(psb.PsbError) as ei:
            psb.sample_filter(qg, b, a)
        assert ei.value.code == psb.ERR_VALUE


def _cases():
    rng = np.random.default_rng(900)
    c = []
    both = (0, 1)             # 0: matrix cores for groups = 1; 1: direct kernel
    c.append(("linear_small", _layer(rng, 5, 37, 9, 1, 1, S=8, xkind="u4", std=0.05), both))
    c.append(("linear_ragged", _layer(rng, 67, 130, 100, 1, 1, S=5, xkind="signed", std=0.05), both))
    c.append(("conv3x3_c20_oc70", _layer(rng, 2, 20, 70, (9, 11), 3, pad=1, S=8), both))
    c.append(("conv3x3_c64", _layer(rng, 1, 64, 64, 14, 3, pad=1, S=16), both))
    c.append(("conv3x3_c96_signed", _layer(rng, 1, 96, 33, 6, 3, pad=1, S=32, xkind="signed"), both))
    c.append(("conv7x7_s2_p3_c3", _layer(rng, 2, 3, 16, (23, 19), 7, stride=2, pad=3, S=8, xkind="signed"), both))
    c.append(("conv1x1_s2", _layer(rng, 2, 24, 40, 9, 1, stride=2, S=4), both))
    c.append(("conv_rect_kernel", _layer(rng, 1, 6, 12, (6, 8), (2, 3), stride=(1, 2), pad=(0, 2), S=3), both))
    c.append(("conv_s1", _layer(rng, 1, 5, 7, 5, 3, pad=1, S=1), both))
    c.append(("conv_pad3_tiny_image", _layer(rng, 1, 4, 8, 2, 3, pad=3, S=4), both))
    c.append(("conv_wide_row", _layer(rng, 1, 8, 32, (3, 150), 3, pad=1, S=8), both))
    c.append(("pruned_pointwise", _layer(rng, 2, 96, 40, 5, 1, S=16, prune=0.9), both))
    c.append(("s255", _layer(rng, 1, 3, 8, 4, 3, pad=1, S=255, std=0.01), both))
    c.append(("s12_three_generator_blocks", _layer(rng, 2, 40, 48, 10, 3, pad=1, S=12), both))
    c.append(("deep_reduction_few_pixels", _layer(rng, 1, 256, 64, 6, 3, pad=1, S=8), both))      # reduction split 4 ways
    c.append(("deep_linear", _layer(rng, 3, 2048, 40, 1, 1, S=4, xkind="u4", std=0.02), both))     # split 4 ways
    c.append(("row_packed_5x5_c6", _layer(rng, 2, 6, 20, (13, 17), 5, stride=2, pad=2, S=8, xkind="signed"), both))
    c.append(("row_packed_1x3_c10", _layer(rng, 1, 10, 8, (4, 9), (1, 3), pad=(0, 1), S=4), both))
    # more pixel tiles than workgroups fit the chip, short reduction: the persistent variant of the matrix-core kernel
    c.append(("many_tiles_short_reduction", _layer(rng, 1, 16, 40, (370, 372), 3, pad=1, S=4), (0,)))
    c.append(("many_tiles_row_packed", _layer(rng, 1, 3, 33, (530, 540), 5, stride=2, pad=2, S=4, xkind="signed"), (0,)))
    # two half tiles per wave without the persistent variant: many channel blocks, few pixel tiles per block
    c.append(("two_half_tiles_many_blocks", _layer(rng, 1, 32, 250, (100, 120), 3, pad=1, S=4), (0,)))
    # 3 x 3, stride 1, padding 1 with both operands in LDS, in each of its shapes: two teams that split the channel
    # blocks (narrow and wide window), one team (ragged sizes, channel padding), one channel block on a wide image,
    # two half tiles per wave with a tile that crosses an image boundary, and tiles that span many tiny images
    c.append(("window_two_teams", _layer(rng, 2, 128, 64, 14, 3, pad=1, S=8), (0,)))
    c.append(("window_two_teams_wide", _layer(rng, 1, 128, 32, 40, 3, pad=1, S=4), (0,)))
    c.append(("window_ragged", _layer(rng, 3, 64, 40, (13, 11), 3, pad=1, S=8), (0,)))
    c.append(("window_one_block_wide", _layer(rng, 1, 20, 33, (37, 45), 3, pad=1, S=4), (0,)))
    c.append(("window_two_half_tiles", _layer(rng, 2, 32, 480, 50, 3, pad=1, S=4), (0,)))
    c.append(("window_many_small_images", _layer(rng, 40, 128, 32, 4, 3, pad=1, S=8, xkind="signed"), (0,)))
    # ... and a weight-heavy layer (every XCD takes an eighth of the channel blocks instead of the pixel tiles)
    c.append(("window_many_channel_blocks", _layer(rng, 3, 128, 250, 6, 3, pad=1, S=8, xkind="signed"), (0,)))
    c.append(("window_sixteen_channel_blocks", _layer(rng, 2, 64, 512, 9, 3, pad=1, S=4), (0,)))
    c.append(("window_one_pixel_images", _layer(rng, 70, 64, 32, 1, 3, pad=1, S=8, xkind="signed"), (0,)))
    c.append(("window_one_column_images", _layer(rng, 9, 64, 32, (17, 1), 3, pad=1, S=8, xkind="signed"), (0,)))
    c.append(("grouped", _layer(rng, 2, 8, 12, 7, 3, pad=1, groups=4, S=8), (0,)))
    c.append(("depthwise", _layer(rng, 2, 70, 70, 9, 3, pad=1, groups=70, S=16), (0,)))
    # 3 x 3 depthwise layers have a kernel of their own: odd channel count, stride 2, two outputs per input channel
    c.append(("depthwise_s2_odd_channels", _layer(rng, 3, 13, 13, (11, 9), 3, stride=2, pad=1, groups=13, S=8), (0,)))
    c.append(("depthwise_multiplier_2_unpadded", _layer(rng, 1, 10, 20, 8, 3, groups=10, S=4, xkind="signed"), (0,)))
    c.append(("depthwise_many_pixels", _layer(rng, 2, 5, 5, (40, 70), 3, pad=1, groups=5, S=8), (0,)))
    c.append(("depthwise_5x5", _layer(rng, 1, 6, 6, 9, 5, pad=2, groups=6, S=8), (0,)))
    return c


@pytest.mark.parametrize("case", _cases(), ids=lambda c: c[0])
def test_layer_bit_exact(psb, orc, case):
    _, L, mappings = case
    ref, over, _ = helpers.oracle_layer(orc, L, shared=True)
    assert over == 0
    qg = helpers.gpu_quantize(psb, L)
    for m in mappings:
        psb.set_mapping(m)
        acc, _ = helpers.gpu_layer(psb, L, qg, shared=True)
        assert np.array_equal(acc, ref), f"mapping {m}"
        acc, _ = helpers.gpu_layer(psb, L, qg, shared=True)      # workspace reuse: same bits
        assert np.array_equal(acc, ref), f"mapping {m}, second call"
    psb.set_mapping(psb.MAPPING_AUTO)


@pytest.mark.parametrize("planes_case", [
    # few taps and a tiny activation range let the window reach deep: filter values up to 2^30
    ("deep_window", dict(exp_bits=5, x_absmax=1, s_max=2), 2),
    ("one_exponent", dict(exp_bits=1, x_absmax=127, s_max=1), 1),
    ("default", dict(exp_bits=0, x_absmax=127, s_max=16), 16),
], ids=lambda c: c[0])
def test_every_digit_plane_count(psb, orc, planes_case):
    """Filters that need 1, 3 and 4 base-256 digit planes."""
    import torch
    _, kw, S = planes_case
    rng = np.random.default_rng(950)
    w = (rng.standard_normal((40, 4, 1, 1)) * 10.0 ** rng.uniform(-6, 0, size=(40, 4, 1, 1))).astype(np.float32)
    x = rng.integers(-kw["x_absmax"], kw["x_absmax"] + 1, size=(3, 4, 9, 9)).astype(np.int8)
    qo = orc.QWeights(w.reshape(40, -1), **kw)
    qg = psb.Weights(torch.from_numpy(w).cuda(), **kw)
    ref, over = orc.conv2d_shared(qo, (40, 4, 1, 1, 1), x, S=S, seed=8, layer_id=2)
    assert over == 0
    acc = psb.conv2d(qg, torch.from_numpy(x).cuda(), S, seed=8, layer_id=2, shared=True).cpu().numpy()
    assert np.array_equal(acc, ref)
    if planes_case[0] == "deep_window":
        assert np.abs(orc.sample_filter(qo, S, seed=8, layer_id=2)).max() >= 2 ** 24      # really four planes


def test_four_digit_planes_on_a_3x3_layer(psb, orc):
    """The both-operands-in-LDS kernel with four planes, with one team and with two."""
    import torch
    rng = np.random.default_rng(951)
    kw = dict(exp_bits=5, x_absmax=1, s_max=2)
    for c, hw in ((64, 9), (128, 12)):
        w = (rng.standard_normal((40, c, 3, 3)) * 10.0 ** rng.uniform(-6, 0, size=(40, c, 3, 3))).astype(np.float32)
        x = rng.integers(-1, 2, size=(3, c, hw, hw)).astype(np.int8)
        qo = orc.QWeights(w.reshape(40, -1), **kw)
        qg = psb.Weights(torch.from_numpy(w).cuda(), **kw)
        ref, over = orc.conv2d_shared(qo, (40, c, 3, 3, 1), x, (1, 1), (1, 1), S=2, seed=8, layer_id=2)
        assert over == 0
        assert np.abs(orc.sample_filter(qo, 2, seed=8, layer_id=2)).max() >= 2 ** 24      # really four planes
        acc = psb.conv2d(qg, torch.from_numpy(x).cuda(), 2, pad=(1, 1), seed=8, layer_id=2, shared=True).cpu().numpy()
        assert np.array_equal(acc, ref), c


def test_filter_value_between_the_ranges_of_two_and_three_digits(psb, orc):
    """W = 64 * (255 + 255) = 32640 has 15 bits but lies above 127 * 257, the largest two-digit balanced number."""
    import torch
    w = np.full((3, 500), np.nextafter(np.float32(2.0), np.float32(0)), np.float32)
    x = np.random.default_rng(955).integers(-128, 128, size=(4, 500)).astype(np.int8)
    qo = orc.QWeights(w, x_absmax=128, s_max=255)
    assert qo.e_top - qo.e_min == 6
    W = orc.sample_filter(qo, 255, seed=1)
    assert W.max() == 32640
    ref, over = orc.conv2d_shared(qo, (3, 500, 1, 1, 1), x.reshape(4, 500, 1, 1), S=255, seed=1)
    qg = psb.Weights(torch.from_numpy(w).cuda(), x_absmax=128, s_max=255)
    acc = psb.linear(qg, torch.from_numpy(x).cuda(), 255, seed=1, shared=True).cpu().numpy()
    assert over == 0 and np.array_equal(acc, ref.reshape(4, 3))


def test_prob_bits_and_seed(psb, orc):
    rng = np.random.default_rng(960)
    L = _layer(rng, 2, 32, 64, 8, 3, pad=1, S=16)
    qo = helpers.oracle_quantize(orc, L, prob_bits=4)
    qg = helpers.gpu_quantize(psb, L, prob_bits=4)
    ref, _, _ = helpers.oracle_layer(orc, L, qo, shared=True)
    acc, _ = helpers.gpu_layer(psb, L, qg, shared=True)
    assert np.array_equal(acc, ref)
    L2 = synth.Layer("t", L.w, L.x, pad=L.pad, S=16, s_max=16, seed=L.seed + 1, layer_id=L.layer_id)
    ref2, _, _ = helpers.oracle_layer(orc, L2, qo, shared=True)
    acc2, _ = helpers.gpu_layer(psb, L2, qg, shared=True)
    assert np.array_equal(acc2, ref2) and not np.array_equal(acc2, acc)
    per_product, _ = helpers.gpu_layer(psb, L, qg)
    assert not np.array_equal(per_product, acc)                   # a different estimator


@pytest.mark.parametrize("mapping", [0, 1])
def test_progressive_bit_exact_and_incremental(psb, orc, mapping):
    rng = np.random.default_rng(970)
    L = _layer(rng, 3, 12, 70, (9, 8), 3, pad=1, S=32, s_max=32)
    oh, ow = L.out_hw
    to = rng.choice([0, 1, 2, 3, 4, 7, 8, 16, 31, 32, 40], size=(3, oh, ow)).astype(np.uint8)   # 40 is clamped to 32
    qo = helpers.oracle_quantize(orc, L)
    ref, over, _ = helpers.oracle_layer(orc, L, qo, budget_to=to, shared=True)
    assert over == 0
    psb.set_mapping(mapping)
    qg = helpers.gpu_quantize(psb, L)
    acc, _ = helpers.gpu_layer(psb, L, qg, budget_to=to, shared=True)
    assert np.array_equal(acc, ref)
    for m in (8, 5):
        first = np.minimum(to, m).astype(np.uint8)
        a1, _ = helpers.gpu_layer(psb, L, qg, budget_to=first, shared=True)
        r1, _, _ = helpers.oracle_layer(orc, L, qo, budget_to=first, shared=True)
        assert np.array_equal(a1, r1)
        a2, _ = helpers.gpu_layer(psb, L, qg, budget_to=to, budget_from=first, acc_in=a1, shared=True)
        assert np.array_equal(a2, ref)
    a3, _ = helpers.gpu_layer(psb, L, qg, budget_to=first, budget_from=to, acc_in=a1, shared=True)   # empty ranges
    assert np.array_equal(a3, a1)
    const, _ = helpers.gpu_layer(psb, L, qg, budget_to=np.full((3, oh, ow), 8, np.uint8), shared=True)
    plain, _ = helpers.gpu_layer(psb, L, qg, S=8, shared=True)
    assert np.array_equal(const, plain)
    psb.set_mapping(psb.MAPPING_AUTO)


def test_progressive_with_many_channel_blocks(psb, orc):
    """Budget segments as masked, accumulating launches of the 3 x 3 kernel with two teams."""
    rng = np.random.default_rng(982)
    L = _layer(rng, 2, 128, 40, 12, 3, pad=1, S=8, s_max=8)
    oh, ow = L.out_hw
    to = rng.choice([0, 2, 4, 8], size=(2, oh, ow)).astype(np.uint8)
    qo, qg = helpers.oracle_quantize(orc, L), helpers.gpu_quantize(psb, L)
    ref, over, _ = helpers.oracle_layer(orc, L, qo, budget_to=to, shared=True)
    assert over == 0
    acc, _ = helpers.gpu_layer(psb, L, qg, budget_to=to, shared=True)
    assert np.array_equal(acc, ref)


def test_progressive_on_a_large_image(psb, orc):
    """Budget segments (masked, accumulating launches) with two half tiles per wave."""
    rng = np.random.default_rng(981)
    L = _layer(rng, 2, 16, 40, (200, 190), 3, pad=1, S=8, s_max=8)
    oh, ow = L.out_hw
    to = rng.choice([0, 2, 4, 8], size=(2, oh, ow)).astype(np.uint8)
    qo, qg = helpers.oracle_quantize(orc, L), helpers.gpu_quantize(psb, L)
    ref, over, _ = helpers.oracle_layer(orc, L, qo, budget_to=to, shared=True)
    assert over == 0
    acc, _ = helpers.gpu_layer(psb, L, qg, budget_to=to, shared=True)
    assert np.array_equal(acc, ref)


def test_activation_pointer_alignment(psb, orc):
    """The layout copy moves 32-bit words when the image plane and the pointer allow it: same integers at any
    byte offset of the input tensor, for planes that are and are not multiples of four bytes."""
    import torch
    rng = np.random.default_rng(983)
    for hw in ((20, 18), (9, 7)):
        L = _layer(rng, 2, 40, 48, hw, 3, pad=1, S=8)
        qo, qg = helpers.oracle_quantize(orc, L), helpers.gpu_quantize(psb, L)
        ref, over, _ = helpers.oracle_layer(orc, L, qo, shared=True)
        assert over == 0
        flat = torch.from_numpy(L.x).reshape(-1)
        for offset in (0, 1, 2, 4):
            buf = torch.zeros(flat.numel() + 8, dtype=torch.int8, device="cuda")
            buf[offset:offset + flat.numel()] = flat.cuda()
            x = buf[offset:offset + flat.numel()].view(L.x.shape)
            acc = psb.conv2d(qg, x, L.S, stride=L.stride, pad=L.pad, seed=L.seed, layer_id=L.layer_id, shared=True)
            assert np.array_equal(acc.cpu().numpy(), ref), (hw, offset)


def test_announced_budget_levels(psb, orc):
    """Budget values announced by the caller (for its next call) instead of read back from the map: same integers
    (exact set, a superset, values above s_max), for the matrix-core and the direct kernel, with and without a
    budget_from map; without the read-back the call can be captured into a HIP graph."""
    import torch
    rng = np.random.default_rng(984)
    for groups in (1, 4):
        L = _layer(rng, 2, 16, 40, (12, 9), 3, pad=1, groups=groups, S=16, s_max=16)
        oh, ow = L.out_hw
        to = rng.choice([4, 8, 16], size=(2, oh, ow)).astype(np.uint8)
        qo, qg = helpers.oracle_quantize(orc, L), helpers.gpu_quantize(psb, L)
        ref, over, _ = helpers.oracle_layer(orc, L, qo, budget_to=to, shared=True)
        assert over == 0
        try:
            for levels in ((4, 8, 16), (16, 4, 8, 2, 12), (4, 8, 200)):          # 200 clamps to s_max = 16
                psb.shared_budget_levels(levels)
                acc, _ = helpers.gpu_layer(psb, L, qg, budget_to=to, shared=True)
                assert np.array_equal(acc, ref), (groups, levels)
            first = np.minimum(to, 8).astype(np.uint8)
            psb.shared_budget_levels((4, 8))
            a1, _ = helpers.gpu_layer(psb, L, qg, budget_to=first, shared=True)
            psb.shared_budget_levels((4, 8, 16))
            a2, _ = helpers.gpu_layer(psb, L, qg, budget_to=to, budget_from=first, acc_in=a1, shared=True)
            assert np.array_equal(a2, ref)
            # captured: replays give the same integers
            x = torch.from_numpy(L.x).cuda()
            bt = torch.from_numpy(to).cuda()
            acc_t = torch.zeros((2, 40, oh, ow), dtype=torch.int32, device="cuda")
            psb.conv2d_progressive(qg, x, bt, stride=L.stride, pad=L.pad, seed=L.seed, layer_id=L.layer_id, acc=acc_t,
                                   shared=True)
            torch.cuda.synchronize()
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph):
                psb.shared_budget_levels((4, 8, 16))          # an announcement is for the next call only
                psb.conv2d_progressive(qg, x, bt, stride=L.stride, pad=L.pad, seed=L.seed, layer_id=L.layer_id,
                                       acc=acc_t, shared=True)
            for _ in range(3):
                acc_t.fill_(-1)
                graph.replay()
                torch.cuda.synchronize()
                assert np.array_equal(acc_t.cpu().numpy(), ref)
        finally:
            psb.shared_budget_levels(None)
    acc, _ = helpers.gpu_layer(psb, L, qg, budget_to=to, shared=True)       # default path again
    assert np.array_equal(acc, ref)


def test_progressive_depthwise(psb, orc):
    """Budget segments through the 3 x 3 depthwise kernel: masked, accumulating launches; refinement in two calls."""
    rng = np.random.default_rng(982)
    L = _layer(rng, 2, 9, 9, (17, 12), 3, pad=1, groups=9, S=16, s_max=16)
    oh, ow = L.out_hw
    to = rng.choice([0, 2, 4, 8, 16], size=(2, oh, ow)).astype(np.uint8)
    qo, qg = helpers.oracle_quantize(orc, L), helpers.gpu_quantize(psb, L)
    ref, over, _ = helpers.oracle_layer(orc, L, qo, budget_to=to, shared=True)
    assert over == 0
    acc, _ = helpers.gpu_layer(psb, L, qg, budget_to=to, shared=True)
    assert np.array_equal(acc, ref)
    first = np.minimum(to, 4).astype(np.uint8)
    a1, _ = helpers.gpu_layer(psb, L, qg, budget_to=first, shared=True)
    a2, _ = helpers.gpu_layer(psb, L, qg, budget_to=to, budget_from=first, acc_in=a1, shared=True)
    assert np.array_equal(a2, ref)


def test_activation_tensor_beyond_the_offset_range_is_refused(psb):
    """The matrix-core kernel addresses the channels-last activations with 32-bit offsets: a tensor that
    reaches 2 GiB in that layout is an error, not a launch."""
    import torch
    w = torch.full((1, 1, 3, 3), 0.25, device="cuda")
    q = psb.Weights(w, x_absmax=127, s_max=8)
    x = torch.zeros((1, 1, 8192, 8192), dtype=torch.int8, device="cuda")    # 8192 * 8192 * 32 bytes once blocked
    acc = torch.empty((1, 1, 8192, 8192), dtype=torch.int32, device="cuda")
    with pytest.raises(psb.PsbError) as ei:
        psb.conv2d(q, x, 8, pad=(1, 1), acc=acc, shared=True)
    assert ei.value.code == psb.ERR_TOO_LARGE
    ok = psb.conv2d(q, x[:, :, :64, :64].contiguous(), 8, pad=(1, 1), shared=True)
    assert int(ok.abs().max()) == 0


@pytest.mark.parametrize("mapping", [0, 1])
def test_rescale_matches_oracle(psb, orc, mapping):
    rng = np.random.default_rng(980)
    L = _layer(rng, 2, 10, 40, 6, 3, pad=1, S=8, s_max=16)
    oc = 40
    mult = (rng.uniform(0.5, 2.0, size=oc) * 2.0 ** -9).astype(np.float32)
    bias = rng.standard_normal(oc).astype(np.float32)
    qo = helpers.oracle_quantize(orc, L)
    qg = helpers.gpu_quantize(psb, L)
    psb.set_mapping(mapping)
    ref, _, _ = helpers.oracle_layer(orc, L, qo, shared=True)
    acc, y = helpers.gpu_layer(psb, L, qg, want_y=True, mult=mult, bias=bias, shared=True)
    assert np.array_equal(acc, ref)
    assert np.array_equal(y, orc.rescale(ref, qo.e_min, S=8, s_max=16, mult=mult, bias=bias))
    oh, ow = L.out_hw
    to = rng.choice([0, 2, 8, 16], size=(2, oh, ow)).astype(np.uint8)
    refp, _, _ = helpers.oracle_layer(orc, L, qo, budget_to=to, shared=True)
    accp, yp = helpers.gpu_layer(psb, L, qg, budget_to=to, want_y=True, shared=True)
    assert np.array_equal(accp, refp)
    assert np.array_equal(yp, orc.rescale(refp, qo.e_min, s_max=16, budget_to=to))
    psb.set_mapping(psb.MAPPING_AUTO)
