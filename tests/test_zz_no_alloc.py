"""psb_conv2d_requant_static (the entry point that allocates nothing) against psb_conv2d_requant, through the C-ABI:
same requantised activations and rescaled values, element for element, on two calls in a row, the second with a
smaller input - the static scratch array keeps the first call's contents."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


def _case(psb, torch, rng, shape_w, shape_x, stride, pad, S, budget, seed, layer_id, with_res):
    from paper_1904_02205_amd import synth
    w = torch.from_numpy(synth.he_normal(shape_w, rng)).cuda()
    x = torch.from_numpy(synth.sparse_relu_int8(shape_x, rng)).cuda()
    q = psb.Weights(w, x_absmax=127, s_max=16)
    n, oc = shape_x[0], shape_w[0]
    oh, ow = psb.conv2d_out_dims(q.wshape, (n, shape_x[2], shape_x[3]) + stride + pad)
    mult = torch.from_numpy((rng.random(oc) * 2.0 ** q.e_min * 0.05 + 1e-9).astype(np.float32)).cuda()
    bias = torch.from_numpy(rng.standard_normal(oc).astype(np.float32)).cuda()
    bt = None
    if budget:
        bt = torch.from_numpy(rng.choice([0, 2, 4, 8, 16], size=(n, oh, ow)).astype(np.uint8)).cuda()
    res = None
    if with_res:
        res = torch.from_numpy(rng.integers(0, 128, size=(n, oc, oh, ow)).astype(np.int8)).cuda()
    kw = dict(S=None if budget else S, budget_to=bt, stride=stride, pad=pad, seed=seed, layer_id=layer_id, mult=mult,
              bias=bias, res_i8=res, res_step=0.03)
    y_ref = torch.empty((n, oc, oh, ow), dtype=torch.float32, device="cuda")
    x_ref = psb.conv2d_requant(q, x, 8.0, y=y_ref, want_acc=False, **kw)
    y = torch.full((n, oc, oh, ow), float("nan"), dtype=torch.float32, device="cuda")
    x_out = torch.full((n, oc, oh, ow), -7, dtype=torch.int8, device="cuda")
    psb.conv2d_requant_static(q, x, 8.0, x_out, y=y, **kw)
    torch.cuda.synchronize()
    assert torch.equal(x_out, x_ref), "requantised activations differ"
    assert torch.equal(y, y_ref), "rescaled values differ"
    assert int((x_out != 0).sum()) > 0
    return q


def test_static_entry_point_matches_the_allocating_one():
    import torch
    from paper_1904_02205_amd import psb
    psb.lib()
    psb.set_mapping(psb.MAPPING_AUTO)
    rng = np.random.default_rng(91)
    # a split tap reduction (K = 576: nine chunks, partial sums meet in the static accumulators), then a smaller
    # input, then a budget map, a single-chunk layer (K = 48) and a layer of the product-list kernel (depthwise)
    keep = [_case(psb, torch, rng, (64, 64, 3, 3), (2, 64, 20, 20), (1, 1), (1, 1), 16, False, 11, 1, True)]
    keep.append(_case(psb, torch, rng, (64, 64, 3, 3), (1, 64, 9, 7), (2, 2), (1, 1), 8, False, 12, 2, False))
    keep.append(_case(psb, torch, rng, (128, 32, 3, 3), (2, 32, 12, 10), (1, 1), (1, 1), 0, True, 13, 3, True))
    keep.append(_case(psb, torch, rng, (64, 48, 1, 1), (3, 48, 6, 6), (1, 1), (0, 0), 4, False, 14, 4, False))
    # more than 2^20 outputs: the tiled pass from the static partial sums to the outputs
    keep.append(_case(psb, torch, rng, (64, 16, 3, 3), (2, 16, 102, 100), (1, 1), (1, 1), 8, False, 15, 5, True))
    # the limit is checked on the host: one output element too many launches nothing
    q = keep[0]
    n = psb.STATIC_MAX_OUTPUTS // (64 * 64 * 64) + 1
    x = torch.zeros((n, 64, 64, 64), dtype=torch.int8, device="cuda")
    x_out = torch.zeros((n, 64, 64, 64), dtype=torch.int8, device="cuda")
    with pytest.raises(psb.PsbError) as ei:
        psb.conv2d_requant_static(q, x, 1.0, x_out, S=8, pad=(1, 1))
    assert ei.value.code == psb.ERR_TOO_LARGE
    psb.conv2d_requant_static(q, x[:n - 1], 1.0, x_out[:n - 1], S=8, pad=(1, 1))      # exactly the limit
    torch.cuda.synchronize()
    # the limit counts the channels rounded up to whole blocks of 64: 96 channels take the room of 128
    q96 = psb.Weights(torch.from_numpy((rng.standard_normal((96, 64, 3, 3)) * 0.05).astype(np.float32)).cuda(), s_max=8)
    rows = psb.STATIC_MAX_OUTPUTS // (128 * 256)
    x = torch.zeros((1, 64, rows + 1, 256), dtype=torch.int8, device="cuda")
    x_out = torch.zeros((1, 96, rows + 1, 256), dtype=torch.int8, device="cuda")
    with pytest.raises(psb.PsbError) as ei:
        psb.conv2d_requant_static(q96, x, 1.0, x_out, S=8, pad=(1, 1))
    assert ei.value.code == psb.ERR_TOO_LARGE
    psb.conv2d_requant_static(q96, x[:, :, :rows].contiguous(), 1.0, x_out[:, :, :rows].contiguous(), S=8, pad=(1, 1))
    torch.cuda.synchronize()
