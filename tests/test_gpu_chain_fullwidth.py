"""The chained shared-filter pass at the width and batch the benchmark times (ResNet-18 shape, 64..512 channels,
batch 32, 224 x 224, S = 8), checked layer by layer against the oracle, teacher-forced: every layer of the oracle is
fed the GPU's previous activation, and compared on all channels of randomly chosen output pixels (corners included)
- shared-filter layer -> rescale -> requantize, with the residual the GPU used.  Pooling layers and the classifier
are compared whole.  (Sect. 4.1 "Setup" and suppl. "Efficient simulation of the forward pass": one sampled filter per
layer and pass.)"""
import numpy as np
import pytest

from paper_1904_02205_amd import resnet_synth as rs

pytestmark = pytest.mark.gpu

PIXELS = 160          # output pixels per layer, each with all its channels: 10,000 .. 82,000 outputs per layer


def _points(rng, n, oc, oh, ow):
    """Flat [N][OC][OH][OW] indices of all channels of PIXELS random pixels, channel-major: [oc][pixel]."""
    total = n * oh * ow
    pix = rng.choice(total, size=min(PIXELS, total), replace=False)
    pix[:4] = [0, ow - 1, total - ow, total - 1]                      # corners of the first and the last image
    pix = np.unique(pix)
    b, r = pix // (oh * ow), pix % (oh * ow)
    pts = (b[None, :] * oc + np.arange(oc)[:, None]) * (oh * ow) + r[None, :]
    return pts.astype(np.int64)                                       # [oc, P]


def test_full_width_chain_teacher_forced(orc):
    import torch
    from paper_1904_02205_amd import network, psb
    psb.lib()
    psb.set_mapping(psb.MAPPING_AUTO)
    S, seed = 8, 3
    net = rs.resnet18(batch=32, hw=224, width=64, classes=1000, device="cuda")
    model = network.ResNet18(net, s_max=S, seed=seed)
    acts = []
    logits = model.forward(S=S, shared=True, collect=acts)            # the chain: blocked layouts, filters up front
    torch.cuda.synchronize()
    acts = [a.cpu().numpy() for a in acts]
    names = [s.name for s in net.specs]
    rng = np.random.default_rng(77)
    inv_relu, inv_block = np.float32(1.0 / rs.STEP_RELU), np.float32(1.0 / rs.STEP_BLOCK)

    def steps(i):
        name = names[i]
        return rs.STEP_RELU if (name == "conv1" or name.endswith("c2") or name.startswith("s1b0")) else rs.STEP_BLOCK

    def layer_at(i, x, pts):
        """Rescaled fp32 values of layer i on input x at the points [oc, P] (oracle only)."""
        sp = net.specs[i]
        q = orc.QWeights(net.weights[i].reshape(sp.cout, -1), x_absmax=127, s_max=S)
        acc, over = orc.conv2d_shared(q, (sp.cout, sp.cin, sp.k, sp.k, 1), x, (sp.stride, sp.stride), (sp.pad, sp.pad),
                                      S=S, s_max=S, seed=seed, layer_id=i, points=pts.ravel())
        assert over == 0
        unit = np.float32(steps(i)) * np.float32(2.0) ** q.e_min
        mult = (net.ch_scale[i] * np.float32(unit)).astype(np.float32)
        y = orc.rescale(acc.reshape(1, sp.cout, -1), q.e_min, S=S, s_max=S, mult=mult, bias=net.ch_bias[i])
        return y.reshape(pts.shape)

    def out_hw(i, h):
        sp = net.specs[i]
        return (h + 2 * sp.pad - sp.k) // sp.stride + 1

    # first convolution and the max-pool
    n = net.x0.shape[0]
    oh = out_hw(0, net.x0.shape[2])
    pts = _points(rng, n, net.specs[0].cout, oh, oh)
    ref = orc.requantize(layer_at(0, net.x0, pts), inv_relu)
    assert np.array_equal(acts[0].ravel()[pts], ref), "conv1"
    assert np.array_equal(acts[1], orc.maxpool_i8(acts[0], (3, 3), (2, 2), (1, 1))), "max-pool"
    a, k, i = acts[1], 2, 1
    step_a = np.float32(rs.STEP_RELU)
    while names[i] != "fc":
        has_sc = names[i + 2].endswith("sc")
        a1, a_out = acts[k], acts[k + 1]
        oh = out_hw(i, a.shape[2])
        oc = net.specs[i].cout
        pts = _points(rng, n, oc, oh, oh)
        assert np.array_equal(a1.ravel()[pts], orc.requantize(layer_at(i, a, pts), inv_relu)), names[i]
        pts = _points(rng, n, oc, oh, oh)
        y2 = layer_at(i + 1, a1, pts)
        if has_sc:
            ref = orc.requantize(y2, inv_block, res_f32=layer_at(i + 2, a, pts))
        else:
            ref = orc.requantize(y2, inv_block, res_i8=a.ravel()[pts], res_step=step_a)
        assert np.array_equal(a_out.ravel()[pts], ref), names[i + 1]
        assert a_out.max() > 0
        a, k = a_out, k + 2
        step_a = np.float32(rs.STEP_BLOCK)
        i += 3 if has_sc else 2
    pooled = acts[k]
    assert np.array_equal(pooled, orc.avgpool_requantize(a, 1.0)), "average pool"
    c = pooled.shape[1]
    sp = net.specs[i]
    q = orc.QWeights(net.weights[i].reshape(sp.cout, -1), x_absmax=127, s_max=S)
    acc, over = orc.conv2d_shared(q, (sp.cout, c, 1, 1, 1), pooled.reshape(n, c, 1, 1), S=S, s_max=S, seed=seed, layer_id=i)
    unit = np.float32(steps(i)) * np.float32(2.0) ** q.e_min
    y = orc.rescale(acc, q.e_min, S=S, s_max=S, mult=(net.ch_scale[i] * np.float32(unit)).astype(np.float32),
                    bias=net.ch_bias[i])
    assert over == 0 and np.array_equal(logits.cpu().numpy(), y.reshape(n, -1)), "classifier"
