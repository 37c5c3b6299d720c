"""A synthetic ResNet-18-shaped network: random weights, a random input batch and a synthetic batch
normalisation, for chaining the layers end to end.

The paper runs pretrained ImageNet classifiers with batch normalisation folded into per-channel affine
maps (Sect. 3, Eq. 2; Sect. 4.3); no trained network is available here, so this module draws He-normal
weights and obtains the affine map of every convolution from ONE ordinary floating-point forward pass of
the same random network on the same batch (scale = 1/std, bias = -mean/std of the channel's
pre-activation).  These arrays are inputs: they are handed unchanged to the GPU library's caller and to
the CPU oracle's caller.  Nothing of the method (no sampling, no integer arithmetic, no requantisation
rule) lives here.
"""
from dataclasses import dataclass
from typing import List

import numpy as np

from . import synth

STEP_INPUT = 4.0 / 127.0      # network input and post-ReLU activations: value = integer * 4/127
STEP_RELU = 4.0 / 127.0
STEP_BLOCK = 6.0 / 127.0      # activations after a residual addition


@dataclass
class Net:
    specs: List[synth.NetLayerSpec]     # forward order: conv1, then per block c1, c2 [, sc], ..., fc
    weights: List[np.ndarray]           # float32 OIHW
    ch_scale: List[np.ndarray]          # float32 [oc]: synthetic batch-norm scale (ones for the classifier)
    ch_bias: List[np.ndarray]           # float32 [oc]
    x0: np.ndarray                      # int8 [batch, 3, hw, hw], value = x0 * STEP_INPUT
    batch: int
    hw: int

    def index(self, name: str) -> int:
        return [s.name for s in self.specs].index(name)


def _float_forward(net_specs, weights, x0_real, device="cpu"):
    """Plain floating-point forward pass; returns per-layer (mean, std) of the pre-activations."""
    import torch
    F = torch.nn.functional
    dt = torch.float32 if device != "cpu" else torch.float64
    W = [torch.from_numpy(w).to(device=device, dtype=dt) for w in weights]
    names = [s.name for s in net_specs]
    stats = [None] * len(net_specs)

    def conv_bn(i, a):
        sp = net_specs[i]
        y = F.conv2d(a, W[i], stride=sp.stride, padding=sp.pad)
        mean = y.mean(dim=(0, 2, 3))
        std = y.std(dim=(0, 2, 3), unbiased=False).clamp_min(1e-6)
        stats[i] = (mean.double().cpu().numpy(), std.double().cpu().numpy())
        return (y - mean[None, :, None, None]) / std[None, :, None, None]

    a = torch.from_numpy(x0_real).to(device=device, dtype=dt)
    a = conv_bn(0, a).clamp(0, 4)
    a = F.max_pool2d(a, 3, 2, 1)
    i = 1
    while names[i] != "fc":
        has_sc = i + 2 < len(names) and names[i + 2].endswith("sc")
        y1 = conv_bn(i, a).clamp(0, 4)
        y2 = conv_bn(i + 1, y1)
        short = conv_bn(i + 2, a) if has_sc else a
        a = (y2 + short).clamp(0, 6)
        i += 3 if has_sc else 2
    return stats


def resnet18(batch=2, hw=64, width=32, classes=10, seed=18, device="cpu") -> Net:
    rng = np.random.default_rng(seed)
    specs = synth.resnet18_specs(hw, width, classes)
    weights = [synth.he_normal((sp.cout, sp.cin, sp.k, sp.k), rng) for sp in specs]
    x0 = synth.gaussian_int8((batch, 3, hw, hw), rng)
    stats = _float_forward(specs, weights, x0.astype(np.float64) * STEP_INPUT, device)
    ch_scale, ch_bias = [], []
    for sp, st in zip(specs, stats):
        if st is None:          # classifier: no normalisation
            ch_scale.append(np.ones(sp.cout, np.float32))
            ch_bias.append(np.zeros(sp.cout, np.float32))
        else:
            mean, std = st
            ch_scale.append((1.0 / std).astype(np.float32))
            ch_bias.append((-mean / std).astype(np.float32))
    return Net(specs, weights, ch_scale, ch_bias, x0, batch, hw)
