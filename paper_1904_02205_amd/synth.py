"""Seeded synthetic inputs shaped like the paper's ImageNet CNN layers.

The paper evaluates pretrained ImageNet classifiers (Sect. 4.3-4.5); neither the
images nor the weights are available, so these tensors stand in for them: same
shapes, He-normal weights, post-ReLU-like sparse int8 activations, a saliency-
blob sample-budget map.  This module is the only code shared by the GPU library's
callers and the CPU oracle's callers, and it contains none of the method's
arithmetic: it only draws inputs.

Every generator takes an explicit numpy Generator; `rng_for(cfg)` gives the
harness seed 1000 + config index.
"""
from dataclasses import dataclass, field
from typing import List, Optional, Tuple

import numpy as np


def rng_for(cfg_index: int) -> np.random.Generator:
    return np.random.default_rng(1000 + cfg_index)


def normal_weights(shape, std, rng) -> np.ndarray:
    return (rng.standard_normal(shape) * std).astype(np.float32)


def he_normal(shape, rng) -> np.ndarray:
    """N(0, 2/fan_in), fan_in = prod(shape[1:]) (OIHW)."""
    fan_in = int(np.prod(shape[1:]))
    return normal_weights(shape, np.sqrt(2.0 / fan_in), rng)


def sparse_relu_int8(shape, rng, zero_frac=0.5, mean=20.0) -> np.ndarray:
    """Half zeros, the rest round(Exp(mean)) clipped to [1,127]: a post-ReLU 8-bit activation."""
    v = np.clip(np.rint(rng.exponential(mean, size=shape)), 1, 127)
    z = rng.random(size=shape) < zero_frac
    v[z] = 0
    return v.astype(np.int8)


def uniform_uint4(shape, rng) -> np.ndarray:
    return rng.integers(0, 16, size=shape).astype(np.int8)


def gaussian_int8(shape, rng) -> np.ndarray:
    """N(0,1) pixels quantised to int8 with step 4/127 (network input)."""
    v = rng.standard_normal(shape)
    return np.clip(np.rint(v * (127.0 / 4.0)), -127, 127).astype(np.int8)


def prune_by_magnitude(w: np.ndarray, frac: float) -> np.ndarray:
    """Zero the `frac` smallest-magnitude weights of the layer (threshold pruning, Sect. 4.4)."""
    a = np.abs(w).ravel()
    n_zero = int(round(frac * a.size))
    if n_zero <= 0:
        return w.copy()
    order = np.argsort(a, kind="stable")
    out = w.copy().ravel()
    out[order[:n_zero]] = 0.0
    return out.reshape(w.shape)


def budget_blob(n, oh, ow, rng, sigma=6.0, levels=(32, 16, 8, 4, 2)) -> np.ndarray:
    """Per-pixel sample budgets: a Gaussian saliency blob at a random centre per image.

    g = exp(-d^2 / (2 sigma^2)); budget = levels[0..4] for g in (0.8,1], (0.6,0.8], (0.4,0.6], (0.2,0.4],
    [0,0.2].
    """
    out = np.zeros((n, oh, ow), dtype=np.uint8)
    yy, xx = np.meshgrid(np.arange(oh), np.arange(ow), indexing="ij")
    for i in range(n):
        cy = int(rng.integers(0, oh))
        cx = int(rng.integers(0, ow))
        g = np.exp(-((yy - cy) ** 2 + (xx - cx) ** 2) / (2.0 * sigma * sigma))
        b = np.full((oh, ow), levels[4], dtype=np.uint8)
        b[g > 0.2] = levels[3]
        b[g > 0.4] = levels[2]
        b[g > 0.6] = levels[1]
        b[g > 0.8] = levels[0]
        out[i] = b
    return out


@dataclass
class Layer:
    """One PSB layer call: weights OIHW (linear: [oc, cin, 1, 1]), activations NCHW (linear: [B, K, 1, 1])."""
    name: str
    w: np.ndarray
    x: np.ndarray
    groups: int = 1
    stride: Tuple[int, int] = (1, 1)
    pad: Tuple[int, int] = (0, 0)
    S: int = 8
    s_max: int = 8
    x_absmax: int = 127
    seed: int = 0
    layer_id: int = 0
    budget_to: Optional[np.ndarray] = None
    linear: bool = False

    @property
    def wshape(self):
        oc, cg, kh, kw = self.w.shape
        return (oc, cg * self.groups, kh, kw, self.groups)

    @property
    def out_hw(self):
        _, _, kh, kw = self.w.shape
        h, w = self.x.shape[2], self.x.shape[3]
        return ((h + 2 * self.pad[0] - kh) // self.stride[0] + 1,
                (w + 2 * self.pad[1] - kw) // self.stride[1] + 1)


def config1(batch=64, k=512, oc=256) -> Layer:
    """Linear 512->256, N(0,0.05^2) weights, uint4 activations, S=8, seed 0."""
    rng = rng_for(1)
    w = normal_weights((oc, k, 1, 1), 0.05, rng)
    x = uniform_uint4((batch, k, 1, 1), rng)
    return Layer("c1_linear", w, x, S=8, s_max=8, x_absmax=15, seed=0, linear=True)


def config2(c=64, hw=56, n=1) -> Layer:
    """3x3 s1 p1 conv, ResNet stage-1 shape, S=16, seed 1."""
    rng = rng_for(2)
    w = he_normal((c, c, 3, 3), rng)
    x = sparse_relu_int8((n, c, hw, hw), rng)
    return Layer("c2_conv3x3", w, x, pad=(1, 1), S=16, s_max=16, seed=1)


def config3(c=128, hw=28, n=8) -> Layer:
    """Progressive 3x3 conv 128->128 @28x28, batch 8, blob budgets from {2,4,8,16,32}, seed 2."""
    rng = rng_for(3)
    w = he_normal((c, c, 3, 3), rng)
    x = sparse_relu_int8((n, c, hw, hw), rng)
    b = budget_blob(n, hw, hw, rng)
    return Layer("c3_progressive", w, x, pad=(1, 1), S=32, s_max=32, seed=2, budget_to=b)


def config5(n=64, c=576, oc=160, hw=14) -> List[Layer]:
    """MobileNet-v2-style block: 90 %-pruned pointwise 576->160 and depthwise 3x3 over 576 channels."""
    rng = rng_for(5)
    w_pw = prune_by_magnitude(he_normal((oc, c, 1, 1), rng), 0.9)
    x_pw = sparse_relu_int8((n, c, hw, hw), rng)
    w_dw = he_normal((c, 1, 3, 3), rng)
    x_dw = sparse_relu_int8((n, c, hw, hw), rng)
    return [Layer("c5_pointwise_pruned", w_pw, x_pw, S=16, s_max=16, seed=4, layer_id=0),
            Layer("c5_depthwise", w_dw, x_dw, groups=c, pad=(1, 1), S=16, s_max=16, seed=4, layer_id=1)]


@dataclass
class NetLayerSpec:
    name: str
    cin: int
    cout: int
    k: int
    stride: int
    pad: int
    hw_in: int


def resnet18_specs(hw=224, width=64, classes=1000) -> List[NetLayerSpec]:
    """The 20 convolutions and the FC layer of a ResNet-18-shaped network, in forward order."""
    specs = [NetLayerSpec("conv1", 3, width, 7, 2, 3, hw)]
    h = (hw + 6 - 7) // 2 + 1          # conv1
    h = (h + 2 - 3) // 2 + 1           # max-pool 3x3 s2 p1
    cin = width
    for stage in range(4):
        cout = width << stage
        for block in range(2):
            s = 2 if (stage > 0 and block == 0) else 1
            specs.append(NetLayerSpec(f"s{stage + 1}b{block}c1", cin, cout, 3, s, 1, h))
            h2 = (h + 2 - 3) // s + 1
            specs.append(NetLayerSpec(f"s{stage + 1}b{block}c2", cout, cout, 3, 1, 1, h2))
            if s == 2:
                specs.append(NetLayerSpec(f"s{stage + 1}b{block}sc", cin, cout, 1, 2, 0, h))
            cin, h = cout, h2
    specs.append(NetLayerSpec("fc", cin, classes, 1, 1, 0, 1))
    return specs


def config4_layers(batch=32, hw=224, width=64, classes=1000) -> List[Layer]:
    """ResNet-18-shaped layer set, each layer with its own synthetic input of the right shape and type.

    Layer inputs are drawn independently (post-ReLU-like int8, Gaussian int8 for the first layer): every
    layer is a full-size, teacher-forced instance of the layer it stands for.  S=8, seed 3,
    layer_id = position in the list.
    """
    rng = rng_for(4)
    layers = []
    for i, sp in enumerate(resnet18_specs(hw, width, classes)):
        w = he_normal((sp.cout, sp.cin, sp.k, sp.k), rng)
        if i == 0:
            x = gaussian_int8((batch, sp.cin, sp.hw_in, sp.hw_in), rng)
        else:
            x = sparse_relu_int8((batch, sp.cin, sp.hw_in, sp.hw_in), rng)
        layers.append(Layer("c4_" + sp.name, w, x, stride=(sp.stride, sp.stride), pad=(sp.pad, sp.pad),
                            S=8, s_max=8, seed=3, layer_id=i, linear=(sp.name == "fc")))
    return layers
