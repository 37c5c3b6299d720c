"""The ResNet-18-shaped network of resnet_synth, run end to end on the CPU oracle (tests only).

Written independently of the GPU driver: it shares the network description and the input arrays with it,
and nothing else."""
import numpy as np

from paper_1904_02205_amd import resnet_synth as rs


def _steps(names):
    out = []
    for name in names:
        if name == "conv1" or name.endswith("c2") or name.startswith("s1b0"):
            out.append(rs.STEP_RELU)
        else:
            out.append(rs.STEP_BLOCK)
    return out


class OracleResNet18:
    def __init__(self, orc, net, s_max=16, prob_bits=23, seed=3):
        self.orc, self.net, self.seed, self.s_max = orc, net, seed, s_max
        self.names = [s.name for s in net.specs]
        self.q = [orc.QWeights(w.reshape(w.shape[0], -1), x_absmax=127, s_max=s_max, prob_bits=prob_bits)
                  for w in net.weights]
        self.mult = []
        for i, st in enumerate(_steps(self.names)):
            unit = np.float32(st) * np.float32(2.0) ** self.q[i].e_min
            self.mult.append((net.ch_scale[i] * np.float32(unit)).astype(np.float32))

    def _conv(self, i, x, S, budget, shared):
        sp, orc = self.net.specs[i], self.orc
        ws = (sp.cout, sp.cin, sp.k, sp.k, 1)
        stride, pad = (sp.stride, sp.stride), (sp.pad, sp.pad)
        bt = None
        if budget is not None:
            oh, ow = orc.out_hw(x.shape[2], x.shape[3], sp.k, sp.k, stride, pad)
            bt = orc.budget_resample(budget, oh, ow)
        kw = dict(S=None if bt is not None else S, s_max=self.s_max, budget_to=bt, seed=self.seed, layer_id=i)
        if shared:
            acc, over = orc.conv2d_shared(self.q[i], ws, x, stride, pad, **kw)
        else:
            acc, over, _ = orc.conv2d(self.q[i], ws, x, stride, pad, **kw)
        assert over == 0
        return orc.rescale(acc, self.q[i].e_min, S=None if bt is not None else S, s_max=self.s_max, budget_to=bt,
                           mult=self.mult[i], bias=self.net.ch_bias[i])

    def forward(self, S=8, budget=None, s_fc=None, shared=False, collect=None):
        orc = self.orc
        keep = (lambda t: collect.append(t)) if collect is not None else (lambda t: None)
        inv_relu, inv_block = np.float32(1.0 / rs.STEP_RELU), np.float32(1.0 / rs.STEP_BLOCK)
        a = orc.requantize(self._conv(0, self.net.x0, S, budget, shared), inv_relu)
        keep(a)
        a = orc.maxpool_i8(a, (3, 3), (2, 2), (1, 1))
        keep(a)
        step_a = np.float32(rs.STEP_RELU)
        i = 1
        while self.names[i] != "fc":
            has_sc = self.names[i + 2].endswith("sc")
            a1 = orc.requantize(self._conv(i, a, S, budget, shared), inv_relu)
            keep(a1)
            y2 = self._conv(i + 1, a1, S, budget, shared)
            if has_sc:
                a = orc.requantize(y2, inv_block, res_f32=self._conv(i + 2, a, S, budget, shared))
            else:
                a = orc.requantize(y2, inv_block, res_i8=a, res_step=step_a)
            keep(a)
            step_a = np.float32(rs.STEP_BLOCK)
            i += 3 if has_sc else 2
        pooled = orc.avgpool_requantize(a, 1.0)
        keep(pooled)
        n, c = pooled.shape
        s = s_fc if s_fc is not None else S
        x = pooled.reshape(n, c, 1, 1)
        if shared:
            acc, over = orc.conv2d_shared(self.q[i], (self.net.specs[i].cout, c, 1, 1, 1), x, S=s, s_max=self.s_max,
                                          seed=self.seed, layer_id=i)
        else:
            acc, over, _ = orc.conv2d(self.q[i], (self.net.specs[i].cout, c, 1, 1, 1), x, S=s, s_max=self.s_max,
                                      seed=self.seed, layer_id=i)
        assert over == 0
        y = orc.rescale(acc, self.q[i].e_min, S=s, s_max=self.s_max, mult=self.mult[i], bias=self.net.ch_bias[i])
        return y.reshape(n, -1)

    def forward_attention(self, s_lo=8, s_hi=16, shared=False):
        acts = []
        self.forward(S=s_lo, shared=shared, collect=acts)
        ent, mean, budget = self.orc.attention_budget(acts[-2], np.float32(rs.STEP_BLOCK), s_lo, s_hi)
        return self.forward(budget=budget, s_fc=s_hi, shared=shared), budget, ent, mean
