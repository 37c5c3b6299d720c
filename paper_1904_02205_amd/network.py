"""A ResNet-18-shaped network run end to end through the C-ABI library: every convolution and the
classifier are stochastically binarized layers (Sect. 3.1), the affine map of the folded batch
normalisation (Sect. 3, Eq. 2) is the mult/bias of the layer call, and the glue between layers (ReLU,
requantisation to 8-bit activations, residual addition, max- and average-pooling; suppl. "ReLU,
Batch-Norm, and Pooling") runs in the library's glue kernels.  Nothing is computed in Python or PyTorch:
this file only orders the calls and owns the device buffers.

Sample budgets: either one sample count S for the whole network, or a per-pixel budget map at any
resolution, which is resampled to the output resolution of every convolution (Sect. 4.5: the regions
apply to the activations of every layer); the classifier then uses `s_fc` samples.
"""
import numpy as np
import torch

from . import psb
from . import resnet_synth as rs


class ResNet18:
    def __init__(self, net: rs.Net, s_max=16, prob_bits=23, seed=3, device="cuda"):
        self.net, self.seed, self.device, self.s_max = net, seed, device, s_max
        self.q, self.mult, self.bias = [], [], []
        self.names = [s.name for s in net.specs]
        step_in = self._input_steps()
        for i, sp in enumerate(net.specs):
            w = torch.from_numpy(net.weights[i]).to(device)
            q = psb.Weights(w, x_absmax=127, s_max=s_max, prob_bits=prob_bits)
            # 2^e_min * step is exact (a power of two times a binary32 number); one rounded product with the scale
            unit = np.float32(np.float32(step_in[i]) * np.float32(2.0) ** q.e_min)
            self.q.append(q)
            self.mult.append(torch.from_numpy((net.ch_scale[i] * unit).astype(np.float32)).to(device))
            self.bias.append(torch.from_numpy(net.ch_bias[i]).to(device))
        self.x0 = torch.from_numpy(net.x0).to(device)
        self.record_inputs = False      # benchmarks: keep the input tensor of every layer of the last pass
        self.inputs = {}
        self._levels = None             # budget values of the pass that is running, if the caller gave them

    def _input_steps(self):
        """Real value of one integer step of each layer's input activations."""
        steps = []
        for i, name in enumerate(self.names):
            if name == "conv1":
                steps.append(rs.STEP_INPUT)
            elif name.endswith("c2"):
                steps.append(rs.STEP_RELU)
            elif name.startswith("s1b0"):
                steps.append(rs.STEP_RELU)          # straight after the max-pool
            else:
                steps.append(rs.STEP_BLOCK)         # block inputs and the classifier
        return steps

    def _conv_requant(self, i, x, S, budget, shared, inv_step, res_f32=None, res_i8=None, res_step=0.0):
        """Convolution i with ReLU, residual and requantisation fused into its epilogue: int8 activations."""
        sp = self.net.specs[i]
        if self.record_inputs:
            self.inputs[i] = x
        bt = None
        if budget is not None:
            oh = (x.shape[2] + 2 * sp.pad - sp.k) // sp.stride + 1
            bt = psb.budget_resample(budget, oh, oh)
            if shared and self._levels is not None:
                psb.shared_budget_levels(self._levels)      # for this call: it need not read the values back
        return psb.conv2d_requant(self.q[i], x, inv_step, S=None if bt is not None else S, budget_to=bt,
                                  stride=(sp.stride, sp.stride), pad=(sp.pad, sp.pad), seed=self.seed, layer_id=i,
                                  res_f32=res_f32, res_i8=res_i8, res_step=res_step, mult=self.mult[i],
                                  bias=self.bias[i], shared=shared, want_acc=False)

    def _conv(self, i, x, S, budget, shared):
        sp = self.net.specs[i]
        if self.record_inputs:
            self.inputs[i] = x
        n, _, h, w = x.shape
        oh = (h + 2 * sp.pad - sp.k) // sp.stride + 1
        y = torch.empty((n, sp.cout, oh, oh), dtype=torch.float32, device=self.device)
        acc = torch.empty((n, sp.cout, oh, oh), dtype=torch.int32, device=self.device)
        kw = dict(stride=(sp.stride, sp.stride), pad=(sp.pad, sp.pad), seed=self.seed, layer_id=i, acc=acc, y=y,
                  mult=self.mult[i], bias=self.bias[i], shared=shared)
        if budget is None:
            psb.conv2d(self.q[i], x, S, **kw)
        else:
            bt = psb.budget_resample(budget, oh, oh)
            if shared and self._levels is not None:
                psb.shared_budget_levels(self._levels)
            psb.conv2d_progressive(self.q[i], x, bt, None, **kw)
        return y

    def _chain_call(self, i, x, x_shape, S, inv_step, layout, budget=None, maps=None, **kw):
        """Convolution i of a chained pass: uniform S, or (budget given) the budget map resampled to the layer's
        output resolution with its values rounded down to self._levels - all sample segments in one launch."""
        sp = self.net.specs[i]
        common = dict(stride=(sp.stride, sp.stride), pad=(sp.pad, sp.pad), seed=self.seed, layer_id=i,
                      mult=self.mult[i], bias=self.bias[i], layout=layout, **kw)
        if budget is None:
            return psb.conv2d_shared_requant_blocked(self.q[i], x, x_shape, inv_step, S, **common)
        oh = (x_shape[2] + 2 * sp.pad - sp.k) // sp.stride + 1
        if oh not in maps:                       # one resampled map per resolution and pass
            maps[oh] = psb.budget_resample(budget, oh, oh)
        return psb.conv2d_shared_budget_requant_blocked(self.q[i], x, x_shape, inv_step, maps[oh], self._levels, **common)

    def _forward_chain(self, S, collect, budget=None, s_fc=None):
        """Shared-filter pass as one chain on the GPU: every filter of the pass is sampled in one launch up front
        (with a budget map: the filters of every segment between its levels), and between the convolutions the
        activations stay in the blocked channels-last layout that the matrix-core kernel reads in place (no layout
        copies).  Same integers as the layer-by-layer pass."""
        def keep(t, shape=None):
            if collect is None:
                return
            if shape is not None:        # diagnostic copy back to [N, C, H, W]
                n, c, h, w = shape
                t = t.permute(0, 2, 4, 1, 3).reshape(n, -1, h, w)[:, :c].contiguous()
            collect.append(t)
        inv_relu, inv_block = float(np.float32(1.0 / rs.STEP_RELU)), float(np.float32(1.0 / rs.STEP_BLOCK))
        n_layers = len(self.q)
        maps = {}
        bkw = dict(budget=budget, maps=maps)
        if budget is None:
            psb.shared_prepare_filters(self.q, S, [self.seed] * n_layers, list(range(n_layers)))
        else:
            psb.shared_prepare_filters_levels(self.q[:-1], self._levels, [self.seed] * (n_layers - 1),
                                              list(range(n_layers - 1)))
        # the first convolution reads the network input as it is and writes the blocked layout; the pooling and
        # every convolution after it read and write that layout
        sp = self.net.specs[0]
        oh = (self.x0.shape[2] + 2 * sp.pad - sp.k) // sp.stride + 1
        shape = (self.x0.shape[0], sp.cout, oh, oh)
        a = self._chain_call(0, self.x0, tuple(self.x0.shape), S, inv_relu, psb.BLOCKED_OUT, **bkw)
        keep(a, shape)
        a = psb.maxpool2d_i8_blocked(a, shape, (3, 3), (2, 2), (1, 1))
        shape = (shape[0], shape[1], (oh + 2 - 3) // 2 + 1, (oh + 2 - 3) // 2 + 1)
        keep(a, shape)
        blocked = True                              # logical [N, C, H, W] of `a` is `shape`
        step_a = rs.STEP_RELU
        i = 1
        B_IN, B_OUT, B_RES = psb.BLOCKED_IN, psb.BLOCKED_OUT, psb.BLOCKED_RES
        while self.names[i] != "fc":
            has_sc = self.names[i + 2].endswith("sc")
            last = self.names[i + (3 if has_sc else 2)] == "fc"
            sp = self.net.specs[i]
            oh = (shape[2] + 2 * sp.pad - sp.k) // sp.stride + 1
            shape1 = (shape[0], sp.cout, oh, oh)
            lin = B_IN if blocked else 0
            a1 = self._chain_call(i, a, shape, S, inv_relu, lin | B_OUT, **bkw)
            keep(a1, shape1)
            lout = 0 if last else B_OUT              # the average pooling reads [N, C, H, W]
            if has_sc:
                ysc = self._chain_call(i + 2, a, shape, S, 0.0, lin, want_x=False, **bkw)
                a = self._chain_call(i + 1, a1, shape1, S, inv_block, B_IN | lout, res_f32=ysc, **bkw)
            else:
                a = self._chain_call(i + 1, a1, shape1, S, inv_block, B_IN | lout | (B_RES if blocked else 0), res_i8=a,
                                     res_step=float(np.float32(step_a)), **bkw)
            shape, blocked = shape1, not last
            keep(a, shape if blocked else None)
            step_a = rs.STEP_BLOCK
            i += 3 if has_sc else 2
        pooled = psb.global_avgpool_requantize(a, 1.0)
        keep(pooled)
        n = pooled.shape[0]
        logits = torch.empty((n, self.net.specs[i].cout), dtype=torch.float32, device=self.device)
        acc = torch.empty((n, self.net.specs[i].cout), dtype=torch.int32, device=self.device)
        psb.linear(self.q[i], pooled, s_fc if s_fc is not None else S, seed=self.seed, layer_id=i, acc=acc, y=logits,
                   mult=self.mult[i], bias=self.bias[i], shared=True)
        return logits

    def forward(self, S=8, budget=None, s_fc=None, shared=False, collect=None, fused=True, chain=None, levels=None):
        """Logits float32 [batch, classes].  collect: optional list that receives every int8 activation tensor.
        fused: requantisation in the epilogue of the layer kernels (default) or as separate glue kernels; the
        activations are the same integers either way.  chain: run a shared-filter pass with a uniform sample count
        as one chain (see _forward_chain); by default whenever that applies.  levels: the values the budget map
        holds, if the caller knows them (nearest-pixel resampling only ever drops values): a shared-filter pass
        then runs as a chain too (every layer takes the levels with its call, all sample segments in one launch), or,
        layer by layer, announces them before every call instead of reading them back from the map."""
        self._levels = None
        if budget is not None and levels is not None:
            self._levels = tuple(sorted({int(v) for v in levels}))
        uniform = budget is None and (s_fc is None or s_fc == S)
        masked = budget is not None and self._levels is not None and len([v for v in self._levels if v > 0]) <= 4
        can_chain = shared and fused and (uniform or masked) and not self.record_inputs
        if chain is None:
            chain = can_chain
        if chain:
            if not can_chain:
                raise ValueError("chain=True needs shared=True, fused=True, and either no budget map and s_fc == S or "
                                 "a budget map with at most four levels given")
            return self._forward_chain(S, collect, budget, s_fc)
        keep = (lambda t: collect.append(t)) if collect is not None else (lambda t: None)
        inv_relu, inv_block = float(np.float32(1.0 / rs.STEP_RELU)), float(np.float32(1.0 / rs.STEP_BLOCK))
        if fused:
            a = self._conv_requant(0, self.x0, S, budget, shared, inv_relu)
        else:
            a = psb.requantize(self._conv(0, self.x0, S, budget, shared), inv_relu)
        keep(a)
        a = psb.maxpool2d_i8(a, (3, 3), (2, 2), (1, 1))
        keep(a)
        step_a = rs.STEP_RELU
        i = 1
        while self.names[i] != "fc":
            has_sc = self.names[i + 2].endswith("sc")
            if fused:
                a1 = self._conv_requant(i, a, S, budget, shared, inv_relu)
                keep(a1)
                if has_sc:
                    a = self._conv_requant(i + 1, a1, S, budget, shared, inv_block,
                                           res_f32=self._conv(i + 2, a, S, budget, shared))
                else:
                    a = self._conv_requant(i + 1, a1, S, budget, shared, inv_block, res_i8=a,
                                           res_step=float(np.float32(step_a)))
            else:
                a1 = psb.requantize(self._conv(i, a, S, budget, shared), inv_relu)
                keep(a1)
                y2 = self._conv(i + 1, a1, S, budget, shared)
                if has_sc:
                    a = psb.requantize(y2, inv_block, res_f32=self._conv(i + 2, a, S, budget, shared))
                else:
                    a = psb.requantize(y2, inv_block, res_i8=a, res_step=float(np.float32(step_a)))
            keep(a)
            step_a = rs.STEP_BLOCK
            i += 3 if has_sc else 2
        pooled = psb.global_avgpool_requantize(a, 1.0)
        keep(pooled)
        if self.record_inputs:
            self.inputs[i] = pooled
        n = pooled.shape[0]
        logits = torch.empty((n, self.net.specs[i].cout), dtype=torch.float32, device=self.device)
        acc = torch.empty((n, self.net.specs[i].cout), dtype=torch.int32, device=self.device)
        psb.linear(self.q[i], pooled, s_fc if s_fc is not None else S, seed=self.seed, layer_id=i, acc=acc, y=logits,
                   mult=self.mult[i], bias=self.bias[i], shared=shared)
        return logits

    def capture(self, S=8, shared=False, budget=None, s_fc=None, levels=None):
        """Record one pass with a uniform sample count into a HIP graph.  Returns (graph, logits): graph.replay()
        reruns the pass (same seed, same bits) into the same logits tensor without any per-launch host work.
        The pass is run once eagerly first, so that every workspace the library allocates on first use exists
        before the capture starts.  A shared-filter pass with a budget map can be captured when its levels are
        given (the map tensor is read at every replay); other passes with a budget map cannot (they read back
        which budget values occur)."""
        kw = dict(S=S, shared=shared, budget=budget, s_fc=s_fc, levels=levels)
        self.forward(**kw)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            logits = self.forward(**kw)
        return graph, logits

    def forward_attention(self, s_lo=8, s_hi=16, shared=False):
        """The two-stage scheme of Sect. 4.5: a low-precision pass everywhere, the entropy mask of the last
        convolutional layer, then the network again with s_hi samples inside the mask and s_lo outside, on all
        layers.  Returns (logits, budget map uint8 [batch, h, w] at the last layer's resolution)."""
        acts = []
        self.forward(S=s_lo, shared=shared, collect=acts)
        last = acts[-2]                                  # output of the last residual block
        _, _, budget = psb.attention_budget(last, float(np.float32(rs.STEP_BLOCK)), s_lo, s_hi)
        return self.forward(budget=budget, s_fc=s_hi, shared=shared, levels=(s_lo, s_hi)), budget
